"""MI355X-native implementation of OptiReduce's per-node gradient-bucket path (arXiv 2310.06993):
randomized Hadamard encode, masked aggregation of N workers' shards, decode -- hand-written HIP for
gfx950 behind the C ABI of include/optireduce.h.  `binding` is the ctypes front of that library;
`workloads` generates the seeded synthetic inputs used by tests and the benchmark."""
