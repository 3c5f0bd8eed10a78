"""MI355X-native approximate kNN-graph construction (EFANNA offline path): HIP kernels
behind the C ABI of include/efanna.h, plus a ctypes binding (`efanna`) and seeded
synthetic workloads (`synth`).  Importing the package loads nothing heavy; the binding
and torch are imported on first use of `paper_1609_07228_amd.efanna`."""
