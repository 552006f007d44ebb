"""MI355X-native packed variable-length causal attention (forward and backward): the
per-replica hot path of Hydraulis (arXiv 2412.07894), as hand-written HIP kernels for gfx950
behind a C-ABI library.  `paper_2412_07894_amd.binding` is the Python front end of that library;
`paper_2412_07894_amd.workloads` generates the seeded synthetic inputs."""
