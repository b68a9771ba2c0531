"""MI355X-native single-GPU hot path of the FlexMoE MoE layer (arXiv 2304.03946).

`binding` exposes the C ABI of libflexmoe.so (HIP kernels for gfx950);
`layer` chains the calls into a forward / backward pass on caller-owned buffers;
`workloads` draws the seeded synthetic inputs.  Importing the package does not
load the library; the first call does, and fails loudly if it is not built.
"""
