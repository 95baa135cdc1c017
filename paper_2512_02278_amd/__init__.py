"""MI355X-native batched graph beam search (one GPU's partition, resident in HBM).

``ann``     thin ctypes binding over the C-ABI library (libann.so, HIP kernels for gfx950)
``inputs``  seeded synthetic partitions, graphs, queries and exact ground truth
``metrics`` bytes-per-query accounting and the paper's traffic model
"""
