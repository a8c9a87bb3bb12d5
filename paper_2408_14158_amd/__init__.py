"""libhfr: the reduction arithmetic of the HFReduce allreduce (K-way in-order
sum, combine-and-average, bucketed chunk-pipelined reduction) as hand-written
HIP kernels for MI355X behind a C ABI, plus this thin ctypes binding."""
