"""CPU oracle for the polar-quantized key-cache path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64/NumPy statement of what the path computes, written from
the paper (Section 3.2 for the encoder and the mid-point dequantizer, Section
3.3 and Appendix A for the query-key product).  It exists to check the HIP
library and to be timed beside it as a CPU baseline.  Only tests, the smoke
check and the benchmark's cpu_baseline leg may import it; the product package
never does, and this package imports nothing from the product.

Modules
  polar.py         pair -> (radius, angle) -> group-wise codes; mid-point dequantizer
  cache_format.py  the packed page layout (an independent write-up of the byte format)
  values.py        token-wise value quantizer (the paper's optional value quantization)
  attention.py     dequantize-then-dot scores, softmax, fp16-V aggregation over a paged cache

Every function is pinned by the CPU tests (closed forms, hand-worked values
under tests/golden/, brute force on tiny inputs, the bits-to-infinity limit);
none is "parity unpinned".
"""
