"""MI355X-native dense tensor operators (GEMM, batched GEMM, NHWC conv2d) behind a C ABI.

`paper_2505_02146_amd.xp` is the ctypes binding of libxp.so (argument marshalling only);
`paper_2505_02146_amd.inputs` holds the seeded synthetic input generators.
Nothing is imported eagerly so that the generators can be used without the GPU library.
"""
__all__ = ["xp", "inputs", "build"]
