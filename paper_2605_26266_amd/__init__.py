"""MI355X-native quantized-KV chunk attention with Jensen-bias correction.

`paper_2605_26266_amd.binding` wraps the C ABI of libkvq.so (see include/kvq.h);
`paper_2605_26266_amd.workloads` produces the seeded synthetic inputs;
`paper_2605_26266_amd.build` compiles the HIP sources for gfx950.
"""
__all__ = ["binding", "workloads", "build"]
