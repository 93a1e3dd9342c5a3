"""MI355X-native SSD (Mamba-2 state space duality) layer core: chunked prefill and the
O(1) cached decode step, as hand-written gfx950 HIP kernels behind a C-ABI library.

``paper_2603_09555_amd.ssd`` is the Python binding (same names as the C entry points);
``paper_2603_09555_amd.inputs`` draws the seeded synthetic workloads.  Nothing is imported
eagerly so that the input generators can be used without the compiled library.
"""
__all__ = ["ssd", "inputs", "build"]
