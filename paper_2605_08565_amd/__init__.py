"""MI355X-native microscaled FP4 quantisation with per-block scale selection.

``paper_2605_08565_amd.mxq`` is the thin Python binding over the C-ABI library ``libmxq.so``
(hand-written HIP kernels for gfx950); ``paper_2605_08565_amd.workloads`` draws the seeded
synthetic inputs.  There is no CPU fallback: the binding raises if the library is missing.
"""
