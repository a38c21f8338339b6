"""MI355X-native hot path of Lagom: chunked reduce-copy / gather-copy kernel, bf16 MFMA
GEMM, two-stream overlap runner, overlap cost model and priority-based parameter search.

The native library is loaded lazily by ``paper_2602_20656_amd.binding``; importing this
package (for instance for ``paper_2602_20656_amd.inputs``) touches no GPU code.
"""
