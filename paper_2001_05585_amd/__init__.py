"""libmfreduce: fp16 -> fp32 arithmetic reduction on MI355X (gfx950).

The sum is encoded as chains of R ones-matrix MFMAs with fp32 partials
(the single-pass variant of "GPU Tensor Cores for fast Arithmetic Reductions",
Section 5.2).  All arithmetic runs in the HIP library ``libmfreduce.so``; this
package only marshals arguments (``binding``), builds the library (``build``)
and generates synthetic inputs (``workloads``).
"""
__all__ = ["binding", "build", "workloads"]
