"""MI355X-native KV-cache codec of Quant VideoGen (semantic-aware smoothing +
progressive residual 2-bit quantization, Sec. 4): encode, decode and decode fused
into attention, as hand-written HIP kernels behind a C ABI.

`binding` wraps the C-ABI library (argument marshalling only); `synth` and
`configs` hold the seeded synthetic workloads.  Importing the package does not
load the GPU library; the first call into `binding` does, and raises if the
library has not been built.
"""
__all__ = ["binding", "configs", "synth"]
