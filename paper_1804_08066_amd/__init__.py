"""MI355X-native hot path of MQGrad (arXiv 1804.08066): b-bit gradient quantize+pack on the
worker side, fused unpack+de-quantize+average+SGD-update on the server side, plus the host MDP
that picks b.  `mqgrad` is the thin binding over the C-ABI library; `workloads` the synthetic inputs.
"""
__all__ = ["mqgrad", "workloads"]
