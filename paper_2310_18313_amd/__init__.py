"""MI355X (gfx950) implementation of the optimizer-side hot path of FP8-LM (arXiv 2310.18313):
per-tensor auto-scaled FP8 gradient quantisation (Sec. 2.1, Appendix A) and the FP8 Adam step
(Sec. 2.2).  The arithmetic lives in csrc/ behind the C ABI of include/fp8lm.h; `binding` marshals
torch tensors into it; `synth` makes seeded synthetic inputs; `state` bundles the flat buffers."""
