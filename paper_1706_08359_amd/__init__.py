"""MI355X-native histogram hot path of histogram-based GBDT training (arXiv 1706.08359).

The product is the C-ABI library built from csrc/ (declared in include/gbdt_hist.h);
`binding` is its thin ctypes front end, `synth` draws seeded synthetic inputs.
Nothing is imported eagerly so that `synth` can be used without the HIP library.
"""
__all__ = ["binding", "synth"]
