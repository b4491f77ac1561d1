"""libeoq: the full-int8 training step of a Fixup residual CNN without BatchNorm
(EOQ, arXiv 2105.13890) as hand-written HIP kernels for MI355X (gfx950).

`eoq` holds the thin binding over the C ABI declared in include/eoq.h (argument
marshalling only); `net` sequences those calls into whole training steps.  There is
no CPU fallback: importing `eoq` fails loudly when libeoq.so is missing.
"""
