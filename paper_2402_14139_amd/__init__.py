"""MI355X-native local training step of adaptive local learning (NeuroFlux, arXiv 2402.14139).

``binding``  ctypes access to libnf.so (the C ABI declared in include/nf.h)
``layer``    device-side state of one local layer + the calls on it
``controller`` partition -> train block by block -> fill caches -> evaluate exits -> select
``layout``   NCHW/OIHW <-> NHWC/KRSC index permutations
``build``    compiles csrc/*.hip into libnf.so for gfx950

Importing the package loads nothing; ``binding.lib()`` raises if libnf.so is not built.
"""
__all__ = ["binding", "layer", "controller", "layout", "build"]
