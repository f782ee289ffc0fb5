"""MI355X-native factorization-machine pass of DS-FACTO (arXiv 2004.13940).

``binding`` wraps the C ABI of ``libfm_mi355x.so`` (see include/fm.h);
``workloads`` synthesises the seeded inputs; ``build`` compiles the HIP sources.
Nothing is loaded at import time; the library is opened on first use and there
is no CPU fallback.
"""
__all__ = ["binding", "workloads", "build"]
