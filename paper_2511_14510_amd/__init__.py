"""MI355X-native QSAC decode step (LiteCache, arXiv 2511.14510, Algorithm 1).

The HIP kernels live in ``csrc/`` behind a C ABI (``include/qsac.h``);
``binding`` marshals arguments to it and nothing else.  Importing the package
does not load the shared library; ``binding.load()`` does, and fails loudly if
it has not been built.
"""
__all__ = ["binding", "workload"]
