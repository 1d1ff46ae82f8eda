"""MI355X-native degraded-block backward of MeCeFO (arxiv 2510.16415).

The compute path lives in the HIP library under ``csrc/`` behind a C ABI;
``binding`` marshals arguments to it.  Importing this package does not load the
library; ``binding.lib()`` does, and raises if it has not been built.
"""
__all__ = ["inputs", "binding", "build"]
