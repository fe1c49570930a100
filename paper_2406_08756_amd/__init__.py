"""MI355X-native per-layer recompute-and-backward of a GPT block shard.

The product is the C-ABI library built from csrc/ (see include/lynx.h);
`binding` marshals arguments to it.  Importing this package loads nothing:
the shared library is opened on first use of `binding`.
"""
__all__ = ["binding", "build"]
