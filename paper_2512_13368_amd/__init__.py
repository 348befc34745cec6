"""MI355X-native Blossom attention (BlossomRec, arXiv 2512.13368, Sec. 3.4-3.6).

The compute path is the HIP library ``libblossom.so`` (C ABI declared in
``include/blossom.h``); ``binding`` marshals torch device tensors into it.
Importing this package loads nothing: the library is opened on first use and a
missing library is an error, never a fallback.
"""
