"""MI355X-native KV-cache migration (pack / pipeline / unpack) behind a C ABI.

``binding`` marshals arguments for ``libnts_kvmig.so``; every step of the path
runs in that library's HIP kernels.  Importing ``binding`` raises if the
library has not been built (``python -m paper_2605_05467_amd.build``).
"""
__all__ = ["binding", "build"]
