"""MI355X-native StructKV scoring / selection / gather path (hand-written HIP behind a C ABI).

`binding` is a thin ctypes layer over libstructkv.so: argument marshalling only.
Importing it fails loudly when the library has not been built
(`python -m paper_2604_06746_amd.build`); there is no CPU fallback.
"""
__all__ = ["binding", "build"]
