"""MI355X-native paged decode attention (GQA, block-table KV cache) behind a C ABI.

``workloads`` draws seeded synthetic decode batches; ``binding`` is the thin ctypes
layer over ``libpa_decode.so`` (built from ``csrc/`` by ``build``).  Importing the
package loads nothing native; the library is opened on first use of ``binding``.
"""
__all__ = ["workloads", "binding", "build"]
