"""MI355X-native tree-verify step of BiTA (arXiv 2401.12522): a thin ctypes binding
over libbita.so.  Importing the package does not load the library; the first use does,
and fails loudly if it has not been built (there is no CPU fallback)."""
from .binding import (lib, BitaError, Model, TreeTemplate, KVState, PagedKVState, StepBuffers,   # noqa: F401
                      pack_weight, packed_bytes, gemm, tree_attention, select, decode_step, prefill, prefill_prepare, prefill_workspace,
                      build_tree, verify_step, accept, compact_kv)
