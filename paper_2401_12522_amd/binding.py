"""ctypes binding of include/bita.h.  Argument marshalling only: every step of the
path runs in the HIP kernels of libbita.so.  torch supplies device memory and the
current stream."""
import ctypes as C
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("BITA_LIBRARY") or os.path.join(_PKG, "libbita.so")   # override: another build of the same ABI
_lib = None

EXPORTS = [
    "bita_packed_bytes", "bita_pack_weight", "bita_model_create", "bita_model_destroy",
    "bita_workspace_bytes", "bita_tree_template_create", "bita_tree_template_destroy",
    "bita_tree_template_info", "bita_build_tree", "bita_verify_step", "bita_accept",
    "bita_compact_kv", "bita_prefill_workspace_bytes", "bita_prefill_prepare", "bita_prefill", "bita_attention_workspace_bytes", "bita_tree_attention",
    "bita_gemm_workspace_bytes", "bita_gemm", "bita_gemm_noalloc_max_scratch_bytes", "bita_gemm_noalloc_scratch_bytes",
    "bita_gemm_noalloc", "bita_select", "bita_tune_gemm", "bita_gemm_plan_info", "bita_profile_enable",
    "bita_profile_disable", "bita_profile_read", "bita_last_error",
]


class BitaError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libbita error {code}: {msg}")
        self.code = code


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim",
                                           "d_ffn", "vocab", "n_prompt", "n_mask", "max_pos")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("tok_emb", "mask_emb", "final_norm", "lm_head")] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "ffn_norm", "wqkv", "wo", "w_gate_up",
                                                     "w_down", "prompt_k", "prompt_v")]


class _KV(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("k_cache", "v_cache", "k_tree", "v_tree")] + \
               [(n, C.c_int32) for n in ("smax", "rows", "batch", "ctx_hint")] + \
               [("block_table", C.c_void_p)] + [(n, C.c_int32) for n in ("page_size", "n_pages", "max_pages")]


def lib():
    """Load libbita.so (once).  Raises if it is missing: the product has no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} not built; run `python __graft_entry__.py` (or "
                           "paper_2401_12522_amd/build.py) first")
    L = C.CDLL(_LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.bita_packed_bytes.restype, L.bita_packed_bytes.argtypes = sz, [i64, i64]
    L.bita_pack_weight.restype, L.bita_pack_weight.argtypes = C.c_int, [vp, i64, i64, vp, i64, i64, i64, vp]
    L.bita_model_create.restype = C.c_int
    L.bita_model_create.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), C.POINTER(vp)]
    L.bita_model_destroy.restype, L.bita_model_destroy.argtypes = None, [vp]
    L.bita_workspace_bytes.restype, L.bita_workspace_bytes.argtypes = sz, [vp, i32, i32]
    L.bita_tree_template_create.restype = C.c_int
    L.bita_tree_template_create.argtypes = [vp, vp, i32, i32, i32, C.POINTER(vp)]
    L.bita_tree_template_destroy.restype, L.bita_tree_template_destroy.argtypes = None, [vp]
    L.bita_tree_template_info.restype, L.bita_tree_template_info.argtypes = i32, [vp, i32]
    L.bita_build_tree.restype = C.c_int
    L.bita_build_tree.argtypes = [vp, vp, vp, i32, i32, vp, vp, i32, vp, vp]
    L.bita_verify_step.restype = C.c_int
    L.bita_verify_step.argtypes = [vp, C.POINTER(_KV), vp, vp, vp, i32, vp, sz, i32, vp, vp, vp, vp, vp]
    L.bita_accept.restype = C.c_int
    L.bita_accept.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
    L.bita_compact_kv.restype = C.c_int
    L.bita_compact_kv.argtypes = [vp, C.POINTER(_KV), vp, i32, vp, vp, i32, vp]
    L.bita_prefill_workspace_bytes.restype, L.bita_prefill_workspace_bytes.argtypes = sz, [vp, i32, i32]
    L.bita_prefill_prepare.restype, L.bita_prefill_prepare.argtypes = C.c_int, [vp, i32, i32]
    L.bita_prefill.restype = C.c_int
    L.bita_prefill.argtypes = [vp, C.POINTER(_KV), vp, i32, vp, vp, i32, i32, vp, sz, vp, vp]
    L.bita_attention_workspace_bytes.restype = sz
    L.bita_attention_workspace_bytes.argtypes = [i32] * 6
    L.bita_tree_attention.restype = C.c_int
    L.bita_tree_attention.argtypes = [vp] * 12 + [i32] * 7 + [vp, sz, vp, vp, vp]
    L.bita_gemm_workspace_bytes.restype, L.bita_gemm_workspace_bytes.argtypes = sz, [i32, i64, i64]
    L.bita_gemm.restype, L.bita_gemm.argtypes = C.c_int, [vp, vp, i32, i64, i64, vp, i64, vp, sz, vp, vp]
    L.bita_gemm_noalloc_max_scratch_bytes.restype, L.bita_gemm_noalloc_max_scratch_bytes.argtypes = sz, []
    L.bita_gemm_noalloc_scratch_bytes.restype, L.bita_gemm_noalloc_scratch_bytes.argtypes = sz, [i32, i64, i64]
    L.bita_gemm_noalloc.restype, L.bita_gemm_noalloc.argtypes = C.c_int, [vp, vp, i32, i64, i64, vp, i64, vp, vp]
    L.bita_select.restype, L.bita_select.argtypes = C.c_int, [vp, vp, i32, i32, i32, vp, vp, vp, vp]
    L.bita_tune_gemm.restype, L.bita_tune_gemm.argtypes = None, [i32, i32]
    L.bita_gemm_plan_info.restype, L.bita_gemm_plan_info.argtypes = C.c_int, [i32, i64, i64, vp]
    L.bita_profile_enable.restype, L.bita_profile_enable.argtypes = C.c_int, [i32]
    L.bita_profile_disable.restype, L.bita_profile_disable.argtypes = None, []
    L.bita_profile_read.restype, L.bita_profile_read.argtypes = C.c_int, [i32, vp, vp, vp]
    L.bita_last_error.restype, L.bita_last_error.argtypes = C.c_char_p, []
    _lib = L
    return L


def _check(rc):
    if rc != 0:
        raise BitaError(rc, lib().bita_last_error().decode())


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def packed_bytes(n_rows, k):
    return lib().bita_packed_bytes(n_rows, k)


def pack_weight(src, dst=None, tile0=0, tile_stride=1, total_rows=None):
    """src: bf16 cuda tensor [N][K].  Returns the packed uint8 buffer (allocated here
    when dst is None, sized for total_rows rows)."""
    n, k = src.shape
    assert src.dtype == torch.bfloat16 and src.is_cuda and src.is_contiguous()
    total_rows = total_rows or n
    if dst is None:
        dst = torch.empty(packed_bytes(total_rows, k), dtype=torch.uint8, device=src.device)
    _check(lib().bita_pack_weight(_ptr(src), n, k, _ptr(dst), total_rows, tile0, tile_stride, _stream()))
    return dst


class TreeTemplate:
    def __init__(self, parent, is_mask, n_tree, n_mask):
        parent = np.ascontiguousarray(parent, np.int32)
        is_mask = np.ascontiguousarray(is_mask, np.uint8)
        self.handle = C.c_void_p()
        _check(lib().bita_tree_template_create(parent.ctypes.data_as(C.c_void_p), is_mask.ctypes.data_as(C.c_void_p),
                                               int(n_tree), int(parent.shape[0]), int(n_mask), C.byref(self.handle)))
        info = lambda w: lib().bita_tree_template_info(self.handle, w)   # noqa: E731
        self.rows, self.n_tree, self.n_groups = info(0), info(1), info(2)
        self.depth, self.kmax, self.words = info(3), info(4), info(5)
        self.n_mask = int(n_mask)

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.bita_tree_template_destroy(self.handle)
            self.handle = None


class Model:
    """Packs the matrices of a weight source (anything with .torch(name, layer) giving bf16
    cuda tensors [out][in]) and creates the library handle.  The packed buffers and the
    small row-major tensors are kept alive here; the library only borrows them."""

    def __init__(self, cfg, weights, max_pos, n_layers=None, free_source=False):
        self.cfg = cfg
        L = cfg.n_layers if n_layers is None else n_layers
        self.n_layers = L
        dev = torch.device("cuda")
        keep = self._keep = []
        hd = cfg.head_dim

        def pack_many(parts, k, interleave=False):
            total = sum(p.shape[0] for p in parts)
            dst = torch.empty(packed_bytes(total, k), dtype=torch.uint8, device=dev)
            if interleave:
                for i, p in enumerate(parts):
                    pack_weight(p.contiguous(), dst, i, len(parts), total_rows=total)
            else:
                row = 0
                for p in parts:
                    pack_weight(p.contiguous(), dst, row // 16, 1, total_rows=total)
                    row += p.shape[0]
            keep.append(dst)
            return dst

        def small(name, layer=None):
            t = weights.torch(name, layer).to(dev).contiguous()
            keep.append(t)
            return t

        def arr(ts):
            a = (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
            keep.append(a)
            return a
        cols = {n: [] for n in ("attn_norm", "ffn_norm", "wqkv", "wo", "w_gate_up", "w_down", "prompt_k", "prompt_v")}
        for l in range(L):
            g = lambda n: weights.torch(n, l).to(dev)     # noqa: E731
            cols["wqkv"].append(pack_many([g("wq"), g("wk"), g("wv")], cfg.d_model))
            cols["wo"].append(pack_many([g("wo")], cfg.n_heads * hd))
            cols["w_gate_up"].append(pack_many([g("w_gate"), g("w_up")], cfg.d_model, interleave=True))
            cols["w_down"].append(pack_many([g("w_down")], cfg.d_ffn))
            cols["attn_norm"].append(small("attn_norm", l))
            cols["ffn_norm"].append(small("ffn_norm", l))
            if cfg.n_prompt > 0:
                cols["prompt_k"].append(small("prompt_k", l))
                cols["prompt_v"].append(small("prompt_v", l))
            if free_source:
                torch.cuda.synchronize()
                for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
                    weights._store.pop((n, l), None)
        w = _Weights()
        w.tok_emb = small("tok_emb").data_ptr()
        w.mask_emb = small("mask_emb").data_ptr() if cfg.n_mask > 0 else None
        w.final_norm = small("final_norm").data_ptr()
        w.lm_head = pack_many([weights.torch("lm_head").to(dev)], cfg.d_model).data_ptr()
        for n, ts in cols.items():
            if ts:
                setattr(w, n, arr(ts))
        c = _Config(L, cfg.d_model, cfg.n_heads, cfg.n_kv_heads, hd, cfg.d_ffn, cfg.vocab, cfg.n_prompt,
                    cfg.n_mask, int(max_pos), cfg.rms_eps, cfg.rope_theta)
        torch.cuda.synchronize()
        self.max_pos = int(max_pos)
        self.handle = C.c_void_p()
        _check(lib().bita_model_create(C.byref(c), C.byref(w), C.byref(self.handle)))

    def workspace_bytes(self, batch, rows):
        return lib().bita_workspace_bytes(self.handle, batch, rows)

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.bita_model_destroy(self.handle)
            self.handle = None


class KVState:
    """Caller-owned KV cache, per-pass tree scratch and ctx_len for `batch` sequences."""

    def __init__(self, cfg, n_layers, batch, smax, rows):
        dev = torch.device("cuda")
        shape_c = (n_layers, batch, cfg.n_kv_heads, smax, cfg.head_dim)
        shape_t = (n_layers, batch, cfg.n_kv_heads, rows, cfg.head_dim)
        self.k_cache = torch.zeros(shape_c, dtype=torch.bfloat16, device=dev)
        self.v_cache = torch.zeros(shape_c, dtype=torch.bfloat16, device=dev)
        self.k_tree = torch.zeros(shape_t, dtype=torch.bfloat16, device=dev)
        self.v_tree = torch.zeros(shape_t, dtype=torch.bfloat16, device=dev)
        self.ctx_len = torch.zeros(batch, dtype=torch.int32, device=dev)
        self.smax, self.rows, self.batch = smax, rows, batch

    def resize_rows(self, n_layers, cfg, rows):
        """Lay the per-pass scratch out for a template of `rows` rows (the template may change from
        step to step).  The memory is kept when it is large enough; the contents are undefined."""
        shape_t = (n_layers, self.batch, cfg.n_kv_heads, rows, cfg.head_dim)
        n = n_layers * self.batch * cfg.n_kv_heads * rows * cfg.head_dim
        for name in ("k_tree", "v_tree"):
            flat = getattr(self, "_" + name + "_flat", None)
            if flat is None:
                flat = getattr(self, name).reshape(-1)
            if flat.numel() < n:
                flat = torch.zeros(n, dtype=torch.bfloat16, device=self.k_cache.device)
            setattr(self, "_" + name + "_flat", flat)
            setattr(self, name, flat[:n].view(shape_t))
        self.rows = rows

    def desc(self, ctx_hint):
        return _KV(self.k_cache.data_ptr(), self.v_cache.data_ptr(), self.k_tree.data_ptr(),
                   self.v_tree.data_ptr(), self.smax, self.rows, self.batch, int(ctx_hint), None, 0, 0, 0)


class PagedKVState(KVState):
    """KV state whose caches are page pools [n_layers][n_pages][n_kv_heads][page_size][head_dim];
    block_table [batch][max_pages] names the pages of every sequence (here: a seeded shuffle of
    the pool, so that neighbouring slots of a sequence are not neighbours in memory)."""

    def __init__(self, cfg, n_layers, batch, smax, rows, page_size, n_pages=None, seed=0):
        dev = torch.device("cuda")
        self.page_size = int(page_size)
        self.max_pages = (smax + page_size - 1) // page_size
        self.n_pages = int(n_pages or batch * self.max_pages)
        assert self.n_pages >= batch * self.max_pages
        shape_c = (n_layers, self.n_pages, cfg.n_kv_heads, page_size, cfg.head_dim)
        shape_t = (n_layers, batch, cfg.n_kv_heads, rows, cfg.head_dim)
        self.k_cache = torch.zeros(shape_c, dtype=torch.bfloat16, device=dev)
        self.v_cache = torch.zeros(shape_c, dtype=torch.bfloat16, device=dev)
        self.k_tree = torch.zeros(shape_t, dtype=torch.bfloat16, device=dev)
        self.v_tree = torch.zeros(shape_t, dtype=torch.bfloat16, device=dev)
        self.ctx_len = torch.zeros(batch, dtype=torch.int32, device=dev)
        self.smax, self.rows, self.batch = smax, rows, batch
        perm = np.random.default_rng(seed).permutation(self.n_pages)[: batch * self.max_pages]
        self.block_table = torch.tensor(perm.reshape(batch, self.max_pages), dtype=torch.int32, device=dev)

    def desc(self, ctx_hint):
        return _KV(self.k_cache.data_ptr(), self.v_cache.data_ptr(), self.k_tree.data_ptr(),
                   self.v_tree.data_ptr(), self.smax, self.rows, self.batch, int(ctx_hint),
                   self.block_table.data_ptr(), self.page_size, self.n_pages, self.max_pages)

    def contiguous(self, b):
        """(k, v) of sequence b as [n_layers][n_kv_heads][max_pages * page_size][head_dim] copies."""
        pages = self.block_table[b].long()
        def one(pool):
            x = pool[:, pages]                                      # [L][max_pages][Hkv][page][hd]
            return x.permute(0, 2, 1, 3, 4).reshape(x.shape[0], x.shape[2], -1, x.shape[4])
        return one(self.k_cache), one(self.v_cache)

    def load_contiguous(self, b, k, v, n):
        """Write slots 0..n-1 of sequence b from k, v [n_layers][n_kv_heads][>= n][head_dim]; sets ctx_len[b] = n."""
        for i in range((n + self.page_size - 1) // self.page_size):
            lo, hi = i * self.page_size, min((i + 1) * self.page_size, n)
            page = int(self.block_table[b, i])
            self.k_cache[:, page, :, : hi - lo] = k[:, :, lo:hi]
            self.v_cache[:, page, :, : hi - lo] = v[:, :, lo:hi]
        self.ctx_len[b] = n


class StepBuffers:
    """Device outputs of one step for a given template and batch."""

    def __init__(self, model, tmpl, batch, kmax, want_logits=False):
        dev = torch.device("cuda")
        i32 = dict(dtype=torch.int32, device=dev)
        self.kmax = int(kmax)
        self.token = torch.zeros((batch, tmpl.rows), **i32)
        self.argmax = torch.zeros((batch, tmpl.n_tree), **i32)
        nm = max(tmpl.n_groups * tmpl.n_mask, 1)
        self.topk_ids = torch.zeros((batch, nm, self.kmax), **i32)
        self.topk_val = torch.zeros((batch, nm, self.kmax), dtype=torch.float32, device=dev)
        self.logits = torch.zeros((batch, tmpl.rows, model.cfg.vocab), dtype=torch.float32, device=dev) if want_logits else None
        self.path = torch.zeros((batch, tmpl.depth + 1), **i32)
        self.n_acc = torch.zeros(batch, **i32)
        self.bonus = torch.zeros(batch, **i32)
        self.emitted = torch.zeros((batch, tmpl.depth + 1), **i32)
        self.next_group = torch.zeros(batch, **i32)
        self.next_shift = torch.zeros(batch, **i32)
        self.workspace = torch.empty(model.workspace_bytes(batch, tmpl.rows), dtype=torch.uint8, device=dev)


def build_tree(tmpl, root_token, cand, group, shift, batch, token_out):
    cand_rows, kmax = (cand.shape[1], cand.shape[2]) if cand is not None else (0, 0)
    _check(lib().bita_build_tree(tmpl.handle, _ptr(root_token), _ptr(cand), cand_rows, kmax, _ptr(group),
                                 _ptr(shift), batch, _ptr(token_out), _stream()))


def verify_step(model, kv, ctx_hint, tmpl, buf, batch):
    d = kv.desc(ctx_hint)
    has_masks = tmpl.n_groups > 0
    _check(lib().bita_verify_step(model.handle, C.byref(d), tmpl.handle, _ptr(buf.token), _ptr(kv.ctx_len), batch,
                                  _ptr(buf.workspace), buf.workspace.numel(), buf.kmax, _ptr(buf.argmax),
                                  _ptr(buf.topk_ids if has_masks else None),
                                  _ptr(buf.topk_val if has_masks else None), _ptr(buf.logits), _stream()))


def accept(tmpl, buf, batch):
    _check(lib().bita_accept(tmpl.handle, _ptr(buf.token), _ptr(buf.argmax), batch, _ptr(buf.path),
                             _ptr(buf.n_acc), _ptr(buf.bonus), _ptr(buf.emitted), _ptr(buf.next_group),
                             _ptr(buf.next_shift), _stream()))


def compact_kv(model, kv, ctx_hint, buf, batch, path=None, n_acc=None):
    d = kv.desc(ctx_hint)
    path = buf.path if path is None else path
    n_acc = buf.n_acc if n_acc is None else n_acc
    _check(lib().bita_compact_kv(model.handle, C.byref(d), _ptr(path), path.shape[1], _ptr(n_acc),
                                 _ptr(kv.ctx_len), batch, _stream()))


def prefill_workspace(model, batch, chunk_rows):
    """A workspace tensor for prefill() with these sizes."""
    need = lib().bita_prefill_workspace_bytes(model.handle, batch, chunk_rows)
    return torch.empty(need, dtype=torch.uint8, device="cuda")


def prefill_prepare(model, n_tokens, chunk_rows):
    """Create the model's chain templates for this chunking ahead of time (needed before a
    prefill is captured into a graph)."""
    _check(lib().bita_prefill_prepare(model.handle, int(n_tokens), int(chunk_rows)))


def prefill(model, kv, ctx_hint, tokens, chunk_rows, seq_len=None, workspace=None, next_token=None):
    """tokens int32 cuda [B][n]; appends them (row b up to seq_len[b]) to the cache by chunked causal
    passes.  Returns the greedy token after each sequence's last one, int32 cuda [B] (written into
    next_token when given; with workspace and next_token supplied nothing is allocated here)."""
    batch, n = tokens.shape
    assert tokens.dtype == torch.int32 and tokens.is_contiguous()
    need = lib().bita_prefill_workspace_bytes(model.handle, batch, chunk_rows)
    if workspace is None or workspace.numel() < need:
        workspace = torch.empty(need, dtype=torch.uint8, device=tokens.device)
    if next_token is None:
        next_token = torch.full((batch,), -1, dtype=torch.int32, device=tokens.device)
    d = kv.desc(ctx_hint)
    _check(lib().bita_prefill(model.handle, C.byref(d), _ptr(tokens), n, _ptr(seq_len), _ptr(kv.ctx_len), batch,
                              int(chunk_rows), _ptr(workspace), workspace.numel(), _ptr(next_token), _stream()))
    return next_token


def decode_step(model, kv, ctx_hint, tmpl, buf, batch, root_token, cand, group=None, shift=None):
    """The four calls of one step, back to back on the current stream (no host sync)."""
    build_tree(tmpl, root_token, cand, group, shift, batch, buf.token)
    verify_step(model, kv, ctx_hint, tmpl, buf, batch)
    accept(tmpl, buf, batch)
    compact_kv(model, kv, ctx_hint, buf, batch)


def profile_enable(max_records):
    _check(lib().bita_profile_enable(int(max_records)))


def profile_read(capacity):
    """Returns (ms[n], weight_bytes[n]) of the GEMM launches recorded since profile_enable."""
    n = C.c_int32(0)
    ms = np.zeros(capacity, np.float32)
    wb = np.zeros(capacity, np.int64)
    _check(lib().bita_profile_read(capacity, C.byref(n), ms.ctypes.data_as(C.c_void_p), wb.ctypes.data_as(C.c_void_p)))
    lib().bita_profile_disable()
    return ms[: n.value], wb[: n.value]


def gemm(a, w_packed, n_rows, k=None, a_lo=None):
    """a (and optionally a_lo, the residual plane): bf16 cuda [M][lda]; returns fp32 [M][n_rows]."""
    m, lda = a.shape
    k = lda if k is None else k
    ws = torch.empty(lib().bita_gemm_workspace_bytes(m, n_rows, k), dtype=torch.uint8, device=a.device)
    out = torch.empty((m, n_rows), dtype=torch.float32, device=a.device)
    _check(lib().bita_gemm(_ptr(a), _ptr(a_lo), m, k, lda, _ptr(w_packed), n_rows, _ptr(ws), ws.numel(), _ptr(out), _stream()))
    return out


def gemm_noalloc(a, w_packed, n_rows, out, k=None, a_lo=None):
    """bita_gemm_noalloc: as gemm(), but the library's static scratch replaces the workspace and the
    caller brings the output (fp32 cuda [M][n_rows]); nothing is allocated by the call."""
    m, lda = a.shape
    k = lda if k is None else k
    assert out.dtype == torch.float32 and out.is_contiguous() and tuple(out.shape) == (m, n_rows)
    _check(lib().bita_gemm_noalloc(_ptr(a), _ptr(a_lo), m, k, lda, _ptr(w_packed), n_rows, _ptr(out), _stream()))
    return out


def gemm_plan_info(m_rows, n_rows, k):
    """{splits, variant, mt_pass, ksteps_per_split} the launch heuristic picks for this GEMM shape."""
    out = (C.c_int32 * 4)()
    _check(lib().bita_gemm_plan_info(int(m_rows), int(n_rows), int(k), out))
    return dict(splits=out[0], variant=out[1], mt_pass=out[2], ksteps_per_split=out[3])


def select(tmpl, logits, kmax):
    """logits fp32 cuda [B][R][vocab] -> (argmax int32 [B][T], topk_ids int32 [B][G*n][kmax], topk_val fp32)."""
    B, R, V = logits.shape
    assert R == tmpl.rows and logits.dtype == torch.float32 and logits.is_contiguous()
    argmax = torch.empty((B, tmpl.n_tree), dtype=torch.int32, device=logits.device)
    n_sel = tmpl.n_groups * tmpl.n_mask
    ids = torch.empty((B, n_sel, kmax), dtype=torch.int32, device=logits.device)
    val = torch.empty((B, n_sel, kmax), dtype=torch.float32, device=logits.device)
    _check(lib().bita_select(tmpl.handle, _ptr(logits), B, V, kmax, _ptr(argmax), _ptr(ids), _ptr(val), _stream()))
    return argmax, ids, val


def tree_attention(tmpl, q, k_cache, v_cache, k_tree, v_tree, prompt_k, prompt_v, ctx_len, ctx_hint, q_lo=None,
                   k_tree_lo=None, v_tree_lo=None, two_plane_out=False):
    """q [B][R][Hq][hd]; k/v_cache [B][Hkv][smax][hd]; k/v_tree [B][Hkv][R][hd];
    prompt_k/v [Hkv][P][hd] or None; q_lo, k_tree_lo, v_tree_lo: optional low bf16 planes.  Returns bf16
    [B][R][Hq*hd], or the pair (hi, lo) of bf16 planes when two_plane_out."""
    B, R, Hq, hd = q.shape
    Hkv, smax = k_cache.shape[1], k_cache.shape[2]
    P = 0 if prompt_k is None else prompt_k.shape[1]
    ws = torch.empty(lib().bita_attention_workspace_bytes(B, R, Hq, hd, int(ctx_hint), P), dtype=torch.uint8, device=q.device)
    out = torch.empty((B, R, Hq * hd), dtype=torch.bfloat16, device=q.device)
    out_lo = torch.empty_like(out) if two_plane_out else None
    _check(lib().bita_tree_attention(tmpl.handle, _ptr(q), _ptr(q_lo), _ptr(k_cache), _ptr(v_cache), _ptr(k_tree), _ptr(v_tree),
                                     _ptr(k_tree_lo), _ptr(v_tree_lo), _ptr(prompt_k), _ptr(prompt_v), _ptr(ctx_len), B, Hq, Hkv, hd, P, smax,
                                     int(ctx_hint), _ptr(ws), ws.numel(), _ptr(out), _ptr(out_lo), _stream()))
    return (out, out_lo) if two_plane_out else out
