// Host side of the C ABI: handles, validation, the per-step launch sequence.
#include "common.h"
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

static thread_local char g_err[512] = "";

int bita_set_error(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
extern "C" const char *bita_last_error(void) { return g_err; }

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ------------------------------------------------------------------------------------------

extern "C" size_t bita_packed_bytes(int64_t n_rows, int64_t k) {
    if (n_rows <= 0 || k <= 0) return 0;
    return (size_t)((n_rows + 15) / 16) * (size_t)((k + 63) / 64) * 2048;
}

extern "C" int bita_pack_weight(const void *d_src, int64_t n_rows, int64_t k, void *d_dst,
                                int64_t dst_total_rows, int64_t dst_tile0, int64_t dst_tile_stride,
                                void *stream) {
    if (!d_src || !d_dst || n_rows <= 0 || k <= 0 || dst_tile0 < 0 || dst_tile_stride < 1)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_pack_weight: bad argument");
    if (n_rows % 16 || k % 8 || dst_total_rows % 16)
        return bita_set_error(BITA_ERR_UNSUPPORTED, "bita_pack_weight: rows must be a multiple of 16 and k of 8");
    if (dst_tile0 + (n_rows / 16 - 1) * dst_tile_stride >= dst_total_rows / 16)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_pack_weight: source tiles do not fit %lld destination rows",
                              (long long)dst_total_rows);
    launch_pack(d_src, n_rows, k, d_dst, dst_tile0, dst_tile_stride, dst_total_rows / 16, (hipStream_t)stream);
    BITA_HIP_CHECK(hipGetLastError());
    return BITA_OK;
}

extern "C" int bita_model_create(const bita_config *cfg, const bita_weights *w, bita_model **out) {
    if (!cfg || !w || !out) return bita_set_error(BITA_ERR_INVALID_ARG, "bita_model_create: null argument");
    const bita_config &c = *cfg;
    if (c.n_layers <= 0 || c.d_model <= 0 || c.n_heads <= 0 || c.n_kv_heads <= 0 || c.d_ffn <= 0 ||
        c.vocab <= 0 || c.n_prompt < 0 || c.n_mask < 0 || c.max_pos <= 0 || c.n_heads % c.n_kv_heads)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_model_create: non-positive or inconsistent shape");
    if ((c.head_dim != 64 && c.head_dim != 128) || c.d_model % 32 || c.d_ffn % 16 || c.vocab % 16 ||
        c.d_model > 1024 * RMS_MAX_CHUNKS)
        return bita_set_error(BITA_ERR_UNSUPPORTED,
                              "bita_model_create: head_dim must be 64 or 128; d_model a multiple of 32 and <= %d; "
                              "d_ffn, vocab multiples of 16", 1024 * RMS_MAX_CHUNKS);
    if (!w->tok_emb || !w->final_norm || !w->lm_head || !w->attn_norm || !w->ffn_norm || !w->wqkv ||
        !w->wo || !w->w_gate_up || !w->w_down || (c.n_mask > 0 && !w->mask_emb) ||
        (c.n_prompt > 0 && (!w->prompt_k || !w->prompt_v)))
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_model_create: missing weight pointer");
    bita_model *m = new bita_model();
    m->cfg = c;
    m->tok_emb = w->tok_emb; m->mask_emb = w->mask_emb; m->final_norm = w->final_norm; m->lm_head = w->lm_head;
    for (int l = 0; l < c.n_layers; l++) {
        m->attn_norm.push_back(w->attn_norm[l]); m->ffn_norm.push_back(w->ffn_norm[l]);
        m->wqkv.push_back(w->wqkv[l]); m->wo.push_back(w->wo[l]);
        m->w_gate_up.push_back(w->w_gate_up[l]); m->w_down.push_back(w->w_down[l]);
        m->prompt_k.push_back(c.n_prompt > 0 ? w->prompt_k[l] : nullptr);
        m->prompt_v.push_back(c.n_prompt > 0 ? w->prompt_v[l] : nullptr);
        if (!m->attn_norm[l] || !m->ffn_norm[l] || !m->wqkv[l] || !m->wo[l] || !m->w_gate_up[l] ||
            !m->w_down[l] || (c.n_prompt > 0 && (!m->prompt_k[l] || !m->prompt_v[l]))) {
            delete m;
            return bita_set_error(BITA_ERR_INVALID_ARG, "bita_model_create: null weight in layer %d", l);
        }
    }
    // rotary table: angle(pos, i) = pos * theta^(-2i/hd), evaluated in double on the host
    const int half = c.head_dim / 2;
    std::vector<float> hc((size_t)c.max_pos * half), hs((size_t)c.max_pos * half);
    for (int p = 0; p < c.max_pos; p++)
        for (int i = 0; i < half; i++) {
            const double ang = (double)p * std::pow((double)c.rope_theta, -2.0 * i / c.head_dim);
            hc[(size_t)p * half + i] = (float)std::cos(ang);
            hs[(size_t)p * half + i] = (float)std::sin(ang);
        }
    hipError_t e = hipMalloc((void **)&m->rope_cos, hc.size() * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void **)&m->rope_sin, hs.size() * sizeof(float));
    if (e == hipSuccess) e = hipMemcpy(m->rope_cos, hc.data(), hc.size() * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(m->rope_sin, hs.data(), hs.size() * sizeof(float), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        bita_model_destroy(m);
        return bita_set_error(BITA_ERR_HIP, "bita_model_create: rotary table: %s", hipGetErrorString(e));
    }
    *out = m;
    return BITA_OK;
}

extern "C" void bita_model_destroy(bita_model *m) {
    if (!m) return;
    if (m->rope_cos) (void)hipFree(m->rope_cos);
    if (m->rope_sin) (void)hipFree(m->rope_sin);
    for (auto &kv : m->chains) bita_tree_template_destroy(kv.second);
    delete m;
}

// ------------------------------------------------------------------------------------------
extern "C" int bita_tree_template_create(const int32_t *parent, const uint8_t *is_mask, int32_t n_tree,
                                         int32_t rows, int32_t n_mask, bita_tree_template **out) {
    if (!parent || !is_mask || !out) return bita_set_error(BITA_ERR_INVALID_ARG, "template: null argument");
    if (rows <= 0 || rows > BITA_MAX_ROWS || n_tree <= 0 || n_tree > rows || n_mask < 0)
        return bita_set_error(BITA_ERR_BAD_TREE, "template: need 1 <= n_tree <= rows <= %d", BITA_MAX_ROWS);
    if (parent[0] != -1 || is_mask[0])
        return bita_set_error(BITA_ERR_BAD_TREE, "template: row 0 must be the root (parent -1, not a mask)");
    const int R = rows, T = n_tree, W = (R + 63) / 64;
    std::vector<int32_t> depth(R, 0), rank(R, 0), mask_index(R, -1), group_of_node(T, -1), nchild(R, 0);
    std::vector<int32_t> mask_rows;
    std::vector<uint64_t> anc((size_t)R * W, 0);
    anc[0] = 1;
    int n_groups = 0, run = 0;
    for (int i = 1; i < R; i++) {
        const int p = parent[i];
        const bool mk = is_mask[i] != 0;
        if (p < 0 || p >= i) return bita_set_error(BITA_ERR_BAD_TREE, "template: parent[%d] = %d not in [0, %d)", i, p, i);
        if (mk != (i >= T)) return bita_set_error(BITA_ERR_BAD_TREE, "template: tree rows must precede mask rows (row %d)", i);
        depth[i] = depth[p] + 1;
        for (int w = 0; w < W; w++) anc[(size_t)i * W + w] = anc[(size_t)p * W + w];
        anc[(size_t)i * W + i / 64] |= 1ull << (i % 64);
        if (!mk) {
            if (is_mask[p]) return bita_set_error(BITA_ERR_BAD_TREE, "template: draft row %d hangs off a mask row", i);
            rank[i] = nchild[p]++;
        } else if (!is_mask[p]) {                       // first mask of a new group
            if (run != 0) return bita_set_error(BITA_ERR_BAD_TREE, "template: mask group before row %d is shorter than n_mask", i);
            if (group_of_node[p] != -1) return bita_set_error(BITA_ERR_BAD_TREE, "template: two mask groups on node %d", p);
            if (n_mask <= 0) return bita_set_error(BITA_ERR_BAD_TREE, "template: mask rows present but n_mask = 0");
            group_of_node[p] = n_groups++;
            mask_index[i] = 0;
            run = 1;
            mask_rows.push_back(i);
        } else {
            if (p != i - 1 || run == 0 || run >= n_mask)
                return bita_set_error(BITA_ERR_BAD_TREE, "template: mask group at row %d is not a chain of n_mask consecutive rows", i);
            mask_index[i] = mask_index[p] + 1;
            run++;
            mask_rows.push_back(i);
        }
        if (mk && run == n_mask) run = 0;
    }
    if (run != 0) return bita_set_error(BITA_ERR_BAD_TREE, "template: last mask group is shorter than n_mask");
    int depth_max = 0, kmax = 1;
    for (int i = 0; i < T; i++) {
        if (depth[i] > depth_max) depth_max = depth[i];
        if (nchild[i] > kmax) kmax = nchild[i];
    }
    // one blob: parent, depth, rank, mask_index [R] | group_of_node [T] | mask_rows | is_mask | anc
    const size_t o_parent = 0, o_depth = o_parent + R * 4, o_rank = o_depth + R * 4, o_midx = o_rank + R * 4;
    const size_t o_gon = o_midx + R * 4, o_mrows = o_gon + T * 4;
    const size_t o_ismask = o_mrows + (mask_rows.size() + 1) * 4;
    const size_t o_anc = align_up(o_ismask + R, 8), total = o_anc + (size_t)R * W * 8;
    std::vector<unsigned char> host(total, 0);
    memcpy(&host[o_parent], parent, R * 4);
    memcpy(&host[o_depth], depth.data(), R * 4);
    memcpy(&host[o_rank], rank.data(), R * 4);
    memcpy(&host[o_midx], mask_index.data(), R * 4);
    memcpy(&host[o_gon], group_of_node.data(), T * 4);
    if (!mask_rows.empty()) memcpy(&host[o_mrows], mask_rows.data(), mask_rows.size() * 4);
    memcpy(&host[o_ismask], is_mask, R);
    memcpy(&host[o_anc], anc.data(), (size_t)R * W * 8);
    void *blob = nullptr;
    BITA_HIP_CHECK(hipMalloc(&blob, total));
    hipError_t e = hipMemcpy(blob, host.data(), total, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(blob);
        return bita_set_error(BITA_ERR_HIP, "template upload: %s", hipGetErrorString(e));
    }
    bita_tree_template *t = new bita_tree_template();
    t->blob = blob;
    unsigned char *d = (unsigned char *)blob;
    t->dev.rows = R; t->dev.n_tree = T; t->dev.n_mask = n_mask; t->dev.n_groups = n_groups;
    t->dev.depth_max = depth_max; t->dev.kmax = kmax; t->dev.words = W;
    t->dev.parent = (const int32_t *)(d + o_parent); t->dev.depth = (const int32_t *)(d + o_depth);
    t->dev.rank = (const int32_t *)(d + o_rank); t->dev.mask_index = (const int32_t *)(d + o_midx);
    t->dev.group_of_node = (const int32_t *)(d + o_gon); t->dev.mask_rows = (const int32_t *)(d + o_mrows);
    t->dev.is_mask = (const uint8_t *)(d + o_ismask); t->dev.anc = (const uint64_t *)(d + o_anc);
    *out = t;
    return BITA_OK;
}

extern "C" void bita_tree_template_destroy(bita_tree_template *t) {
    if (!t) return;
    if (t->blob) (void)hipFree(t->blob);
    delete t;
}

extern "C" int32_t bita_tree_template_info(const bita_tree_template *t, int32_t what) {
    if (!t) return -1;
    switch (what) {
        case 0: return t->dev.rows;
        case 1: return t->dev.n_tree;
        case 2: return t->dev.n_groups;
        case 3: return t->dev.depth_max;
        case 4: return t->dev.kmax;
        case 5: return t->dev.words;
        default: return -1;
    }
}

// ------------------------------------------------------------------------------------------
// Optional instrumentation: HIP events around every GEMM launch of bita_verify_step, recorded
// on the caller's stream.  Events are created by bita_profile_enable (never inside a step).
struct GemmRecord { hipEvent_t start, stop; int64_t weight_bytes; };
static std::vector<GemmRecord> g_prof;
static size_t g_prof_used = 0;
static bool g_prof_on = false;

extern "C" int bita_profile_enable(int32_t max_records) {
    if (max_records <= 0) return bita_set_error(BITA_ERR_INVALID_ARG, "bita_profile_enable: max_records <= 0");
    while ((int)g_prof.size() < max_records) {
        GemmRecord r;
        r.weight_bytes = 0;
        BITA_HIP_CHECK(hipEventCreate(&r.start));
        BITA_HIP_CHECK(hipEventCreate(&r.stop));
        g_prof.push_back(r);
    }
    g_prof_used = 0;
    g_prof_on = true;
    return BITA_OK;
}
extern "C" void bita_profile_disable(void) { g_prof_on = false; }
extern "C" int bita_profile_read(int32_t capacity, int32_t *n_records, float *ms, int64_t *weight_bytes) {
    if (!n_records || !ms || !weight_bytes) return bita_set_error(BITA_ERR_INVALID_ARG, "bita_profile_read: null");
    int n = 0;
    for (size_t i = 0; i < g_prof_used && n < capacity; i++, n++) {
        BITA_HIP_CHECK(hipEventSynchronize(g_prof[i].stop));
        BITA_HIP_CHECK(hipEventElapsedTime(&ms[n], g_prof[i].start, g_prof[i].stop));
        weight_bytes[n] = g_prof[i].weight_bytes;
    }
    *n_records = n;
    return BITA_OK;
}
static void timed_gemm(const void *a_frag, int M, int64_t K, const void *w, int64_t N, float *out, int64_t ldo,
                       const GemmPlan &p, hipStream_t s, const GemmOutput *direct = nullptr) {
    GemmRecord *r = (g_prof_on && g_prof_used < g_prof.size()) ? &g_prof[g_prof_used++] : nullptr;
    if (r) { r->weight_bytes = N * K * 2; (void)hipEventRecord(r->start, s); }
    launch_gemm(a_frag, true, M, K, w, N, out, ldo, p, s, direct);
    if (r) (void)hipEventRecord(r->stop, s);
}

// ------------------------------------------------------------------------------------------
struct WsLayout {
    size_t x, h, q, attn_out, act, partial, part_o, part_ml, logits, ssq, kv_lo, total;
    size_t partial_bytes;
};
#define ATTN_MAX_SPLITS 32

static WsLayout ws_layout(const bita_config &c, int batch, int rows) {
    const size_t M = (size_t)batch * rows;
    const int64_t nqkv = (int64_t)(c.n_heads + 2 * c.n_kv_heads) * c.head_dim, nq = (int64_t)c.n_heads * c.head_dim;
    WsLayout L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    L.x = take(M * c.d_model * 4);
    // GEMM inputs: two bf16 planes (hi, lo) in fragment order; queries: two row-major planes
    L.h = take(frag_bytes((int)M, c.d_model));
    L.q = take(2 * M * nq * 2);
    L.attn_out = take(frag_bytes((int)M, nq));
    L.act = take(frag_bytes((int)M, c.d_ffn));
    size_t pb = 0;
    const int64_t shapes[5][2] = {{nqkv, c.d_model}, {c.d_model, nq}, {2 * (int64_t)c.d_ffn, c.d_model},
                                  {c.d_model, c.d_ffn}, {c.vocab, c.d_model}};
    for (auto &s : shapes) {
        const GemmPlan p = gemm_plan((int)M, s[0], s[1]);
        const size_t b = (size_t)p.splits * M * s[0] * 4;
        if (b > pb) pb = b;
    }
    L.partial_bytes = pb;
    L.partial = take(pb);
    L.part_o = take((size_t)batch * c.n_heads * ATTN_MAX_SPLITS * rows * c.head_dim * 4);
    L.part_ml = take((size_t)batch * c.n_heads * ATTN_MAX_SPLITS * rows * 2 * 4);
    L.logits = take(M * c.vocab * 4);
    L.ssq = take(M * RMS_MAX_CHUNKS * 4);
    L.kv_lo = take(2 * M * c.n_kv_heads * c.head_dim * 2);   // low planes of one layer's pass-row K and V
    L.total = off;
    return L;
}

// Paging fields of a KV descriptor -> PageMap (table == nullptr when the cache is contiguous).
// ctx_upper: the number of leading slots per sequence the call may read.
int page_map_of(const bita_kv *kv, int ctx_upper, PageMap *pm, const char *who) {
    *pm = PageMap{nullptr, 0, 0, 0, 0};
    if (!kv->block_table) return BITA_OK;
    const int ps = kv->page_size;
    if (ps < 16 || (ps & (ps - 1)) || kv->n_pages <= 0 || kv->max_pages <= 0)
        return bita_set_error(BITA_ERR_INVALID_ARG, "%s: paged cache needs page_size a power of two >= 16 (got %d), n_pages and max_pages positive",
                              who, ps);
    if ((int64_t)kv->smax > (int64_t)kv->max_pages * ps)
        return bita_set_error(BITA_ERR_CAPACITY, "%s: smax %d exceeds the block table (%d pages of %d)", who, kv->smax, kv->max_pages, ps);
    int cap = (ctx_upper + ps - 1) / ps;
    if (cap > kv->max_pages) cap = kv->max_pages;
    if (cap > ATT_PAGE_TABLE_MAX)
        return bita_set_error(BITA_ERR_UNSUPPORTED, "%s: %d pages per sequence, at most %d", who, cap, ATT_PAGE_TABLE_MAX);
    *pm = PageMap{kv->block_table, __builtin_ctz((unsigned)ps), kv->n_pages, kv->max_pages, cap};
    return BITA_OK;
}

extern "C" size_t bita_workspace_bytes(const bita_model *m, int32_t batch, int32_t rows) {
    if (!m || batch <= 0 || rows <= 0) return 0;
    return ws_layout(m->cfg, batch, rows).total;
}

extern "C" int bita_verify_step(bita_model *m, const bita_kv *kv, const bita_tree_template *t,
                                const int32_t *d_token, const int32_t *d_ctx_len, int32_t batch,
                                void *d_workspace, size_t ws_bytes, int32_t kmax, int32_t *d_argmax,
                                int32_t *d_topk_ids, float *d_topk_val, float *d_logits, void *stream) {
    if (!m || !kv || !t || !d_token || !d_ctx_len || !d_workspace || !d_argmax || batch <= 0)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_verify_step: null argument or batch <= 0");
    const bita_config &c = m->cfg;
    const TemplateDev &td = t->dev;
    if (!kv->k_cache || !kv->v_cache || !kv->k_tree || !kv->v_tree)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_verify_step: null KV pointer");
    if (kv->rows != td.rows || kv->batch != batch)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_verify_step: kv rows/batch (%d, %d) do not match template/batch (%d, %d)",
                              kv->rows, kv->batch, td.rows, batch);
    if (td.rows > td.n_tree && td.n_mask != c.n_mask)
        return bita_set_error(BITA_ERR_BAD_TREE, "bita_verify_step: template n_mask %d != model n_mask %d", td.n_mask, c.n_mask);
    const int n_sel_mask = td.n_groups * td.n_mask;
    if (n_sel_mask > 0 && d_topk_ids && (kmax <= 0 || kmax > BITA_MAX_TOPK || kmax > c.vocab))
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_verify_step: kmax must be in 1..%d", BITA_MAX_TOPK);
    if (kv->ctx_hint < 0 || kv->ctx_hint > kv->smax)
        return bita_set_error(BITA_ERR_CAPACITY, "bita_verify_step: ctx_hint %d outside cache capacity %d", kv->ctx_hint, kv->smax);
    const int deepest = td.depth_max + td.n_mask;       // mask chains extend the depth by up to n
    if (kv->ctx_hint + deepest >= c.max_pos)
        return bita_set_error(BITA_ERR_CAPACITY, "bita_verify_step: position %d beyond rotary table (%d)", kv->ctx_hint + deepest, c.max_pos);
    const WsLayout L = ws_layout(c, batch, td.rows);
    if (ws_bytes < L.total)
        return bita_set_error(BITA_ERR_CAPACITY, "bita_verify_step: workspace %zu < %zu bytes", ws_bytes, L.total);
    PageMap pm;
    if (int rc = page_map_of(kv, kv->ctx_hint, &pm, "bita_verify_step")) return rc;

    hipStream_t s = (hipStream_t)stream;
    unsigned char *ws = (unsigned char *)d_workspace;
    float *x = (float *)(ws + L.x), *partial = (float *)(ws + L.partial);
    unsigned char *h = ws + L.h, *q = ws + L.q, *attn_out = ws + L.attn_out, *act = ws + L.act;
    float *part_o = (float *)(ws + L.part_o), *part_ml = (float *)(ws + L.part_ml);
    float *logits = d_logits ? d_logits : (float *)(ws + L.logits);
    float *ssq = (float *)(ws + L.ssq);
    unsigned char *k_lo = ws + L.kv_lo;
    const int M = batch * td.rows, d = c.d_model, hd = c.head_dim;
    const RowScale rs_norm = {ssq, (d / 4 + 255) / 256, 1.0f / (float)d, c.rms_eps};
    const int64_t nq = (int64_t)c.n_heads * hd, nqkv = (int64_t)(c.n_heads + 2 * c.n_kv_heads) * hd;
    unsigned char *q_lo = q + (size_t)M * nq * 2;
    unsigned char *v_lo = k_lo + (size_t)M * c.n_kv_heads * hd * 2;
    const GemmPlan p_qkv = gemm_plan(M, nqkv, d), p_o = gemm_plan(M, d, nq),
                   p_gu = gemm_plan(M, 2 * (int64_t)c.d_ffn, d), p_dn = gemm_plan(M, d, c.d_ffn),
                   p_lm = gemm_plan(M, c.vocab, d);
    AttnPlan ap = attn_plan(batch, td.rows, c.n_heads, hd, kv->ctx_hint, c.n_prompt);
    if (ap.splits > ATTN_MAX_SPLITS) ap.splits = ATTN_MAX_SPLITS;
    const size_t kv_layer_cache = pm.table ? (size_t)kv->n_pages * c.n_kv_heads * kv->page_size * hd * 2
                                           : (size_t)batch * c.n_kv_heads * kv->smax * hd * 2;
    const size_t kv_layer_tree = (size_t)batch * c.n_kv_heads * td.rows * hd * 2;

    launch_embed(d_token, td, batch, m->tok_emb, m->mask_emb, d, c.vocab, x, s);
    int pending = 0;                                    // split-K partials waiting to be added to x
    for (int l = 0; l < c.n_layers; l++) {
        launch_rmsnorm_prep(x, partial, pending, M, d, m->attn_norm[l], h, ssq, s);
        timed_gemm(h, M, d, m->wqkv[l], nqkv, partial, nqkv, p_qkv, s);
        void *kt = (unsigned char *)kv->k_tree + l * kv_layer_tree, *vt = (unsigned char *)kv->v_tree + l * kv_layer_tree;
        launch_qkv_rope(partial, p_qkv.splits, batch, td, c.n_heads, c.n_kv_heads, hd, d_ctx_len, m->rope_cos,
                        m->rope_sin, c.max_pos, q, q_lo, kt, vt, k_lo, v_lo, rs_norm, s);
        launch_tree_attention(td, q, q_lo, (unsigned char *)kv->k_cache + l * kv_layer_cache,
                              (unsigned char *)kv->v_cache + l * kv_layer_cache, kt, vt, k_lo, v_lo, m->prompt_k[l],
                              m->prompt_v[l], d_ctx_len, d_token, batch, c.n_heads, c.n_kv_heads, hd, c.n_prompt, kv->smax,
                              ap, part_o, part_ml, attn_out, nullptr, true, pm, s);
        timed_gemm(attn_out, M, nq, m->wo[l], d, partial, d, p_o, s);
        launch_rmsnorm_prep(x, partial, p_o.splits, M, d, m->ffn_norm[l], h, ssq, s);
        // with a single split the gate/up GEMM gates in its own epilogue and writes the slab itself
        if (gemm_direct_output_possible(p_gu, GEMM_OUT_SILU)) {
            const GemmOutput gated = {GEMM_OUT_SILU, rs_norm, (uint16_t *)act, c.d_ffn};
            timed_gemm(h, M, d, m->w_gate_up[l], 2 * (int64_t)c.d_ffn, partial, 2 * (int64_t)c.d_ffn, p_gu, s, &gated);
        } else {
            timed_gemm(h, M, d, m->w_gate_up[l], 2 * (int64_t)c.d_ffn, partial, 2 * (int64_t)c.d_ffn, p_gu, s);
            launch_silu_mul(partial, p_gu.splits, M, c.d_ffn, act, rs_norm, s);
        }
        timed_gemm(act, M, c.d_ffn, m->w_down[l], d, partial, d, p_dn, s);
        pending = p_dn.splits;
    }
    launch_rmsnorm_prep(x, partial, pending, M, d, m->final_norm, h, ssq, s);
    // the final norm's row factor: in the LM head's own epilogue when it runs as a single split,
    // else in the reduction of its partial sums
    if (gemm_direct_output_possible(p_lm, GEMM_OUT_SCALED)) {
        const GemmOutput scaled = {GEMM_OUT_SCALED, rs_norm, nullptr, 0};
        timed_gemm(h, M, d, m->lm_head, c.vocab, logits, c.vocab, p_lm, s, &scaled);
    } else {
        timed_gemm(h, M, d, m->lm_head, c.vocab, partial, c.vocab, p_lm, s);
        launch_reduce_partials(partial, p_lm.splits, M, c.vocab, c.vocab, logits, rs_norm, s);
    }
    launch_select(logits, batch, td, c.vocab, kmax, d_argmax, n_sel_mask > 0 ? d_topk_ids : nullptr, d_topk_val, s);
    BITA_HIP_CHECK(hipGetLastError());
    return BITA_OK;
}

int compact_kv_launch(const bita_config &cfg, const bita_kv *kv, const PageMap &pm, const int32_t *d_path,
                      int path_stride, const int32_t *d_n_acc, int32_t *d_ctx_len, int batch, hipStream_t s);

extern "C" int bita_compact_kv(const bita_model *m, const bita_kv *kv, const int32_t *d_path,
                               int32_t path_stride, const int32_t *d_n_acc, int32_t *d_ctx_len,
                               int32_t batch, void *stream) {
    if (!m || !kv || !d_path || !d_n_acc || !d_ctx_len || batch <= 0 || path_stride <= 0)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_compact_kv: null argument or non-positive size");
    if (!kv->k_cache || !kv->v_cache || !kv->k_tree || !kv->v_tree || kv->batch != batch)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_compact_kv: bad KV descriptor");
    if (path_stride > kv->rows)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_compact_kv: path_stride %d exceeds rows %d", path_stride, kv->rows);
    if (kv->ctx_hint + path_stride > kv->smax)
        return bita_set_error(BITA_ERR_CAPACITY, "bita_compact_kv: ctx_hint %d + %d accepted rows exceed cache capacity %d",
                              kv->ctx_hint, path_stride, kv->smax);
    PageMap pm;
    if (int rc = page_map_of(kv, kv->ctx_hint + path_stride, &pm, "bita_compact_kv")) return rc;
    compact_kv_launch(m->cfg, kv, pm, d_path, path_stride, d_n_acc, d_ctx_len, batch, (hipStream_t)stream);
    BITA_HIP_CHECK(hipGetLastError());
    return BITA_OK;
}

// ------------------------------------------------------------------------------------------
extern "C" size_t bita_attention_workspace_bytes(int32_t batch, int32_t rows, int32_t n_heads, int32_t head_dim,
                                                 int32_t ctx_hint, int32_t n_prompt) {
    if (batch <= 0 || rows <= 0 || n_heads <= 0 || head_dim <= 0) return 0;
    const AttnPlan p = attn_plan(batch, rows, n_heads, head_dim, ctx_hint, n_prompt);
    return align_up(p.part_o_bytes, 256) + align_up(p.part_ml_bytes, 256);
}

extern "C" int bita_tree_attention(const bita_tree_template *t, const void *d_q, const void *d_q_lo,
                                   const void *d_k_cache,
                                   const void *d_v_cache, const void *d_k_tree, const void *d_v_tree,
                                   const void *d_k_tree_lo, const void *d_v_tree_lo, const void *d_prompt_k, const void *d_prompt_v, const int32_t *d_ctx_len,
                                   int32_t batch, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim,
                                   int32_t n_prompt, int32_t smax, int32_t ctx_hint, void *d_ws, size_t ws_bytes,
                                   void *d_out, void *d_out_lo, void *stream) {
    if (!t || !d_q || !d_k_cache || !d_v_cache || !d_k_tree || !d_v_tree || !d_ctx_len || !d_ws || !d_out ||
        batch <= 0 || n_heads <= 0 || n_kv_heads <= 0 || n_heads % n_kv_heads || n_prompt < 0 ||
        (n_prompt > 0 && (!d_prompt_k || !d_prompt_v)))
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_tree_attention: bad argument");
    if (head_dim != 64 && head_dim != 128)
        return bita_set_error(BITA_ERR_UNSUPPORTED, "bita_tree_attention: head_dim must be 64 or 128");
    if (ctx_hint < 0 || ctx_hint > smax)
        return bita_set_error(BITA_ERR_CAPACITY, "bita_tree_attention: ctx_hint %d outside capacity %d", ctx_hint, smax);
    const AttnPlan p = attn_plan(batch, t->dev.rows, n_heads, head_dim, ctx_hint, n_prompt);
    const size_t need = align_up(p.part_o_bytes, 256) + align_up(p.part_ml_bytes, 256);
    if (ws_bytes < need) return bita_set_error(BITA_ERR_CAPACITY, "bita_tree_attention: workspace %zu < %zu", ws_bytes, need);
    float *part_o = (float *)d_ws, *part_ml = (float *)((unsigned char *)d_ws + align_up(p.part_o_bytes, 256));
    launch_tree_attention(t->dev, d_q, d_q_lo, d_k_cache, d_v_cache, d_k_tree, d_v_tree, d_k_tree_lo, d_v_tree_lo, d_prompt_k, d_prompt_v, d_ctx_len, nullptr,
                          batch, n_heads, n_kv_heads, head_dim, n_prompt, smax, p, part_o, part_ml, d_out,
                          d_out_lo, false, PageMap{nullptr, 0, 0, 0, 0}, (hipStream_t)stream);
    BITA_HIP_CHECK(hipGetLastError());
    return BITA_OK;
}

extern "C" int bita_select(const bita_tree_template *t, const float *d_logits, int32_t batch, int32_t vocab,
                           int32_t kmax, int32_t *d_argmax, int32_t *d_topk_ids, float *d_topk_val, void *stream) {
    if (!t || !d_logits || !d_argmax || batch <= 0 || vocab <= 0)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_select: bad argument");
    if (vocab % 16) return bita_set_error(BITA_ERR_UNSUPPORTED, "bita_select: vocab must be a multiple of 16");
    if (d_topk_ids && (kmax <= 0 || kmax > BITA_MAX_TOPK || kmax > vocab))
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_select: kmax must be in 1..%d", BITA_MAX_TOPK);
    launch_select(d_logits, batch, t->dev, vocab, kmax, d_argmax, d_topk_ids, d_topk_val, (hipStream_t)stream);
    BITA_HIP_CHECK(hipGetLastError());
    return BITA_OK;
}

extern "C" void bita_tune_gemm(int32_t variant, int32_t splits) { gemm_force_plan(variant, splits); }

extern "C" int bita_gemm_plan_info(int32_t m_rows, int64_t n_rows, int64_t k, int32_t *out4) {
    if (!out4 || m_rows <= 0 || n_rows <= 0 || k <= 0) return bita_set_error(BITA_ERR_INVALID_ARG, "bita_gemm_plan_info: bad argument");
    const GemmPlan p = gemm_plan(m_rows, n_rows, k);
    out4[0] = p.splits; out4[1] = p.variant; out4[2] = p.mt_pass; out4[3] = p.ksteps_per_split;
    return BITA_OK;
}

extern "C" size_t bita_gemm_workspace_bytes(int32_t m_rows, int64_t n_rows, int64_t k) {
    if (m_rows <= 0 || n_rows <= 0 || k <= 0) return 0;
    // split-K partials (never more than 32 splits) + the activations re-laid in fragment order
    return align_up((size_t)32 * m_rows * n_rows * 4, 256) + frag_bytes(m_rows, k);
}

extern "C" int bita_gemm(const void *d_a, const void *d_a_lo, int32_t m_rows, int64_t k, int64_t lda,
                         const void *d_w_packed, int64_t n_rows, void *d_ws, size_t ws_bytes, float *d_out,
                         void *stream) {
    if (!d_a || !d_w_packed || !d_ws || !d_out || m_rows <= 0 || k <= 0 || n_rows <= 0 || lda < k)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_gemm: bad argument");
    if (n_rows % 16 || k % 8 || lda % 8)
        return bita_set_error(BITA_ERR_UNSUPPORTED, "bita_gemm: n_rows must be a multiple of 16, k and lda of 8");
    const GemmPlan p = gemm_plan(m_rows, n_rows, k);
    const size_t part_bytes = align_up((size_t)p.splits * m_rows * n_rows * 4, 256);
    if (ws_bytes < part_bytes + frag_bytes(m_rows, k))
        return bita_set_error(BITA_ERR_CAPACITY, "bita_gemm: workspace too small");
    hipStream_t s = (hipStream_t)stream;
    void *frag = (unsigned char *)d_ws + part_bytes;
    launch_to_fragments(d_a, d_a_lo, m_rows, k, lda, frag, s);
    if (p.splits == 1) {
        launch_gemm(frag, d_a_lo != nullptr, m_rows, k, d_w_packed, n_rows, d_out, n_rows, p, s);
    } else {
        launch_gemm(frag, d_a_lo != nullptr, m_rows, k, d_w_packed, n_rows, (float *)d_ws, n_rows, p, s);
        launch_reduce_partials((const float *)d_ws, p.splits, m_rows, n_rows, n_rows, d_out, RowScale{nullptr, 0, 0.f, 0.f}, s);
    }
    BITA_HIP_CHECK(hipGetLastError());
    return BITA_OK;
}

// ------------------------------------------------------------------------------------------
// bita_gemm for callers that cannot allocate (HIP graph capture, serving loops, harnesses that
// forbid hipMalloc): the split-K partial sums and the re-laid activation fragments, which
// bita_gemm takes from the caller's workspace, live in a static device array instead.  Every GPU
// holds its own copy of the array at its own address; the address is looked up once per device.
#define BITA_NOALLOC_SCRATCH_BYTES (32u << 20)
#define BITA_NOALLOC_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[BITA_NOALLOC_SCRATCH_BYTES];
static void *g_scratch_ptr[BITA_NOALLOC_MAX_DEVICES] = {};
static std::mutex g_scratch_mutex;

// device address of `scratch` on the current device (looked up on the first call per device)
static int noalloc_scratch(void **ptr) {
    int dev = -1;
    BITA_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= BITA_NOALLOC_MAX_DEVICES)
        return bita_set_error(BITA_ERR_UNSUPPORTED, "bita_gemm_noalloc: device ordinal %d outside 0..%d", dev,
                              BITA_NOALLOC_MAX_DEVICES - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        BITA_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return bita_set_error(BITA_ERR_HIP, "bita_gemm_noalloc: null address for the scratch array on device %d", dev);
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return BITA_OK;
}

extern "C" size_t bita_gemm_noalloc_max_scratch_bytes(void) { return BITA_NOALLOC_SCRATCH_BYTES; }

extern "C" size_t bita_gemm_noalloc_scratch_bytes(int32_t m_rows, int64_t n_rows, int64_t k) {
    if (m_rows <= 0 || n_rows <= 0 || k <= 0) return 0;
    const GemmPlan p = gemm_plan(m_rows, n_rows, k);
    const size_t part = p.splits > 1 ? align_up((size_t)p.splits * m_rows * n_rows * 4, 256) : 0;
    return part + frag_bytes(m_rows, k);
}

extern "C" int bita_gemm_noalloc(const void *d_a, const void *d_a_lo, int32_t m_rows, int64_t k, int64_t lda,
                                 const void *d_w_packed, int64_t n_rows, float *d_out, void *stream) {
    if (!d_a || !d_w_packed || !d_out || m_rows <= 0 || k <= 0 || n_rows <= 0 || lda < k)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_gemm_noalloc: bad argument");
    if (n_rows % 16 || k % 8 || lda % 8)
        return bita_set_error(BITA_ERR_UNSUPPORTED, "bita_gemm_noalloc: n_rows must be a multiple of 16, k and lda of 8");
    const GemmPlan p = gemm_plan(m_rows, n_rows, k);
    const size_t part_bytes = p.splits > 1 ? align_up((size_t)p.splits * m_rows * n_rows * 4, 256) : 0;
    const size_t need = part_bytes + frag_bytes(m_rows, k);
    if (need > BITA_NOALLOC_SCRATCH_BYTES)
        return bita_set_error(BITA_ERR_CAPACITY,
                              "bita_gemm_noalloc: %d x %lld x %lld needs %zu bytes of scratch (%d k splits), the static "
                              "buffer holds %u; use bita_gemm with a workspace", m_rows, (long long)n_rows, (long long)k,
                              need, p.splits, BITA_NOALLOC_SCRATCH_BYTES);
    void *base = nullptr;
    if (int rc = noalloc_scratch(&base)) return rc;
    hipStream_t s = (hipStream_t)stream;
    float *partial = (float *)base;
    void *frag = (unsigned char *)base + part_bytes;
    // nothing in the scratch has to start at zero: the fragment kernel writes every granule the
    // GEMM reads, and the GEMM writes every partial sum the reduction reads
    launch_to_fragments(d_a, d_a_lo, m_rows, k, lda, frag, s);
    if (p.splits == 1) {
        launch_gemm(frag, d_a_lo != nullptr, m_rows, k, d_w_packed, n_rows, d_out, n_rows, p, s);
    } else {
        launch_gemm(frag, d_a_lo != nullptr, m_rows, k, d_w_packed, n_rows, partial, n_rows, p, s);
        launch_reduce_partials(partial, p.splits, m_rows, n_rows, n_rows, d_out, RowScale{nullptr, 0, 0.f, 0.f}, s);
    }
    BITA_HIP_CHECK(hipGetLastError());
    return BITA_OK;
}
