// Context prefill as chunked chain passes (Algorithm 1, the pass over the input before the
// first draft exists; Sec. 3.2: ordinary tokens attend causally).  A chain template (row i's
// parent is row i-1, no mask rows) makes the verify pass a causal forward over
// [cache ‖ chunk]; committing rows 0..m-1 in order appends the chunk to the cache.
#include "common.h"
#include <vector>

// One launch per chunk: the chunk's token rows (gathered from the [B][n_tokens] input, -1 =
// inactive row beyond a sequence's end), the identity path and the number of rows to commit.
__global__ void prefill_chunk_kernel(const int32_t *__restrict__ tokens, int n_tokens,
                                     const int32_t *__restrict__ seq_len, int done, int m,
                                     int32_t *__restrict__ tok, int32_t *__restrict__ path,
                                     int32_t *__restrict__ n_acc) {
    const int b = blockIdx.x;
    const int len = seq_len ? min(max(seq_len[b], 0), n_tokens) : n_tokens;
    for (int i = threadIdx.x; i < m; i += blockDim.x) {
        tok[b * m + i] = done + i < len ? tokens[(int64_t)b * n_tokens + done + i] : -1;
        path[b * m + i] = i;
    }
    if (threadIdx.x == 0) n_acc[b] = min(max(len - done, 0), m);
}

// Greedy token after a sequence's last context token, once the chunk holding it has run.
__global__ void prefill_pick_kernel(const int32_t *__restrict__ argmax, const int32_t *__restrict__ seq_len,
                                    int n_tokens, int done, int m, int batch, int32_t *__restrict__ next_token) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    const int len = seq_len ? min(max(seq_len[b], 0), n_tokens) : n_tokens;
    const int last = len - 1 - done;
    if (last >= 0 && last < m) next_token[b] = argmax[b * m + last];
}

namespace {
struct PrefillWs { size_t step, tok, argmax, path, n_acc, total; };
PrefillWs prefill_layout(const bita_model *m, int batch, int chunk_rows) {
    PrefillWs L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) & ~(size_t)255; return o; };
    L.step = take(bita_workspace_bytes(m, batch, chunk_rows));
    L.tok = take((size_t)batch * chunk_rows * 4);
    L.argmax = take((size_t)batch * chunk_rows * 4);
    L.path = take((size_t)batch * chunk_rows * 4);
    L.n_acc = take((size_t)batch * 4);
    L.total = off;
    return L;
}
// The model's chain template of `rows` rows.  Created (device allocation and a blocking copy) the
// first time a row count is asked for, unless may_create is false: then a missing template is an
// error, which is how a call under stream capture stays free of allocations.
int chain_template(bita_model *m, int rows, bool may_create, bita_tree_template **out) {
    std::lock_guard<std::mutex> lock(m->chain_mutex);
    auto it = m->chains.find(rows);
    if (it != m->chains.end()) { *out = it->second; return BITA_OK; }
    if (!may_create)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_prefill: the stream is capturing and no chain template of %d rows "
                              "exists yet; call bita_prefill_prepare first", rows);
    std::vector<int32_t> parent(rows);
    std::vector<uint8_t> is_mask(rows, 0);
    for (int i = 0; i < rows; i++) parent[i] = i - 1;
    bita_tree_template *t = nullptr;
    if (int rc = bita_tree_template_create(parent.data(), is_mask.data(), rows, rows, 0, &t)) return rc;
    m->chains[rows] = t;
    *out = t;
    return BITA_OK;
}
}  // namespace

extern "C" int bita_prefill_prepare(bita_model *m, int32_t n_tokens, int32_t chunk_rows) {
    if (!m || n_tokens < 0 || chunk_rows <= 0 || chunk_rows > BITA_MAX_ROWS)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_prefill_prepare: null model, n_tokens < 0 or chunk_rows outside 1..%d",
                              BITA_MAX_ROWS);
    bita_tree_template *t = nullptr;
    if (n_tokens >= chunk_rows)
        if (int rc = chain_template(m, chunk_rows, true, &t)) return rc;
    if (n_tokens % chunk_rows)
        if (int rc = chain_template(m, n_tokens % chunk_rows, true, &t)) return rc;
    return BITA_OK;
}

extern "C" size_t bita_prefill_workspace_bytes(const bita_model *m, int32_t batch, int32_t chunk_rows) {
    if (!m || batch <= 0 || chunk_rows <= 0 || chunk_rows > BITA_MAX_ROWS) return 0;
    return prefill_layout(m, batch, chunk_rows).total;
}

extern "C" int bita_prefill(bita_model *m, const bita_kv *kv, const int32_t *d_tokens, int32_t n_tokens,
                            const int32_t *d_seq_len, int32_t *d_ctx_len, int32_t batch, int32_t chunk_rows,
                            void *d_workspace, size_t ws_bytes, int32_t *d_next_token, void *stream) {
    if (!m || !kv || (!d_tokens && n_tokens != 0) || !d_ctx_len || !d_workspace || batch <= 0 || n_tokens < 0)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_prefill: null argument, batch <= 0 or n_tokens < 0");
    if (chunk_rows <= 0 || chunk_rows > BITA_MAX_ROWS)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_prefill: chunk_rows must be in 1..%d", BITA_MAX_ROWS);
    if (kv->rows < chunk_rows || kv->batch != batch)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_prefill: tree scratch holds %d rows for %d sequences, need %d rows for %d",
                              kv->rows, kv->batch, chunk_rows, batch);
    if (kv->ctx_hint < 0 || (int64_t)kv->ctx_hint + n_tokens > kv->smax)
        return bita_set_error(BITA_ERR_CAPACITY, "bita_prefill: ctx_hint %d + %d tokens exceed cache capacity %d",
                              kv->ctx_hint, n_tokens, kv->smax);
    if ((int64_t)kv->ctx_hint + n_tokens > m->cfg.max_pos)
        return bita_set_error(BITA_ERR_CAPACITY, "bita_prefill: position %lld beyond rotary table (%d)",
                              (long long)kv->ctx_hint + n_tokens - 1, m->cfg.max_pos);
    const PrefillWs L = prefill_layout(m, batch, chunk_rows);
    if (ws_bytes < L.total)
        return bita_set_error(BITA_ERR_CAPACITY, "bita_prefill: workspace %zu < %zu bytes", ws_bytes, L.total);
    if (n_tokens == 0) return BITA_OK;

    hipStream_t s = (hipStream_t)stream;
    unsigned char *ws = (unsigned char *)d_workspace;
    int32_t *tok = (int32_t *)(ws + L.tok), *argmax = (int32_t *)(ws + L.argmax);
    int32_t *path = (int32_t *)(ws + L.path), *n_acc = (int32_t *)(ws + L.n_acc);

    // at most two templates (full chunks and the ragged last one), kept in the model handle; a
    // capturing stream must find them there
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (s) (void)hipStreamIsCapturing(s, &cap);
    (void)hipGetLastError();
    const bool may_create = cap == hipStreamCaptureStatusNone;
    int rc = BITA_OK;
    for (int done = 0; done < n_tokens && rc == BITA_OK; done += chunk_rows) {
        const int rows = n_tokens - done < chunk_rows ? n_tokens - done : chunk_rows;
        bita_tree_template *tmpl = nullptr;
        rc = chain_template(m, rows, may_create, &tmpl);
        if (rc != BITA_OK) break;
        bita_kv chunk_kv = *kv;
        chunk_kv.rows = rows;                           // tree scratch laid out as [L][B][Hkv][rows][hd]
        chunk_kv.ctx_hint = kv->ctx_hint + done;
        prefill_chunk_kernel<<<batch, 256, 0, s>>>(d_tokens, n_tokens, d_seq_len, done, rows, tok, path, n_acc);
        rc = bita_verify_step(m, &chunk_kv, tmpl, tok, d_ctx_len, batch, ws + L.step, L.tok - L.step, 1,
                              argmax, nullptr, nullptr, nullptr, stream);
        if (rc != BITA_OK) break;
        rc = bita_compact_kv(m, &chunk_kv, path, rows, n_acc, d_ctx_len, batch, stream);
        if (rc != BITA_OK) break;
        if (d_next_token)
            prefill_pick_kernel<<<(batch + 255) / 256, 256, 0, s>>>(argmax, d_seq_len, n_tokens, done, rows, batch,
                                                                    d_next_token);
    }
    if (rc != BITA_OK) return rc;
    BITA_HIP_CHECK(hipGetLastError());
    return BITA_OK;
}
