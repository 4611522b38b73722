// Integer kernels of the streamlined generation-and-verification loop (Sec. 3.2, Algorithm 1):
// next-tree token assignment, the greedy acceptance walk, and the K/V commit of accepted rows.
#include "common.h"

// token[v] of the next pass: draft row at depth dv with sibling rank j carries the j-th
// ranked prediction of mask (dv-1+shift) of the chosen group; rows without a prediction
// are inactive (-1); mask rows carry their index in the group; row 0 is the last emitted token.
__global__ void build_tree_kernel(TemplateDev t, const int32_t *__restrict__ root_token,
                                  const int32_t *__restrict__ cand, const int32_t *__restrict__ group,
                                  const int32_t *__restrict__ shift, int cand_rows, int kmax,
                                  int32_t *__restrict__ token) {
    const int b = blockIdx.x;
    const int g = group ? group[b] : 0;
    const int sh = shift ? shift[b] : 0;
    for (int v = threadIdx.x; v < t.rows; v += blockDim.x) {
        int tok;
        if (v == 0) {
            tok = root_token[b];
        } else if (v < t.n_tree) {
            const int lvl = t.depth[v] - 1 + sh;
            const int row = g * t.n_mask + lvl;
            // g < 0: the previous pass had no mask group to offer (accept writes -1 then): no drafts
            tok = (g >= 0 && lvl >= 0 && lvl < t.n_mask && row < cand_rows && t.rank[v] < kmax)
                      ? cand[((int64_t)b * cand_rows + row) * kmax + t.rank[v]] : -1;
        } else {
            tok = t.mask_index[v];
        }
        token[(int64_t)b * t.rows + v] = tok;
    }
}

// One wavefront per sequence.  At node v with greedy token a, the lanes test rows
// v+1.. in parallel for "tree child of v, active, token == a"; the lowest such row wins.
__global__ __launch_bounds__(64) void accept_kernel(TemplateDev t, const int32_t *__restrict__ token,
                                                    const int32_t *__restrict__ argmax,
                                                    int32_t *__restrict__ path, int32_t *__restrict__ n_acc,
                                                    int32_t *__restrict__ bonus, int32_t *__restrict__ emitted,
                                                    int32_t *__restrict__ next_group,
                                                    int32_t *__restrict__ next_shift) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int32_t *tok = token + (int64_t)b * t.rows;
    const int32_t *am = argmax + (int64_t)b * t.n_tree;
    const int stride = t.depth_max + 1;
    int32_t *p = path + (int64_t)b * stride, *e = emitted + (int64_t)b * stride;
    for (int i = lane; i < stride; i += 64) { p[i] = -1; e[i] = -1; }
    __syncthreads();
    int v = 0, len = 1;
    if (lane == 0) p[0] = 0;
    int a = am[0];
    while (len <= t.depth_max) {
        int found = -1;
        for (int base = v + 1; base < t.n_tree && found < 0; base += 64) {
            const int c = base + lane;
            const bool hit = c < t.n_tree && t.parent[c] == v && tok[c] >= 0 && tok[c] == a;
            const unsigned long long m = __ballot(hit);
            if (m) found = base + __ffsll((long long)m) - 1;
        }
        if (found < 0) break;
        if (lane == 0) { p[len] = found; e[len - 1] = a; }
        v = found;
        len++;
        a = am[v];
    }
    if (lane == 0) {
        e[len - 1] = a;
        n_acc[b] = len;
        bonus[b] = a;
        const int g = t.group_of_node[v];
        if (next_group) next_group[b] = g >= 0 ? g : t.group_of_node[0];
        if (next_shift) next_shift[b] = g >= 0 ? 0 : len - 1;
    }
}

// cache[l][b][h][ctx_len + i][:] <- tree[l][b][h][path[i]][:], 16 bytes per lane.
// grid: (layer * kv-head, slot i, sequence).  ctx_len is advanced by a second tiny kernel so
// every workgroup of this one reads the old value.
__global__ void compact_kv_kernel(uint4 *__restrict__ k_cache, uint4 *__restrict__ v_cache,
                                  const uint4 *__restrict__ k_tree, const uint4 *__restrict__ v_tree,
                                  const int32_t *__restrict__ path, int path_stride,
                                  const int32_t *__restrict__ n_acc, const int32_t *__restrict__ ctx_len,
                                  int batch, int Hkv, int smax, int rows, int row_u4, PageMap pm) {
    const int lh = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
    const int n = n_acc[b];
    if (i >= n) return;
    const int lc = ctx_len[b];
    if (lc + n > smax) return;
    const int src_row = path[(int64_t)b * path_stride + i];
    if (src_row < 0 || src_row >= rows) return;
    const int l = lh / Hkv, h = lh % Hkv;
    const int64_t src = ((((int64_t)l * batch + b) * Hkv + h) * rows + src_row) * row_u4;
    int64_t dst = ((((int64_t)l * batch + b) * Hkv + h) * smax + lc + i) * row_u4;
    if (pm.table) {                                     // page pools [L][n_pages][Hkv][page][hd]
        const int slot = lc + i;
        const int page = min(max(pm.table[(int64_t)b * pm.max_pages + (slot >> pm.page_lg)], 0), pm.n_pages - 1);
        dst = (((((int64_t)l * pm.n_pages + page) * Hkv + h) << pm.page_lg) + (slot & ((1 << pm.page_lg) - 1))) * row_u4;
    }
    for (int j = threadIdx.x; j < row_u4; j += blockDim.x) {
        k_cache[dst + j] = k_tree[src + j];
        v_cache[dst + j] = v_tree[src + j];
    }
}
__global__ void advance_ctx_kernel(const int32_t *__restrict__ n_acc, int32_t *__restrict__ ctx_len,
                                   int batch, int smax) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < batch && ctx_len[b] + n_acc[b] <= smax) ctx_len[b] += n_acc[b];
}

extern "C" int bita_build_tree(const bita_tree_template *t, const int32_t *d_root_token,
                               const int32_t *d_cand, int32_t cand_rows, int32_t kmax,
                               const int32_t *d_group, const int32_t *d_shift, int32_t batch,
                               int32_t *d_token, void *stream) {
    if (!t || !d_root_token || !d_token || batch <= 0)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_build_tree: null argument or batch <= 0");
    if (t->dev.n_tree > 1 && (!d_cand || cand_rows <= 0 || kmax <= 0 || kmax > BITA_MAX_TOPK))
        return bita_set_error(BITA_ERR_INVALID_ARG,
                              "bita_build_tree: candidates needed, cand_rows > 0, 1 <= kmax <= %d",
                              BITA_MAX_TOPK);
    hipLaunchKernelGGL(build_tree_kernel, dim3(batch), dim3(64), 0, (hipStream_t)stream, t->dev,
                       d_root_token, d_cand, d_group, d_shift, cand_rows, kmax, d_token);
    BITA_HIP_CHECK(hipGetLastError());
    return BITA_OK;
}

extern "C" int bita_accept(const bita_tree_template *t, const int32_t *d_token, const int32_t *d_argmax,
                           int32_t batch, int32_t *d_path, int32_t *d_n_acc, int32_t *d_bonus,
                           int32_t *d_emitted, int32_t *d_next_group, int32_t *d_next_shift,
                           void *stream) {
    if (!t || !d_token || !d_argmax || !d_path || !d_n_acc || !d_bonus || !d_emitted || batch <= 0)
        return bita_set_error(BITA_ERR_INVALID_ARG, "bita_accept: null argument or batch <= 0");
    hipLaunchKernelGGL(accept_kernel, dim3(batch), dim3(64), 0, (hipStream_t)stream, t->dev, d_token,
                       d_argmax, d_path, d_n_acc, d_bonus, d_emitted, d_next_group, d_next_shift);
    BITA_HIP_CHECK(hipGetLastError());
    return BITA_OK;
}

int compact_kv_launch(const bita_config &cfg, const bita_kv *kv, const PageMap &pm, const int32_t *d_path,
                      int path_stride, const int32_t *d_n_acc, int32_t *d_ctx_len, int batch, hipStream_t s) {
    const int row_u4 = cfg.head_dim * 2 / 16;
    dim3 grid(cfg.n_layers * cfg.n_kv_heads, path_stride, batch);
    hipLaunchKernelGGL(compact_kv_kernel, grid, dim3(16), 0, s, (uint4 *)kv->k_cache, (uint4 *)kv->v_cache,
                       (const uint4 *)kv->k_tree, (const uint4 *)kv->v_tree, d_path, path_stride, d_n_acc,
                       d_ctx_len, batch, cfg.n_kv_heads, kv->smax, kv->rows, row_u4, pm);
    hipLaunchKernelGGL(advance_ctx_kernel, dim3((batch + 63) / 64), dim3(64), 0, s, d_n_acc, d_ctx_len,
                       batch, kv->smax);
    return BITA_OK;
}
