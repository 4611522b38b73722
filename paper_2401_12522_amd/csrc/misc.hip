// Row-wise kernels of the verify step: embedding gather, RMSNorm (fused with the split-K
// reduction and the residual add), rotary embedding + tree K/V write, SwiGLU gating, and the
// vocabulary argmax / top-k selection with wavefront-shuffle reductions.
#include "common.h"

// ---------------------------------------------------------------------------------------
// Embedding: tree rows take tok_emb[token], mask rows mask_emb[index] (Sec. 3.1), inactive
// rows (token < 0) the zero vector.  x is the fp32 residual stream [B*R][d].
__global__ void embed_kernel(const int32_t *__restrict__ token, TemplateDev t,
                             const uint16_t *__restrict__ tok_emb, const uint16_t *__restrict__ mask_emb,
                             int d, int vocab, float *__restrict__ x) {
    const int row = blockIdx.x, r = row % t.rows;
    const int tok = token[row];
    const uint16_t *src = nullptr;
    if (t.is_mask[r]) {
        src = mask_emb + (int64_t)t.mask_index[r] * d;
    } else if (tok >= 0 && tok < vocab) {
        src = tok_emb + (int64_t)tok * d;
    }
    // d is a multiple of 32: 8 elements (16 bytes in, 32 out) per thread and iteration
    float4 *dst = reinterpret_cast<float4 *>(x + (int64_t)row * d);
#pragma unroll 4
    for (int i8 = threadIdx.x; i8 < (d >> 3); i8 += blockDim.x) {
        const uint4 q = src ? reinterpret_cast<const uint4 *>(src)[i8] : make_uint4(0, 0, 0, 0);
        dst[2 * i8] = make_float4(__uint_as_float(q.x << 16), __uint_as_float(q.x & 0xFFFF0000u),
                                  __uint_as_float(q.y << 16), __uint_as_float(q.y & 0xFFFF0000u));
        dst[2 * i8 + 1] = make_float4(__uint_as_float(q.z << 16), __uint_as_float(q.z & 0xFFFF0000u),
                                      __uint_as_float(q.w << 16), __uint_as_float(q.w & 0xFFFF0000u));
    }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// RMSNorm, first half.  Grid (row, 1024-column chunk): x += sum_s partial[s] (fixed order), then
// the *unnormalised* x * gain is written as two bf16 planes (hi, lo) in the GEMM's fragment
// order, and the chunk's sum of squares goes to ssq[row][chunk].  The row factor
// rsqrt(mean(x^2) + eps) is a scalar per row and commutes with the matrix product, so the GEMM
// applies it to its output rows; that keeps this kernel free of any row-wide reduction and
// lets all CUs share the split-K partial traffic.
__global__ __launch_bounds__(256) void rmsnorm_prep_kernel(float *__restrict__ x, const float *__restrict__ partial,
                                                           int splits, int M, int d,
                                                           const uint16_t *__restrict__ gain,
                                                           uint16_t *__restrict__ h_frag, float *__restrict__ ssq) {
    __shared__ float red[4];
    const int row = blockIdx.x, chunk = blockIdx.y, tid = threadIdx.x;
    const int n_ksteps = (d + 31) >> 5, m_tiles = (M + 15) >> 4;
    const int c = chunk * 256 + tid;                         // float4 column
    float ss = 0.f;
    if (c < (d >> 2)) {
        float4 *xr = reinterpret_cast<float4 *>(x + (int64_t)row * d);
        // Everything this thread reads is requested before anything is looked at (one memory
        // round trip): the residual, the gain and the first eight splits (the loads of a group
        // are independent; indices past the last split re-read it and are left out of the sum).
        // The partial sums are added in split order.
        float4 p[8];
        if (splits > 0) {
#pragma unroll
            for (int u = 0; u < 8; u++)
                p[u] = reinterpret_cast<const float4 *>(partial + ((int64_t)min(u, splits - 1) * M + row) * d)[c];
        }
        float4 v = xr[c];
        const uint2 gq = reinterpret_cast<const uint2 *>(gain)[c];
        if (splits > 0) {
#pragma unroll
            for (int u = 0; u < 8; u++)
                if (u < splits) { v.x += p[u].x; v.y += p[u].y; v.z += p[u].z; v.w += p[u].w; }
        }
        for (int s0 = 8; s0 < splits; s0 += 8) {
#pragma unroll
            for (int u = 0; u < 8; u++)
                p[u] = reinterpret_cast<const float4 *>(partial + ((int64_t)min(s0 + u, splits - 1) * M + row) * d)[c];
#pragma unroll
            for (int u = 0; u < 8; u++)
                if (s0 + u < splits) { v.x += p[u].x; v.y += p[u].y; v.z += p[u].z; v.w += p[u].w; }
        }
        if (splits > 0) xr[c] = v;
        ss = v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        const float o[4] = {v.x * bf16_to_f32((uint16_t)(gq.x & 0xFFFFu)), v.y * bf16_to_f32((uint16_t)(gq.x >> 16)),
                            v.z * bf16_to_f32((uint16_t)(gq.y & 0xFFFFu)), v.w * bf16_to_f32((uint16_t)(gq.y >> 16))};
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; e++) split_bf16(o[e], hi[e], lo[e]);
        uint2 ph, pl;
        ph.x = hi[0] | ((uint32_t)hi[1] << 16); ph.y = hi[2] | ((uint32_t)hi[3] << 16);
        pl.x = lo[0] | ((uint32_t)lo[1] << 16); pl.y = lo[2] | ((uint32_t)lo[3] << 16);
        const int pack_off = frag_pack_offset(M);
        *reinterpret_cast<uint2 *>(h_frag + frag_index(0, row, 4 * c, n_ksteps, m_tiles, pack_off)) = ph;
        *reinterpret_cast<uint2 *>(h_frag + frag_index(1, row, 4 * c, n_ksteps, m_tiles, pack_off)) = pl;
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    if (tid == 0) ssq[(int64_t)row * RMS_MAX_CHUNKS + chunk] = red[0] + red[1] + red[2] + red[3];
}

// ---------------------------------------------------------------------------------------
// QKV epilogue: sum split-K partials, rotate q and k by the row's position
// ctx_len + depth(row) in the half-split pairing, write q [B][R][Hq][hd] and the rows'
// k/v into the per-pass tree scratch [B][Hkv][R][hd].  q, k and v are all written as hi and lo
// bf16 planes; only the hi planes of accepted rows are ever committed to the cache.
#define ROPE_HEADS_PER_WG 4      // one wave per head: fewer, larger workgroups to dispatch
__global__ __launch_bounds__(64 * ROPE_HEADS_PER_WG) void qkv_rope_kernel(
    // (what the first loads depend on sits in the first 14 dwords, which arrive in registers)
    const float *__restrict__ partial, const int32_t *__restrict__ ctx_len, const int32_t *__restrict__ depth,
    const float *__restrict__ rs_ssq, int splits, int M, int R, int Hq, int Hkv, int hd, int max_pos,
    const float *__restrict__ rope_cos, const float *__restrict__ rope_sin, uint16_t *__restrict__ q,
    uint16_t *__restrict__ q_lo, uint16_t *__restrict__ k_tree, uint16_t *__restrict__ v_tree,
    uint16_t *__restrict__ k_tree_lo, uint16_t *__restrict__ v_tree_lo, int rs_chunks, float rs_inv_d, float rs_eps) {
    const int row = blockIdx.x, head = blockIdx.y * ROPE_HEADS_PER_WG + (threadIdx.x >> 6);   // head over Hq + 2*Hkv
    if (head >= Hq + 2 * Hkv) return;
    const int b = row / R, r = row % R;
    const int half = hd >> 1, i = threadIdx.x & 63;
    if (i >= half) return;
    // Two memory round trips: the row's position and the sums behind its norm factor, then the
    // rotary table entry together with the partial sums (the table is read for value heads too,
    // and ignored).
    const int row_ctx = ctx_len[b], row_depth = depth[r];
    const RowScale rs{rs_ssq, rs_chunks, rs_inv_d, rs_eps};
    const float sc = row_scale(rs, row);          // RMSNorm's row factor, deferred past the GEMM
    int pos = row_ctx + row_depth;
    pos = pos < max_pos ? pos : max_pos - 1;          // host checks capacity; stay in bounds
    const float tab_c = rope_cos[(int64_t)pos * half + i], tab_s = rope_sin[(int64_t)pos * half + i];
    const int64_t ncols = (int64_t)(Hq + 2 * Hkv) * hd;
    const int64_t col = (int64_t)head * hd + i;
    float lo = 0.f, hi = 0.f;
    for (int s0 = 0; s0 < splits; s0 += 8) {     // eight splits per round trip, summed in split order
        float pl[8], ph[8];
#pragma unroll
        for (int u = 0; u < 8; u++) {
            const float *p = partial + ((int64_t)min(s0 + u, splits - 1) * M + row) * ncols + col;
            pl[u] = p[0];
            ph[u] = p[half];
        }
#pragma unroll
        for (int u = 0; u < 8; u++)
            if (s0 + u < splits) { lo += pl[u]; hi += ph[u]; }
    }
    lo *= sc;
    hi *= sc;
    uint16_t *dst, *dst_lo = nullptr;
    if (head < Hq) {
        dst = q + ((int64_t)row * Hq + head) * hd;
        dst_lo = q_lo + ((int64_t)row * Hq + head) * hd;
    } else if (head < Hq + Hkv) {
        const int64_t o = (((int64_t)b * Hkv + (head - Hq)) * R + r) * hd;
        dst = k_tree + o;
        dst_lo = k_tree_lo + o;      // the pass keeps the rounding residual of its own K/V rows
    } else {
        const int64_t o = (((int64_t)b * Hkv + (head - Hq - Hkv)) * R + r) * hd;
        dst = v_tree + o;
        dst_lo = v_tree_lo + o;
    }
    if (head < Hq + Hkv) {
        const float nlo = lo * tab_c - hi * tab_s, nhi = hi * tab_c + lo * tab_s;
        lo = nlo;
        hi = nhi;
    }
    uint16_t a_hi, a_lo, b_hi, b_lo;
    split_bf16(lo, a_hi, a_lo);
    split_bf16(hi, b_hi, b_lo);
    dst[i] = a_hi;
    dst[i + half] = b_hi;
    if (dst_lo) {
        dst_lo[i] = a_lo;
        dst_lo[i + half] = b_lo;
    }
}

// ---------------------------------------------------------------------------------------
// SwiGLU gating on the gate/up GEMM output whose 16-column tiles alternate gate, up.  One
// thread per 8 consecutive features: sums the split-K partials, writes both bf16 planes of
// silu(gate) * up as one 16-byte store each into the down-projection's activation slab
// (fragment order; features beyond d_ffn inside the last k-step are written as zeros).
__global__ void silu_mul_kernel(const float *__restrict__ partial, int splits, int M, int F,
                                uint16_t *__restrict__ act_frag, RowScale rs) {
    const int f8 = blockIdx.x * blockDim.x + threadIdx.x;
    const int row = blockIdx.y;
    const int n_ksteps = (F + 31) >> 5, m_tiles = (M + 15) >> 4;
    const int f = f8 * 8;
    if (f >= n_ksteps * 32) return;
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; e++) o[e] = 0.f;
    if (f < F) {
        const int64_t cg = (int64_t)(f >> 4) * 32 + (f & 15);
        float g[8], u[8];
#pragma unroll
        for (int e = 0; e < 8; e++) g[e] = u[e] = 0.f;
        for (int s = 0; s < splits; s++) {
            const float4 *p = reinterpret_cast<const float4 *>(partial + ((int64_t)s * M + row) * (2 * (int64_t)F) + cg);
            const float4 g0 = p[0], g1 = p[1], u0 = p[4], u1 = p[5];
            g[0] += g0.x; g[1] += g0.y; g[2] += g0.z; g[3] += g0.w; g[4] += g1.x; g[5] += g1.y; g[6] += g1.z; g[7] += g1.w;
            u[0] += u0.x; u[1] += u0.y; u[2] += u0.z; u[3] += u0.w; u[4] += u1.x; u[5] += u1.y; u[6] += u1.z; u[7] += u1.w;
        }
        const float sc = row_scale(rs, row);      // RMSNorm's row factor, deferred past the GEMM
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const float gs = g[e] * sc;
            o[e] = gs / (1.0f + expf(-gs)) * (u[e] * sc);
        }
    }
    uint16_t hi[8], lo[8];
#pragma unroll
    for (int e = 0; e < 8; e++) split_bf16(o[e], hi[e], lo[e]);
    uint4 ph, pl;
    ph.x = hi[0] | ((uint32_t)hi[1] << 16); ph.y = hi[2] | ((uint32_t)hi[3] << 16);
    ph.z = hi[4] | ((uint32_t)hi[5] << 16); ph.w = hi[6] | ((uint32_t)hi[7] << 16);
    pl.x = lo[0] | ((uint32_t)lo[1] << 16); pl.y = lo[2] | ((uint32_t)lo[3] << 16);
    pl.z = lo[4] | ((uint32_t)lo[5] << 16); pl.w = lo[6] | ((uint32_t)lo[7] << 16);
    const int pack_off = frag_pack_offset(M);
    *reinterpret_cast<uint4 *>(act_frag + frag_index(0, row, f, n_ksteps, m_tiles, pack_off)) = ph;
    *reinterpret_cast<uint4 *>(act_frag + frag_index(1, row, f, n_ksteps, m_tiles, pack_off)) = pl;
}

// ---------------------------------------------------------------------------------------
// Selection over the vocabulary.  Order: value descending, lower id first among equals.
// One workgroup per selected row; pass p finds the best entry that comes strictly after
// the previous winner in that order, so k passes give the sorted top-k and pass 0 alone
// is the greedy argmax.  Reductions: per-lane scan (16-byte loads), wave shuffles, then the
// workgroup's 16 waves via LDS.
// (value, index) as one unsigned 64-bit key whose order is "larger value first, lower index on
// equal values": the float's bits made monotone (sign flip for positives, complement for
// negatives; -0 is first turned into +0) above the complemented index.  Logits are finite.
__device__ __forceinline__ unsigned long long select_key(float v, int i) {
    uint32_t u = __float_as_uint(v + 0.0f);
    u ^= (u & 0x80000000u) ? 0xFFFFFFFFu : 0x80000000u;
    return ((unsigned long long)u << 32) | (uint32_t)(0x7FFFFFFF - i);
}
__device__ __forceinline__ float select_key_value(unsigned long long k) {
    uint32_t u = (uint32_t)(k >> 32);
    u ^= (u & 0x80000000u) ? 0x80000000u : 0xFFFFFFFFu;
    return __uint_as_float(u);
}
#define SELECT_THREADS 1024
__global__ __launch_bounds__(SELECT_THREADS) void select_kernel(const float *__restrict__ logits, TemplateDev t,
                                                                int vocab, int kmax, int32_t *__restrict__ argmax,
                                                                int32_t *__restrict__ topk_ids,
                                                                float *__restrict__ topk_val) {
    constexpr int NW = SELECT_THREADS / 64;
    __shared__ unsigned long long sk[NW];
    const int b = blockIdx.y;
    const int sel = blockIdx.x;                       // 0..T-1 tree rows, then G*n mask rows
    const bool is_tree = sel < t.n_tree;
    const int r = is_tree ? sel : t.mask_rows[sel - t.n_tree];
    const int k = is_tree ? 1 : kmax;
    const float4 *row = reinterpret_cast<const float4 *>(logits + ((int64_t)b * t.rows + r) * vocab);   // vocab % 16 == 0
    // A row of up to 32768 logits is fetched once (8 independent 16-byte loads per thread) and
    // stays in registers for all k passes; longer rows are re-read from L2 pass by pass.
    constexpr int CACHE = 8;
    const int n4 = vocab >> 2;
    const bool cached = n4 <= CACHE * SELECT_THREADS;
    float4 cq[CACHE];
    if (cached) {
#pragma unroll
        for (int j = 0; j < CACHE; j++) {
            const int i4 = threadIdx.x + j * SELECT_THREADS;
            cq[j] = row[min(i4, n4 - 1)];                  // (slots past the row are skipped below)
        }
    }
    unsigned long long prev = ~0ull;                      // pass p selects the largest key below pass p-1's
    for (int p = 0; p < k; p++) {
        unsigned long long best = 0;                      // below every real key (indices are < 2^31 - 1)
        auto scan = [&](const float4 &q, int i4) __attribute__((always_inline)) {
            const float v[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const unsigned long long key = select_key(v[e], 4 * i4 + e);
                best = (key < prev && key > best) ? key : best;
            }
        };
        if (cached) {
#pragma unroll
            for (int j = 0; j < CACHE; j++) {
                const int i4 = threadIdx.x + j * SELECT_THREADS;
                if (i4 < n4) scan(cq[j], i4);
            }
        } else {
            for (int i4 = threadIdx.x; i4 < n4; i4 += SELECT_THREADS) scan(row[i4], i4);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const unsigned long long other = __shfl_xor(best, o, 64);
            best = other > best ? other : best;
        }
        if ((threadIdx.x & 63) == 0) sk[threadIdx.x >> 6] = best;
        __syncthreads();
        best = sk[0];
#pragma unroll
        for (int w = 1; w < NW; w++) best = sk[w] > best ? sk[w] : best;
        __syncthreads();
        prev = best;
        if (threadIdx.x == 0) {
            const int bi = 0x7FFFFFFF - (int)(uint32_t)(best & 0xFFFFFFFFu);
            if (is_tree) {
                argmax[b * t.n_tree + sel] = bi;
            } else {
                const int64_t o = ((int64_t)b * (t.n_groups * t.n_mask) + (sel - t.n_tree)) * kmax + p;
                topk_ids[o] = bi;
                if (topk_val) topk_val[o] = select_key_value(best);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
void launch_embed(const int32_t *token, const TemplateDev &t, int batch, const void *tok_emb,
                  const void *mask_emb, int d, int vocab, float *x, hipStream_t s) {
    hipLaunchKernelGGL(embed_kernel, dim3(batch * t.rows), dim3(256), 0, s, token, t,
                       (const uint16_t *)tok_emb, (const uint16_t *)mask_emb, d, vocab, x);
}
void launch_rmsnorm_prep(float *x, const float *partial, int splits, int M, int d, const void *gain,
                         void *h_frag, float *ssq, hipStream_t s) {
    const int chunks = (d / 4 + 255) / 256;
    hipLaunchKernelGGL(rmsnorm_prep_kernel, dim3(M, chunks), dim3(256), 0, s, x, partial, splits, M, d,
                       (const uint16_t *)gain, (uint16_t *)h_frag, ssq);
}
void launch_qkv_rope(const float *partial, int splits, int batch, const TemplateDev &t, int Hq,
                     int Hkv, int hd, const int32_t *ctx_len, const float *rope_cos,
                     const float *rope_sin, int max_pos, void *q, void *q_lo, void *k_tree, void *v_tree,
                     void *k_tree_lo, void *v_tree_lo, const RowScale &rs, hipStream_t s) {
    hipLaunchKernelGGL(qkv_rope_kernel, dim3(batch * t.rows, (Hq + 2 * Hkv + ROPE_HEADS_PER_WG - 1) / ROPE_HEADS_PER_WG),
                       dim3(64 * ROPE_HEADS_PER_WG), 0, s, partial, ctx_len, t.depth,
                       rs.ssq, splits, batch * t.rows, t.rows, Hq, Hkv, hd, max_pos, rope_cos, rope_sin,
                       (uint16_t *)q, (uint16_t *)q_lo, (uint16_t *)k_tree, (uint16_t *)v_tree,
                       (uint16_t *)k_tree_lo, (uint16_t *)v_tree_lo, rs.chunks, rs.inv_d, rs.eps);
}
void launch_silu_mul(const float *partial, int splits, int M, int F, void *act_frag, const RowScale &rs,
                     hipStream_t s) {
    const int n8 = ((F + 31) / 32) * 4;                       // threads (8 features each) per row
    hipLaunchKernelGGL(silu_mul_kernel, dim3((n8 + 127) / 128, M), dim3(128), 0, s, partial, splits, M, F,
                       (uint16_t *)act_frag, rs);
}
void launch_select(const float *logits, int batch, const TemplateDev &t, int vocab, int kmax,
                   int32_t *argmax, int32_t *topk_ids, float *topk_val, hipStream_t s) {
    const int n_sel = t.n_tree + (topk_ids ? t.n_groups * t.n_mask : 0);
    hipLaunchKernelGGL(select_kernel, dim3(n_sel, batch), dim3(SELECT_THREADS), 0, s, logits, t, vocab, kmax,
                       argmax, topk_ids, topk_val);
}
