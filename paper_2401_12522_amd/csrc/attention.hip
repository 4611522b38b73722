// Tree-masked attention of the verify pass (Sec. 3.2, "tree-based attention"): every row of
// the pass attends to all cached tokens and to its ancestors-or-self among the rows of the
// pass; mask-token rows additionally attend to the per-layer prompt prefix.
//
// Flash-style, one workgroup per (sequence, query head, key split):
//  * the key axis [prefix | cache | pass rows] is cut into 128-key tiles; K tiles are staged
//    in LDS row-major, V tiles transposed, so both feed v_mfma_f32_16x16x32_bf16 with one
//    16-byte LDS read per operand;
//  * the 4 wavefronts split each tile's keys (32 each) and keep their own online-softmax
//    state for all query rows, merged through LDS at the end (fixed order, deterministic);
//  * S^T = K Q^T is computed so that its accumulator layout is already the B-operand layout
//    of O^T = V^T P^T: the probabilities never leave registers;
//  * the tree mask is derived from per-row ancestor bitsets and only evaluated in tiles that
//    touch the prefix or the pass rows; pure cache tiles take an unmasked path;
//  * the K/V of the pass rows are not yet rounded to the cache format: they come as two bf16
//    planes.  Tiles over the pass rows hold 64 keys, each followed (4 slots later inside a
//    lane's 8-key group) by a partner slot carrying the low plane; the two scores are added
//    and the probability is copied to the partner before P.V, all lane-locally.
// Partial (m, l, O) per split are combined by attn_merge_kernel.
#include "common.h"

#define ATT_TK 128
#define ATT_WAVES 4
#define ATT_PAD 8   // bf16 elements of row padding in both LDS tiles

// 2^x for x <= 0 or -inf (softmax arguments): the bare hardware instruction, without the
// denormal-range fix-up of exp2f (results below 2^-126 flush to zero, which is what we want)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// two floats -> packed bf16 pair, round to nearest even (gfx950 has a native conversion)
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <int HD>
struct AttSmem {
    static constexpr int K_STRIDE = HD + ATT_PAD;          // bf16 per K row
    static constexpr int V_STRIDE = ATT_TK + ATT_PAD;      // bf16 per V^T row
    static constexpr int K_BYTES = ATT_TK * K_STRIDE * 2;
    static constexpr int V_BYTES = HD * V_STRIDE * 2;
    static constexpr int TILE_BYTES = K_BYTES + V_BYTES;
};

// LDS map: [K tile | V^T tile] (reused by the final merge) followed by the query fragments
// (two bf16 planes, MFMA operand order).
template <int HD, int MT>
constexpr int att_tile_region() {
    const int tile = AttSmem<HD>::TILE_BYTES;
    (void)MT;
    return tile;
}
template <int HD, int MT>
constexpr int att_smem_bytes() {
    return att_tile_region<HD, MT>() + 2 * MT * (HD / 32) * 1024;
}

template <int HD, int MT>
__global__ __launch_bounds__(ATT_WAVES * 64) void tree_attn_kernel(
    TemplateDev t, const uint16_t *__restrict__ q, const uint16_t *__restrict__ q_lo,
    const uint16_t *__restrict__ k_cache,
    const uint16_t *__restrict__ v_cache, const uint16_t *__restrict__ k_tree,
    const uint16_t *__restrict__ v_tree, const uint16_t *__restrict__ k_tree_lo,
    const uint16_t *__restrict__ v_tree_lo, const uint16_t *__restrict__ prompt_k,
    const uint16_t *__restrict__ prompt_v, const int32_t *__restrict__ ctx_len, int Hq, int Hkv,
    int P, int smax, int n_splits, int n_qblk, float scale_log2, float *__restrict__ part_o,
    float *__restrict__ part_ml) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int GPK = HD / 8;                    // 16-byte granules per key row
    constexpr int KSN = HD / 32;                   // k-steps of the QK^T contraction
    constexpr int NTN = HD / 16;                   // 16-wide tiles of the head dimension
    constexpr int K_IT = ATT_TK * GPK / 256;       // K granules per thread per tile
    constexpr int V_IT = ATT_TK / 2 * GPK / 256;   // V key-pair granules per thread per tile
    constexpr int KSTR = AttSmem<HD>::K_STRIDE * 2, VSTR = AttSmem<HD>::V_STRIDE * 2;   // bytes
    unsigned char *ks_lds = smem, *vt_lds = smem + AttSmem<HD>::K_BYTES;
    uint4 *q_lds = reinterpret_cast<uint4 *>(smem + att_tile_region<HD, MT>());   // [2][MT][KSN][64]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, c = lane & 15;
    const int split = blockIdx.x, h = blockIdx.y / n_qblk, qblk = blockIdx.y % n_qblk, b = blockIdx.z;
    const int kvh = h / (Hq / Hkv);
    const int R = t.rows, Lc = ctx_len[b];
    // key axis: tiles over [prefix | cache] (128 keys each), then tiles over the pass rows
    // (64 keys + 64 low-plane partner slots each)
    const int n_ctx_keys = P + Lc;
    const int n_ct = (n_ctx_keys + ATT_TK - 1) / ATT_TK;
    const int n_tiles = n_ct + (R + ATT_TK / 2 - 1) / (ATT_TK / 2);
    const int per_split = (n_tiles + n_splits - 1) / n_splits;
    const int tile_begin = split * per_split;
    const int tile_end = min(n_tiles, tile_begin + per_split);
    const int row0 = qblk * MT * 16;

    const uint16_t *pk = prompt_k + (int64_t)kvh * P * HD, *pv = prompt_v + (int64_t)kvh * P * HD;
    const uint16_t *ck = k_cache + ((int64_t)b * Hkv + kvh) * smax * HD;
    const uint16_t *cv = v_cache + ((int64_t)b * Hkv + kvh) * smax * HD;
    const int64_t tree_off = ((int64_t)b * Hkv + kvh) * R * HD;
    const uint16_t *tk = k_tree + tree_off, *tv = v_tree + tree_off;
    const uint16_t *tk_lo = k_tree_lo ? k_tree_lo + tree_off : nullptr;
    const uint16_t *tv_lo = v_tree_lo ? v_tree_lo + tree_off : nullptr;

    // Query fragments (B operand of S^T = K Q^T) go to LDS once, as two bf16 planes (value and
    // rounding residual): fragment (plane, mt, ks) holds, for lane (g, c),
    // Q[row0 + 16mt + c][32ks + 8g .. +8].  Rows beyond R are zero.
    bool row_ok[MT], row_mask[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        const int r = row0 + mt * 16 + c;
        row_ok[mt] = r < R;
        row_mask[mt] = row_ok[mt] && t.is_mask[r];
    }
    for (int f = wave; f < 2 * MT * KSN; f += ATT_WAVES) {
        const int plane = f / (MT * KSN), mt = (f / KSN) % MT, ks = f % KSN;
        const int r = row0 + mt * 16 + c;
        const uint16_t *src = plane ? q_lo : q;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r < R && src)
            v = *reinterpret_cast<const uint4 *>(src + (((int64_t)b * R + r) * Hq + h) * HD + ks * 32 + g * 8);
        q_lds[f * 64 + lane] = v;
    }

    f32x4 o_acc[NTN][MT];
    float m_run[MT], l_run[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        m_run[mt] = -INFINITY;
        l_run[mt] = 0.f;
#pragma unroll
        for (int nt = 0; nt < NTN; nt++) o_acc[nt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    uint4 k_stage[K_IT], v_stage[V_IT][2];
    // source row of slot `slot` of tile `tile` (nullptr: padding, staged as zeros)
    auto src_row = [&](int tile, int slot, const uint16_t *pp, const uint16_t *cp, const uint16_t *tp,
                       const uint16_t *tp_lo) -> const uint16_t * {
        if (tile < n_ct) {
            const int kidx = tile * ATT_TK + slot;
            if (kidx < P) return pp + (int64_t)kidx * HD;
            if (kidx < n_ctx_keys) return cp + (int64_t)(kidx - P) * HD;
            return nullptr;
        }
        const int j = (tile - n_ct) * (ATT_TK / 2) + (slot >> 3) * 4 + (slot & 3);   // pass row
        if (j >= R) return nullptr;
        if (slot & 4) return tp_lo ? tp_lo + (int64_t)j * HD : nullptr;            // partner slot
        return tp + (int64_t)j * HD;
    };
    auto prefetch = [&](int tile) {
#pragma unroll
        for (int it = 0; it < K_IT; it++) {
            const int id = it * 256 + tid, key = id / GPK, part = id % GPK;
            const uint16_t *p = src_row(tile, key, pk, ck, tk, tk_lo);
            k_stage[it] = p ? *reinterpret_cast<const uint4 *>(p + part * 8) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int it = 0; it < V_IT; it++) {
            const int id = it * 256 + tid, kp = id / GPK, part = id % GPK;
#pragma unroll
            for (int e = 0; e < 2; e++) {
                const uint16_t *p = src_row(tile, 2 * kp + e, pv, cv, tv, tv_lo);
                v_stage[it][e] = p ? *reinterpret_cast<const uint4 *>(p + part * 8) : make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto stage_to_lds = [&]() {
#pragma unroll
        for (int it = 0; it < K_IT; it++) {
            const int id = it * 256 + tid, key = id / GPK, part = id % GPK;
            *reinterpret_cast<uint4 *>(ks_lds + key * KSTR + part * 16) = k_stage[it];
        }
#pragma unroll
        for (int it = 0; it < V_IT; it++) {
            const int id = it * 256 + tid, kp = id / GPK, part = id % GPK;
            const uint32_t a[4] = {v_stage[it][0].x, v_stage[it][0].y, v_stage[it][0].z, v_stage[it][0].w};
            const uint32_t d[4] = {v_stage[it][1].x, v_stage[it][1].y, v_stage[it][1].z, v_stage[it][1].w};
#pragma unroll
            for (int j = 0; j < 4; j++) {
                // hd element 2j of both keys, then element 2j+1
                const uint32_t even = (a[j] & 0xFFFFu) | (d[j] << 16);
                const uint32_t odd = (a[j] >> 16) | (d[j] & 0xFFFF0000u);
                *reinterpret_cast<uint32_t *>(vt_lds + (part * 8 + 2 * j) * VSTR + kp * 4) = even;
                *reinterpret_cast<uint32_t *>(vt_lds + (part * 8 + 2 * j + 1) * VSTR + kp * 4) = odd;
            }
        }
    };

    if (tile_begin < tile_end) prefetch(tile_begin);
    const int kb = wave * 32;                                // this wave's keys inside a tile
    for (int tile = tile_begin; tile < tile_end; tile++) {
        __syncthreads();                                     // previous tile fully consumed
        stage_to_lds();
        __syncthreads();
        if (tile + 1 < tile_end) prefetch(tile + 1);
        const int base = tile * ATT_TK;
        const bool tree_tile = tile >= n_ct;
        const int tree_j0 = (tile - n_ct) * (ATT_TK / 2);   // first pass row of a pass-row tile
        if (tree_tile ? (tree_j0 + (kb >> 1) >= R) : (base + kb >= n_ctx_keys)) continue;   // only padding

        // S^T[key][q]: rows of sub-tile tt are keys 8*(i/4) + 4*tt + i%4, so that a lane ends
        // up with 8 consecutive keys (8g .. 8g+7) for its query row.
        f32x4 s_acc[MT][2];
#pragma unroll
        for (int mt = 0; mt < MT; mt++) s_acc[mt][0] = s_acc[mt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        bf16x8 kf[2][KSN];
#pragma unroll
        for (int tt = 0; tt < 2; tt++) {
            const int key = kb + 8 * (c >> 2) + 4 * tt + (c & 3);
#pragma unroll
            for (int ks = 0; ks < KSN; ks++)
                kf[tt][ks] = __builtin_bit_cast(
                    bf16x8, *reinterpret_cast<const uint4 *>(ks_lds + key * KSTR + (ks * 32 + g * 8) * 2));
        }
#pragma unroll
        for (int ks = 0; ks < KSN; ks++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                const bf16x8 qh = __builtin_bit_cast(bf16x8, q_lds[((0 * MT + mt) * KSN + ks) * 64 + lane]);
                const bf16x8 ql = __builtin_bit_cast(bf16x8, q_lds[((1 * MT + mt) * KSN + ks) * 64 + lane]);
#pragma unroll
                for (int tt = 0; tt < 2; tt++) {
                    s_acc[mt][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tt][ks], qh, s_acc[mt][tt], 0, 0, 0);
                    s_acc[mt][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tt][ks], ql, s_acc[mt][tt], 0, 0, 0);
                }
            }

        const bool need_mask = tree_tile || (base < P) || (base + ATT_TK > n_ctx_keys);
        bf16x8 pf[MT], pf_lo[MT];
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            float sv[8];
#pragma unroll
            for (int tt = 0; tt < 2; tt++)
#pragma unroll
                for (int r = 0; r < 4; r++) sv[tt * 4 + r] = s_acc[mt][tt][r] * scale_log2;
            if (tree_tile) {                 // score = q.k_hi + q.k_lo; partner slots leave the softmax
#pragma unroll
                for (int e = 0; e < 4; e++) sv[e] += sv[e + 4];
            }
            if (need_mask) {
                // 8-bit visibility word for this lane's slots, built with integer selects only:
                // prefix -> mask rows, cache -> all rows, pass rows -> ancestor bits.
                const int rq = row0 + mt * 16 + c;
                uint32_t bits = 0;
                if (row_ok[mt]) {
                    if (tree_tile) {
                        const int j0 = tree_j0 + ((kb >> 3) + g) * 4;     // this lane's 4 pass rows (4-aligned)
                        uint32_t four = 0;
                        if (j0 < R) four = (uint32_t)(t.anc[(int64_t)rq * t.words + (j0 >> 6)] >> (j0 & 63)) & 0xFu;
#pragma unroll
                        for (int e = 0; e < 4; e++)
                            bits |= ((j0 + e < R) ? ((four >> e) & 1u) : 0u) << e;
                    } else {
                        const int k0 = base + kb + 8 * g;
#pragma unroll
                        for (int e = 0; e < 8; e++) {
                            const int kidx = k0 + e;
                            const uint32_t in_prefix = kidx < P ? 1u : 0u;
                            const uint32_t in_cache = (kidx >= P && kidx < n_ctx_keys) ? 1u : 0u;
                            bits |= ((in_prefix & (row_mask[mt] ? 1u : 0u)) | in_cache) << e;
                        }
                    }
                }
#pragma unroll
                for (int e = 0; e < 8; e++) sv[e] = ((bits >> e) & 1u) ? sv[e] : -INFINITY;
            }
            float mx = sv[0];
#pragma unroll
            for (int e = 1; e < 8; e++) mx = fmaxf(mx, sv[e]);
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[mt], mx);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = fast_exp2(m_run[mt] - m_use);
            m_run[mt] = m_new;
            // probabilities as two bf16 planes (value and rounding residual), like every other
            // MFMA input of the pass
            float ps = 0.f;
            uint32_t pk2[4], pl2[4];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const float p0 = fast_exp2(sv[e] - m_use), p1 = fast_exp2(sv[e + 1] - m_use);
                ps += p0 + p1;
                const uint32_t hi = cvt_pk_bf16(p0, p1);
                pk2[e >> 1] = hi;
                pl2[e >> 1] = cvt_pk_bf16(p0 - __uint_as_float(hi << 16), p1 - __uint_as_float(hi & 0xFFFF0000u));
            }
            if (tree_tile) {                 // the low-plane value rows take the same probabilities
                pk2[2] = pk2[0];
                pk2[3] = pk2[1];
                pl2[2] = pl2[0];
                pl2[3] = pl2[1];
            }
            l_run[mt] = l_run[mt] * alpha + ps;
            pf[mt] = __builtin_bit_cast(bf16x8, make_uint4(pk2[0], pk2[1], pk2[2], pk2[3]));
            pf_lo[mt] = __builtin_bit_cast(bf16x8, make_uint4(pl2[0], pl2[1], pl2[2], pl2[3]));
#pragma unroll
            for (int nt = 0; nt < NTN; nt++) o_acc[nt][mt] *= alpha;
        }
        // O^T[hd][q] += V^T[hd][keys 8g..8g+7] * P^T
#pragma unroll
        for (int nt = 0; nt < NTN; nt++) {
            const bf16x8 vf = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const uint4 *>(vt_lds + (nt * 16 + c) * VSTR + (kb + 8 * g) * 2));
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                o_acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[mt], o_acc[nt][mt], 0, 0, 0);
                o_acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf_lo[mt], o_acc[nt][mt], 0, 0, 0);
            }
        }
    }

    // ---- merge the 4 wavefronts (each saw a disjoint key subset) --------------------------
    // Row statistics go through two small LDS arrays; the O accumulators are added pairwise
    // (3 <- nothing, 2+3 -> regions, 0 += 2, 1 += 3, then 0 += 1) through LDS in register order,
    // so every LDS access is a linear 1 KiB sweep, and wave 0 stores the result from registers.
    __syncthreads();
    float *sm = reinterpret_cast<float *>(smem), *sl = sm + ATT_WAVES * MT * 16;
    float4 *region = reinterpret_cast<float4 *>(smem + 2 * ATT_WAVES * MT * 16 * 4);   // 2 x [NTN*MT][64]
    constexpr int REGION_F4 = NTN * MT * 64;
    static_assert(2 * ATT_WAVES * MT * 16 * 4 + 2 * REGION_F4 * 16 <= att_smem_bytes<HD, MT>(), "merge scratch fits");
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        float l = l_run[mt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        l_run[mt] = l;
        if (g == 0) {
            sm[wave * MT * 16 + mt * 16 + c] = m_run[mt];
            sl[wave * MT * 16 + mt * 16 + c] = l;
        }
    }
    __syncthreads();
    float m_tot[MT], l_tot[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        float m = -INFINITY;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; w++) m = fmaxf(m, sm[w * MT * 16 + mt * 16 + c]);
        const float m_use = (m == -INFINITY) ? 0.f : m;
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; w++)
            l += sl[w * MT * 16 + mt * 16 + c] * fast_exp2(sm[w * MT * 16 + mt * 16 + c] - m_use);
        const float f = fast_exp2(m_run[mt] - m_use);
        m_tot[mt] = m;
        l_tot[mt] = l;
#pragma unroll
        for (int nt = 0; nt < NTN; nt++) o_acc[nt][mt] *= f;
    }
    auto park = [&](int which) {
#pragma unroll
        for (int nt = 0; nt < NTN; nt++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
                region[which * REGION_F4 + (nt * MT + mt) * 64 + lane] =
                    make_float4(o_acc[nt][mt][0], o_acc[nt][mt][1], o_acc[nt][mt][2], o_acc[nt][mt][3]);
    };
    auto absorb = [&](int which) {
#pragma unroll
        for (int nt = 0; nt < NTN; nt++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                const float4 v = region[which * REGION_F4 + (nt * MT + mt) * 64 + lane];
                o_acc[nt][mt][0] += v.x; o_acc[nt][mt][1] += v.y; o_acc[nt][mt][2] += v.z; o_acc[nt][mt][3] += v.w;
            }
    };
    if (wave >= 2) park(wave - 2);
    __syncthreads();
    if (wave < 2) absorb(wave);
    __syncthreads();
    if (wave == 1) park(0);
    __syncthreads();
    if (wave != 0) return;
    absorb(0);
    // ---- write the split's partial result: lane (g, c) holds O[row c][hd 16nt + 4g .. +4] ------
    const int64_t pbase = (((int64_t)b * Hq + h) * n_splits + split) * R;
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        const int r = row0 + mt * 16 + c;
        if (r < R) {
#pragma unroll
            for (int nt = 0; nt < NTN; nt++)
                *reinterpret_cast<float4 *>(part_o + (pbase + r) * HD + nt * 16 + 4 * g) =
                    make_float4(o_acc[nt][mt][0], o_acc[nt][mt][1], o_acc[nt][mt][2], o_acc[nt][mt][3]);
            if (g == 0) {
                part_ml[(pbase + r) * 2] = m_tot[mt];
                part_ml[(pbase + r) * 2 + 1] = l_tot[mt];
            }
        }
    }
}

// out[b][r][h*HD + 4i .. +4] = sum_s w_s O_s / sum_s w_s l_s,  w_s = 2^(m_s - max m).
// One thread per 4 head-dim elements; blockDim = (HD/4) * heads_per_block.
__global__ void attn_merge_kernel(const float *__restrict__ part_o, const float *__restrict__ part_ml,
                                  int R, int Hq, int HD, int n_splits, uint16_t *__restrict__ out,
                                  int as_fragments, int m_tiles) {
    const int per_head = HD >> 2;
    const int r = blockIdx.x, b = blockIdx.z;
    const int h = blockIdx.y * (blockDim.x / per_head) + threadIdx.x / per_head, i4 = threadIdx.x % per_head;
    if (h >= Hq) return;
    const int64_t pbase = ((int64_t)b * Hq + h) * n_splits;
    float m = -INFINITY;
    for (int s = 0; s < n_splits; s++) m = fmaxf(m, part_ml[((pbase + s) * R + r) * 2]);
    const float m_use = (m == -INFINITY) ? 0.f : m;
    float l = 0.f;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < n_splits; s++) {
        const float2 ml = *reinterpret_cast<const float2 *>(part_ml + ((pbase + s) * R + r) * 2);
        const float w = fast_exp2(ml.x - m_use);
        const float4 o = *reinterpret_cast<const float4 *>(part_o + ((pbase + s) * R + r) * HD + i4 * 4);
        l += w * ml.y;
        acc.x += w * o.x; acc.y += w * o.y; acc.z += w * o.z; acc.w += w * o.w;
    }
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    const float v[4] = {acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv};
    uint16_t hi[4], lo[4];
#pragma unroll
    for (int e = 0; e < 4; e++) split_bf16(v[e], hi[e], lo[e]);
    uint2 ph, pl;
    ph.x = hi[0] | ((uint32_t)hi[1] << 16); ph.y = hi[2] | ((uint32_t)hi[3] << 16);
    pl.x = lo[0] | ((uint32_t)lo[1] << 16); pl.y = lo[2] | ((uint32_t)lo[3] << 16);
    if (as_fragments) {                     // two planes, the O-projection's activation slab
        const int mrow = b * R + r, k = h * HD + i4 * 4, n_ksteps = (Hq * HD) >> 5;
        *reinterpret_cast<uint2 *>(out + frag_index(0, mrow, k, n_ksteps, m_tiles)) = ph;
        *reinterpret_cast<uint2 *>(out + frag_index(1, mrow, k, n_ksteps, m_tiles)) = pl;
    } else {
        *reinterpret_cast<uint2 *>(out + (((int64_t)b * R + r) * Hq + h) * HD + i4 * 4) = ph;
    }
}

AttnPlan attn_plan(int batch, int rows, int n_heads, int hd, int ctx_hint, int n_prompt) {
    AttnPlan p;
    const int n_tiles = (n_prompt + ctx_hint + ATT_TK - 1) / ATT_TK + (rows + ATT_TK / 2 - 1) / (ATT_TK / 2);
    const int n_qblk = (rows + 79) / 80;
    const int wgs = batch * n_heads * n_qblk;
    // the kernel's LDS footprint allows one workgroup per CU: ask for one round of <= 256
    int splits = 256 / wgs;
    if (splits > n_tiles) splits = n_tiles;
    if (splits < 1) splits = 1;
    if (splits > 32) splits = 32;
    // equal shares: with per = ceil(tiles/splits) tiles each, drop the splits left without work
    const int per = (n_tiles + splits - 1) / splits;
    splits = (n_tiles + per - 1) / per;
    p.splits = splits;
    p.part_o_bytes = (size_t)batch * n_heads * splits * rows * hd * sizeof(float);
    p.part_ml_bytes = (size_t)batch * n_heads * splits * rows * 2 * sizeof(float);
    return p;
}

template <int HD, int MT>
static void launch_attn_t(const TemplateDev &t, const void *q, const void *q_lo, const void *k_cache, const void *v_cache,
                          const void *k_tree, const void *v_tree, const void *k_tree_lo, const void *v_tree_lo,
                          const void *prompt_k,
                          const void *prompt_v, const int32_t *ctx_len, int batch, int Hq, int Hkv, int P,
                          int smax, const AttnPlan &p, float *part_o, float *part_ml, hipStream_t s) {
    constexpr int smem = att_smem_bytes<HD, MT>();
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)tree_attn_kernel<HD, MT>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        attr_set = true;
    }
    const int n_qblk = (t.rows + MT * 16 - 1) / (MT * 16);
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
    dim3 grid(p.splits, Hq * n_qblk, batch);
    hipLaunchKernelGGL((tree_attn_kernel<HD, MT>), grid, dim3(ATT_WAVES * 64), smem, s, t,
                       (const uint16_t *)q, (const uint16_t *)q_lo, (const uint16_t *)k_cache, (const uint16_t *)v_cache,
                       (const uint16_t *)k_tree, (const uint16_t *)v_tree, (const uint16_t *)k_tree_lo,
                       (const uint16_t *)v_tree_lo, (const uint16_t *)prompt_k,
                       (const uint16_t *)prompt_v, ctx_len, Hq, Hkv, P, smax, p.splits, n_qblk, scale_log2,
                       part_o, part_ml);
}

void launch_tree_attention(const TemplateDev &t, const void *q, const void *q_lo, const void *k_cache, const void *v_cache,
                           const void *k_tree, const void *v_tree, const void *k_tree_lo, const void *v_tree_lo,
                           const void *prompt_k,
                           const void *prompt_v, const int32_t *ctx_len, int batch, int Hq, int Hkv, int hd,
                           int P, int smax, const AttnPlan &p, float *part_o, float *part_ml, void *out,
                           bool out_as_fragments, hipStream_t s) {
    const bool small = t.rows <= 16;
    if (hd == 128) {
        if (small) launch_attn_t<128, 1>(t, q, q_lo, k_cache, v_cache, k_tree, v_tree, k_tree_lo, v_tree_lo, prompt_k, prompt_v, ctx_len, batch, Hq, Hkv, P, smax, p, part_o, part_ml, s);
        else launch_attn_t<128, 5>(t, q, q_lo, k_cache, v_cache, k_tree, v_tree, k_tree_lo, v_tree_lo, prompt_k, prompt_v, ctx_len, batch, Hq, Hkv, P, smax, p, part_o, part_ml, s);
    } else {
        if (small) launch_attn_t<64, 1>(t, q, q_lo, k_cache, v_cache, k_tree, v_tree, k_tree_lo, v_tree_lo, prompt_k, prompt_v, ctx_len, batch, Hq, Hkv, P, smax, p, part_o, part_ml, s);
        else launch_attn_t<64, 5>(t, q, q_lo, k_cache, v_cache, k_tree, v_tree, k_tree_lo, v_tree_lo, prompt_k, prompt_v, ctx_len, batch, Hq, Hkv, P, smax, p, part_o, part_ml, s);
    }
    const int heads_per_block = (256 / (hd / 4)) < Hq ? (256 / (hd / 4)) : Hq;
    hipLaunchKernelGGL(attn_merge_kernel, dim3(t.rows, (Hq + heads_per_block - 1) / heads_per_block, batch),
                       dim3(heads_per_block * (hd / 4)), 0, s, part_o, part_ml, t.rows,
                       Hq, hd, p.splits, (uint16_t *)out, out_as_fragments ? 1 : 0, (batch * t.rows + 15) / 16);
}
