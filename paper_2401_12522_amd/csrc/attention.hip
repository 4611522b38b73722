// Tree-masked attention of the verify pass (Sec. 3.2, "tree-based attention"): every row of
// the pass attends to all cached tokens and to its ancestors-or-self among the rows of the
// pass; mask-token rows additionally attend to the per-layer prompt prefix.
//
// Flash-style, one workgroup per (sequence, query head, 16 query rows, key split):
//  * A workgroup owns one m-tile of 16 query rows and walks the key axis
//    [prefix | cache | pass rows] in chunks of 32 key slots.  Its 8 wavefronts (two per SIMD,
//    so that one wave's softmax arithmetic overlaps the other's matrix instructions) take
//    chunks round-robin and never synchronise inside the loop: each keeps its own
//    online-softmax state, merged through LDS once at the end (fixed order, deterministic).  With 16 rows
//    per workgroup no split over the keys is needed to fill the chip at the verify shapes,
//    so the output is normalised and written in place (no partial results, no second kernel)
//    unless the context is long enough for the planner to ask for key splits.
//  * Workgroups that read the same K/V head are placed on the same XCD (consecutive workgroup
//    ids go round-robin over the 8 XCDs), so a head's K/V comes from HBM once and from that
//    XCD's L2 for the other m-tiles and query heads of the group.
//  * K and V chunks go straight into LDS with global->LDS loads, row-major with an XOR swizzle
//    of the 16-byte columns; K is read back as A-operand fragments, V transposed
//    (ds_read_tr16_b64) as the A operand of O^T = V^T P^T.  A wave owns one 16 KiB chunk buffer:
//    it pulls all fragments of a chunk into registers first and refills the buffer with the
//    next chunk while it multiplies, the loads interleaved with the QK^T matrix instructions.
//  * S^T = K Q^T is computed so that its accumulator layout is already the B-operand layout
//    of O^T = V^T P^T: the probabilities never leave registers.  Queries, probabilities and
//    the pass rows' K/V are each two bf16 planes (value and rounding residual).
//  * The K/V of the pass rows are not yet rounded to the cache format.  A chunk over the pass
//    rows holds 16 keys, each followed (4 slots later inside a lane's 8-slot group) by a
//    partner slot carrying the low plane; the two scores are added and the probability is
//    copied to the partner before P.V, all lane-locally.
//  * The tree mask is derived from per-row ancestor bitsets and only evaluated in chunks that
//    touch the prefix, the ragged end of the cache or the pass rows.  A parent always has a
//    smaller row index than its child, so m-tile mt skips pass-row chunks beyond its own.
#include "common.h"
#include <type_traits>

#define ATT_WAVES 8
#define ATT_CHUNK 32            // key slots per chunk

// one all-zero K/V row (head dim <= 128): padding slots read it like any other row
static __device__ uint4 g_att_zero_row[16] = {};

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

// max / sum over the 4 lanes l, l^16, l^32, l^48 (the 16-lane groups of a wave) with the
// gfx950 row swaps: permlane32_swap(a, b) returns ([a.lanes0-31, b.lanes0-31],
// [a.lanes32-63, b.lanes32-63]); permlane16_swap does the same with rows 1 and 2 of each half
__device__ __forceinline__ float max_over_lane_groups(float x) {
    typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;
    u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_over_lane_groups(float x) {
    typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;
    u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// wait until at most N vector-memory operations of this wave are outstanding and all of its
// LDS reads have returned; nothing may be moved across it
template <int N>
__device__ __forceinline__ void att_wait() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0x0 << 8));
    asm volatile("" ::: "memory");
}
template <int I, int N, typename F>
__device__ __forceinline__ void att_static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        att_static_for<I + 1, N>(f);
    }
}

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// Transposed 16-bit LDS read (ds_read_b64_tr_b16): lane j of a 16-lane group receives, as
// element e, column j%4 of the four 16-bit values that lane 4e + j/4 of the group addressed.
// Issued as bare instructions: the V chunks reach LDS through global->LDS loads whose
// completion this kernel tracks itself (att_wait), and the compiler, unable to tell the ring
// slots apart, would otherwise drain every outstanding load before each such read.  The
// results are only valid after lds_wait_all().
template <int OFFSET>
__device__ __forceinline__ s16x4 lds_read_tr16(uint32_t lds_addr) {
    static_assert(OFFSET >= 0 && OFFSET < 65536, "ds offset field");
    s16x4 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(lds_addr), "n"(OFFSET));
    return v;
}
template <int OFFSET>
__device__ __forceinline__ u32x4 lds_read_b128(uint32_t lds_addr) {
    static_assert(OFFSET >= 0 && OFFSET < 65536, "ds offset field");
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(lds_addr), "n"(OFFSET));
    return v;
}
// wait for every LDS read of this wave; the registers pass through the statements so that no
// use of them can be scheduled ahead of the wait
template <int N, int M>
__device__ __forceinline__ void lds_wait_all(u32x4 (&k)[2][N], s16x4 (&v)[M][2]) {
    static_assert((N == 2 && M == 4) || (N == 4 && M == 8), "head dim 64 or 128");
    if constexpr (N == 4) {
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(k[0][0]), "+v"(k[0][1]), "+v"(k[0][2]), "+v"(k[0][3]), "+v"(k[1][0]), "+v"(k[1][1]),
                       "+v"(k[1][2]), "+v"(k[1][3]));
        asm volatile("" : "+v"(v[0][0]), "+v"(v[0][1]), "+v"(v[1][0]), "+v"(v[1][1]), "+v"(v[2][0]), "+v"(v[2][1]),
                          "+v"(v[3][0]), "+v"(v[3][1]));
        asm volatile("" : "+v"(v[4][0]), "+v"(v[4][1]), "+v"(v[5][0]), "+v"(v[5][1]), "+v"(v[6][0]), "+v"(v[6][1]),
                          "+v"(v[7][0]), "+v"(v[7][1]));
    } else {
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(k[0][0]), "+v"(k[0][1]), "+v"(k[1][0]), "+v"(k[1][1]));
        asm volatile("" : "+v"(v[0][0]), "+v"(v[0][1]), "+v"(v[1][0]), "+v"(v[1][1]), "+v"(v[2][0]), "+v"(v[2][1]),
                          "+v"(v[3][0]), "+v"(v[3][1]));
    }
}

template <int HD, int U>
struct AttCfg {
    static constexpr int KSN = HD / 32;                       // k-steps of the QK^T contraction
    static constexpr int NTN = HD / 16;                       // 16-wide tiles of the head dimension
    static constexpr int GPR = HD / 8;                        // 16-byte granules per K/V row
    static constexpr int RPI = 64 / GPR;                      // V rows per global->LDS instruction
    static constexpr int NVI = ATT_CHUNK / RPI;               // such instructions per chunk
    static constexpr int LOADS = 2 * NVI + 1;                 // vector-memory loads per wave per chunk (K, V, mask word)
    static constexpr int KV_BYTES = ATT_CHUNK * HD * 2;       // the K (or V) rows of one chunk
    static constexpr int CHUNK_BYTES = 2 * KV_BYTES;          // one ring slot: [K rows | V rows]
    static constexpr int RING_BYTES = ATT_WAVES * CHUNK_BYTES;       // one buffer per wave
    static constexpr int MERGE_BYTES = 2 * ATT_WAVES * 16 * 4 + ATT_WAVES * NTN * 64 * 16;
    static constexpr int SMEM = RING_BYTES > MERGE_BYTES ? RING_BYTES : MERGE_BYTES;
};

// LDS row of key slot s inside a V chunk: the two 4-slot halves of each lane group's 8 slots
// are kept 16 rows apart, so that one transposed read (16 rows x 32 bytes per half wave)
// touches 8 consecutive rows per 32 lanes.
__device__ __forceinline__ int att_slot_of_row(int rho) { return 8 * ((rho & 15) >> 2) + 4 * (rho >> 4) + (rho & 3); }
// XOR swizzle of the 32-byte column pairs of an LDS row (in 16-byte granules): 8 consecutive
// rows land on 8 different bank groups
template <int HD>
__device__ __forceinline__ constexpr int att_swizzle(int rho) { return HD == 128 ? 2 * (rho & 7) : 2 * ((rho >> 1) & 3); }
// The K rows are read as A-operand fragments, 16 lanes fetching the same 16-byte column of 16
// consecutive rows: there the granule index is XORed with 4 (3) bits of the row.
template <int HD>
__device__ __forceinline__ constexpr int att_swizzle_k(int rho) { return HD == 128 ? (rho & 15) : ((rho >> 1) & 7); }

// PAGED: the cache operands are page pools [n_pages][Hkv][page][HD] and key slot s of sequence b
// lives in page table[b][s >> page_lg] at row s & (page - 1); the sequence's table entries are
// copied to LDS (behind the chunk buffers) once per workgroup.
template <int HD, int U, bool PAGED>
__global__ __launch_bounds__(ATT_WAVES * 64) __attribute__((amdgpu_waves_per_eu(ATT_WAVES / 4, ATT_WAVES / 4))) void tree_attn_kernel(
    // the first 14 dwords arrive in scalar registers with the wave (kernel-argument preload):
    // what the workgroup needs to find its work and to issue its first loads comes first
    const int32_t *__restrict__ ctx_len, int batch, int Hq, int Hkv, int n_mt, int n_splits, int P, int R, int smax,
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ q_lo,
    TemplateDev t, const uint16_t *__restrict__ k_cache, const uint16_t *__restrict__ v_cache,
    const uint16_t *__restrict__ k_tree, const uint16_t *__restrict__ v_tree,
    const uint16_t *__restrict__ k_tree_lo, const uint16_t *__restrict__ v_tree_lo,
    const uint16_t *__restrict__ prompt_k, const uint16_t *__restrict__ prompt_v,
    const int32_t *__restrict__ token, float scale_log2, float *__restrict__ part_o, float *__restrict__ part_ml,
    uint16_t *__restrict__ out, uint16_t *__restrict__ out_lo, int as_fragments, int m_tiles_out, PageMap pm) {
    using C = AttCfg<HD, U>;
    constexpr int KSN = C::KSN, NTN = C::NTN, GPR = C::GPR, RPI = C::RPI, NVI = C::NVI;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 4, c = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, and known to be
    // ---- workgroup id -> (kv group, query head of the group, m-tile, split), kv groups dealt
    //      round-robin to the XCDs
    const int qpk = Hq / Hkv;                                // query heads per K/V head
    const int per_group = (qpk / U) * n_mt * n_splits;       // U query heads of the group per workgroup
    const int xcd = blockIdx.x & 7, slot_in_xcd = blockIdx.x >> 3;
    const int group = xcd + 8 * (slot_in_xcd / per_group);  // (sequence, kv head)
    if (group >= batch * Hkv) return;
    int w_in = slot_in_xcd % per_group;
    const int split = w_in % n_splits; w_in /= n_splits;
    const int mt = n_mt - 1 - (w_in % n_mt);                 // long m-tiles first
    const int qh = w_in / n_mt;
    const int b = group / Hkv, kvh = group % Hkv, h0 = kvh * qpk + qh * U;   // heads h0 .. h0+U-1

    int Lc = ctx_len[b];
    const int32_t *tbl = reinterpret_cast<const int32_t *>(smem + C::SMEM);
    const int page_lg = pm.page_lg, page_mask = (1 << pm.page_lg) - 1;
    if (PAGED) {
        // never walk past the table entries the launch made room for; page ids are clamped to
        // the pool, so a bad table gives wrong data, not a fault
        Lc = min(Lc, pm.tbl_cap << page_lg);
        int32_t *dst = reinterpret_cast<int32_t *>(smem + C::SMEM);
        const int n_used = (Lc + page_mask) >> page_lg;
        for (int i = tid; i < n_used; i += ATT_WAVES * 64)
            dst[i] = min(max(pm.table[(int64_t)b * pm.max_pages + i], 0), pm.n_pages - 1);
        __syncthreads();
    }
    const int row0 = mt * 16;
    const int n_ctx_keys = P + Lc;
    const int n_cc = (n_ctx_keys + ATT_CHUNK - 1) / ATT_CHUNK;           // chunks over [prefix | cache]
    const int n_tc = min((R + 15) >> 4, mt + 1);                         // chunks over the pass rows
    const int n_chunks = n_cc + n_tc;
    const int per_split = (n_chunks + n_splits - 1) / n_splits;
    const int chunk_begin = split * per_split;
    const int chunk_end = min(n_chunks, chunk_begin + per_split);
    // this wave's chunks: chunk_begin + wave + ATT_WAVES * i, i < n_my
    const int n_my = max(0, (chunk_end - chunk_begin - wave + ATT_WAVES - 1) / ATT_WAVES);

    const uint16_t *pk = prompt_k + (int64_t)kvh * P * HD, *pv = prompt_v + (int64_t)kvh * P * HD;
    const int64_t page_stride = (int64_t)Hkv * HD << page_lg;           // elements per page (all kv heads)
    const uint16_t *ck = k_cache + (PAGED ? ((int64_t)kvh * HD << page_lg) : ((int64_t)b * Hkv + kvh) * smax * HD);
    const uint16_t *cv = v_cache + (PAGED ? ((int64_t)kvh * HD << page_lg) : ((int64_t)b * Hkv + kvh) * smax * HD);
    // element offset of cache slot j of this (sequence, kv head) from ck / cv
    auto slot_off = [&](int j) __attribute__((always_inline)) -> int64_t {
        if (!PAGED) return (int64_t)j * HD;
        return (int64_t)tbl[j >> page_lg] * page_stride + (int64_t)(j & page_mask) * HD;
    };
    // a chunk of cache slots j0 .. j0+ATT_CHUNK-1 has one base address (always, when contiguous)
    auto one_page = [&](int j0) __attribute__((always_inline)) -> bool {
        return !PAGED || (j0 >> page_lg) == ((j0 + ATT_CHUNK - 1) >> page_lg);
    };
    const int64_t tree_off = ((int64_t)b * Hkv + kvh) * R * HD;
    const uint16_t *tk = k_tree + tree_off, *tv = v_tree + tree_off;
    const uint16_t *tk_lo = k_tree_lo ? k_tree_lo + tree_off : nullptr;
    const uint16_t *tv_lo = v_tree_lo ? v_tree_lo + tree_off : nullptr;
    const uint16_t *zero = reinterpret_cast<const uint16_t *>(g_att_zero_row);

    // ---- query fragments (B operand of S^T = K Q^T) stay in registers: lane (g, c) holds
    //      Q[row0 + c][32ks + 8g .. +8] of both planes; rows beyond R are zero
    //      All loads of this prologue (mask byte, token, query fragments) are unconditional, from
    //      a clamped row, and their values are first looked at behind the wait for the first chunk:
    //      one memory round trip instead of one per dependent condition.
    const int rq = row0 + c;
    const bool row_ok = rq < R;
    const int rqc = min(rq, R - 1);
    const uint32_t mask_byte = t.is_mask[rqc];
    const int32_t *tok_src = token ? token + (int64_t)b * R + rqc : reinterpret_cast<const int32_t *>(g_att_zero_row);
    const int32_t tok_val = *tok_src;
    bool row_mask = false;                               // set behind the first wait
    bf16x8 qf[U][2][KSN];
#pragma unroll
    for (int u = 0; u < U; u++)
#pragma unroll
        for (int pl = 0; pl < 2; pl++) {
            const uint16_t *src = (pl && q_lo) ? q_lo : q;
            const bool live = row_ok && (pl == 0 || q_lo);
#pragma unroll
            for (int ks = 0; ks < KSN; ks++) {
                uint4 v = *reinterpret_cast<const uint4 *>(src + (((int64_t)b * R + rqc) * Hq + h0 + u) * HD + ks * 32 + g * 8);
                if (!live) v = make_uint4(0, 0, 0, 0);
                qf[u][pl][ks] = __builtin_bit_cast(bf16x8, v);
            }
        }

    f32x4 o_acc[U][NTN];
    float m_run[U], l_run[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
#pragma unroll
        for (int nt = 0; nt < NTN; nt++) o_acc[u][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        m_run[u] = -INFINITY;
        l_run[u] = 0.f;
    }

    unsigned char *v_ring = smem + wave * C::CHUNK_BYTES;              // this wave's private chunk buffer
    // LDS addresses of this lane's transposed V reads inside ring slot 0: lane (g, c) addresses
    // V[slot 8g + 4half + c/4][16nt + 4(c%4) .. +4] and receives V[slots 8g + 4half .. +4][16nt + c]
    // ... and of its K fragment reads: sub-tile tt, k-step ks = row 16tt + c, granule 4ks + g
    // (both swizzles ignore bit 4 of the row, so the second sub-tile / half is the same address
    // plus 16 rows: an immediate offset of the read)
    static_assert(att_swizzle_k<HD>(16) == 0 && att_swizzle<HD>(16) == 0, "row bit 4 outside the swizzles");
    constexpr int ROWS16 = 16 * HD * 2;
    uint32_t k_addr[KSN];
#pragma unroll
    for (int ks = 0; ks < KSN; ks++)
        k_addr[ks] = (uint32_t)(size_t)((__attribute__((address_space(3))) unsigned char *)v_ring) +
                     c * (HD * 2) + (((4 * ks + g) ^ att_swizzle_k<HD>(c)) * 16);
    uint32_t v_addr[NTN];
#pragma unroll
    for (int nt = 0; nt < NTN; nt++) {
        const int rho = 4 * g + (c >> 2);
        const int gran = (2 * nt + ((c & 3) >> 1)) ^ att_swizzle<HD>(rho);
        v_addr[nt] = (uint32_t)(size_t)((__attribute__((address_space(3))) unsigned char *)v_ring) +
                     C::KV_BYTES + rho * (HD * 2) + gran * 16 + (c & 1) * 8;
    }

    // Per-lane byte offsets of the fast path (a chunk that lies wholly inside the cache).  Both
    // operands are copied row-major, 1 KiB (RPI rows) per global->LDS instruction: instruction
    // iv fills LDS rows iv*RPI .., LDS row rho holds key slot att_slot_of_row(rho), and the lane
    // at granule position p of that row fetches granule p ^ swizzle(rho).  The swizzles depend
    // on iv only through iv%4 (K) and iv%2 (V).
    // In a chunk over the pass rows slot s is pass row 4*(s>>3) + (s&3) of the chunk's 16, plane
    // (s>>2)&1; the instruction's first slot and the lane's slot inside the instruction occupy
    // disjoint bits, so row and plane split the same way (the plane is uniform per instruction).
    const int v_lane_row = lane / GPR;                                  // row inside one instruction
    const int lane_slot = att_slot_of_row(v_lane_row);
    const int lane_tree_row = 4 * (lane_slot >> 3) + (lane_slot & 3);
    uint32_t k_gran[4], v_gran[2];                                      // source granule (bytes) at this lane's position
#pragma unroll
    for (int par = 0; par < 4; par++) {
        const int rho = par * RPI + v_lane_row;
        k_gran[par] = ((lane % GPR) ^ att_swizzle_k<HD>(rho)) * 16;
        if (par < 2) v_gran[par] = ((lane % GPR) ^ att_swizzle<HD>(rho)) * 16;
    }

    // The two global->LDS loads (one K, one V instruction) number iv < NVI of this wave's stage i,
    // the mask word riding with the last.  A chunk wholly inside the cache takes one uniform base
    // per operand plus the constant lane offsets; the other cases select per lane.
    typedef const __attribute__((address_space(1))) unsigned char *gptr;   // keeps the loads global, not flat
    uint64_t anc_next = 0;                                              // ancestor bits for the stage in flight
    auto emit = [&](int i, int iv) __attribute__((always_inline)) {
        const int chunk = chunk_begin + wave + ATT_WAVES * i;
        const int base = chunk * ATT_CHUNK;
        const unsigned char *zero_b = reinterpret_cast<const unsigned char *>(zero);
        const int slot0 = att_slot_of_row(iv * RPI);                    // slot of the instruction's first row
        gptr k_src, v_src, a_src = (gptr)(zero_b + (lane & 1) * 8);
        if (base >= P && base + ATT_CHUNK <= n_ctx_keys && one_page(base - P)) {
            const int64_t row_bytes = (slot_off(base - P) + (int64_t)(slot0 + lane_slot) * HD) * 2;
            k_src = (gptr)(reinterpret_cast<const unsigned char *>(ck) + row_bytes + k_gran[iv & 3]);
            v_src = (gptr)(reinterpret_cast<const unsigned char *>(cv) + row_bytes + v_gran[iv & 1]);
        } else if (chunk >= n_cc) {
            // over the pass rows: one plane and 4-row group per instruction, rows beyond R are zero
            const int j_first = (chunk - n_cc) * 16;
            if (row_ok) a_src = (gptr)(t.anc + (int64_t)rq * t.words + (j_first >> 6));   // ancestor bits of these 16 rows
            const int j = j_first + 4 * (slot0 >> 3) + lane_tree_row;
            const uint16_t *kp = (slot0 & 4) ? tk_lo : tk, *vp = (slot0 & 4) ? tv_lo : tv;   // uniform
            const bool k_ok = j < R && kp, v_ok = j < R && vp;
            k_src = (gptr)(reinterpret_cast<const unsigned char *>(k_ok ? kp + (int64_t)j * HD : zero) + k_gran[iv & 3]);
            v_src = (gptr)(reinterpret_cast<const unsigned char *>(v_ok ? vp + (int64_t)j * HD : zero) + v_gran[iv & 1]);
        } else {
            // a chunk with prefix rows or the ragged end of the cache
            const int kidx = base + slot0 + lane_slot;
            const bool in_prefix = kidx < P, in_cache = kidx >= P && kidx < n_ctx_keys;
            const int64_t off = in_cache ? slot_off(kidx - P) : 0;
            const uint16_t *krow = in_prefix ? pk + (int64_t)kidx * HD : (in_cache ? ck + off : zero);
            const uint16_t *vrow = in_prefix ? pv + (int64_t)kidx * HD : (in_cache ? cv + off : zero);
            k_src = (gptr)(reinterpret_cast<const unsigned char *>(krow) + k_gran[iv & 3]);
            v_src = (gptr)(reinterpret_cast<const unsigned char *>(vrow) + v_gran[iv & 1]);
        }
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)k_src,
                                         (__attribute__((address_space(3))) void *)(v_ring + iv * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)v_src,
                                         (__attribute__((address_space(3))) void *)(v_ring + C::KV_BYTES + iv * 1024), 16, 0, 0);
        if (iv == NVI - 1) anc_next = *(const __attribute__((address_space(1))) uint64_t *)a_src;
    };

    // The same two loads for a chunk known to lie wholly inside the cache (all but a handful):
    // one uniform base per operand, the lane's constant offset, the instruction's constant row.
    const uint32_t lane_row_bytes = (uint32_t)lane_slot * (HD * 2);
    auto emit_cache = [&](const unsigned char *kb, const unsigned char *vb, int iv) __attribute__((always_inline)) {
        const uint32_t row0_bytes = (uint32_t)att_slot_of_row(iv * RPI) * (HD * 2);      // compile-time per iv
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gptr)(kb + (lane_row_bytes + k_gran[iv & 3] + row0_bytes)),
                                         (__attribute__((address_space(3))) void *)(v_ring + iv * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gptr)(vb + (lane_row_bytes + v_gran[iv & 1] + row0_bytes)),
                                         (__attribute__((address_space(3))) void *)(v_ring + C::KV_BYTES + iv * 1024), 16, 0, 0);
    };

    // One chunk.  Its K and V fragments are all pulled into registers first, which frees the
    // wave's LDS buffer: the next chunk's loads are issued into it right away, interleaved
    // with the QK^T matrix instructions, and have the rest of the step to land.
    auto compute = [&](int i, bool more) __attribute__((always_inline)) {
        const uint64_t anc_cur = anc_next;
        const int chunk = chunk_begin + wave + ATT_WAVES * i;
        const bool tree_chunk = chunk >= n_cc;
        const int base = chunk * ATT_CHUNK;
        u32x4 kf[2][KSN];
#pragma unroll
        for (int tt = 0; tt < 2; tt++)
#pragma unroll
            for (int ks = 0; ks < KSN; ks++)
                kf[tt][ks] = tt ? lds_read_b128<ROWS16>(k_addr[ks]) : lds_read_b128<0>(k_addr[ks]);
        s16x4 vh[NTN][2];
#pragma unroll
        for (int nt = 0; nt < NTN; nt++) {
            vh[nt][0] = lds_read_tr16<0>(v_addr[nt]);
            vh[nt][1] = lds_read_tr16<ROWS16>(v_addr[nt]);
        }
        lds_wait_all(kf, vh);
        f32x4 s_acc[U][2];
#pragma unroll
        for (int u = 0; u < U; u++) s_acc[u][0] = s_acc[u][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        static_assert(NVI == 2 * KSN, "one (k-step, sub-tile) pair per load slot");
        auto qk = [&](int iv) __attribute__((always_inline)) {
            const int ks = iv >> 1, tt = iv & 1;
            const bf16x8 ka = __builtin_bit_cast(bf16x8, kf[tt][ks]);
#pragma unroll
            for (int u = 0; u < U; u++) {
                s_acc[u][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qf[u][0][ks], s_acc[u][tt], 0, 0, 0);
                s_acc[u][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qf[u][1][ks], s_acc[u][tt], 0, 0, 0);
            }
        };
        const int base_n = base + ATT_WAVES * ATT_CHUNK;                 // the wave's next chunk
        // (with two heads per workgroup the second code path costs registers the kernel does not have)
        if (U == 1 && more && base_n >= P && base_n + ATT_CHUNK <= n_ctx_keys && one_page(base_n - P)) {   // wave-uniform
            const int64_t off_n = slot_off(base_n - P) * 2;
            const unsigned char *kb = reinterpret_cast<const unsigned char *>(ck) + off_n;
            const unsigned char *vb = reinterpret_cast<const unsigned char *>(cv) + off_n;
#pragma unroll
            for (int iv = 0; iv < NVI; iv++) {
                emit_cache(kb, vb, iv);
                __builtin_amdgcn_sched_barrier(0);
                qk(iv);
                __builtin_amdgcn_sched_barrier(0);
            }
            anc_next = 0;
        } else {
#pragma unroll
            for (int iv = 0; iv < NVI; iv++) {
                if (more) emit(i + 1, iv);
                __builtin_amdgcn_sched_barrier(0);
                qk(iv);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // the visibility of a key depends on the row and the key only: one mask word for all heads
        const bool need_mask = tree_chunk || (base < P) || (base + ATT_CHUNK > n_ctx_keys);
        uint32_t bits = 0xFFu;
        if (need_mask) {
            // 8-bit visibility word for this lane's slots, built with integer selects only:
            // prefix -> mask rows, cache -> all rows, pass rows -> ancestor bits.
            bits = 0;
            if (row_ok) {
                if (tree_chunk) {
                    const int j0 = (chunk - n_cc) * 16 + 4 * g;          // this lane's 4 pass rows (4-aligned)
                    const uint32_t four = (uint32_t)(anc_cur >> (j0 & 63)) & 0xFu;
#pragma unroll
                    for (int e = 0; e < 4; e++) bits |= ((j0 + e < R) ? ((four >> e) & 1u) : 0u) << e;
                } else {
                    const int k0 = base + 8 * g;
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        const int kidx = k0 + e;
                        const uint32_t in_prefix = kidx < P ? 1u : 0u;
                        const uint32_t in_cache = (kidx >= P && kidx < n_ctx_keys) ? 1u : 0u;
                        bits |= ((in_prefix & (row_mask ? 1u : 0u)) | in_cache) << e;
                    }
                }
            }
        }
        s16x8 v8[NTN];
#pragma unroll
        for (int nt = 0; nt < NTN; nt++)
            v8[nt] = s16x8{vh[nt][0][0], vh[nt][0][1], vh[nt][0][2], vh[nt][0][3],
                           vh[nt][1][0], vh[nt][1][1], vh[nt][1][2], vh[nt][1][3]};
#pragma unroll
        for (int u = 0; u < U; u++) {
            float sv[8];
#pragma unroll
            for (int tt = 0; tt < 2; tt++)
#pragma unroll
                for (int r = 0; r < 4; r++) sv[tt * 4 + r] = s_acc[u][tt][r] * scale_log2;
            if (tree_chunk) {                // score = q.k_hi + q.k_lo; partner slots leave the softmax
#pragma unroll
                for (int e = 0; e < 4; e++) sv[e] += sv[e + 4];
            }
            if (need_mask) {
#pragma unroll
                for (int e = 0; e < 8; e++) sv[e] = ((bits >> e) & 1u) ? sv[e] : -INFINITY;
            }
            float mx = sv[0];
#pragma unroll
            for (int e = 1; e < 8; e++) mx = fmaxf(mx, sv[e]);
            mx = max_over_lane_groups(mx);
            const float m_new = fmaxf(m_run[u], mx);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = fast_exp2(m_run[u] - m_use);
            m_run[u] = m_new;
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
            if (tree_chunk) {                // the low-plane value rows take the same probabilities
                pk2[2] = pk2[0];
                pk2[3] = pk2[1];
                pl2[2] = pl2[0];
                pl2[3] = pl2[1];
            }
            l_run[u] = l_run[u] * alpha + ps;
            // O^T[hd][q] = alpha * O^T + V^T[hd][slots 8g..8g+7] * P^T; the running maximum rarely
            // moves after the first chunks, and then alpha is exactly 1 in every lane
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int nt = 0; nt < NTN; nt++) o_acc[u][nt] *= alpha;
            }
            const bf16x8 pf = __builtin_bit_cast(bf16x8, make_uint4(pk2[0], pk2[1], pk2[2], pk2[3]));
            const bf16x8 pf_lo = __builtin_bit_cast(bf16x8, make_uint4(pl2[0], pl2[1], pl2[2], pl2[3]));
#pragma unroll
            for (int nt = 0; nt < NTN; nt++) {
                const bf16x8 vf = __builtin_bit_cast(bf16x8, v8[nt]);
                o_acc[u][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf, o_acc[u][nt], 0, 0, 0);
                o_acc[u][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf_lo, o_acc[u][nt], 0, 0, 0);
            }
        }
    };

    // ---- per-wave loop: one chunk in flight behind the one being multiplied -------------------
    if (n_my > 0) {
#pragma unroll
        for (int iv = 0; iv < NVI; iv++) emit(0, iv);
    }
    att_wait<0>();                                      // the first chunk and the prologue's loads have landed
    // a tree row without a candidate (negative token) is absent from the pass: its output is zero
    int row_flags = (row_ok && mask_byte ? 1 : 0) | (row_ok && (mask_byte || tok_val >= 0) ? 2 : 0);
    asm volatile("" : "+v"(row_flags));                 // (looked at here, not inside the loop)
    row_mask = (row_flags & 1) != 0;
    const bool row_present = (row_flags & 2) != 0;
    for (int i = 0; i < n_my; i++) {
        compute(i, i + 1 < n_my);
        att_wait<0>();                                  // the next chunk has landed
    }

    // ---- merge the wavefronts (disjoint key subsets), head by head: every wave leaves its rescaled
    //      tiles in LDS, wave nt then sums tile nt of the head dimension over the waves in wave order
    //      (fixed order, deterministic) and finishes and stores those 16 columns -----------------------
    float *sm = reinterpret_cast<float *>(smem), *sl = sm + ATT_WAVES * 16;
    float4 *region = reinterpret_cast<float4 *>(smem + 2 * ATT_WAVES * 16 * 4);   // [WAVES][NTN][64]
#pragma unroll
    for (int u = 0; u < U; u++) {
        const int h = h0 + u;
        __syncthreads();                     // the chunk buffers (first head) or the previous head's sums are done with
        const float l = sum_over_lane_groups(l_run[u]);
        if (g == 0) {
            sm[wave * 16 + c] = m_run[u];
            sl[wave * 16 + c] = l;
        }
        __syncthreads();
        float m_tot = -INFINITY;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; w++) m_tot = fmaxf(m_tot, sm[w * 16 + c]);
        const float m_use = (m_tot == -INFINITY) ? 0.f : m_tot;
        float l_tot = 0.f;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; w++) l_tot += sl[w * 16 + c] * fast_exp2(sm[w * 16 + c] - m_use);
        const float f = fast_exp2(m_run[u] - m_use);
#pragma unroll
        for (int nt = 0; nt < NTN; nt++)
            region[(wave * NTN + nt) * 64 + lane] =
                make_float4(o_acc[u][nt][0] * f, o_acc[u][nt][1] * f, o_acc[u][nt][2] * f, o_acc[u][nt][3] * f);
        __syncthreads();
        if (wave >= NTN || !row_ok) continue;
        const int nt = wave;                 // this wave's 16 columns of the head
        float4 o = region[nt * 64 + lane];
#pragma unroll
        for (int w = 1; w < ATT_WAVES; w++) {
            const float4 v = region[(w * NTN + nt) * 64 + lane];
            o.x += v.x; o.y += v.y; o.z += v.z; o.w += v.w;
        }
        // ---- lane (g, c) holds O[row rq][hd 16nt + 4g .. +4] -----------------------------------
        if (n_splits > 1) {                  // unnormalised partial for attn_merge_kernel
            const int64_t prow = (((int64_t)b * Hq + h) * n_splits + split) * R + rq;
            *reinterpret_cast<float4 *>(part_o + prow * HD + nt * 16 + 4 * g) = o;
            if (nt == 0 && g == 0) {
                part_ml[prow * 2] = m_tot;
                part_ml[prow * 2 + 1] = row_present ? l_tot : 0.f;      // (a zero sum makes the merge write zeros)
            }
            continue;
        }
        const float inv = (l_tot > 0.f && row_present) ? 1.0f / l_tot : 0.f;
        const int mrow = b * R + rq, n_ksteps = (Hq * HD) >> 5;
        const float ov[4] = {o.x * inv, o.y * inv, o.z * inv, o.w * inv};
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; e++) split_bf16(ov[e], hi[e], lo[e]);
        uint2 ph, pl;
        ph.x = hi[0] | ((uint32_t)hi[1] << 16); ph.y = hi[2] | ((uint32_t)hi[3] << 16);
        pl.x = lo[0] | ((uint32_t)lo[1] << 16); pl.y = lo[2] | ((uint32_t)lo[3] << 16);
        const int k = h * HD + nt * 16 + 4 * g;
        if (as_fragments) {                  // two planes, the O-projection's activation slab
            const int pack_off = frag_pack_offset(batch * R);
            *reinterpret_cast<uint2 *>(out + frag_index(0, mrow, k, n_ksteps, m_tiles_out, pack_off)) = ph;
            *reinterpret_cast<uint2 *>(out + frag_index(1, mrow, k, n_ksteps, m_tiles_out, pack_off)) = pl;
        } else {
            *reinterpret_cast<uint2 *>(out + (int64_t)mrow * Hq * HD + k) = ph;
            if (out_lo) *reinterpret_cast<uint2 *>(out_lo + (int64_t)mrow * Hq * HD + k) = pl;
        }
    }
}

// out[b][r][h*HD + 4i .. +4] = sum_s w_s O_s / sum_s w_s l_s,  w_s = 2^(m_s - max m).
// One thread per 4 head-dim elements; blockDim = (HD/4) * heads_per_block.
__global__ void attn_merge_kernel(const float *__restrict__ part_o, const float *__restrict__ part_ml,
                                  int R, int Hq, int HD, int n_splits, uint16_t *__restrict__ out,
                                  uint16_t *__restrict__ out_lo, int as_fragments, int m_tiles) {
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
        const int pack_off = frag_pack_offset((int)gridDim.z * R);
        *reinterpret_cast<uint2 *>(out + frag_index(0, mrow, k, n_ksteps, m_tiles, pack_off)) = ph;
        *reinterpret_cast<uint2 *>(out + frag_index(1, mrow, k, n_ksteps, m_tiles, pack_off)) = pl;
    } else {
        *reinterpret_cast<uint2 *>(out + (((int64_t)b * R + r) * Hq + h) * HD + i4 * 4) = ph;
        if (out_lo) *reinterpret_cast<uint2 *>(out_lo + (((int64_t)b * R + r) * Hq + h) * HD + i4 * 4) = pl;
    }
}

AttnPlan attn_plan(int batch, int rows, int n_heads, int hd, int ctx_hint, int n_prompt) {
    AttnPlan p;
    const int n_mt = (rows + 15) / 16;
    const int n_chunks = (n_prompt + ctx_hint + ATT_CHUNK - 1) / ATT_CHUNK + n_mt;
    const int wgs = batch * n_heads * n_mt;
    // No key split while one workgroup's walk stays moderate (256 chunks = 8192 keys, 32 per
    // wave); beyond that, or when the row tiles alone leave most CUs idle on a long context,
    // split the key axis (partials + merge kernel) into shares of at least 16 chunks.
    int splits = (n_chunks + 255) / 256;
    if (wgs * splits < 128) {
        int fill = 256 / wgs;
        if (fill > n_chunks / 16) fill = n_chunks / 16;
        if (fill > splits) splits = fill;
    }
    if (splits < 1) splits = 1;
    if (splits > 64) splits = 64;
    const int per = (n_chunks + splits - 1) / splits;
    splits = (n_chunks + per - 1) / per;
    p.splits = splits;
    p.part_o_bytes = (size_t)batch * n_heads * splits * rows * hd * sizeof(float);
    p.part_ml_bytes = (size_t)batch * n_heads * splits * rows * 2 * sizeof(float);
    return p;
}

template <int HD, int U, bool PAGED>
static void launch_attn_t(const TemplateDev &t, const void *q, const void *q_lo, const void *k_cache, const void *v_cache,
                          const void *k_tree, const void *v_tree, const void *k_tree_lo, const void *v_tree_lo,
                          const void *prompt_k, const void *prompt_v, const int32_t *ctx_len, const int32_t *token,
                          int batch, int Hq,
                          int Hkv, int P, int smax, const AttnPlan &p, float *part_o, float *part_ml, void *out,
                          void *out_lo, bool out_as_fragments, const PageMap &pm, hipStream_t s) {
    using C = AttCfg<HD, U>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)tree_attn_kernel<HD, U, PAGED>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize,
                                  C::SMEM + (PAGED ? ATT_PAGE_TABLE_MAX * 4 : 0));
        attr_set = true;
    }
    const size_t smem_bytes = C::SMEM + (PAGED ? (size_t)((pm.tbl_cap + 3) / 4) * 16 : 0);
    const int n_mt = (t.rows + 15) / 16;
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
    const int groups = batch * Hkv, per_group = (Hq / Hkv / U) * n_mt * p.splits;
    const int grid = 8 * ((groups + 7) / 8) * per_group;
    hipLaunchKernelGGL((tree_attn_kernel<HD, U, PAGED>), dim3(grid), dim3(ATT_WAVES * 64), smem_bytes, s,
                       ctx_len, batch, Hq, Hkv, n_mt, p.splits, P, t.rows, smax, (const uint16_t *)q, (const uint16_t *)q_lo, t,
                       (const uint16_t *)k_cache, (const uint16_t *)v_cache,
                       (const uint16_t *)k_tree, (const uint16_t *)v_tree, (const uint16_t *)k_tree_lo,
                       (const uint16_t *)v_tree_lo, (const uint16_t *)prompt_k, (const uint16_t *)prompt_v, token,
                       scale_log2, part_o, part_ml, (uint16_t *)out,
                       (uint16_t *)out_lo, out_as_fragments ? 1 : 0, (batch * t.rows + 15) / 16, pm);
}

void launch_tree_attention(const TemplateDev &t, const void *q, const void *q_lo, const void *k_cache, const void *v_cache,
                           const void *k_tree, const void *v_tree, const void *k_tree_lo, const void *v_tree_lo,
                           const void *prompt_k,
                           const void *prompt_v, const int32_t *ctx_len, const int32_t *token, int batch, int Hq, int Hkv, int hd,
                           int P, int smax, const AttnPlan &p, float *part_o, float *part_ml, void *out,
                           void *out_lo, bool out_as_fragments, const PageMap &pm, hipStream_t s) {
    // grouped-query models: two query heads of a K/V head per workgroup share its chunk loads
    const bool pair = (Hq / Hkv) % 2 == 0;
#define ATT_LAUNCH_P(HD_, U_, PG_) launch_attn_t<HD_, U_, PG_>(t, q, q_lo, k_cache, v_cache, k_tree, v_tree, k_tree_lo, v_tree_lo, prompt_k, \
                                                   prompt_v, ctx_len, token, batch, Hq, Hkv, P, smax, p, part_o, part_ml, out, out_lo, out_as_fragments, pm, s)
#define ATT_LAUNCH(HD_, U_) do { if (pm.table) ATT_LAUNCH_P(HD_, U_, true); else ATT_LAUNCH_P(HD_, U_, false); } while (0)
    if (hd == 128) {
        if (pair) ATT_LAUNCH(128, 2); else ATT_LAUNCH(128, 1);
    } else {
        if (pair) ATT_LAUNCH(64, 2); else ATT_LAUNCH(64, 1);
    }
#undef ATT_LAUNCH_P
#undef ATT_LAUNCH
    if (p.splits > 1) {
        const int heads_per_block = (256 / (hd / 4)) < Hq ? (256 / (hd / 4)) : Hq;
        hipLaunchKernelGGL(attn_merge_kernel, dim3(t.rows, (Hq + heads_per_block - 1) / heads_per_block, batch),
                           dim3(heads_per_block * (hd / 4)), 0, s, part_o, part_ml, t.rows,
                           Hq, hd, p.splits, (uint16_t *)out, (uint16_t *)out_lo, out_as_fragments ? 1 : 0, (batch * t.rows + 15) / 16);
    }
}
