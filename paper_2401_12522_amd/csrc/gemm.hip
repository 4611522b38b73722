// Skinny weight-streaming GEMM for the verify step: Y[M][N] = A[M][K] * W[N][K]^T with
// M = (tree + mask rows) * batch, i.e. a few dozen rows, so the kernel is bound by the one
// pass over W in HBM (the paper's premise, Sec. 3.2: inference is memory-bandwidth bound,
// extra rows are nearly free).
//
// Layout choices for gfx950:
//  * W is pre-packed into 1 KiB blocks, each exactly one v_mfma_f32_16x16x32_bf16 B-operand
//    (16 rows x 32 k; lane l holds W[16t + l%16][32s + 8(l/16) .. +8]), so a wave loads its
//    fragments with fully coalesced 16-byte-per-lane loads straight into MFMA registers; W
//    never touches LDS.  Blocks are ordered k-major: [k-step pair][16-row tile][2 k-steps].
//    Waves that run side by side work on neighbouring tiles of the same k range, so what
//    the chip reads at any moment is one contiguous region (as in a plain copy), instead of
//    thousands of streams a power-of-two stride apart that would pile onto few HBM channels.
//  * The activation slab is small and shared by every wave.  Producers write it to global
//    memory already in A-operand fragment order (1 KiB per (plane, k-step, m-tile): lane l
//    holds A[16mt + l%16][32ks + 8(l/16) .. +8]), so one direct global->LDS load per
//    fragment reads 1 KiB contiguous, lands in LDS in operand order (conflict-free linear
//    reads) and spends no VGPRs on staging.  Each fragment read from LDS feeds NW weight
//    tiles; with two planes the slab traffic from L2 is what limits narrow NW.
//  * Activations may come as two bf16 planes (hi = bf16(x), lo = bf16(x - hi)); both are
//    multiplied with the same weight fragment.  That removes the activation rounding from
//    the error budget at the price of 2x MFMA work, which the kernel has to spare (at 68
//    rows it needs ~1/4 of the matrix-core rate the HBM stream could feed).
//  * A three-stage software pipeline keeps two stages of W (registers) and A (LDS ring) in
//    flight behind the one being multiplied; waits are on the oldest stage only.
//  * Parallelism comes from N (16*NW rows per wave) and, where N alone cannot fill 256 CUs,
//    from split-K with fp32 partial sums reduced in a fixed order by the consumer
//    (deterministic, no float atomics).
#include "common.h"
#include <string.h>
#include <stdlib.h>
#include <type_traits>

// index of the 1 KiB block holding rows 16t..16t+15, k 32ks..32ks+31 (k-major order)
__host__ __device__ __forceinline__ int64_t packed_block(int64_t t, int64_t ks, int64_t n_tiles) {
    return ((ks >> 1) * n_tiles + t) * 2 + (ks & 1);
}

// wait until at most N vector-memory operations of this wave are outstanding and all of its
// LDS reads have returned
template <int N>
__device__ __forceinline__ void wait_vmcnt_lds() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0x0 << 8));
}

// Workgroup barrier without the memory fences of __syncthreads(): those would drain every
// outstanding vector-memory operation (vmcnt(0)) and with it the prefetched stages.  The
// data hazards are covered explicitly by the wait that precedes it: the wave's own LDS-bound
// loads of the stage about to be read have landed, and its LDS reads of the previous stage
// (whose slot is refilled after the barrier) have returned.
__device__ __forceinline__ void wg_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// LDS reads of activation fragments as bare instructions with their own staged waits: the
// k-step's reads are all issued up front and each MFMA group waits only for the fragment it
// uses (the compiler's own placement was one wait for all of them).  lgkmcnt counts this
// wave's outstanding LDS reads, which return in order.
template <int OFFSET>
__device__ __forceinline__ bf16x8 lds_read_frag(uint32_t lds_addr) {
    static_assert(OFFSET >= 0 && OFFSET < 65536, "ds offset field");
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(lds_addr), "n"(OFFSET));
    return v;
}
template <int OUTSTANDING>
__device__ __forceinline__ void lds_wait_frag(bf16x8 &a) {
    static_assert(OUTSTANDING >= 0 && OUTSTANDING < 16, "lgkmcnt range");
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(OUTSTANDING));
}

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// MT m-tiles of 16 rows, NW n-tiles per wave, SPLIT = two activation planes, KC k-steps (of 32)
// per pipeline stage, D stages in the ring (D-1 in flight behind the one being multiplied),
// WAVES wavefronts per workgroup, of which KG groups of WN = WAVES/KG waves each take one
// contiguous part of the workgroup's k range (with their own activation ring) and are summed
// through LDS at the end: twice the waves per partial sum written.
// PACK: the slab's last m-tile (the pass' tile MT-1) keeps both planes of its rows in its high
// plane's fragment (frag_pack_offset): the stage has one fragment less, the last of the list.
template <int MT, int NW, bool SPLIT, int KC, int D, int WAVES, int KG, bool PACK = false>
struct GemmCfg {
    static_assert(!PACK || (SPLIT && KC == 1), "packing folds the low plane into the high one");
    static constexpr int WN = WAVES / KG;                       // waves side by side along N
    static constexpr int PL = SPLIT ? 2 : 1;
    static constexpr int NFRAG = PL * MT * KC - (PACK ? 1 : 0); // A fragments per stage
    static constexpr int FPW = (NFRAG + WN - 1) / WN;           // fetched per wave per stage
    static constexpr int LOADS = NW * KC + FPW;                 // vector-memory loads per wave per stage
    // every wave issues FPW fragment loads per stage (the vmcnt bookkeeping counts on it);
    // those beyond NFRAG land in one shared dump slot after the ring
    static constexpr int RING = KG * D * NFRAG * 1024;          // one ring per k group
    static constexpr int MERGE = KG > 1 ? WN * MT * NW * 1024 : 0;   // accumulators of one k group
    static constexpr int STAGE = NW % 2 == 0 ? 2 * (WN * NW * 8 / 16) * MT * 512 : 0;    // gated output slab of the workgroup
    static constexpr int SMEM = (RING > MERGE ? (RING > STAGE ? RING : STAGE) : (MERGE > STAGE ? MERGE : STAGE)) + 1024;
    static_assert((D - 2) * LOADS < 64, "vmcnt counter range");
};

template <int MT, int NW, bool SPLIT, int KC, int D, int WAVES, int KG, bool DIRECT, bool PACK>
__global__ __launch_bounds__(WAVES * 64) void gemm_skinny_kernel(
    // The first 14 dwords of the argument block arrive in scalar registers with the wave
    // (kernel-argument preload); everything the first loads depend on is among them, the grid's
    // extent included: read through gridDim it costs one dependent scalar load per component
    // before the first weight load can be issued.
    const uint4 *__restrict__ A_frag, const uint4 *__restrict__ Wp, int planes_stride_f, int M, int m_tiles,
    int NT, int KS, int ksteps_per_split, int grid_x, int grid_y, int grid_z,
    float *__restrict__ out, int64_t ldo, GemmOutput direct) {
    using C = GemmCfg<MT, NW, SPLIT, KC, D, WAVES, KG, PACK>;
    constexpr int WN = C::WN;
    extern __shared__ __attribute__((aligned(16))) uint4 smem_u4[];   // [KG][D][NFRAG][64] + dump slot

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, and known to be: addresses on the scalar unit
    const int kg = wave / WN, wn = wave % WN;                  // k group, position along N
    // (column group, k split, row pass) of this workgroup.  With several row passes (more rows
    // than one pass holds) the passes over the same weights are made neighbours on one XCD:
    // dispatch index L goes to XCD L % 8, so the passes of a (column group, split) pair take
    // indices 8 apart and run side by side on that XCD, the later ones finding the weight
    // blocks in its L2 instead of fetching them again.
    int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    if (grid_z > 1) {
        const int X = grid_x, Z = grid_z, T = X * grid_y, Tb = T & ~7;
        const int L = bx + X * (by + grid_y * bz);
        int pair;
        if (L < Tb * Z) {
            const int q = L >> 3;
            bz = q % Z;
            pair = (q / Z) * 8 + (L & 7);
        } else {                                               // the last T % 8 pairs, pass-major
            const int r = L - Tb * Z;
            bz = r % Z;
            pair = Tb + r / Z;
        }
        bx = pair % X;
        by = pair / X;
    }
    else if (grid_y > 1) {
        // Split-K launch: workgroups of one k split read the same k range of the activation
        // slab.  With a power-of-two number of splits each split is given to its own XCD(s), so
        // that every k range is fetched into one L2 (or few) instead of all eight.
        const int X = grid_x, Y = grid_y, L = bx + X * by;
        if ((Y & (Y - 1)) == 0 && ((X * Y) & 7) == 0) {
            if (Y >= 8) {
                const int per = Y >> 3;                        // splits per XCD
                by = (L & 7) + 8 * ((L >> 3) % per);
                bx = (L >> 3) / per;
            } else {
                const int per = 8 / Y;                         // XCDs per split
                by = (L & 7) / per;
                bx = (L >> 3) * per + (L & 7) % per;
            }
        }
    }
    const int t0 = (bx * WN + wn) * NW;
    // the workgroup's k range, cut into KG contiguous parts of equal stage count
    const int wg_begin = by * ksteps_per_split;
    const int wg_end = min(KS, wg_begin + ksteps_per_split);
    const int per_group = (wg_end - wg_begin + KG - 1) / KG;
    const int ks_begin = wg_begin + kg * per_group;
    const int ks_end = min(wg_end, ks_begin + per_group);
    const int m_base = bz * (MT * 16);
    const int n_stages = (per_group + KC - 1) / KC;            // same for every wave: barriers in lockstep
    uint4 *a_lds = smem_u4 + kg * (D * C::NFRAG * 64);         // this k group's ring
    uint4 *dump = smem_u4 + KG * D * C::NFRAG * 64;            // target of padding fetches

    // lane -> lane holding the same k granule of the last existing row of the slab's last m-tile
    // (packed tile: of the last existing row of the lane's plane)
    const int rows_last = M - (m_tiles - 1) * 16, pack_off = PACK ? frag_pack_offset(M) : 16;
    const int lane_row = lane & 15;
    const int lane_last = (lane & ~15) | (lane_row < pack_off ? min(lane_row, rows_last - 1)
                                                              : pack_off + min(lane_row - pack_off, rows_last - 1));

    f32x4 acc[MT][NW];
#pragma unroll
    for (int i = 0; i < MT; i++)
#pragma unroll
        for (int j = 0; j < NW; j++) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    uint4 w[D][NW][KC];
    // byte address in LDS of this lane's 16 bytes of the k group's fragment 0
    const uint32_t lds_lane_base = (uint32_t)(size_t)((__attribute__((address_space(3))) uint4 *)a_lds) + lane * 16;

    // Issue all loads of pipeline stage `stage` into ring slot SLOT: NW*KC weight fragments to
    // registers and this wave's FPW activation fragments to LDS.  Every wave issues exactly
    // C::LOADS vector-memory operations, which is what the vmcnt waits below count on.
    // Every address is valid and computed without a select (all terms are wave-uniform but the
    // lane's 16 bytes): tiles past the matrix, k-steps past the group's range, m-tiles past the
    // slab and the padding fetches re-read the nearest existing fragment.  What they bring is
    // either never multiplied (k-steps: see compute) or lands in accumulators that are never
    // stored (rows and columns beyond the output).
    auto issue = [&](auto slot_c, int stage) {
        constexpr int SLOT = decltype(slot_c)::value;
        const int ks0 = ks_begin + stage * KC;
#pragma unroll
        for (int j = 0; j < NW; j++)
#pragma unroll
            for (int s = 0; s < KC; s++) {
                const int t = min(t0 + j, NT - 1), ks = min(ks0 + s, KS - 1);
                typedef uint32_t __attribute__((ext_vector_type(4))) u32x4_t;
                const u32x4_t q = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(Wp + packed_block(t, ks, NT) * 64 + lane));
                w[SLOT][j][s] = make_uint4(q.x, q.y, q.z, q.w);
            }
#pragma unroll
        for (int i = 0; i < C::FPW; i++) {
            const int f = i * WN + wn;                            // fragment id inside the stage
            const int fc = min(f, C::NFRAG - 1);
            const int plane = fc / (MT * KC), mt = (fc / KC) % MT, s = fc % KC;
            const int mtg = min(bz * MT + mt, m_tiles - 1);   // m-tile in the whole slab
            const int ks = min(ks0 + s, KS - 1);
            // fragment (plane, ks, mtg) starts at ((plane * KS + ks) * m_tiles + mtg) * 64 uint4
            // The slab's last m-tile may hold fewer than 16 rows (4 of the 68 of a 64-node tree):
            // the lanes of its missing rows re-read the last row that exists, so the fragment
            // costs the L1 the cache lines of its real rows only (same-address lanes coalesce).
            // The copies land in accumulator rows that are never stored.
            const int src_lane = mtg == m_tiles - 1 ? lane_last : lane;   // wave-uniform choice
            const uint4 *src = A_frag + ((int64_t)plane * planes_stride_f + (int64_t)ks * m_tiles + mtg) * 64 + src_lane;
            uint4 *dst = f < C::NFRAG ? a_lds + (SLOT * C::NFRAG + f) * 64 : dump;   // wave-uniform; lane l lands at dst[l]
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)dst, 16, 0, 0);
        }
    };
    auto compute = [&](auto slot_c, int stage) {
        constexpr int SLOT = decltype(slot_c)::value;
#pragma unroll
        for (int s = 0; s < KC; s++) {
            // a k group whose share of the range is shorter than the others' skips the k-steps
            // past its end (wave-uniform)
            if (ks_begin + stage * KC + s >= ks_end) continue;
            if constexpr (MT <= 5) {
                // all LDS reads of the k-step are issued before its first MFMA; fragment f is
                // waited for with the NF-1-f later reads still in flight
                constexpr int NF = C::PL * MT - (PACK ? 1 : 0);
                static_assert(NF <= 16, "lgkmcnt range");
                bf16x8 a[NF];
                static_for<0, NF>([&](auto f_c) {
                    constexpr int F = decltype(f_c)::value;
                    a[F] = lds_read_frag<((SLOT * C::NFRAG + F * KC) * 64) * 16>(lds_lane_base + s * 1024);
                });
                static_for<0, NF>([&](auto f_c) {
                    constexpr int F = decltype(f_c)::value, i = F % MT;
                    lds_wait_frag<NF - 1 - F>(a[F]);
#pragma unroll
                    for (int j = 0; j < NW; j++)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            a[F], __builtin_bit_cast(bf16x8, w[SLOT][j][s]), acc[i][j], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);          // keeps the next fragment's wait behind these MFMAs
                });
            } else {
                // tall passes (6 to 10 m-tiles): the fragments of a k-step are read in batches of
                // AB, so that the accumulators (MT x NW tiles) leave room for them
                static_assert(!PACK, "tall passes never pack");
                constexpr int NF = C::PL * MT, AB = 4, NB = (NF + AB - 1) / AB;
                static_for<0, NB>([&](auto b_c) {
                    constexpr int B0 = decltype(b_c)::value * AB, BN = (NF - B0) < AB ? (NF - B0) : AB;
                    bf16x8 a[BN];
                    static_for<0, BN>([&](auto f_c) {
                        constexpr int F = B0 + decltype(f_c)::value;
                        a[F - B0] = lds_read_frag<((SLOT * C::NFRAG + F * KC) * 64) * 16>(lds_lane_base + s * 1024);
                    });
                    static_for<0, BN>([&](auto f_c) {
                        constexpr int F = B0 + decltype(f_c)::value, i = F % MT;
                        lds_wait_frag<BN - 1 - (F - B0)>(a[F - B0]);
#pragma unroll
                        for (int j = 0; j < NW; j++)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                a[F - B0], __builtin_bit_cast(bf16x8, w[SLOT][j][s]), acc[i][j], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    });
                });
            }
        }
    };
    // One pipeline step for stage c living in slot U: wait for its data (leaving the D-2 newer
    // stages in flight), make it visible to the workgroup, refill the slot freed by stage
    // c-1, multiply.  Every step issues exactly C::LOADS loads, also for stages past the end
    // (those read the zero granule), so the wait count is a compile-time constant and the
    // compiler's own wait-count analysis sees every register dependency satisfied by it; with
    // data-dependent counts it drains the whole ring at the loop head instead.
    // The k groups take the two halves of a step in opposite order: behind the barrier one
    // group queues its loads on the vector-memory path while the other is on LDS and the
    // matrix cores (waves of different groups share a SIMD), then they swap.  Two copies of the
    // loop, chosen once per wave: with both orders inside one body the compiler's wait-count
    // analysis loses track at the join and drains the ring (vmcnt(0)) before every multiply.
    auto main_loop = [&](auto multiply_first_c) __attribute__((always_inline)) {
        constexpr bool MULTIPLY_FIRST = decltype(multiply_first_c)::value;
        int c = 0;
        for (; c + D <= n_stages; c += D)        // branch-free body: D steps, slots 0..D-1
            static_for<0, D>([&](auto u_c) {
                constexpr int U = decltype(u_c)::value;
                constexpr int PRE = (U + D - 1) % D;
                wait_vmcnt_lds<(D - 2) * C::LOADS>();
                wg_barrier();
                if constexpr (MULTIPLY_FIRST) {
                    compute(u_c, c + U);
                    issue(std::integral_constant<int, PRE>{}, c + U + D - 1);
                } else {
                    issue(std::integral_constant<int, PRE>{}, c + U + D - 1);
                    compute(u_c, c + U);
                }
            });
        return c;
    };

    // A launch that finishes its own output needs the row factors of its rows at the end.  The sums
    // behind them are requested here, ahead of the first stages' loads (every thread fetches, from
    // a clamped row, and where there is nothing to fetch from the slab instead: no branch around
    // the loads), and reduced to the one factor right behind those loads, where the wave has to
    // wait for its first stage anyway: a single register lives through the loop.
    RowScaleSums my_row_sums;
    if constexpr (DIRECT) {
        const bool have = direct.kind != GEMM_OUT_PARTIAL && direct.rs.ssq != nullptr;
        const float4 *src = have ? reinterpret_cast<const float4 *>(direct.rs.ssq + (int64_t)min(m_base + (tid % (MT * 16)), M - 1) * RMS_MAX_CHUNKS)
                                 : reinterpret_cast<const float4 *>(A_frag);
        my_row_sums.q0 = src[0]; my_row_sums.q1 = src[1]; my_row_sums.q2 = src[2]; my_row_sums.q3 = src[3];
    }
    static_for<0, D - 1>([&](auto u_c) { issue(u_c, decltype(u_c)::value); });
    float my_row_scale = 0.f;
    if constexpr (DIRECT) {
        if (direct.kind != GEMM_OUT_PARTIAL && m_base + (tid % (MT * 16)) < M) my_row_scale = row_scale_finish(direct.rs, my_row_sums);
    }
    int c;
    if (KG > 1 && (kg & 1)) c = main_loop(std::true_type{});
    else c = main_loop(std::false_type{});
    // Remaining n_stages % D steps: nothing more to fetch.  Stages c .. c+D-2 were issued by the
    // loop above (or the prologue) with C::LOADS loads each, so step U leaves D-2-U stages in
    // flight.  (Issuing dummy loads here instead would not keep the count: the compiler drops
    // the register loads whose values are never used, and the wait would then cover too little.)
    static_for<0, D - 1>([&](auto u_c) {
        constexpr int U = decltype(u_c)::value;
        if (c + U < n_stages) {
            wait_vmcnt_lds<(D - 2 - U) * C::LOADS>();
            wg_barrier();
            compute(u_c, c + U);
        }
    });

    if constexpr (KG > 1) {
        // sum the k groups through LDS, group by group in a fixed order; group 0 stores
        wait_vmcnt_lds<0>();                                 // incl. this wave's fetches of stages past the end
        float4 *mrg = reinterpret_cast<float4 *>(smem_u4) + wn * (MT * NW * 64);
#pragma unroll
        for (int src = 1; src < KG; src++) {
            __syncthreads();
            if (kg == src) {
#pragma unroll
                for (int i = 0; i < MT; i++)
#pragma unroll
                    for (int j = 0; j < NW; j++)
                        mrg[(i * NW + j) * 64 + lane] = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
            }
            __syncthreads();
            if (kg == 0) {
#pragma unroll
                for (int i = 0; i < MT; i++)
#pragma unroll
                    for (int j = 0; j < NW; j++) {
                        const float4 v = mrg[(i * NW + j) * 64 + lane];
                        acc[i][j][0] += v.x; acc[i][j][1] += v.y; acc[i][j][2] += v.z; acc[i][j][3] += v.w;
                    }
            }
        }
        if (kg != 0) return;
    }
    if constexpr (PACK) {
        // the packed tile's low-plane products sit pack_off rows (pack_off / 4 lane groups)
        // further down: add them to the rows they belong to
#pragma unroll
        for (int j = 0; j < NW; j++)
#pragma unroll
            for (int r = 0; r < 4; r++) acc[MT - 1][j][r] += __shfl_down(acc[MT - 1][j][r], 4 * pack_off, 64);
    }
    // D layout: lane (g = lane/16, c = lane%16) holds rows 4g..4g+3, column c of each tile.
    const int g = lane >> 4, cc = lane & 15;
    // Stores of the wave's MT x NW tiles (k group 0 after the merge).  With k groups they go
    // through the wave's own LDS region (the one its partners wrote into, private since the
    // merge) and leave as 16 bytes per lane: whole NW*64-byte row segments instead of 64-byte
    // pieces.  Rows of 4-row group g sit in the half of the row given by g's parity (two-way
    // instead of four-way bank conflicts).
    auto store_tiles = [&](float *o, auto &&value) __attribute__((always_inline)) {
        if constexpr (KG > 1) {
            constexpr int CPR = NW * 4, RPI = 64 / CPR;       // 16-byte chunks per row, rows per store instruction
            float *stage = reinterpret_cast<float *>(smem_u4) + wn * (MT * NW * 256);
#pragma unroll
            for (int i = 0; i < MT; i++)
#pragma unroll
                for (int j = 0; j < NW; j++)
#pragma unroll
                    for (int r = 0; r < 4; r++) {
                        const int row = i * 16 + 4 * g + r, chunk = (j * 4 + (cc >> 2)) ^ ((CPR / 2) * (g & 1));
                        stage[row * (NW * 16) + chunk * 4 + (cc & 3)] = value(i, j, r);
                    }
            // (the same wave wrote and reads: LDS keeps a wave's accesses in order)
#pragma unroll
            for (int k = 0; k < MT * 16 / RPI; k++) {
                const int row = k * RPI + lane / CPR, chunk = lane % CPR;
                const int phys = chunk ^ ((CPR / 2) * ((row >> 2) & 1));
                const float4 v = *reinterpret_cast<const float4 *>(stage + row * (NW * 16) + phys * 4);
                const int m = m_base + row, t = t0 + (chunk >> 2);
                if (m < M && t < NT) *reinterpret_cast<float4 *>(o + (int64_t)m * ldo + t0 * 16 + chunk * 4) = v;
            }
        } else {
#pragma unroll
            for (int j = 0; j < NW; j++) {
                const int t = t0 + j;
                if (t >= NT) continue;
#pragma unroll
                for (int i = 0; i < MT; i++)
#pragma unroll
                    for (int r = 0; r < 4; r++) {
                        const int m = m_base + i * 16 + 4 * g + r;
                        if (m < M) o[(int64_t)m * ldo + t * 16 + cc] = value(i, j, r);
                    }
            }
        }
    };
    if (DIRECT && direct.kind != GEMM_OUT_PARTIAL) {
        // single split: the sums are complete.  The row factors of the block's rows are computed
        // once per workgroup (one thread per row) and handed out through LDS.
        float *scale_lds = reinterpret_cast<float *>(smem_u4 + (C::SMEM - 1024) / 16);   // the dump slot
        if constexpr (KG == 1) wait_vmcnt_lds<0>();          // (KG > 1: done before the merge)
        __syncthreads();
        if (tid < MT * 16) scale_lds[tid] = my_row_scale;
        __syncthreads();
        float sc[MT][4];
#pragma unroll
        for (int i = 0; i < MT; i++)
#pragma unroll
            for (int r = 0; r < 4; r++) sc[i][r] = scale_lds[i * 16 + 4 * g + r];
        if (direct.kind == GEMM_OUT_SCALED) {
            // (the row factors sit in the dump slot behind the ring, outside the staging regions)
            store_tiles(out, [&](int i, int j, int r) { return acc[i][j][r] * sc[i][r]; });
        } else if constexpr (NW % 2 == 0) {
            // Tiles alternate gate, up: accumulators (j, j+1) hold gate and up of the same 16
            // features for the same rows and lanes.  The workgroup's WN*NW*8 features are whole
            // k-steps of the next GEMM: the gated values are laid out as its fragments in LDS
            // (two planes) and leave as whole 1 KiB fragments, 16 bytes per lane.
            constexpr int FEATS = WN * NW * 8, HK = FEATS / 16;           // features, half k-steps per workgroup
            static_assert(FEATS % 16 == 0, "whole half fragments");
            static_assert(2 * HK * MT * 512 <= C::SMEM, "staging fits the ring");
            // a fragment (16 rows x 32 features) is two contiguous halves of 16 features
            // (512 bytes: [feature octet][row][8 features]); the workgroup's features are whole halves
            const int F = direct.d_ffn, n_ksteps = (F + 31) >> 5, mt_all = (M + 15) >> 4;
            uint16_t *stage = reinterpret_cast<uint16_t *>(smem_u4);     // [plane][HK][MT][256]
            // (every wave is past the ring and the merge area: synchronised above)
#pragma unroll
            for (int j = 0; j < NW; j += 2) {
                const int f_local = (wn * NW + j) * 8 + cc;              // feature inside the workgroup
                const int hk = f_local >> 4, pos = ((f_local >> 3) & 1) * 128 + (f_local & 7);
                const bool live = (t0 + j) < NT;
#pragma unroll
                for (int i = 0; i < MT; i++)
#pragma unroll
                    for (int r = 0; r < 4; r++) {
                        const float gs = acc[i][j][r] * sc[i][r];
                        const float v = live ? gs / (1.0f + expf(-gs)) * (acc[i][j + 1][r] * sc[i][r]) : 0.f;
                        uint16_t hi, lo;
                        split_bf16(v, hi, lo);
                        const int at = pos + (4 * g + r) * 8;            // row 4g+r of m-tile i
                        if (PACK && i == MT - 1) {                       // the output slab packs its last tile the same way
                            if (4 * g + r < pack_off) stage[((0 * HK + hk) * MT + i) * 256 + at] = hi;
                            if (4 * g + r < rows_last) stage[((0 * HK + hk) * MT + i) * 256 + at + pack_off * 8] = lo;
                        } else {
                            stage[((0 * HK + hk) * MT + i) * 256 + at] = hi;
                            stage[((1 * HK + hk) * MT + i) * 256 + at] = lo;
                        }
                    }
            }
            __syncthreads();
            // fragment (plane, ks, mt) of the slab starts at ((plane * n_ksteps + ks) * mt_all + mt) KiB;
            // k-steps at or beyond n_ksteps and m-tiles beyond the slab do not exist.
            // One store instruction moves two halves (32 lanes x 16 bytes each).
            const int hk0 = bx * HK, mt0 = bz * MT, half_lane = lane >> 5, l32 = lane & 31;
            for (int pr = wn; pr < HK * MT * 2 / 2; pr += WN) {
                const int idx = pr * 2 + half_lane;                      // (plane, hk, i) flattened, as staged
                const int plane = idx / (HK * MT), hk = (idx / MT) % HK, i = idx % MT;
                const int hkg = hk0 + hk;                                // half k-step in the whole slab
                if ((hkg >> 1) >= n_ksteps || mt0 + i >= mt_all) continue;   // (a last half past F holds zeros)
                if (PACK && plane == 1 && i == MT - 1) continue;             // lives in the high plane's fragment
                const uint4 v = reinterpret_cast<const uint4 *>(stage)[idx * 32 + l32];
                reinterpret_cast<uint4 *>(direct.act_frag)[(((int64_t)plane * n_ksteps + (hkg >> 1)) * mt_all + mt0 + i) * 64 +
                                                           (hkg & 1) * 32 + l32] = v;
            }
            // A feature count that is an odd number of 16-feature halves leaves the second half of
            // the slab's last k-step without a feature.  Where the grid's columns run past F, the
            // loop above has stored zeros there (tiles beyond the matrix are not live); where they
            // end exactly at F, the workgroup that owns the last half clears it here: the down
            // projection multiplies it by zero-padded weights, and 0 x NaN of stale memory is NaN.
            const int n_half = F >> 4;
            if ((n_half & 1) && hk0 + HK == n_half && lane < 32) {
                for (int pr = wn; pr < 2 * MT; pr += WN) {
                    const int plane = pr / MT, i = pr % MT;
                    if (mt0 + i >= mt_all || (PACK && plane == 1 && i == MT - 1)) continue;
                    reinterpret_cast<uint4 *>(direct.act_frag)[(((int64_t)plane * n_ksteps + (n_half >> 1)) * mt_all + mt0 + i) * 64 +
                                                               32 + lane] = make_uint4(0u, 0u, 0u, 0u);
                }
            }
        }
        return;
    }
    store_tiles(out + (int64_t)by * M * ldo, [&](int i, int j, int r) { return acc[i][j][r]; });
}

// out[m][n] = rowscale(m) * sum over splits of partial[s][m][n], in split order
__global__ void reduce_partials_kernel(const float *__restrict__ partial, int splits, int M,
                                       int64_t N, int64_t ld, float *__restrict__ out, RowScale rs) {
    const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int m = blockIdx.y;
    if (n >= N) return;
    float acc = 0.f;
    for (int s = 0; s < splits; s++) acc += partial[((int64_t)s * M + m) * ld + n];
    out[(int64_t)m * N + n] = acc * row_scale(rs, m);
}

// Pure permutation: row-major [N][K] bf16 -> packed tiles (see file header).
__global__ void pack_weight_kernel(const uint16_t *__restrict__ src, int64_t N, int64_t K, int64_t KS,
                                   uint4 *__restrict__ dst, int64_t tile0, int64_t tile_stride,
                                   int64_t total_tiles) {
    const int64_t blk = blockIdx.x;            // (source tile, k-step incl. the padding step)
    const int64_t t = blk / KS, s = blk % KS;
    const int lane = threadIdx.x;
    const int64_t n = t * 16 + (lane & 15), k = s * 32 + (lane >> 4) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (k < K) v = *reinterpret_cast<const uint4 *>(src + n * K + k);
    dst[packed_block(tile0 + t * tile_stride, s, total_tiles) * 64 + lane] = v;
}

// Row-major bf16 planes -> A-operand fragment order (used by the stand-alone GEMM entry point;
// inside the verify step the producing kernels write this layout directly).
__global__ void to_fragments_kernel(const uint16_t *__restrict__ a_hi, const uint16_t *__restrict__ a_lo, int M,
                                    int K, int64_t lda, int KS, int m_tiles, uint4 *__restrict__ dst) {
    const int ks = blockIdx.x, mt = blockIdx.y, plane = blockIdx.z, lane = threadIdx.x;
    const uint16_t *src = plane ? a_lo : a_hi;
    const int m = mt * 16 + (lane & 15), k = ks * 32 + (lane >> 4) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (src && m < M && k < K) v = *reinterpret_cast<const uint4 *>(src + (int64_t)m * lda + k);
    const int pack_off = a_lo ? frag_pack_offset(M) : 0;
    if (pack_off && mt == m_tiles - 1) {
        // both planes of a packed last tile share the high plane's fragment (disjoint rows)
        const int row = lane & 15;
        if (plane == 0 && row < pack_off) dst[((int64_t)ks * m_tiles + mt) * 64 + lane] = v;
        if (plane == 1 && m < M) dst[((int64_t)ks * m_tiles + mt) * 64 + lane + pack_off] = v;
        return;
    }
    dst[(((int64_t)plane * KS + ks) * m_tiles + mt) * 64 + lane] = v;
}

// Launch shapes.  Wide groups reuse each activation fragment for more weight tiles (the
// L2->LDS slab traffic is what limits narrow ones) but produce wider split-K partials; deep
// rings and more waves keep more weight bytes in flight per CU.
struct GemmVariant { int nw, waves, depth, kgroups; };
static const GemmVariant g_variants[] = {
    {1, 4, 4, 1}, {2, 4, 4, 1}, {4, 4, 4, 1}, {2, 8, 6, 1}, {4, 8, 6, 1},
    {2, 8, 4, 2}, {4, 8, 4, 2}, {1, 8, 4, 2}, {2, 8, 3, 2}, {2, 16, 3, 2}, {2, 6, 3, 2}, {2, 14, 3, 2},
    {4, 8, 3, 2},     // 12: tall passes (6 to 9 m-tiles per pass), 16 tiles per k group
};
#define GEMM_N_VARIANTS ((int)(sizeof(g_variants) / sizeof(g_variants[0])))
static int g_force_variant = -1, g_force_splits = -1;
// variant: >= 0 forces that workgroup shape, -1 the heuristic, -2 the heuristic without tall passes
void gemm_force_plan(int variant, int splits) { g_force_variant = variant < -2 ? -1 : variant; g_force_splits = splits; }

GemmPlan gemm_plan(int m_rows, int64_t n_rows, int64_t k) {
    GemmPlan p;
    const int64_t NT = n_rows / 16, KS = (k + 31) / 32;
    // Shapes measured on MI355X at 68 rows (7B- and 70B-like widths): 2 k groups of 4 waves
    // with 2 tiles per wave (128 columns per workgroup) or of 8 waves (256 columns); as many
    // splits as give one round of 256 equal workgroups, but no more than 8 for the narrow ones,
    // whose partial sums are re-read by a row-wise consumer.
    const int m_tiles = (m_rows + 15) / 16;
    p.variant = NT < 3000 ? 8 : 6;
    // 16 waves (256 columns per workgroup, half the activation-slab traffic per weight byte)
    // for the widest matrices, the QKV-like widths and narrow matrices with a very long k;
    // these and the 6- and 14-wave forms are instantiated for 1 and 5 m-tiles per pass
    const bool wide16 = NT >= 3000 || (NT >= 512 && NT < 1024 && (NT >= 640 || KS >= 512));
    const bool mt_1_or_5 = !(m_tiles == 2 || m_tiles == 3 || m_tiles == 6 || m_tiles == 7);
    if (wide16 && mt_1_or_5) p.variant = 9;
    // matrices wide enough for a single k split: the workgroup width (3, 4, 7 or 8 waves of 2
    // tiles per k group) that puts the most workgroups on the 256 CUs in one round
    if (NT >= 1024 && mt_1_or_5) {
        static const int wn_of[4] = {3, 4, 7, 8}, variant_of[4] = {10, 8, 11, 9};
        int64_t best = 0;
        for (int i = 0; i < 4; i++) {
            const int64_t wgs = (NT + 2 * wn_of[i] - 1) / (2 * wn_of[i]);
            if (wgs <= 256 && wgs >= best) { best = wgs; p.variant = variant_of[i]; }
        }
    }
    if (m_tiles == 6 || m_tiles == 7) p.variant = 8;            // one pass: 4 tiles per wave x 7 m-tiles of accumulators would spill
    // Many rows (prefill chunks, batches, per-node mask groups on large trees): the launch
    // makes `passes` row passes of 5 m-tiles over the weights, every pass its own set of
    // workgroups.  The passes fill the CUs, so fewer k splits are needed, and the widest
    // workgroups (16 waves, or 14 on the gate/up-like widths) share each activation fragment
    // among the most weight tiles.
    int passes = m_tiles > 7 ? (m_tiles + 4) / 5 : 1;
    if (passes >= 2) p.variant = (NT >= 1024 && NT < 3000) ? 11 : 9;
    p.mt_pass = 0;
    // Tall passes (6 to 9 m-tiles per pass, variant 12): fewer passes over the weights and 16
    // weight tiles per activation fragment, against fewer, fatter workgroups.  What decides is the
    // traffic through one CU's vector L1 (weights + activation slab of the workgroup's k range) times
    // the number of rounds the workgroups take on the 256 CUs, plus the split-K partial sums; the
    // same estimate for both forms, the tall one taken where it predicts at least a fifth less
    // (measured on the 7B-shaped matrices at 105 to 512 rows: the estimate ranks the forms right
    // beyond that margin and the choice is then 12 to 36 % faster; inside it they are within 5 %).
    if (m_tiles >= 6 && g_force_variant == -1) {
        auto estimate = [&](int mt, int n_pass, int tiles_wg, int *splits_out) {
            const int64_t wgs_n = (NT + tiles_wg - 1) / tiles_wg;
            int64_t sp = 256 / (wgs_n * n_pass);
            if (sp > KS / 8) sp = KS / 8;
            if (NT < 512 && sp > 8) sp = 8;
            if (sp > 32) sp = 32;
            if (g_force_splits > 0) sp = g_force_splits;
            if (sp < 1) sp = 1;
            const int64_t per = (KS + sp - 1) / sp;
            sp = (KS + per - 1) / per;
            const double per_wg = (double)(tiles_wg + 2 * mt) * 1024.0 * (double)per;
            const double rounds = (double)((wgs_n * n_pass * sp + 255) / 256);
            double t = rounds * per_wg / 41e9;                              // ~17 B/clk through one CU's L1
            if (sp > 1) t += 2.0 * (double)sp * m_rows * (double)n_rows * 4.0 / 4e12;
            *splits_out = (int)sp;
            return t;
        };
        int sp_now = 1;
        const GemmVariant &vn = g_variants[m_tiles <= 7 ? 8 : p.variant];
        const double t_now = estimate(m_tiles <= 7 ? m_tiles : 5, passes, vn.nw * vn.waves / vn.kgroups, &sp_now);
        double t_best = 0.8 * t_now;
        for (int cap = 9; cap >= 6; cap--) {
            const int n_pass = (m_tiles + cap - 1) / cap, mt = (m_tiles + n_pass - 1) / n_pass;
            if (mt < 6) continue;
            int sp = 1;
            const double t = estimate(mt, n_pass, 16, &sp);
            if (t < t_best) { t_best = t; p.mt_pass = mt; passes = n_pass; p.variant = 12; }
        }
    }
    if (g_force_variant >= 0 && g_force_variant < GEMM_N_VARIANTS) p.variant = g_force_variant;
    const GemmVariant &v = g_variants[p.variant];
    const int tiles_wg = v.nw * v.waves / v.kgroups;
    const int64_t wgs_n = (NT + tiles_wg - 1) / tiles_wg;
    int64_t splits = (v.waves > 4 ? 256 : 512) / (wgs_n * passes);
    const int64_t max_splits = KS / 8;                          // at least 8 stages per split
    if (splits > max_splits) splits = max_splits;
    if (NT < 512 && splits > 8) splits = 8;
    if (splits > 32) splits = 32;
    if (g_force_splits > 0) splits = g_force_splits;
    if (splits < 1) splits = 1;
    const int64_t per = (KS + splits - 1) / splits;
    p.ksteps_per_split = (int)per;
    p.splits = (int)((KS + per - 1) / per);
    return p;
}

template <int MT, int NW, bool SPLIT, int WAVES, int D, int KG, bool DIRECT, bool PACK = false>
static void launch_gemm_t(const void *a_frag, int M, int64_t K, const void *w, int64_t N, float *out, int64_t ldo,
                          const GemmPlan &p, hipStream_t s, const GemmOutput &direct) {
    constexpr int KC = 1;
    using C = GemmCfg<MT, NW, SPLIT, KC, D, WAVES, KG, PACK>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)gemm_skinny_kernel<MT, NW, SPLIT, KC, D, WAVES, KG, DIRECT, PACK>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM);
        attr_set = true;
    }
    const int NT = (int)(N / 16), KS = (int)((K + 31) / 32), m_tiles = (M + 15) / 16;
    dim3 grid((NT + C::WN * NW - 1) / (C::WN * NW), p.splits, (m_tiles + MT - 1) / MT);
    hipLaunchKernelGGL((gemm_skinny_kernel<MT, NW, SPLIT, KC, D, WAVES, KG, DIRECT, PACK>), grid, dim3(WAVES * 64), C::SMEM, s,
                       (const uint4 *)a_frag, (const uint4 *)w, KS * m_tiles, M, m_tiles, NT, KS, p.ksteps_per_split,
                       (int)grid.x, (int)grid.y, (int)grid.z, out, ldo, direct);
}

template <int MT, bool SPLIT>
static void launch_gemm_v(const void *a_frag, int M, int64_t K, const void *w, int64_t N, float *out, int64_t ldo,
                          const GemmPlan &p, hipStream_t s, const GemmOutput &direct) {
    // the instantiations with an output epilogue exist for the k-group shapes only
    // a two-plane slab whose last m-tile is packed (frag_pack_offset) takes the instantiation
    // that reads it so; both exist for one and five m-tiles, the only slabs that pack
    constexpr bool CAN_PACK = SPLIT && (MT == 1 || MT == 5);
    const bool pack = CAN_PACK && frag_pack_offset(M) != 0;
#define T(nw, waves, d, kg, dir) do { \
        if constexpr (CAN_PACK) { \
            if (pack) { launch_gemm_t<MT, nw, SPLIT, waves, d, kg, dir, true>(a_frag, M, K, w, N, out, ldo, p, s, direct); break; } \
        } \
        launch_gemm_t<MT, nw, SPLIT, waves, d, kg, dir, false>(a_frag, M, K, w, N, out, ldo, p, s, direct); \
    } while (0)
#define V(i, nw, waves, d, kg) case i: T(nw, waves, d, kg, false); break;
#define W(i, nw, waves, d, kg) case i: \
        if (direct.kind != GEMM_OUT_PARTIAL) T(nw, waves, d, kg, true); \
        else T(nw, waves, d, kg, false); \
        break;
    switch (p.variant) {
        V(0, 1, 4, 4, 1) V(1, 2, 4, 4, 1) V(2, 4, 4, 4, 1) V(3, 2, 8, 6, 1) V(4, 4, 8, 6, 1)
        W(5, 2, 8, 4, 2) W(6, 4, 8, 4, 2) V(7, 1, 8, 4, 2) W(8, 2, 8, 3, 2) W(9, 2, 16, 3, 2) W(10, 2, 6, 3, 2) W(11, 2, 14, 3, 2)
    }
#undef V
#undef W
#undef T
}

// two planes, the planner's variants (6 and 8) only; more than 5 m-tiles with variant 8 alone (registers, LDS ring)
template <int MT>
static void launch_gemm_k(const void *a_frag, int M, int64_t K, const void *w, int64_t N, float *out, int64_t ldo,
                          const GemmPlan &p, hipStream_t s, const GemmOutput &direct) {
    const bool d = direct.kind != GEMM_OUT_PARTIAL;
    if constexpr (MT <= 5) {
        if (p.variant == 6) {
            if (d) launch_gemm_t<MT, 4, true, 8, 4, 2, true>(a_frag, M, K, w, N, out, ldo, p, s, direct);
            else launch_gemm_t<MT, 4, true, 8, 4, 2, false>(a_frag, M, K, w, N, out, ldo, p, s, direct);
            return;
        }
    }
    if (d) launch_gemm_t<MT, 2, true, 8, 3, 2, true>(a_frag, M, K, w, N, out, ldo, p, s, direct);
    else launch_gemm_t<MT, 2, true, 8, 3, 2, false>(a_frag, M, K, w, N, out, ldo, p, s, direct);
}

// a_frag: activations in fragment order, [planes][k-steps][m-tiles][64] x 16 bytes;
// out_partial: [splits][M][ldo] fp32.
void launch_gemm(const void *a_frag, bool two_planes, int M, int64_t K, const void *w, int64_t N,
                 float *out, int64_t ldo, const GemmPlan &p, hipStream_t s, const GemmOutput *directp) {
    GemmOutput direct;
    memset(&direct, 0, sizeof(direct));
    // direct outputs need complete sums and, for the gating, gate/up tile pairs inside one wave
    if (directp && gemm_direct_output_possible(p, directp->kind)) direct = *directp;
    const int m_tiles = (M + 15) / 16;
    if (p.mt_pass >= 6 && two_planes) {
        const bool d = direct.kind != GEMM_OUT_PARTIAL;
#define TALL(MT_) case MT_: \
            if (d) launch_gemm_t<MT_, 4, true, 8, 3, 2, true>(a_frag, M, K, w, N, out, ldo, p, s, direct); \
            else launch_gemm_t<MT_, 4, true, 8, 3, 2, false>(a_frag, M, K, w, N, out, ldo, p, s, direct); \
            return;
        switch (p.mt_pass) { TALL(6) TALL(7) TALL(8) TALL(9) }
#undef TALL
    }
    if (M <= 16) {
        if (two_planes) launch_gemm_v<1, true>(a_frag, M, K, w, N, out, ldo, p, s, direct);
        else launch_gemm_v<1, false>(a_frag, M, K, w, N, out, ldo, p, s, direct);
        return;
    }
    // Row counts other than the 65..80 of the 64-node tree (Sec. 4.3.4, Table 4: 16 or 21 tree rows for
    // the efficient tree, 105 rows with a mask group behind each of its nodes): one pass over
    // the weights with 2, 3 or 7 m-tiles, for the planner's two variants.  Beyond 7 m-tiles
    // the weight stream no longer bounds the kernel, and passes of 5 m-tiles (grid z)
    // measured as fast as fewer passes of 7 or 10.
    const bool planner_variant = p.variant == 6 || p.variant == 8;
    if (two_planes && planner_variant && (m_tiles <= 3 || (m_tiles >= 6 && m_tiles <= 7 && p.variant == 8))) {
        if (m_tiles == 2) launch_gemm_k<2>(a_frag, M, K, w, N, out, ldo, p, s, direct);
        else if (m_tiles == 3) launch_gemm_k<3>(a_frag, M, K, w, N, out, ldo, p, s, direct);
        else launch_gemm_k<7>(a_frag, M, K, w, N, out, ldo, p, s, direct);
        return;
    }
    GemmPlan q = p;
    if (q.variant == 12) q.variant = 9;     // (a single-plane slab has no tall form: passes of 5 m-tiles, same splits)
    if (two_planes) launch_gemm_v<5, true>(a_frag, M, K, w, N, out, ldo, q, s, direct);
    else launch_gemm_v<5, false>(a_frag, M, K, w, N, out, ldo, q, s, direct);
}
bool gemm_direct_output_possible(const GemmPlan &p, int kind) {
    (void)kind;
    return p.splits == 1 && (p.variant == 5 || p.variant == 6 || p.variant >= 8);   // (12: four tiles per wave)   // even tiles per wave, see launch_gemm_v
}

size_t frag_bytes(int m_rows, int64_t k) {                     // two planes
    return (size_t)2 * ((k + 31) / 32) * ((m_rows + 15) / 16) * 1024;
}

void launch_to_fragments(const void *a_hi, const void *a_lo, int M, int64_t K, int64_t lda, void *dst,
                         hipStream_t s) {
    const int KS = (int)((K + 31) / 32), m_tiles = (M + 15) / 16;
    hipLaunchKernelGGL(to_fragments_kernel, dim3(KS, m_tiles, 2), dim3(64), 0, s, (const uint16_t *)a_hi,
                       (const uint16_t *)a_lo, M, (int)K, lda, KS, m_tiles, (uint4 *)dst);
}

void launch_reduce_partials(const float *partial, int splits, int M, int64_t N, int64_t ld,
                            float *out, const RowScale &rs, hipStream_t s) {
    dim3 grid((unsigned)((N + 255) / 256), M);
    hipLaunchKernelGGL(reduce_partials_kernel, grid, dim3(256), 0, s, partial, splits, M, N, ld, out, rs);
}

void launch_pack(const void *src, int64_t N, int64_t K, void *dst, int64_t tile0, int64_t tile_stride,
                 int64_t total_tiles, hipStream_t s) {
    const int64_t KS = ((K + 63) / 64) * 2;                 // k-steps incl. zero padding to a pair
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((N / 16) * KS)), dim3(64), 0, s,
                       (const uint16_t *)src, N, K, KS, (uint4 *)dst, tile0, tile_stride, total_tiles);
}
