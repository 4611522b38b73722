// Skinny weight-streaming GEMM for the verify step: Y[M][N] = A[M][K] * W[N][K]^T with
// M = (tree + mask rows) * batch, i.e. a few dozen rows, so the kernel is bound by the one
// pass over W in HBM (the paper's premise, Sec. 3.2: inference is memory-bandwidth bound,
// extra rows are nearly free).
//
// Layout choices for gfx950:
//  * W is pre-packed into 16-row tiles whose K range is a run of 1 KiB blocks, each block
//    being exactly one v_mfma_f32_16x16x32_bf16 B-operand (lane l holds
//    W[16t + l%16][32s + 8(l/16) .. +8]).  A wave therefore streams its tile with fully
//    coalesced 16-byte-per-lane loads straight into MFMA registers; W never touches LDS.
//  * The activation slab is small and shared by every wave, so it is staged through LDS in
//    A-operand fragment order (conflict-free linear reads), double buffered along K.
//  * Parallelism comes from N (16*NW rows per wave, 4 waves per workgroup) and, where N
//    alone cannot fill 256 CUs, from split-K with fp32 partial sums reduced in a fixed
//    order by the consumer (deterministic, no float atomics).
#include "common.h"

#define GEMM_KC 4          // k-steps (of 32) per LDS chunk
#define GEMM_WAVES 4

template <int MT, int NW>
__global__ __launch_bounds__(GEMM_WAVES * 64) void gemm_skinny_kernel(
    const uint16_t *__restrict__ A, int M, int K, int64_t lda, const uint4 *__restrict__ Wp,
    int NT, int KS, float *__restrict__ out, int64_t ldo, int ksteps_per_split) {
    __shared__ uint4 a_lds[2][MT * GEMM_KC * 64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = (blockIdx.x * GEMM_WAVES + wave) * NW;
    const int ks_begin = blockIdx.y * ksteps_per_split;
    const int ks_end = min(KS, ks_begin + ksteps_per_split);
    const int m_base = blockIdx.z * (MT * 16);
    const int n_chunks = (ks_end - ks_begin + GEMM_KC - 1) / GEMM_KC;

    f32x4 acc[MT][NW];
#pragma unroll
    for (int i = 0; i < MT; i++)
#pragma unroll
        for (int j = 0; j < NW; j++) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    uint4 w_next[NW][GEMM_KC];
    uint4 a_stage[MT];
    const uint4 zero4 = make_uint4(0, 0, 0, 0);

    // staging map: thread tid of pass `it` owns row it*16 + tid%16, k-group tid/16
    const int a_row = tid & 15, a_q = tid >> 4;

    auto load_w = [&](int chunk) {
        const int ks0 = ks_begin + chunk * GEMM_KC;
#pragma unroll
        for (int j = 0; j < NW; j++)
#pragma unroll
            for (int s = 0; s < GEMM_KC; s++) {
                const int t = t0 + j, ks = ks0 + s;
                w_next[j][s] = (t < NT && ks < ks_end)
                                   ? Wp[((int64_t)t * KS + ks) * 64 + lane] : zero4;
            }
    };
    auto load_a = [&](int chunk) {
        const int k = (ks_begin + chunk * GEMM_KC) * 32 + a_q * 8;
#pragma unroll
        for (int it = 0; it < MT; it++) {
            const int m = m_base + it * 16 + a_row;
            a_stage[it] = (m < M && k < K && k < ks_end * 32)
                              ? *reinterpret_cast<const uint4 *>(A + (int64_t)m * lda + k) : zero4;
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int it = 0; it < MT; it++) a_lds[buf][it * 256 + tid] = a_stage[it];
    };

    if (n_chunks > 0) {
        load_w(0);
        load_a(0);
        store_a(0);
    }
    __syncthreads();
    for (int c = 0; c < n_chunks; c++) {
        uint4 w_cur[NW][GEMM_KC];
#pragma unroll
        for (int j = 0; j < NW; j++)
#pragma unroll
            for (int s = 0; s < GEMM_KC; s++) w_cur[j][s] = w_next[j][s];
        const bool more = (c + 1 < n_chunks);
        if (more) {
            load_w(c + 1);
            load_a(c + 1);
        }
        const int buf = c & 1;
#pragma unroll
        for (int s = 0; s < GEMM_KC; s++) {
#pragma unroll
            for (int i = 0; i < MT; i++) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, a_lds[buf][(i * GEMM_KC + s) * 64 + lane]);
#pragma unroll
                for (int j = 0; j < NW; j++)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        a, __builtin_bit_cast(bf16x8, w_cur[j][s]), acc[i][j], 0, 0, 0);
            }
        }
        if (more) store_a(buf ^ 1);
        __syncthreads();
    }

    // D layout: lane (g = lane/16, c = lane%16) holds rows 4g..4g+3, column c of each tile.
    const int g = lane >> 4, cc = lane & 15;
    float *o = out + (int64_t)blockIdx.y * M * ldo;
#pragma unroll
    for (int j = 0; j < NW; j++) {
        const int t = t0 + j;
        if (t >= NT) continue;
#pragma unroll
        for (int i = 0; i < MT; i++)
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const int m = m_base + i * 16 + 4 * g + r;
                if (m < M) o[(int64_t)m * ldo + t * 16 + cc] = acc[i][j][r];
            }
    }
}

// out[m][n] = sum over splits of partial[s][m][n], in split order
__global__ void reduce_partials_kernel(const float *__restrict__ partial, int splits, int M,
                                       int64_t N, int64_t ld, float *__restrict__ out) {
    const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int m = blockIdx.y;
    if (n >= N) return;
    float acc = 0.f;
    for (int s = 0; s < splits; s++) acc += partial[((int64_t)s * M + m) * ld + n];
    out[(int64_t)m * N + n] = acc;
}

// Pure permutation: row-major [N][K] bf16 -> packed tiles (see file header).
__global__ void pack_weight_kernel(const uint16_t *__restrict__ src, int64_t N, int64_t K, int64_t KS,
                                   uint4 *__restrict__ dst, int64_t tile0, int64_t tile_stride) {
    const int64_t blk = blockIdx.x;            // (source tile, k-step)
    const int64_t t = blk / KS, s = blk % KS;
    const int lane = threadIdx.x;
    const int64_t n = t * 16 + (lane & 15), k = s * 32 + (lane >> 4) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (k < K) v = *reinterpret_cast<const uint4 *>(src + n * K + k);
    dst[((tile0 + t * tile_stride) * KS + s) * 64 + lane] = v;
}

GemmPlan gemm_plan(int m_rows, int64_t n_rows, int64_t k) {
    GemmPlan p;
    const int64_t NT = n_rows / 16, KS = (k + 31) / 32;
    p.nw = (NT >= 2048) ? 2 : 1;
    const int64_t wgs_n = (NT + GEMM_WAVES * p.nw - 1) / (GEMM_WAVES * p.nw);
    int64_t splits = (1024 + wgs_n - 1) / wgs_n;          // aim at >= ~4 workgroups per CU
    const int64_t max_splits = (KS + 2 * GEMM_KC - 1) / (2 * GEMM_KC);  // >= 2 chunks per split
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    if (splits > 16) splits = 16;
    int64_t per = (KS + splits - 1) / splits;
    per = (per + GEMM_KC - 1) / GEMM_KC * GEMM_KC;        // whole chunks
    p.ksteps_per_split = (int)per;
    p.splits = (int)((KS + per - 1) / per);
    (void)m_rows;
    return p;
}

template <int MT, int NW>
static void launch_gemm_t(const void *a, int M, int64_t K, int64_t lda, const void *w, int64_t N,
                          float *out, int64_t ldo, const GemmPlan &p, hipStream_t s) {
    const int NT = (int)(N / 16), KS = (int)((K + 31) / 32);
    dim3 grid((NT + GEMM_WAVES * NW - 1) / (GEMM_WAVES * NW), p.splits, (M + MT * 16 - 1) / (MT * 16));
    hipLaunchKernelGGL((gemm_skinny_kernel<MT, NW>), grid, dim3(GEMM_WAVES * 64), 0, s,
                       (const uint16_t *)a, M, (int)K, lda, (const uint4 *)w, NT, KS, out, ldo,
                       p.ksteps_per_split);
}

void launch_gemm(const void *a, int M, int64_t K, int64_t lda, const void *w, int64_t N, float *out,
                 int64_t ldo, const GemmPlan &p, hipStream_t s) {
    if (M <= 16) {
        if (p.nw == 2) launch_gemm_t<1, 2>(a, M, K, lda, w, N, out, ldo, p, s);
        else launch_gemm_t<1, 1>(a, M, K, lda, w, N, out, ldo, p, s);
    } else {
        if (p.nw == 2) launch_gemm_t<5, 2>(a, M, K, lda, w, N, out, ldo, p, s);
        else launch_gemm_t<5, 1>(a, M, K, lda, w, N, out, ldo, p, s);
    }
}

void launch_reduce_partials(const float *partial, int splits, int M, int64_t N, int64_t ld,
                            float *out, hipStream_t s) {
    dim3 grid((unsigned)((N + 255) / 256), M);
    hipLaunchKernelGGL(reduce_partials_kernel, grid, dim3(256), 0, s, partial, splits, M, N, ld, out);
}

void launch_pack(const void *src, int64_t N, int64_t K, void *dst, int64_t tile0, int64_t tile_stride,
                 hipStream_t s) {
    const int64_t KS = (K + 31) / 32;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((N / 16) * KS)), dim3(64), 0, s,
                       (const uint16_t *)src, N, K, KS, (uint4 *)dst, tile0, tile_stride);
}
