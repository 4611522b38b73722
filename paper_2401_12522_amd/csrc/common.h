// Internal declarations shared by the HIP sources of libbita (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <map>
#include <mutex>
#include <vector>
#include "../../include/bita.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define BITA_WAVE 64

// bf16 <-> fp32 on raw bits (round to nearest even; inputs are finite)
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
// x ~= hi + lo with both parts bf16: the pair carries ~16 mantissa bits of x
__device__ __forceinline__ void split_bf16(float x, uint16_t &hi, uint16_t &lo) {
    hi = f32_to_bf16(x);
    lo = f32_to_bf16(x - bf16_to_f32(hi));
}
// Position (in bf16 elements) of A[m][k] of plane p inside an activation slab kept in MFMA
// A-operand fragment order: 1 KiB per (plane, k-step of 32, m-tile of 16), lane l of a
// fragment holding A[16mt + l%16][32ks + 8(l/16) .. +8].
// A last m-tile that is at most half full keeps BOTH planes of its rows in the high plane's
// fragment: the low plane of row r sits at row r + off (off = 4 for up to 4 rows, 8 for up to 8).
// One fragment and one matrix instruction per weight tile then serve both planes of those rows;
// the two partial products come out as different accumulator rows and are added once, after the
// k loop.  frag_pack_offset gives off (0 = not packed) from the slab's row count alone, so
// producers and the GEMM agree; it applies to the slabs whose GEMM always takes every m-tile in
// one pass with as many accumulator tiles: one m-tile (M <= 8: the one-row pass) or five
// (65..72 rows: the 64-node tree with its mask rows).
__host__ __device__ __forceinline__ int frag_pack_offset(int M) {
    const int m_tiles = (M + 15) >> 4, v = M - 16 * (m_tiles - 1);
    if ((m_tiles != 1 && m_tiles != 5) || v > 8) return 0;
    return v <= 4 ? 4 : 8;
}
__device__ __forceinline__ int64_t frag_index(int plane, int m, int k, int n_ksteps, int m_tiles, int pack_off) {
    if (pack_off && plane == 1 && (m >> 4) == m_tiles - 1) {
        plane = 0;
        m += pack_off;
    }
    const int ks = k >> 5, kq = (k >> 3) & 3, e = k & 7;
    return ((((int64_t)plane * n_ksteps + ks) * m_tiles + (m >> 4)) * 64 + kq * 16 + (m & 15)) * 8 + e;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// ---- host-side error plumbing -------------------------------------------------
int  bita_set_error(int code, const char *fmt, ...);
#define BITA_HIP_CHECK(expr)                                                                 \
    do {                                                                                     \
        hipError_t _e = (expr);                                                              \
        if (_e != hipSuccess)                                                                \
            return bita_set_error(BITA_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(_e)); \
    } while (0)

// ---- device mirror of a pass layout ---------------------------------------------
struct TemplateDev {
    int32_t rows, n_tree, n_mask, n_groups, depth_max, kmax, words;
    const int32_t *parent;        // [R]
    const int32_t *depth;         // [R]
    const int32_t *rank;          // [R] sibling rank of a tree row
    const int32_t *mask_index;    // [R] index inside its group, -1 for tree rows
    const int32_t *group_of_node; // [T] group attached to a tree row or -1
    const int32_t *mask_rows;     // [G*n] row of mask i of group g
    const uint8_t *is_mask;       // [R]
    const uint64_t *anc;          // [R][words] ancestor-or-self bitsets
};
struct bita_tree_template {
    TemplateDev dev;
    void *blob;                   // one device allocation backing all arrays
};

// ---- the model handle: borrowed weight pointers plus the rotary table it owns --------
struct bita_model {
    bita_config cfg;
    const void *tok_emb, *mask_emb, *final_norm, *lm_head;
    std::vector<const void *> attn_norm, ffn_norm, wqkv, wo, w_gate_up, w_down, prompt_k, prompt_v;
    float *rope_cos = nullptr, *rope_sin = nullptr;     // [max_pos][hd/2]
    // chain templates of the prefill chunks by row count, created once and kept until the
    // handle is destroyed (the enqueued kernels read their device arrays)
    std::mutex chain_mutex;
    std::map<int, bita_tree_template *> chains;
};

// ---- kernel launchers (each only enqueues) --------------------------------------
#define RMS_MAX_CHUNKS 16          // 1024 columns each: d_model <= 16384
struct RowScale { const float *ssq; int chunks; float inv_d, eps; };   // ssq == nullptr: no scaling
// second half of RMSNorm: rsqrt(mean(x^2) + eps) of row m from the per-chunk sums of squares.
// In two steps, so that a kernel can request the sums early and look at them late: all 16 slots of
// the row are fetched at once (independent loads, one round trip) and summed in chunk order;
// slots at or beyond rs.chunks are never written and are left out.
struct RowScaleSums { float4 q0, q1, q2, q3; };
__device__ __forceinline__ RowScaleSums row_scale_fetch(const RowScale &rs, int m) {
    RowScaleSums r;
    r.q0 = r.q1 = r.q2 = r.q3 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (!rs.ssq) return r;
    const float4 *p = reinterpret_cast<const float4 *>(rs.ssq + (int64_t)m * RMS_MAX_CHUNKS);
    r.q0 = p[0]; r.q1 = p[1]; r.q2 = p[2]; r.q3 = p[3];
    return r;
}
__device__ __forceinline__ float row_scale_finish(const RowScale &rs, const RowScaleSums &r) {
    if (!rs.ssq) return 1.0f;
    const float v[RMS_MAX_CHUNKS] = {r.q0.x, r.q0.y, r.q0.z, r.q0.w, r.q1.x, r.q1.y, r.q1.z, r.q1.w,
                                     r.q2.x, r.q2.y, r.q2.z, r.q2.w, r.q3.x, r.q3.y, r.q3.z, r.q3.w};
    float tot = 0.f;
#pragma unroll
    for (int ch = 0; ch < RMS_MAX_CHUNKS; ch++) tot += ch < rs.chunks ? v[ch] : 0.f;
    return 1.0f / sqrtf(tot * rs.inv_d + rs.eps);
}
__device__ __forceinline__ float row_scale(const RowScale &rs, int m) { return row_scale_finish(rs, row_scale_fetch(rs, m)); }
// mt_pass: m-tiles per row pass of a tall launch (6..9), 0 = the variant's own row handling
struct GemmPlan { int splits, ksteps_per_split, variant, mt_pass; };
// What a GEMM launch with a single split (complete sums in its accumulators) may do instead of
// storing fp32 partials: apply the deferred RMSNorm row factor and store the result, or apply it
// and the SwiGLU gating to its tile-interleaved gate/up columns and store the next GEMM's
// activation slab (two bf16 planes, fragment order).
enum { GEMM_OUT_PARTIAL = 0, GEMM_OUT_SCALED = 1, GEMM_OUT_SILU = 2 };
struct GemmOutput { int kind; RowScale rs; uint16_t *act_frag; int d_ffn; };
bool gemm_direct_output_possible(const GemmPlan &p, int kind);
void gemm_force_plan(int variant, int splits);   // tuning aid: < 0 restores the heuristic
GemmPlan gemm_plan(int m_rows, int64_t n_rows, int64_t k);
size_t frag_bytes(int m_rows, int64_t k);        // bytes of a two-plane activation slab
// a_frag: activations in fragment order (see frag_index); out_partial: [splits][m_rows][ldo] fp32
void launch_gemm(const void *a_frag, bool two_planes, int m_rows, int64_t k, const void *w_packed,
                 int64_t n_rows, float *out_partial, int64_t ldo, const GemmPlan &p, hipStream_t s,
                 const GemmOutput *direct = nullptr);
void launch_to_fragments(const void *a_hi, const void *a_lo, int m_rows, int64_t k, int64_t lda, void *dst,
                         hipStream_t s);
void launch_reduce_partials(const float *partial, int splits, int m_rows, int64_t n, int64_t ld,
                            float *out, const RowScale &rs, hipStream_t s);
void launch_pack(const void *src, int64_t n_rows, int64_t k, void *dst, int64_t tile0,
                 int64_t tile_stride, int64_t total_tiles, hipStream_t s);

void launch_embed(const int32_t *token, const TemplateDev &t, int batch, const void *tok_emb,
                  const void *mask_emb, int d, int vocab, float *x, hipStream_t s);
// x += sum of partials (optional), then h = rmsnorm(x) * gain as bf16 with row stride ldh
// RMSNorm is split: the prep kernel writes x*gain (two planes, fragment order) and per-chunk
// sums of squares ssq[m_rows][RMS_MAX_CHUNKS]; the row factor rsqrt(sum(ssq)/d + eps) commutes
// with the matrix product and is applied by the kernel that consumes the GEMM output.
void launch_rmsnorm_prep(float *x, const float *partial, int splits, int m_rows, int d,
                         const void *gain, void *h_frag, float *ssq, hipStream_t s);
void launch_qkv_rope(const float *partial, int splits, int batch, const TemplateDev &t,
                     int n_heads, int n_kv_heads, int hd, const int32_t *ctx_len,
                     const float *rope_cos, const float *rope_sin, int max_pos,
                     void *q, void *q_lo, void *k_tree, void *v_tree, void *k_tree_lo, void *v_tree_lo,
                     const RowScale &rs, hipStream_t s);
void launch_silu_mul(const float *partial, int splits, int m_rows, int d_ffn, void *act_frag,
                     const RowScale &rs, hipStream_t s);
void launch_select(const float *logits, int batch, const TemplateDev &t, int vocab, int kmax,
                   int32_t *argmax, int32_t *topk_ids, float *topk_val, hipStream_t s);

// Where the cache rows live: contiguous per sequence (table == nullptr) or in pages of
// 1 << page_lg key slots, page ids per sequence in table[b][0 .. max_pages).  tbl_cap: table
// entries per sequence a launch makes room for (covers the call's ctx_hint).
#define ATT_PAGE_TABLE_MAX 4096
struct PageMap { const int32_t *table; int page_lg, n_pages, max_pages, tbl_cap; };
struct AttnPlan { int splits; size_t part_o_bytes, part_ml_bytes; };
AttnPlan attn_plan(int batch, int rows, int n_heads, int hd, int ctx_hint, int n_prompt);
// k_tree_lo / v_tree_lo: low bf16 plane of the pass rows' K/V (nullable); out_lo: low plane of
// the row-major output (nullable; unused when the output is written as fragments)
void launch_tree_attention(const TemplateDev &t, const void *q, const void *q_lo, const void *k_cache,
                           const void *v_cache, const void *k_tree, const void *v_tree,
                           const void *k_tree_lo, const void *v_tree_lo,
                           const void *prompt_k, const void *prompt_v, const int32_t *ctx_len,
                           const int32_t *token /* [B][R] or nullptr: rows with a negative token are absent */,
                           int batch, int n_heads, int n_kv_heads, int hd, int n_prompt, int smax,
                           const AttnPlan &p, float *part_o, float *part_ml, void *out, void *out_lo,
                           bool out_as_fragments, const PageMap &pm, hipStream_t s);
