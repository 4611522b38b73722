/*
 * bita.h -- C ABI of the MI355X (gfx950) tree-verify step of BiTA
 * (Bi-directional Tuning for lossless Acceleration, arXiv 2401.12522).
 *
 * One decode step of the paper's streamlined generation-and-verification loop
 * (Sec. 3.2, Appendix B, Algorithm 1) is four calls on one HIP stream:
 *
 *   bita_build_tree   candidates of the previous pass -> token of every row
 *   bita_verify_step  one decoder forward F(T, O, C, M; P) over the flattened
 *                     token tree plus mask tokens, under tree-based attention
 *   bita_accept       greedy verification walk (Algorithm 1, inner loops)
 *   bita_compact_kv   commit the accepted rows' K/V to the cache
 *
 * and the context is brought into the cache beforehand by
 *
 *   bita_prefill      chunked causal passes over the context (the same kernels)
 *
 * Conventions
 *   - Every call returns an int status: BITA_OK or a negative BITA_ERR_* code;
 *     bita_last_error() returns a human-readable message for the calling thread.
 *     Nothing aborts or throws.
 *   - Pointers named d_* (and every pointer inside bita_weights / bita_kv) are
 *     DEVICE pointers BORROWED from the caller; the library never frees them.
 *     Pointers without the prefix are HOST pointers, read during the call only.
 *   - `stream` is a hipStream_t passed as void*.  The four step calls and bita_prefill only
 *     enqueue work: no allocation, no host synchronisation, no host read of
 *     device memory.  Results are valid once the caller has synchronised the
 *     stream.  They may be captured into a HIP graph by the caller.
 *   - Row layout of a pass ("template"): R rows per sequence.  Row 0 is the root
 *     (the last emitted token, whose K/V is not cached yet), rows 1..T-1 the
 *     draft-token tree flattened in level order (Sec. 3.2), rows T..R-1 mask
 *     tokens.  A group of n mask tokens attached to node v is the parent chain
 *     v -> m_1 -> ... -> m_n, so one parent array covers both kinds of row.
 *   - All floating-point tensors are bf16 unless stated; accumulation, the
 *     residual stream, softmax and logits are fp32.
 */
#ifndef BITA_H
#define BITA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BITA_OK               0
#define BITA_ERR_INVALID_ARG -1   /* null pointer, non-positive size, misaligned shape        */
#define BITA_ERR_BAD_TREE    -2   /* parent[i] >= i, root not row 0, mask groups malformed    */
#define BITA_ERR_CAPACITY    -3   /* KV cache, rotary table or workspace too small            */
#define BITA_ERR_UNSUPPORTED -4   /* shape outside what the kernels are built for             */
#define BITA_ERR_HIP         -5   /* a HIP runtime call failed; see bita_last_error()         */

#define BITA_MAX_ROWS   512      /* R limit of one template                                   */
#define BITA_MAX_TOPK    64      /* kmax limit                                                */

/* Decoder shape.  LLaMA-2 architecture (the paper's base models, Sec. 4.1.2):
 * RMSNorm, rotary embeddings in the half-split pairing (i, i + head_dim/2),
 * SwiGLU, grouped-query attention, no biases, untied LM head.
 * Supported: head_dim 64 or 128; d_model a multiple of 32, at most 16384; d_ffn and
 * vocab multiples of 16. */
typedef struct bita_config {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t n_prompt;   /* P: prompt-prefix tokens per layer (may be 0)             */
    int32_t n_mask;     /* n: mask tokens per group                                 */
    int32_t max_pos;    /* rotary table covers positions 0 .. max_pos-1             */
    float   rms_eps, rope_theta;
} bita_config;

/* Device weight table.  The four matrices of a layer are given PACKED (see
 * bita_pack_weight); everything else is plain row-major bf16.
 *   wqkv[l]     packed rows: Wq (n_heads*hd), then Wk, then Wv (n_kv_heads*hd each), K = d_model
 *   wo[l]       packed [d_model] x K = n_heads*hd
 *   w_gate_up[l] packed, 16-row tiles interleaved: tile 2j = rows 16j.. of W_gate,
 *               tile 2j+1 = rows 16j.. of W_up; K = d_model
 *   w_down[l]   packed [d_model] x K = d_ffn
 *   lm_head     packed [vocab] x K = d_model
 *   prompt_k/v[l] [n_kv_heads][P][head_dim]: per-layer prompt prefix, used as
 *               stored (no rotary, no projection), visible to mask rows only
 *               (Sec. 3.1 and the tree-based attention of Sec. 3.2).
 * The per-layer members are HOST arrays of n_layers device pointers. */
typedef struct bita_weights {
    const void *tok_emb;      /* [vocab][d_model]  */
    const void *mask_emb;     /* [n_mask][d_model] (Sec. 3.1, mask tokens) */
    const void *final_norm;   /* [d_model] */
    const void *lm_head;      /* packed */
    const void *const *attn_norm, *const *ffn_norm;            /* [d_model] each */
    const void *const *wqkv, *const *wo, *const *w_gate_up, *const *w_down;
    const void *const *prompt_k, *const *prompt_v;
} bita_weights;

/* KV state, all device memory owned by the caller.
 *   k_cache, v_cache [n_layers][batch][n_kv_heads][smax][head_dim]: K/V of the
 *       tokens of the result sequence; slots < ctx_len are never written by
 *       bita_verify_step.
 *   k_tree, v_tree   [n_layers][batch][n_kv_heads][rows][head_dim]: K/V of the R
 *       rows of the current pass (scratch; only accepted rows are ever committed).
 *   ctx_hint: HOST upper bound on every sequence's ctx_len for this call, used
 *       only to size launches and to check capacity without reading device memory.
 * Paged cache (block_table != NULL; the paper runs batch 1 with one contiguous
 * cache, Sec. 4.1; pages serve batches whose sequences grow unevenly): the caches
 * are page pools
 *   k_cache, v_cache [n_layers][n_pages][n_kv_heads][page_size][head_dim]
 * and key slot s of sequence b lives in page block_table[b][s / page_size], row
 * s % page_size.  block_table is device memory, [batch][max_pages] int32;
 * page_size a power of two >= 16; smax (the capacity of one sequence in slots)
 * <= max_pages * page_size and <= 4096 pages.  The entries that cover slots
 * 0 .. ctx_len + rows committed by the call must name distinct pages in
 * [0, n_pages) across all sequences: the library does not check that (ids are
 * clamped to the pool: a bad table gives wrong data, never a fault).
 * block_table == NULL: contiguous layout above; the three sizes are ignored. */
typedef struct bita_kv {
    void *k_cache, *v_cache;
    void *k_tree, *v_tree;
    int32_t smax, rows, batch, ctx_hint;
    const int32_t *block_table;
    int32_t page_size, n_pages, max_pages;
} bita_kv;

typedef struct bita_model bita_model;                 /* opaque */
typedef struct bita_tree_template bita_tree_template; /* opaque */

/* Bytes needed for the packed form of an [N][K] matrix (N, K as given to
 * bita_pack_weight; N multiple of 16, K multiple of 8). */
size_t bita_packed_bytes(int64_t n_rows, int64_t k);

/* Re-lay rows of a row-major bf16 matrix d_src[N][K] (y = x W^T convention) into the
 * streaming order of the skinny-GEMM kernel.  The packed matrix of dst_total_rows rows
 * is a sequence of 1 KiB blocks, each one MFMA operand (16 rows x 32 k), ordered
 * [pair of k-steps][16-row tile][k-step of the pair], K zero-padded to a multiple of 64.
 * Source tile j is written to destination tile dst_tile0 + j*dst_tile_stride, which lets
 * several matrices share one packed buffer (QKV concatenation, gate/up interleave).  A
 * pure permutation of bits.  d_dst must hold bita_packed_bytes(dst_total_rows, K). */
int bita_pack_weight(const void *d_src, int64_t n_rows, int64_t k, void *d_dst,
                     int64_t dst_total_rows, int64_t dst_tile0, int64_t dst_tile_stride,
                     void *stream);

/* Create a model handle: copies the pointer table and builds the rotary
 * cos/sin table (allocates device memory once; freed by bita_model_destroy). */
int  bita_model_create(const bita_config *cfg, const bita_weights *w, bita_model **out);
void bita_model_destroy(bita_model *m);

/* Workspace bytes bita_verify_step needs for `batch` sequences of `rows` rows. */
size_t bita_workspace_bytes(const bita_model *m, int32_t batch, int32_t rows);

/* Validate a pass layout and mirror it to the device: depths, sibling ranks,
 * mask-group structure and ancestor-or-self bitsets (what a row attends to
 * inside the pass, Sec. 3.2) are derived here, once.  parent and is_mask are HOST
 * arrays of `rows` entries; the first n_tree rows are the token tree.  Every mask
 * group must be n_mask consecutive rows forming a chain. */
int  bita_tree_template_create(const int32_t *parent, const uint8_t *is_mask, int32_t n_tree,
                               int32_t rows, int32_t n_mask, bita_tree_template **out);
void bita_tree_template_destroy(bita_tree_template *t);
/* Host-side facts about a template: 0 rows, 1 n_tree, 2 n_groups, 3 tree depth,
 * 4 kmax (largest sibling count), 5 bitset words per row. */
int32_t bita_tree_template_info(const bita_tree_template *t, int32_t what);

/* Tokens of the next pass (Algorithm 1: the candidate set C^t becomes the tree).
 *   d_root_token [B]            the token emitted last (previous bonus token)
 *   d_cand [B][cand_rows][kmax] top-k ids of the previous pass' mask rows
 *                               (cand_rows = its number of groups times n)
 *   d_group [B] or NULL (=0)    which group of the previous pass feeds the tree
 *   d_shift [B] or NULL (=0)    how many of its leading masks are stale
 *   d_token [B][R] out          draft row at depth dv, sibling rank j gets
 *                               cand[group*n + dv-1+shift][j]; rows with no
 *                               prediction are inactive (-1); mask rows carry
 *                               their index inside the group. */
int bita_build_tree(const bita_tree_template *t, const int32_t *d_root_token,
                    const int32_t *d_cand, int32_t cand_rows, int32_t kmax,
                    const int32_t *d_group, const int32_t *d_shift,
                    int32_t batch, int32_t *d_token, void *stream);

/* One forward pass over B sequences of R rows each (Algorithm 1, the call to F).
 * Row r of sequence b is embedded (tok_emb[token] / mask_emb[index]), placed at rotary
 * position ctx_len[b] + depth(r), and attends to the
 * prompt prefix (mask rows only), to cache slots 0..ctx_len[b]-1 and to its
 * ancestors-or-self among the rows of the pass.  Writes the rows' K/V to
 * kv->k_tree/v_tree.  A tree row with a negative token is absent from the pass (no
 * candidate exists for it): it attends to nothing, and its K/V and logits are zero.
 *   d_argmax   [B][T]            greedy token of every tree row (ties: lowest id)
 *   d_topk_ids [B][G*n][kmax]    top-k of every mask row, value descending, ties by
 *                                lower id (may be NULL if the template has no masks)
 *   d_topk_val same shape, fp32, or NULL
 *   d_logits   [B][R][vocab] fp32 or NULL (then kept in the workspace)
 * Errors: CAPACITY if ctx_hint + depth exceeds max_pos or smax, or ws too small. */
int bita_verify_step(bita_model *m, const bita_kv *kv, const bita_tree_template *t,
                     const int32_t *d_token, const int32_t *d_ctx_len, int32_t batch,
                     void *d_workspace, size_t ws_bytes, int32_t kmax,
                     int32_t *d_argmax, int32_t *d_topk_ids, float *d_topk_val,
                     float *d_logits, void *stream);

/* Greedy verification (Sec. 3.2; Algorithm 1): from the root, step to the child
 * whose token equals the current row's greedy token (lowest row if several), until
 * none does.
 *   d_path    [B][depth+1]  accepted rows, root first, padded with -1
 *   d_n_acc   [B]           path length, 1 .. depth+1
 *   d_bonus   [B]           greedy token of the last accepted row (always emitted)
 *   d_emitted [B][depth+1]  tokens of path[1:], then the bonus, padded with -1
 *   d_next_group, d_next_shift [B]  mask group feeding the next tree: the one on the
 *       last accepted row (shift 0), else the root's with shift = n_acc-1. */
int bita_accept(const bita_tree_template *t, const int32_t *d_token, const int32_t *d_argmax,
                int32_t batch, int32_t *d_path, int32_t *d_n_acc, int32_t *d_bonus,
                int32_t *d_emitted, int32_t *d_next_group, int32_t *d_next_shift, void *stream);

/* For every layer and kv-head: cache[ctx_len + i] <- tree[path[i]], i < n_acc;
 * then ctx_len += n_acc.  Bit-exact copies.  path_stride is the row length of
 * d_path.  Rows that would land beyond smax are dropped and ctx_len is left
 * unchanged for that sequence (the host-side ctx_hint check normally prevents it). */
int bita_compact_kv(const bita_model *m, const bita_kv *kv, const int32_t *d_path,
                    int32_t path_stride, const int32_t *d_n_acc, int32_t *d_ctx_len,
                    int32_t batch, void *stream);

/* Context prefill (Algorithm 1: the pass over the input that precedes the first
 * draft; Sec. 3.2: ordinary tokens attend causally).  Runs the decoder over the
 * context in chunks of at most chunk_rows rows; a chunk is a verify pass whose
 * tree is a chain (row i hangs off row i-1), which is causal attention over
 * [cache, chunk], followed by committing every row of the chunk to the cache.
 * Same kernels and arithmetic as bita_verify_step / bita_compact_kv.
 *   d_tokens     [B][n_tokens]  context tokens, row b valid up to its length
 *   d_seq_len    [B] or NULL    per-sequence lengths (clamped to 0..n_tokens);
 *                               NULL = every sequence has n_tokens tokens
 *   d_ctx_len    [B] in/out     advanced by each sequence's length
 *   kv           cache as for bita_verify_step; kv->rows is the CAPACITY of the
 *                tree scratch in rows (>= chunk_rows; each chunk lays it out for
 *                its own row count), kv->ctx_hint an upper bound of ctx_len on
 *                entry
 *   chunk_rows   1..BITA_MAX_ROWS
 *   d_workspace  bita_prefill_workspace_bytes(m, batch, chunk_rows) bytes
 *   d_next_token [B] or NULL    greedy token that follows each sequence's last
 *                               context token (untouched for empty sequences)
 * The chain templates (at most two row counts per call: chunk_rows and the ragged last
 * chunk) belong to the model handle: bita_prefill_prepare creates them (a device allocation
 * and a blocking copy each, once per row count; freed by bita_model_destroy).  bita_prefill
 * itself then only enqueues on `stream`: no allocation, no host synchronisation, so it may
 * be captured into a HIP graph like the step calls.  Outside capture bita_prefill creates a
 * missing template itself; on a capturing stream a missing template is INVALID_ARG.
 * Errors: CAPACITY if ctx_hint + n_tokens exceeds smax or max_pos or the
 * workspace is too small (checked before anything is enqueued). */
size_t bita_prefill_workspace_bytes(const bita_model *m, int32_t batch, int32_t chunk_rows);
int bita_prefill_prepare(bita_model *m, int32_t n_tokens, int32_t chunk_rows);
int bita_prefill(bita_model *m, const bita_kv *kv, const int32_t *d_tokens, int32_t n_tokens,
                 const int32_t *d_seq_len, int32_t *d_ctx_len, int32_t batch, int32_t chunk_rows,
                 void *d_workspace, size_t ws_bytes, int32_t *d_next_token, void *stream);

/* Tree-masked attention alone (the kernel bita_verify_step runs per layer), for
 * kernel-level tests and measurement.  d_q [B][R][n_heads][hd] (already rotated; d_q_lo
 * is an optional second bf16 plane of the same shape with the rounding residual),
 * K/V arguments are one layer's slices laid out as in bita_kv; d_k_tree_lo / d_v_tree_lo
 * are optional second planes of d_k_tree / d_v_tree (the pass rows' K/V before they are
 * rounded to the cache format: value = hi + lo; NULL = zero); d_out
 * [B][R][n_heads*hd] bf16; d_out_lo (optional, same shape) receives the rounding residual
 * of d_out, so that d_out + d_out_lo carries the kernel's fp32 result to about 16 bits, which
 * is the form bita_verify_step hands to the output projection.  d_ws needs
 * bita_attention_workspace_bytes(). */
size_t bita_attention_workspace_bytes(int32_t batch, int32_t rows, int32_t n_heads,
                                      int32_t head_dim, int32_t ctx_hint, int32_t n_prompt);
int bita_tree_attention(const bita_tree_template *t, const void *d_q, const void *d_q_lo,
                        const void *d_k_cache, const void *d_v_cache,
                        const void *d_k_tree, const void *d_v_tree,
                        const void *d_k_tree_lo, const void *d_v_tree_lo,
                        const void *d_prompt_k, const void *d_prompt_v,
                        const int32_t *d_ctx_len, int32_t batch, int32_t n_heads,
                        int32_t n_kv_heads, int32_t head_dim, int32_t n_prompt, int32_t smax,
                        int32_t ctx_hint, void *d_ws, size_t ws_bytes, void *d_out, void *d_out_lo,
                        void *stream);

/* Selection alone (the last kernel of bita_verify_step; Sec. 3.2: the greedy token of every
 * draft row and the top-kmax candidates of every mask row), for kernel-level tests.
 * d_logits [B][R][vocab] fp32 (device, finite values; -0 counts as +0).  d_argmax [B][T]:
 * index of the largest logit of each of the T tree rows, the lowest index among equal
 * values.  d_topk_ids / d_topk_val [B][G*n][kmax] (device, both optional): the kmax
 * largest logits of every mask row in the same order (value descending, lower index first
 * among equals).  vocab must be a multiple of 16.  Returns BITA_OK or an error code. */
int bita_select(const bita_tree_template *t, const float *d_logits, int32_t batch, int32_t vocab,
                int32_t kmax, int32_t *d_argmax, int32_t *d_topk_ids, float *d_topk_val, void *stream);

/* Skinny GEMM alone: d_out[M][N] (fp32) = A[M][K] times the packed [N][K] matrix
 * transposed.  A = d_a (bf16, row stride lda) plus, if d_a_lo is not NULL, a second bf16
 * plane of the same shape holding the rounding residual (A = hi + lo), which is how
 * bita_verify_step feeds its activations.  d_ws needs bita_gemm_workspace_bytes(). */
size_t bita_gemm_workspace_bytes(int32_t m_rows, int64_t n_rows, int64_t k);
int bita_gemm(const void *d_a, const void *d_a_lo, int32_t m_rows, int64_t k, int64_t lda,
              const void *d_w_packed, int64_t n_rows, void *d_ws, size_t ws_bytes, float *d_out,
              void *stream);

/* bita_gemm for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and
 * result (bit for bit) as bita_gemm, minus the workspace: the split-K partial sums and the
 * re-laid activations live in a static device array of bita_gemm_noalloc_max_scratch_bytes()
 * = 32 MiB that every GPU the library runs on holds until the process ends.  The call
 * allocates nothing (no hipMalloc / hipFree, no allocating library routine), only enqueues on
 * `stream`, and returns BITA_ERR_CAPACITY, with the sizes in bita_last_error(), when the shape
 * needs more than that (bita_gemm_noalloc_scratch_bytes(m_rows, n_rows, k) says how much a
 * shape needs).  d_a, d_a_lo, d_w_packed, d_out are device pointers owned by the caller.
 * All calls on one GPU share that GPU's array, which keeps the last call's contents (nothing in
 * it needs to start at zero): calls that overlap in time on one GPU, on different streams or
 * from different threads, race and must be ordered by the caller. */
size_t bita_gemm_noalloc_max_scratch_bytes(void);
size_t bita_gemm_noalloc_scratch_bytes(int32_t m_rows, int64_t n_rows, int64_t k);
int bita_gemm_noalloc(const void *d_a, const void *d_a_lo, int32_t m_rows, int64_t k, int64_t lda,
                      const void *d_w_packed, int64_t n_rows, float *d_out, void *stream);

/* Measurement aid: while enabled, bita_verify_step brackets each of its GEMM launches with
 * a pair of HIP events on the caller's stream (not usable under graph capture).
 * bita_profile_enable creates the events (up to max_records launches are recorded from the
 * next step on); bita_profile_read waits for them and returns, per recorded launch, the
 * elapsed milliseconds and the bytes of the weight matrix it streamed (HOST arrays of
 * `capacity` entries). */
int  bita_profile_enable(int32_t max_records);
void bita_profile_disable(void);
int  bita_profile_read(int32_t capacity, int32_t *n_records, float *ms, int64_t *weight_bytes);

/* Tuning aid: override the GEMM launch heuristic for all later launches of this process
 * (variant = workgroup shape index, splits = split-K factor; a negative value restores the
 * heuristic for that knob; variant -2 = the heuristic without tall row passes).  Results are
 * unchanged, only speed.
 * Threads: the step calls, bita_prefill and the kernel-level calls may run from several host
 * threads at once on different model handles and streams (error text is per thread).  The two
 * aids, bita_tune_gemm and bita_profile_*, keep process-wide state and must not be called
 * while another thread is inside the library. */
void bita_tune_gemm(int32_t variant, int32_t splits);
/* What the launch heuristic chooses for an [m_rows] x [n_rows] x [k] GEMM (for tests and
 * reports): out4 (HOST) = {k splits, workgroup shape index, m-tiles per row pass of a tall
 * launch (0 = the shape's own row handling: one pass, or passes of 5 m-tiles), k-steps per split}. */
int bita_gemm_plan_info(int32_t m_rows, int64_t n_rows, int64_t k, int32_t *out4);

const char *bita_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BITA_H */
