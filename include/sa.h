/*
 * sa.h - C ABI of the SampleAttention prefill hot path for AMD MI355X (gfx950).
 *
 * The library computes causal prefill attention under an adaptive structured
 * sparse mask (SampleAttention, arXiv 2406.15486, Algorithm 1):
 *
 *   stage 1  sa_sample_scores   exact causal softmax rows of a sampled subset
 *                               of queries, accumulated into per-key column
 *                               scores and per-offset slash scores
 *   stage 2  sa_select_strips   fewest column / slash strips whose score mass
 *                               reaches the CRA thresholds alpha_c / alpha_s
 *   attend   sa_sparse_attn     flash-style attention over the merged mask
 *   baseline sa_dense_attn      dense causal flash-style attention (Eq. 1-2)
 *
 * The same path at block granularity (Algorithm 1 "block_reduction", blk = 128
 * in the paper): sa_sample_scores with granularity > 1 (or sa_block_scores on
 * per-token scores), sa_select_blocks, sa_block_sparse_attn.  With chunk_n > 1
 * ("Query-Guided Chunked Sampling", Sec. 4.2): sa_sample_scores with n_chunks > 1,
 * sa_select_chunked, sa_sparse_attn_chunked.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 * - Every tensor pointer is a DEVICE pointer owned by the caller.  The library
 *   never allocates, frees or keeps them; scratch memory comes only from the
 *   caller's workspace (size from sa_workspace_bytes, 256-byte aligned).
 * - Tensors are row-major and contiguous: Q and O are [batch, n_q_heads,
 *   seq_len, head_dim]; K and V are [batch, n_kv_heads, seq_len, head_dim];
 *   query head h reads KV head h / (n_q_heads / n_kv_heads) (grouped-query
 *   attention, Sec. 5.1).  Q, K, V are bf16.  Per-head vectors (scores, index
 *   lists, lse) are [batch * n_q_heads, seq_len] (or [.., n_sample_rows]).
 * - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   Calls only enqueue work and return without synchronising; counts and
 *   index lists stay on the device, so the stages chain without a host sync.
 * - Errors are return codes.  All argument checks (null pointers, shapes,
 *   ranges, workspace size) run on the host before anything is launched, so
 *   they work on a machine without a GPU.  SA_ERR_DEVICE reports a failed
 *   launch (hipGetLastError).
 * - Two calls that share a workspace must not overlap in time.
 */
#ifndef SA_H
#define SA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SA_OK = 0,
  SA_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, value out of range */
  SA_ERR_UNSUPPORTED = 2, /* a valid request this build does not implement       */
  SA_ERR_WORKSPACE = 3,   /* workspace missing, misaligned or too small          */
  SA_ERR_DEVICE = 4,      /* the HIP runtime reported an error on launch         */
  SA_ERR_TOO_LARGE = 5    /* sa_dense_attn_static: needs more than its static
                             scratch holds                                       */
} sa_status;

/* Problem shape.  head_dim must be 128 and causal must be 1 (the method is
 * defined for decoder-only prefill); n_q_heads % n_kv_heads == 0;
 * seq_len <= 2^24 and batch * n_q_heads <= 65535 (else SA_ERR_UNSUPPORTED). */
typedef struct {
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t seq_len;
  int32_t head_dim;
  int32_t causal;
  float softmax_scale; /* 0 -> 1/sqrt(head_dim) (Eq. 1) */
} sa_shape;

/* Stage-1 sampling.  n_sample_rows: the last n rows of the sequence are the
 * sampled queries (Algorithm 1 with chunk_n = 1), 1 <= n <= seq_len.
 * n_chunks and granularity are the paper's chunk_n and blk.  With n_chunks =
 * C > 1 the queries are cut into C segments of itv = floor(seq_len / C) rows
 * (the last segment takes the remainder) and the last n rows of EACH segment
 * are sampled (n <= itv, C <= seq_len).  granularity 1 keeps scores per key /
 * per offset; 64, 128 or 256 sums them over blocks of that many keys /
 * offsets (multiples of the kernels' 64-key tile that divide their 256-row
 * query tile; the paper uses 128); other values return SA_ERR_UNSUPPORTED. */
typedef struct {
  int32_t n_sample_rows;
  int32_t n_chunks;
  int32_t granularity;
} sa_sampling;

typedef enum { SA_OUT_BF16 = 0, SA_OUT_F32 = 1 } sa_out_dtype;

typedef enum {
  SA_OP_SAMPLE_SCORES = 0,
  SA_OP_SELECT_STRIPS = 1,
  SA_OP_SPARSE_ATTN = 2,
  SA_OP_DENSE_ATTN = 3,
  SA_OP_BLOCK_SPARSE_ATTN = 4,
  SA_OP_SAMPLE_SCORES_MIN = 5 /* the least sa_sample_scores works with */
} sa_op;

/* Bytes of device workspace `op` needs for this shape (sampling may be NULL
 * for ops that neither sample nor work on blocks; SA_OP_BLOCK_SPARSE_ATTN
 * reads sampling->granularity only).  Returns 0 for invalid arguments.
 * Host only. */
size_t sa_workspace_bytes(int op, const sa_shape* shape, const sa_sampling* sampling);

/* 64 * ceil(ratio * seq_len / 64), clamped to [min(64, seq_len), seq_len]:
 * the sampled-row count for a sample ratio.  Host only. */
int32_t sa_rows_from_ratio(int32_t seq_len, float ratio);

/*
 * Stage 1 (Algorithm 1 "Query-Guided Chunked Attention Sampling", Sec. 4.2).
 * For every query head and every sampled row i in R = [S - n, S):
 *   p_ij = softmax_j(q_i . k_j * scale), j <= i            (exact, causal)
 *   col_scores[h, j]   = sum_{i in R, i >= j} p_ij
 *   slash_scores[h, o] = sum_{i in R, i >= o} p_{i, i-o}    (offset o = i - j)
 * in:  q, k (bf16, layouts above)
 * out: col_scores, slash_scores  fp32 [batch*n_q_heads, seq_len]
 *      row_lse (nullable)        fp32 [batch*n_q_heads, n] natural-log
 *                                sum-exp of each sampled row
 * With sampling->granularity = blk > 1 the outputs are the block scores of
 * Algorithm 1's block_reduction instead, fp32 [batch*n_q_heads, n_blocks] with
 * n_blocks = ceil(seq_len / blk):
 *   col_scores[h, J]   = sum of the per-key scores of keys   [blk*J, blk*J + blk)
 *   slash_scores[h, b] = sum of the per-offset scores of offsets [blk*b, blk*b + blk)
 * With sampling->n_chunks = C > 1 the outputs carry a leading chunk dimension,
 * [C, batch*n_q_heads, n]: chunk m holds the scores of the last n_sample_rows
 * rows of segment m (rows [(m+1)*itv - n_sample_rows, (m+1)*itv); the last
 * segment ends at seq_len), exactly as above (causal: those rows see keys up to
 * their own position); row_lse must then be NULL.
 * The sums are formed in a fixed order: repeated calls give identical bits.
 * Workspace: with sa_workspace_bytes(SA_OP_SAMPLE_SCORES, ..) all heads are
 * processed at once.  Any smaller size down to SA_OP_SAMPLE_SCORES_MIN is
 * accepted as well: the heads are then taken as many at a time as fit (whole
 * KV heads, or an equal part of one KV head's query heads), pass after pass,
 * with the same result - which bounds the workspace for long sequences (it
 * grows with seq_len * n_sample_rows per head, Sec. 5.4).
 */
sa_status sa_sample_scores(const sa_shape* shape, const sa_sampling* sampling,
                           const void* q, const void* k,
                           float* col_scores, float* slash_scores, float* row_lse,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Stage 2 (Algorithm 1 "Score-Based Key-Value Block Filtering", Sec. 4.3).
 * Independently per head and per direction: order candidates by (score
 * descending, index ascending), take the smallest k >= 0 whose first-k score
 * sum (fp64) reaches alpha * total; alpha == 1 keeps all seq_len candidates,
 * alpha == 0 keeps none.  Scores are expected finite and >= 0; a negative,
 * infinite or NaN score counts as 0 (it carries no mass and is kept last).
 * in:  col_scores, slash_scores  fp32 [batch*n_q_heads, seq_len]
 *      alpha_c, alpha_s          CRA thresholds in [0, 1] (SA_ERR_INVALID_ARG
 *                                otherwise, NaN included)
 * out: col_idx, slash_idx  int32 [batch*n_q_heads, seq_len]; the first cnt[h]
 *                          entries of row h are the kept indices in ASCENDING
 *                          order, the rest is unspecified
 *      col_cnt, slash_cnt  int32 [batch*n_q_heads]
 */
sa_status sa_select_strips(const sa_shape* shape,
                           const float* col_scores, const float* slash_scores,
                           float alpha_c, float alpha_s,
                           int32_t* col_idx, int32_t* col_cnt,
                           int32_t* slash_idx, int32_t* slash_cnt,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Block granularity (Algorithm 1 block_reduction, Sec. 4.2-4.3; granularity is
 * the paper's blk and must be 64, 128 or 256, n_blocks = ceil(seq_len / blk)).
 *
 * sa_block_scores: per-token scores [batch*n_q_heads, seq_len] -> block scores
 * [batch*n_q_heads, n_blocks] as defined at sa_sample_scores (what that call
 * does itself when sampling->granularity > 1).  No workspace.
 *
 * sa_select_blocks: sa_select_strips over the n_blocks candidates of each
 * direction; index lists are int32 [batch*n_q_heads, n_blocks], ascending.
 *
 * sa_block_sparse_attn: attention under the block mask (Fig. 6: the selected
 * blocks extended over the matrix and merged).  With block(x) = x / blk,
 *   M[i, j] = (j <= i) and (block(j) in I_c[h]  or  block(i) - block(j) in D[h])
 * where D holds the block diagonals on which a full blk x blk block contains
 * a kept offset: b and b + 1 for every selected offset block b in I_s[h] (its
 * offsets [blk*b, blk*b + blk) spread over both), and every delta with
 * blk*delta - (blk - 1) <= local_window - 1 (delta = 0 always: local_window
 * >= 1).  Kept blocks are computed whole; only the causal edge is masked.
 * Lists: ascending, duplicate-free block indices in [0, n_blocks), counts in
 * [0, n_blocks].  Outputs as for sa_sparse_attn.  Workspace:
 * sa_workspace_bytes(SA_OP_BLOCK_SPARSE_ATTN, shape, sampling).
 */
sa_status sa_block_scores(const sa_shape* shape, int32_t granularity,
                          const float* col_scores, const float* slash_scores,
                          float* col_block_scores, float* slash_block_scores, void* stream);

sa_status sa_select_blocks(const sa_shape* shape, int32_t granularity,
                           const float* col_block_scores, const float* slash_block_scores,
                           float alpha_c, float alpha_s,
                           int32_t* col_blocks, int32_t* col_cnt,
                           int32_t* slash_blocks, int32_t* slash_cnt,
                           void* workspace, size_t workspace_bytes, void* stream);

sa_status sa_block_sparse_attn(const sa_shape* shape, int32_t granularity,
                               const void* q, const void* k, const void* v,
                               const int32_t* col_blocks, const int32_t* col_cnt,
                               const int32_t* slash_blocks, const int32_t* slash_cnt,
                               int32_t local_window,
                               void* out, int out_dtype, float* out_lse, uint64_t* tiles,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * chunk_n > 1 (Algorithm 1: itv, Q_slice, merge_index(I_c, I_s, itv); Sec. 4.2-4.3).
 * sampling gives n_chunks = C and granularity (n_sample_rows is not read); all
 * score, index and count arrays carry a leading chunk dimension:
 * [C, batch*n_q_heads, n] and [C, batch*n_q_heads], n = seq_len candidates at
 * granularity 1, ceil(seq_len / blk) at block granularity.
 *
 * sa_select_chunked: the selection of sa_select_strips / sa_select_blocks for
 * every (chunk, head, direction) independently.
 *
 * sa_sparse_attn_chunked: what is selected from chunk m masks the query rows of
 * segment m, [m*itv, (m+1)*itv) with itv = floor(seq_len / C), the last segment
 * running to seq_len: for those rows the mask is that of
 * sa_sparse_attn (granularity 1) or sa_block_sparse_attn with chunk m's lists.
 * Workspace: that of SA_OP_SPARSE_ATTN or SA_OP_BLOCK_SPARSE_ATTN.  `tiles`
 * counts over all segments.
 */
sa_status sa_select_chunked(const sa_shape* shape, const sa_sampling* sampling,
                            const float* col_scores, const float* slash_scores,
                            float alpha_c, float alpha_s,
                            int32_t* col_idx, int32_t* col_cnt,
                            int32_t* slash_idx, int32_t* slash_cnt,
                            void* workspace, size_t workspace_bytes, void* stream);

sa_status sa_sparse_attn_chunked(const sa_shape* shape, const sa_sampling* sampling,
                                 const void* q, const void* k, const void* v,
                                 const int32_t* col_idx, const int32_t* col_cnt,
                                 const int32_t* slash_idx, const int32_t* slash_cnt,
                                 int32_t local_window,
                                 void* out, int out_dtype, float* out_lse, uint64_t* tiles,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Merge + attend (Algorithm 1 merge_index and sparse_flash_attn; Eq. 3 with
 * masked entries contributing exactly zero).  The mask of head h is
 *   M[i, j] = (j <= i) and (j in I_c[h]  or  (i-j) in I_s[h]  or  i-j < local_window)
 * and O_i = softmax over {j : M[i,j]} of (q_i . k_j * scale) times V.
 * in:  q, k, v; col_idx/col_cnt, slash_idx/slash_cnt as written by
 *      sa_select_strips - or any other ascending, duplicate-free lists with
 *      entries in [0, seq_len) and counts in [0, seq_len];
 *      local_window >= 1 (every row keeps at least its own key)
 * out: out      [batch, n_q_heads, seq_len, head_dim], bf16 or fp32
 *      out_lse  (nullable) fp32 [batch*n_q_heads, seq_len], natural log of
 *               the masked sum-exp
 *      tiles    (nullable) uint64 [batch*n_q_heads]: number of 32x64
 *               (query rows x keys) score tiles the kernel computed for the
 *               head (one wave's unit of work: 4*head_dim*32*64 flop each)
 */
sa_status sa_sparse_attn(const sa_shape* shape, const void* q, const void* k, const void* v,
                         const int32_t* col_idx, const int32_t* col_cnt,
                         const int32_t* slash_idx, const int32_t* slash_cnt,
                         int32_t local_window,
                         void* out, int out_dtype, float* out_lse, uint64_t* tiles,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * sa_sparse_attn with bounded workspace, for long sequences (Sec. 5.4: above
 * 256K tokens the paper splits the sequence into chunks and partitions the
 * attention by head "to avoid memory issues").  The heads are processed
 * heads_per_pass at a time - the workspace then holds the metadata and the
 * gathered K / V of one pass only, about
 *   batch * n_kv_heads * S_pad * 256  +  heads_per_pass * S_pad * 520  bytes
 * (S_pad = seq_len rounded up to 256) instead of the second term times all
 * batch * n_q_heads heads - and the query rows of a pass in n_query_segments
 * consecutive launches of (nearly) equal numbers of 256-row query tiles.
 * Values larger than the number of heads / query tiles are clamped; both must
 * be >= 1.  The result (out, out_lse, tiles) is bit-identical to
 * sa_sparse_attn's: every (head, query tile) is computed by one workgroup in
 * the same order of operations whatever the partition.
 * Workspace: sa_partitioned_workspace_bytes(shape, partition) (0 for invalid
 * arguments; host only).
 */
typedef struct {
  int32_t heads_per_pass;
  int32_t n_query_segments;
} sa_partition;

size_t sa_partitioned_workspace_bytes(const sa_shape* shape, const sa_partition* partition);

sa_status sa_sparse_attn_partitioned(const sa_shape* shape, const sa_partition* partition,
                                     const void* q, const void* k, const void* v,
                                     const int32_t* col_idx, const int32_t* col_cnt,
                                     const int32_t* slash_idx, const int32_t* slash_cnt,
                                     int32_t local_window,
                                     void* out, int out_dtype, float* out_lse, uint64_t* tiles,
                                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * Dense causal attention (Eq. 1-2 with keys j <= i), the in-library baseline
 * the sparse path is compared against.  Same layouts and outputs as above.
 */
sa_status sa_dense_attn(const sa_shape* shape, const void* q, const void* k, const void* v,
                        void* out, int out_dtype, float* out_lse,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * sa_dense_attn for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and kernels as sa_dense_attn, but
 * the transposed copy of V lives in a device array that is part of the library
 * (SA_STATIC_SCRATCH_BYTES per GPU, held until the process ends) instead of a
 * caller workspace, and the call allocates nothing.
 * Limit: batch * n_kv_heads * head_dim * roundup(seq_len, 256) * 2 bytes must
 * fit the array, i.e. batch * n_kv_heads * roundup(seq_len, 256) <= 65536 -
 * otherwise SA_ERR_TOO_LARGE, before anything is launched.
 * All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams or threads) race.  The array keeps the last
 * call's contents; every call rewrites the part it reads.  The first call on
 * a device looks up the array's address (hipGetSymbolAddress, with the
 * caller's current device): make it outside any graph capture.
 */
#define SA_STATIC_SCRATCH_BYTES (16u << 20)
sa_status sa_dense_attn_static(const sa_shape* shape, const void* q, const void* k, const void* v,
                               void* out, int out_dtype, float* out_lse, void* stream);

/*
 * Measurement aid (no part of the method).  While enabled, the library
 * records a HIP event pair on the caller's stream around each of its kernels
 * (or kernel groups), into a ring of SA_PROFILE_SLOTS slots per kernel id.
 * sa_profile_read waits for the recorded events and copies the durations, in
 * milliseconds and oldest first, of up to `cap` launches recorded since the
 * last sa_profile_enable(1) into `ms` (a HOST array); it returns the number
 * written, or -1 for a bad argument.  Event records do not synchronise.
 * Not thread-safe.
 */
typedef enum {
  SA_K_ROW_LSE = 0,        /* stage 1 pass 1: flash sweep giving row log-sum-exp
                              (and the combination of its key splits)              */
  SA_K_SCORE_ACCUM = 1,    /* stage 1 pass 2: column / slash accumulation          */
  SA_K_SCORE_FINAL = 2,    /* stage 1: fixed-order sum of the partials, block
                              reduction                                            */
  SA_K_SELECT = 3,         /* stage 2: the selection launch (both directions)      */
  SA_K_MASK_PREP = 4,      /* merge: bitmaps, tile-diagonal list, K/V gathers (once
                              per pass over a group of heads)                      */
  SA_K_SPARSE_FLASH = 5,   /* strip-masked flash attention kernel                  */
  SA_K_DENSE_FLASH = 6,    /* dense flash attention kernel                         */
  SA_K_TRANSPOSE_V = 7,    /* V -> V^T (dense and strip-masked paths)              */
  SA_K_COUNT = 8
} sa_kernel_id;
#define SA_PROFILE_SLOTS 64
sa_status sa_profile_enable(int enable);
int sa_profile_read(int kernel, float* ms, int cap);

/*
 * Measurement aids (no part of the method): what this GPU reaches on the two
 * resources the kernels are priced against.  Both only enqueue; time them with
 * events on `stream`.
 * sa_probe_mfma: waves_per_simd (1..8) waves on each of the 1024 SIMDs issue
 *   iters * 16 back-to-back 32x32x16 bf16 MFMAs (32768 flop each) from
 *   registers: 1024 * waves_per_simd * iters * 16 * 32768 flop in all.  sink: a
 *   device float, never written in practice.
 * sa_probe_copy: a plain copy of bytes (a multiple of 16) from src to dst
 *   (device pointers, 16-byte aligned): bytes read plus bytes written.
 */
sa_status sa_probe_mfma(int32_t iters, int32_t waves_per_simd, float* sink, void* stream);
sa_status sa_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

const char* sa_status_string(int status);
int sa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SA_H */
