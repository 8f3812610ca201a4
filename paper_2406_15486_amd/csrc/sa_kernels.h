// Host-visible declarations of the kernel launchers (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sa {

constexpr int kHeadDim = 128;  // the only supported head dimension
constexpr int kFlashBQ = 256;  // query rows per workgroup of the flash kernels
constexpr int kFlashBK = 64;   // keys per tile

struct FlashParams {
  const uint16_t* q;        // [n_bh, S, 128] bf16
  const uint16_t* k;        // [n_bkv, S, 128] bf16
  const uint16_t* vt;       // [n_bkv, 128, S_pad] bf16 (V transposed, zero padded)
  void* out;                // [n_bh, S, 128] bf16 or fp32
  float* lse;               // nullable
  int S, S_pad;
  int n_bh, n_bkv, group;   // batch*q-heads, batch*kv-heads, q heads per kv head
  int head0;                // strip-masked mode: q, out, lse, tiles and the per-head metadata start at this
                            // (batch*q-)head, n_bh counts the heads of this pass; KV head = (head0 + h) / group
  float scale_log2;         // softmax scale * log2(e)
  int n_qtiles;             // 256-row query tiles to process
  int qtile0;               // strip-masked mode: the first of them (a segment of the queries)
  int q_row0, n_qrows;      // first query row and number of rows (sampled rows in mode 1)
  int cols_in_place;        // strip-masked mode, block lists: column tiles are read from k / vt themselves
                            // (kc, vct unused); col_idx_pad then holds runs of 64 consecutive keys per tile
  int row_lo;               // strip-masked mode: rows below it are neither computed for nor written
                            // (rows [row_lo, n_qrows) of the launch's query tiles are; q_row0 = 0 there)
  int k_splits;             // mode 1: the keys of a query tile are cut into this many workgroups (>= 1);
                            // lse is then [k_splits, n_bh, n_qrows] partial values (launch_lse_combine)
  // strip-masked mode only
  const uint16_t* kc;           // [n_bh, S_pad, 128] K rows gathered by column index
  const uint16_t* vct;          // [n_bh, 128, S_pad] V rows gathered and transposed
  const int32_t* col_idx_pad;   // [n_bh, cidx_stride] ascending, padded with INT_MAX
  const int32_t* col_cnt;       // [n_bh]
  const uint32_t* col_bits;     // [n_bh, cb_words]  bit j: key j is a selected column
  const uint32_t* off_bits;     // [n_bh, rb_words]  bit x: offset off_max - x is kept
  const int32_t* dlist;         // [n_bh, dlist_stride] ascending touched tile-diagonals
  const int32_t* dcnt;          // [n_bh]
  unsigned long long* tiles;    // nullable [n_bh]
  int cidx_stride, cb_words, rb_words, dlist_stride, off_max;
};

// mode 0: dense causal; 1: row log-sum-exp of rows [q_row0, q_row0+n_qrows); 2: strip mask
hipError_t launch_flash(int mode, bool out_f32, const FlashParams& P, hipStream_t st);
int lse_key_splits(int row_first, int n_s, int n_bh);
hipError_t launch_lse_combine(const float* part, float* out, size_t n, int k, hipStream_t st);

// out[g][d][c] = src[kv(g)][idx ? idx[g][c] : c][d] for c < cnt (zero beyond, up to C_pad);
// optionally also rows_out[g][c][:] = src[kv(g)][idx[g][c]][:]
struct GatherParams {
  const uint16_t* src;      // [n_src, S, 128]; may be null when only idx_pad is wanted
  const int32_t* idx;       // nullable [n_out, idx_stride]
  const int32_t* cnt;       // nullable [n_out]; null -> S
  uint16_t* out_t;          // [n_out, 128, C_pad]
  uint16_t* out_rows;       // nullable [n_out, C_pad, 128]
  int32_t* idx_pad;         // nullable [n_out, idx_pad_stride]: copy of idx padded with INT_MAX
  int n_out, group;         // source head of output g is (head0 + g) / group
  int head0;
  int S, C_pad, idx_stride, idx_pad_stride;
  int key_limit;            // > 0: the list ascends and no reader looks at a key >= key_limit; tiles of 64 list entries
                            // that start there are not gathered (their idx_pad entries still are written)
};
hipError_t launch_gather_transpose(const GatherParams& P, hipStream_t st);

struct MaskPrepParams {
  const int32_t* col_idx; const int32_t* col_cnt;      // [n_bh, S], [n_bh]
  const int32_t* slash_idx; const int32_t* slash_cnt;
  uint32_t* col_bits; uint32_t* off_bits;              // zero-filled by the launcher
  int32_t* dlist; int32_t* dcnt;
  int n_bh, S, window, cb_words, rb_words, dlist_stride, off_max;
};
hipError_t launch_mask_prep(const MaskPrepParams& P, hipStream_t st);
hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t st);

// block granularity: lists of selected key blocks / offset blocks of blk tokens
struct BlockPrepParams {
  const int32_t* col_blk; const int32_t* col_bcnt;     // [n_bh, nb], [n_bh]
  const int32_t* slash_blk; const int32_t* slash_bcnt;
  int32_t* tok_idx; int32_t* tok_cnt;                  // [n_bh, S], [n_bh]: the key blocks as token columns
  uint32_t* diag_bits;                                 // [n_bh, db_words]: kept block diagonals
  uint32_t* col_bits; uint32_t* off_bits;
  int32_t* dlist; int32_t* dcnt;
  int n_bh, S, window, cb_words, rb_words, dlist_stride, off_max;
  int blk, nb, db_words;
};
hipError_t launch_block_prep(const BlockPrepParams& P, hipStream_t st);
// out[r][b] = sum of in[r][b*blk .. (b+1)*blk), r < n_rows, rows of S floats
hipError_t launch_block_reduce(const float* in, float* out, int n_rows, int S, int blk, hipStream_t st);

struct ScoreParams {
  const uint16_t* q; const uint16_t* k;
  const float* lse;         // [n_bh, n_s] natural log
  float* col;               // [n_bh, S]
  float* slash;             // [n_bh, S]
  float* partial;           // workspace for slash partial sums
  int S, n_s, n_bh, n_bkv, group;
  int row_first;            // the sampled rows are [row_first, row_first + n_s)
  float scale_log2;
  int n_kblocks, n_chunks, chunk_rows, win;   // win = floats per (key block, chunk) partial
};
hipError_t launch_score_accumulate(const ScoreParams& P, hipStream_t st);
hipError_t launch_score_finalize(const ScoreParams& P, hipStream_t st);
size_t score_partial_floats(int S, int n_s, int n_bh);
void score_geometry(int S, int n_s, int* n_kblocks, int* n_chunks, int* chunk_rows, int* win);

// measurement aids: back-to-back MFMA loop and plain copy
hipError_t launch_probe_mfma(int iters, int waves_per_simd, float* sink, hipStream_t st);
hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t st);

struct SelectParams {
  const float* scores;      // [n_prob, S]
  int32_t* idx;             // [n_prob, S]
  int32_t* cnt;             // [n_prob]
  int n_prob, S;
  float alpha;
  // optional second set of n_prob problems of the same size, solved by the same launch
  const float* scores2; int32_t* idx2; int32_t* cnt2; float alpha2;
};
hipError_t launch_select(const SelectParams& P, hipStream_t st);

}  // namespace sa
