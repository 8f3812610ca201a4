// C ABI of the library: host-side argument validation, workspace carving and
// kernel launches.  Every check runs before the first launch, so error paths
// need no GPU.  Declarations and contracts: include/sa.h.
#include <math.h>
#include <string.h>

#include <mutex>

#include "../../include/sa.h"
#include "sa_kernels.h"

// Static device scratch of the entry point that allocates nothing (sa_dense_attn_static):
// one copy per GPU that loads the library, held until the process ends.
static __device__ __align__(256) unsigned char scratch[SA_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Dims {
  int S, S_pad, n_bh, n_bkv, group;
  float scale;
};

sa_status check_shape(const sa_shape* s, Dims* d) {
  if (s == nullptr) return SA_ERR_INVALID_ARG;
  if (s->batch < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->seq_len < 1) return SA_ERR_INVALID_ARG;
  if (s->n_q_heads % s->n_kv_heads != 0) return SA_ERR_INVALID_ARG;
  if (!(s->softmax_scale >= 0.0f) || !isfinite(s->softmax_scale)) return SA_ERR_INVALID_ARG;
  if (s->head_dim != sa::kHeadDim) return SA_ERR_UNSUPPORTED;
  if (s->causal != 1) return SA_ERR_UNSUPPORTED;
  if ((long long)s->batch * s->n_q_heads > 65535) return SA_ERR_UNSUPPORTED;
  if (s->seq_len > (1 << 24)) return SA_ERR_UNSUPPORTED;   // kernels keep 32-bit byte offsets into V^T
  d->S = s->seq_len;
  d->S_pad = (s->seq_len + sa::kFlashBQ - 1) / sa::kFlashBQ * sa::kFlashBQ;
  d->n_bh = s->batch * s->n_q_heads;
  d->n_bkv = s->batch * s->n_kv_heads;
  d->group = s->n_q_heads / s->n_kv_heads;
  d->scale = (s->softmax_scale == 0.0f) ? 1.0f / sqrtf((float)s->head_dim) : s->softmax_scale;
  return SA_OK;
}

// block sizes the block path is built for: multiples of the 64-key tile that divide
// the 256-row query tile (the paper fixes blk = 128)
sa_status check_granularity(int g) {
  if (g < 1) return SA_ERR_INVALID_ARG;
  return (g == 64 || g == 128 || g == 256) ? SA_OK : SA_ERR_UNSUPPORTED;
}

sa_status check_sampling(const sa_sampling* sm, const Dims& d) {
  if (sm == nullptr) return SA_ERR_INVALID_ARG;
  if (sm->n_sample_rows < 1 || sm->n_sample_rows > d.S) return SA_ERR_INVALID_ARG;
  if (sm->n_chunks < 1 || sm->granularity < 1) return SA_ERR_INVALID_ARG;
  if (sm->granularity != 1 && check_granularity(sm->granularity) != SA_OK) return SA_ERR_UNSUPPORTED;
  if (sm->n_chunks > d.S) return SA_ERR_INVALID_ARG;
  // segments of itv = floor(S / chunk_n) rows (the last one runs to S): the sampled rows must fit
  if (sm->n_sample_rows > d.S / sm->n_chunks) return SA_ERR_INVALID_ARG;
  return SA_OK;
}

sa_status check_ws(const void* ws, size_t have, size_t need) {
  if (need == 0) return SA_OK;
  if (ws == nullptr || have < need) return SA_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) % kAlign != 0) return SA_ERR_WORKSPACE;
  return SA_OK;
}

// chunk_n and blk of the calls that take no sampled-row count
sa_status check_chunks(const Dims& d, int n_chunks, int granularity) {
  if (n_chunks < 1 || granularity < 1) return SA_ERR_INVALID_ARG;
  if (granularity != 1 && check_granularity(granularity) != SA_OK) return SA_ERR_UNSUPPORTED;
  if (n_chunks > d.S) return SA_ERR_INVALID_ARG;
  return SA_OK;
}

// ---- workspace layouts --------------------------------------------------------
constexpr int kMaxKeySplits = 8;
struct SampleWs { size_t lse, lse_part, partial, tok_col, tok_slash, total; };
SampleWs sample_ws(const Dims& d, int n_s, int granularity) {
  SampleWs w;
  size_t at = 0;
  w.lse = at;      at += align_up((size_t)d.n_bh * n_s * sizeof(float));
  w.lse_part = at; at += align_up((size_t)kMaxKeySplits * d.n_bh * n_s * sizeof(float));
  w.partial = at; at += align_up(sa::score_partial_floats(d.S, n_s, d.n_bh) * sizeof(float));
  w.tok_col = w.tok_slash = at;
  if (granularity > 1) {   // per-token scores, reduced to blocks afterwards
    w.tok_col = at;   at += align_up((size_t)d.n_bh * d.S * sizeof(float));
    w.tok_slash = at; at += align_up((size_t)d.n_bh * d.S * sizeof(float));
  }
  w.total = at;
  return w;
}

// The heads [h0, h0 + nh) as a problem of their own: nh is a multiple of the heads per KV
// head (whole KV heads) or divides it (part of one KV head), so that head h of the pass
// still reads KV head h / group of the pass once the K pointer is moved to the pass's first.
Dims pass_dims(const Dims& d, int nh) {
  Dims p = d;
  p.n_bh = nh;
  p.n_bkv = nh >= d.group ? nh / d.group : 1;
  p.group = nh >= d.group ? d.group : nh;
  return p;
}

// how many heads one pass of sa_sample_scores may take with `have` bytes of workspace
int sample_heads_per_pass(const Dims& d, int n_s, int blk, size_t have) {
  if (sample_ws(d, n_s, blk).total <= have) return d.n_bh;
  for (int nkv = d.n_bkv - 1; nkv >= 1; --nkv)
    if (sample_ws(pass_dims(d, nkv * d.group), n_s, blk).total <= have) return nkv * d.group;
  for (int nh = d.group - 1; nh >= 1; --nh)
    if (d.group % nh == 0 && sample_ws(pass_dims(d, nh), n_s, blk).total <= have) return nh;
  return 0;
}

struct SparseWs {
  size_t vt, kc, vct, cidx, cbits, obits, dlist, dcnt, total;
  int cb_words, rb_words, dlist_stride, off_max;
};
// n_heads: the (batch * query) heads whose metadata and gathered K/V are resident at once;
// gathered: room for the per-head copies of the kept columns' K and V^T (the strip path;
// the block path reads its key blocks in place)
SparseWs sparse_ws(const Dims& d, int n_heads, bool gathered = true) {
  SparseWs w;
  w.cb_words = d.S_pad / 32 + 2;
  w.rb_words = d.S_pad / 32 + 24;
  w.dlist_stride = d.S_pad / 64 + 8;
  w.off_max = d.S_pad - 1;
  size_t at = 0;
  w.vt = at;    at += align_up((size_t)d.n_bkv * sa::kHeadDim * d.S_pad * 2);
  w.kc = at;    at += gathered ? align_up((size_t)n_heads * d.S_pad * sa::kHeadDim * 2) : 0;
  w.vct = at;   at += gathered ? align_up((size_t)n_heads * sa::kHeadDim * d.S_pad * 2) : 0;
  w.cidx = at;  at += align_up((size_t)n_heads * d.S_pad * 4);
  w.cbits = at; at += align_up((size_t)n_heads * w.cb_words * 4);
  w.obits = at; at += align_up((size_t)n_heads * w.rb_words * 4);
  w.dlist = at; at += align_up((size_t)n_heads * w.dlist_stride * 4);
  w.dcnt = at;  at += align_up((size_t)n_heads * 4);
  w.total = at;
  return w;
}

struct BlockWs { SparseWs sp; size_t tok_idx, tok_cnt, dbits, total; int nb, db_words; };
BlockWs block_ws(const Dims& d, int blk, int n_heads) {
  BlockWs w;
  w.sp = sparse_ws(d, n_heads, false);
  w.nb = (d.S + blk - 1) / blk;
  w.db_words = (w.nb + 1) / 32 + 1;
  size_t at = w.sp.total;
  w.tok_idx = at; at += align_up((size_t)n_heads * d.S * 4);
  w.tok_cnt = at; at += align_up((size_t)n_heads * 4);
  w.dbits = at;   at += align_up((size_t)n_heads * w.db_words * 4);
  w.total = at;
  return w;
}

// heads per pass and query segments of a partitioned call, validated
sa_status check_partition(const sa_partition* p, const Dims& d, int* heads_per_pass, int* n_segments) {
  if (p == nullptr) return SA_ERR_INVALID_ARG;
  if (p->heads_per_pass < 1 || p->n_query_segments < 1) return SA_ERR_INVALID_ARG;
  *heads_per_pass = p->heads_per_pass < d.n_bh ? p->heads_per_pass : d.n_bh;
  const int n_qtiles = d.S_pad / sa::kFlashBQ;
  *n_segments = p->n_query_segments < n_qtiles ? p->n_query_segments : n_qtiles;
  return SA_OK;
}

size_t dense_ws(const Dims& d) { return align_up((size_t)d.n_bkv * sa::kHeadDim * d.S_pad * 2); }

// rows [*lo, *hi) of query segment m of chunk_n (Algorithm 1: itv = S_q / chunk_n; here
// itv = floor(S / chunk_n) and the last segment takes the remainder)
inline void segment_rows(int S, int n_chunks, int m, int* lo, int* hi) {
  const int itv = S / n_chunks;
  *lo = m * itv;
  *hi = (m + 1 < n_chunks) ? (m + 1) * itv : S;
}

inline sa_status dev(hipError_t e) { return e == hipSuccess ? SA_OK : SA_ERR_DEVICE; }

// ---- optional event-pair profiling around kernels -----------------------------
struct Profiler {
  bool on = false;
  bool created = false;
  hipEvent_t start[SA_K_COUNT][SA_PROFILE_SLOTS];
  hipEvent_t stop[SA_K_COUNT][SA_PROFILE_SLOTS];
  long long count[SA_K_COUNT];
} g_prof;

struct Scope {   // records start now and stop at destruction
  int k; int slot; hipStream_t st; bool live;
  Scope(int kernel, hipStream_t s) : k(kernel), slot(0), st(s), live(g_prof.on) {
    if (!live) return;
    slot = (int)(g_prof.count[k] % SA_PROFILE_SLOTS);
    (void)hipEventRecord(g_prof.start[k][slot], st);
  }
  ~Scope() {
    if (!live) return;
    (void)hipEventRecord(g_prof.stop[k][slot], st);
    g_prof.count[k]++;
  }
};

// ---- address of the static scratch array on the current device ------------------
// In host code the array's name is only a handle for the runtime, not a device
// address: the address is looked up once per device (with that device current) and
// kept; kernels, fills and copies get that pointer.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

sa_status static_scratch(void** out) {
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return SA_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return SA_ERR_DEVICE;
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return SA_OK;
}

sa::FlashParams base_flash(const Dims& d, const void* q, const void* k) {
  sa::FlashParams P;
  memset(&P, 0, sizeof(P));
  P.q = static_cast<const uint16_t*>(q);
  P.k = static_cast<const uint16_t*>(k);
  P.S = d.S; P.S_pad = d.S_pad;
  P.n_bh = d.n_bh; P.n_bkv = d.n_bkv; P.group = d.group;
  P.scale_log2 = d.scale * 1.4426950408889634f;
  P.n_qtiles = (d.S + sa::kFlashBQ - 1) / sa::kFlashBQ;
  P.q_row0 = 0; P.n_qrows = d.S;
  P.k_splits = 1;
  return P;
}

hipError_t transpose_v(const Dims& d, const void* v, uint16_t* vt, hipStream_t st) {
  sa::GatherParams G;
  memset(&G, 0, sizeof(G));
  G.src = static_cast<const uint16_t*>(v);
  G.out_t = vt;
  G.n_out = d.n_bkv; G.group = 1;
  G.S = d.S; G.C_pad = d.S_pad;
  return sa::launch_gather_transpose(G, st);
}

}  // namespace

extern "C" {

size_t sa_workspace_bytes(int op, const sa_shape* shape, const sa_sampling* sampling) {
  Dims d;
  if (check_shape(shape, &d) != SA_OK) return 0;
  switch (op) {
    case SA_OP_SAMPLE_SCORES:
      if (check_sampling(sampling, d) != SA_OK) return 0;
      return sample_ws(d, sampling->n_sample_rows, sampling->granularity).total;
    case SA_OP_SAMPLE_SCORES_MIN:
      if (check_sampling(sampling, d) != SA_OK) return 0;
      return sample_ws(pass_dims(d, 1), sampling->n_sample_rows, sampling->granularity).total;
    case SA_OP_SELECT_STRIPS: return 0;
    case SA_OP_SPARSE_ATTN: return sparse_ws(d, d.n_bh).total;
    case SA_OP_DENSE_ATTN: return dense_ws(d);
    case SA_OP_BLOCK_SPARSE_ATTN:
      if (sampling == nullptr || check_granularity(sampling->granularity) != SA_OK) return 0;
      return block_ws(d, sampling->granularity, d.n_bh).total;
    default: return 0;
  }
}

int32_t sa_rows_from_ratio(int32_t seq_len, float ratio) {
  if (seq_len < 1 || !(ratio > 0.0f)) return 0;
  double blocks = ceil((double)ratio * (double)seq_len / 64.0 - 1e-9);
  if (blocks < 1.0) blocks = 1.0;
  double n = 64.0 * blocks;
  return (n > (double)seq_len) ? seq_len : (int32_t)n;
}

sa_status sa_sample_scores(const sa_shape* shape, const sa_sampling* sampling,
                           const void* q, const void* k,
                           float* col_scores, float* slash_scores, float* row_lse,
                           void* workspace, size_t workspace_bytes, void* stream) {
  Dims d;
  sa_status s = check_shape(shape, &d);
  if (s != SA_OK) return s;
  s = check_sampling(sampling, d);
  if (s != SA_OK) return s;
  if (q == nullptr || k == nullptr || col_scores == nullptr || slash_scores == nullptr) return SA_ERR_INVALID_ARG;
  const int n_s = sampling->n_sample_rows;
  const int blk = sampling->granularity;
  const int n_chunks = sampling->n_chunks;
  if (row_lse != nullptr && n_chunks != 1) return SA_ERR_UNSUPPORTED;
  // all heads at once if the workspace allows, else as many as fit, pass after pass
  s = check_ws(workspace, workspace_bytes, sample_ws(pass_dims(d, 1), n_s, blk).total);
  if (s != SA_OK) return s;
  const int heads_per_pass = sample_heads_per_pass(d, n_s, blk, workspace_bytes);
  if (heads_per_pass < 1) return SA_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  const size_t n_cand = (size_t)(d.S + blk - 1) / blk;       // scores per head and direction
  const size_t head_elems = (size_t)d.S * sa::kHeadDim;

  for (int m = 0; m < n_chunks; ++m) {
    // chunk m: the last n_s rows of the m-th of n_chunks query segments
    int seg_lo, seg_hi;
    segment_rows(d.S, n_chunks, m, &seg_lo, &seg_hi);
    const int row_first = seg_hi - n_s;
    for (int h0 = 0; h0 < d.n_bh; h0 += heads_per_pass) {
      const int nh = (d.n_bh - h0 < heads_per_pass) ? d.n_bh - h0 : heads_per_pass;
      const Dims pd = pass_dims(d, nh);
      const SampleWs w = sample_ws(pd, n_s, blk);
      const void* q_pass = static_cast<const uint16_t*>(q) + (size_t)h0 * head_elems;
      const void* k_pass = static_cast<const uint16_t*>(k) + (size_t)(h0 / d.group) * head_elems;
      float* lse = row_lse ? row_lse + (size_t)h0 * n_s : reinterpret_cast<float*>(ws + w.lse);
      float* out_col = col_scores + ((size_t)m * d.n_bh + h0) * n_cand;
      float* out_slash = slash_scores + ((size_t)m * d.n_bh + h0) * n_cand;
      float* tok_col = blk > 1 ? reinterpret_cast<float*>(ws + w.tok_col) : out_col;
      float* tok_slash = blk > 1 ? reinterpret_cast<float*>(ws + w.tok_slash) : out_slash;

      // pass 1: log-sum-exp of every sampled row (flash sweep without V)
      sa::FlashParams P = base_flash(pd, q_pass, k_pass);
      P.k_splits = sa::lse_key_splits(row_first, n_s, pd.n_bh);
      if (P.k_splits > kMaxKeySplits) P.k_splits = kMaxKeySplits;
      P.lse = P.k_splits > 1 ? reinterpret_cast<float*>(ws + w.lse_part) : lse;
      P.q_row0 = row_first;
      P.n_qrows = n_s;
      P.n_qtiles = (n_s + sa::kFlashBQ - 1) / sa::kFlashBQ;
      {
        Scope sc(SA_K_ROW_LSE, st);
        s = dev(sa::launch_flash(1, false, P, st));
        if (s == SA_OK && P.k_splits > 1)
          s = dev(sa::launch_lse_combine(P.lse, lse, (size_t)pd.n_bh * n_s, P.k_splits, st));
      }
      if (s != SA_OK) return s;

      // pass 2: recompute the probabilities and accumulate columns and diagonals
      sa::ScoreParams C;
      memset(&C, 0, sizeof(C));
      C.q = static_cast<const uint16_t*>(q_pass);
      C.k = static_cast<const uint16_t*>(k_pass);
      C.lse = lse;
      C.col = tok_col; C.slash = tok_slash;
      C.partial = reinterpret_cast<float*>(ws + w.partial);
      C.S = d.S; C.n_s = n_s; C.n_bh = pd.n_bh; C.n_bkv = pd.n_bkv; C.group = pd.group;
      C.row_first = row_first;
      C.scale_log2 = P.scale_log2;
      {
        Scope sc(SA_K_SCORE_ACCUM, st);
        s = dev(sa::launch_score_accumulate(C, st));
      }
      if (s != SA_OK) return s;
      {
        Scope sc(SA_K_SCORE_FINAL, st);
        s = dev(sa::launch_score_finalize(C, st));
        // block_reduction: the per-token scores summed over blocks of blk keys / offsets
        if (s == SA_OK && blk > 1) s = dev(sa::launch_block_reduce(tok_col, out_col, pd.n_bh, d.S, blk, st));
        if (s == SA_OK && blk > 1) s = dev(sa::launch_block_reduce(tok_slash, out_slash, pd.n_bh, d.S, blk, st));
      }
      if (s != SA_OK) return s;
    }
  }
  return SA_OK;
}

sa_status sa_block_scores(const sa_shape* shape, int32_t granularity,
                          const float* col_scores, const float* slash_scores,
                          float* col_block_scores, float* slash_block_scores, void* stream) {
  Dims d;
  sa_status s = check_shape(shape, &d);
  if (s != SA_OK) return s;
  s = check_granularity(granularity);
  if (s != SA_OK) return s;
  if (col_scores == nullptr || slash_scores == nullptr || col_block_scores == nullptr || slash_block_scores == nullptr)
    return SA_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Scope sc(SA_K_SCORE_FINAL, st);
  s = dev(sa::launch_block_reduce(col_scores, col_block_scores, d.n_bh, d.S, granularity, st));
  if (s != SA_OK) return s;
  return dev(sa::launch_block_reduce(slash_scores, slash_block_scores, d.n_bh, d.S, granularity, st));
}

}  // extern "C"

namespace {
// both selections over n candidates per head (keys / offsets, or blocks of them)
sa_status select_both(const sa_shape* shape, int n_chunks, int granularity,
                      const float* col_scores, const float* slash_scores,
                      float alpha_c, float alpha_s,
                      int32_t* col_idx, int32_t* col_cnt,
                      int32_t* slash_idx, int32_t* slash_cnt, void* stream) {
  Dims d;
  sa_status s = check_shape(shape, &d);
  if (s != SA_OK) return s;
  s = check_chunks(d, n_chunks, granularity);
  if (s != SA_OK) return s;
  if (col_scores == nullptr || slash_scores == nullptr || col_idx == nullptr || col_cnt == nullptr ||
      slash_idx == nullptr || slash_cnt == nullptr)
    return SA_ERR_INVALID_ARG;
  // the CRA thresholds of Algorithm 1 are fractions of the sampled mass
  if (!(alpha_c >= 0.0f && alpha_c <= 1.0f) || !(alpha_s >= 0.0f && alpha_s <= 1.0f)) return SA_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Scope sc(SA_K_SELECT, st);
  sa::SelectParams P;
  P.n_prob = n_chunks * d.n_bh;   // every (chunk, head) is a problem of its own
  P.S = (d.S + granularity - 1) / granularity;
  // both directions in one launch: twice the workgroups on an otherwise mostly idle chip
  P.scores = col_scores; P.idx = col_idx; P.cnt = col_cnt; P.alpha = alpha_c;
  P.scores2 = slash_scores; P.idx2 = slash_idx; P.cnt2 = slash_cnt; P.alpha2 = alpha_s;
  return dev(sa::launch_select(P, st));
}
}  // namespace

extern "C" {

sa_status sa_select_strips(const sa_shape* shape,
                           const float* col_scores, const float* slash_scores,
                           float alpha_c, float alpha_s,
                           int32_t* col_idx, int32_t* col_cnt,
                           int32_t* slash_idx, int32_t* slash_cnt,
                           void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  return select_both(shape, 1, 1, col_scores, slash_scores, alpha_c, alpha_s, col_idx, col_cnt, slash_idx,
                     slash_cnt, stream);
}

sa_status sa_select_blocks(const sa_shape* shape, int32_t granularity,
                           const float* col_block_scores, const float* slash_block_scores,
                           float alpha_c, float alpha_s,
                           int32_t* col_blocks, int32_t* col_cnt,
                           int32_t* slash_blocks, int32_t* slash_cnt,
                           void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  if (granularity < 1) return SA_ERR_INVALID_ARG;
  if (granularity == 1) return SA_ERR_UNSUPPORTED;   // per-token selection is sa_select_strips
  return select_both(shape, 1, granularity, col_block_scores, slash_block_scores, alpha_c, alpha_s, col_blocks,
                     col_cnt, slash_blocks, slash_cnt, stream);
}

sa_status sa_select_chunked(const sa_shape* shape, const sa_sampling* sampling,
                            const float* col_scores, const float* slash_scores,
                            float alpha_c, float alpha_s,
                            int32_t* col_idx, int32_t* col_cnt,
                            int32_t* slash_idx, int32_t* slash_cnt,
                            void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  if (sampling == nullptr) return SA_ERR_INVALID_ARG;
  return select_both(shape, sampling->n_chunks, sampling->granularity, col_scores, slash_scores, alpha_c, alpha_s,
                     col_idx, col_cnt, slash_idx, slash_cnt, stream);
}

}  // extern "C"

namespace {
// merge_index for the heads [h0, h0 + nh) under one set of lists: bitmaps, tile-diagonal
// list and the gathered K / V^T of the kept columns, all in workspace slots 0 .. nh-1.
// granularity 1: strip lists (per key / per offset); otherwise lists of blocks.
// On return *cnt_used points at the column counts the kernel must read (slot-indexed).
sa_status prepare_heads(const Dims& d, const BlockWs& bw, int granularity, int h0, int nh, size_t n_cand,
                        const void* k, const void* v,
                        const int32_t* col_idx, const int32_t* col_cnt,
                        const int32_t* slash_idx, const int32_t* slash_cnt, int32_t local_window, int row_hi,
                        char* ws, hipStream_t st, const int32_t** cnt_used) {
  const SparseWs& w = bw.sp;
  const bool blocks = granularity != 1;
  Scope sc(SA_K_MASK_PREP, st);
  // this pass's rows of the caller's lists
  col_idx += (size_t)h0 * n_cand; slash_idx += (size_t)h0 * n_cand;
  col_cnt += h0; slash_cnt += h0;
  sa_status s = SA_OK;
  uint32_t* col_bits = reinterpret_cast<uint32_t*>(ws + w.cbits);
  uint32_t* off_bits = reinterpret_cast<uint32_t*>(ws + w.obits);
  int32_t* dlist = reinterpret_cast<int32_t*>(ws + w.dlist);
  int32_t* dcnt = reinterpret_cast<int32_t*>(ws + w.dcnt);
  if (!blocks) {
    // slash side: bitmaps of kept columns / offsets and touched tile diagonals
    sa::MaskPrepParams M;
    memset(&M, 0, sizeof(M));
    M.col_bits = col_bits; M.off_bits = off_bits; M.dlist = dlist; M.dcnt = dcnt;
    M.col_idx = col_idx; M.col_cnt = col_cnt; M.slash_idx = slash_idx; M.slash_cnt = slash_cnt;
    M.n_bh = nh; M.S = d.S; M.window = local_window;
    M.cb_words = w.cb_words; M.rb_words = w.rb_words; M.dlist_stride = w.dlist_stride; M.off_max = w.off_max;
    s = dev(sa::launch_mask_prep(M, st));
  } else {
    // the same metadata from block lists; from here on the selected key blocks are
    // the token columns they hold
    sa::BlockPrepParams B;
    memset(&B, 0, sizeof(B));
    B.col_blk = col_idx; B.col_bcnt = col_cnt; B.slash_blk = slash_idx; B.slash_bcnt = slash_cnt;
    B.tok_idx = reinterpret_cast<int32_t*>(ws + bw.tok_idx);
    B.tok_cnt = reinterpret_cast<int32_t*>(ws + bw.tok_cnt);
    B.diag_bits = reinterpret_cast<uint32_t*>(ws + bw.dbits);
    B.col_bits = col_bits; B.off_bits = off_bits; B.dlist = dlist; B.dcnt = dcnt;
    B.n_bh = nh; B.S = d.S; B.window = local_window;
    B.cb_words = w.cb_words; B.rb_words = w.rb_words; B.dlist_stride = w.dlist_stride; B.off_max = w.off_max;
    B.blk = granularity; B.nb = bw.nb; B.db_words = bw.db_words;
    s = dev(sa::launch_block_prep(B, st));
    col_idx = B.tok_idx; col_cnt = B.tok_cnt;
  }
  if (s != SA_OK) return s;
  *cnt_used = col_cnt;

  // column side: compact K rows and V^T columns of the kept keys, per query head.  Key
  // blocks are runs of consecutive keys and are read in place: only the padded index
  // list (the tiles' key indices) is written then.
  sa::GatherParams G;
  memset(&G, 0, sizeof(G));
  G.idx = col_idx; G.cnt = col_cnt; G.idx_stride = d.S;
  G.idx_pad = reinterpret_cast<int32_t*>(ws + w.cidx); G.idx_pad_stride = d.S_pad;
  G.n_out = nh; G.group = d.group; G.head0 = h0; G.S = d.S; G.C_pad = d.S_pad;
  G.key_limit = row_hi < d.S ? row_hi : 0;     // the rows of this segment end at row_hi: later keys are never read
  if (blocks) return dev(sa::launch_gather_transpose(G, st));
  G.src = static_cast<const uint16_t*>(v);
  G.out_t = reinterpret_cast<uint16_t*>(ws + w.vct);
  s = dev(sa::launch_gather_transpose(G, st));
  if (s != SA_OK) return s;
  // K rows: gather only
  G.src = static_cast<const uint16_t*>(k);
  G.out_rows = reinterpret_cast<uint16_t*>(ws + w.kc);
  G.out_t = nullptr;
  G.idx_pad = nullptr;
  return dev(sa::launch_gather_transpose(G, st));
}

// the strip-masked kernel on query tiles [qtile0, qtile0 + n_qtiles) of the heads [h0, h0 + nh)
sa_status launch_attend(const Dims& d, const SparseWs& w, bool blocks, int h0, int nh, int qtile0, int n_qtiles,
                        int row_lo, int row_hi, const void* q, const void* k, const int32_t* col_cnt,
                        void* out, int out_dtype, float* out_lse, uint64_t* tiles, char* ws, hipStream_t st) {
  sa::FlashParams P = base_flash(d, q, k);
  const size_t head_elems = (size_t)d.S * sa::kHeadDim;
  P.q = static_cast<const uint16_t*>(q) + (size_t)h0 * head_elems;
  P.out = static_cast<char*>(out) + (size_t)h0 * head_elems * (out_dtype == SA_OUT_F32 ? 4 : 2);
  P.lse = out_lse ? out_lse + (size_t)h0 * d.S : nullptr;
  P.tiles = tiles ? reinterpret_cast<unsigned long long*>(tiles) + h0 : nullptr;
  P.n_bh = nh; P.head0 = h0;
  P.qtile0 = qtile0;
  P.n_qtiles = n_qtiles;
  // only rows [row_lo, row_hi) are computed and written (a query tile that straddles two
  // segments is visited by both launches, each writing its own rows)
  P.row_lo = row_lo;
  P.n_qrows = row_hi;
  P.vt = reinterpret_cast<const uint16_t*>(ws + w.vt);
  P.cols_in_place = blocks ? 1 : 0;
  P.kc = blocks ? nullptr : reinterpret_cast<const uint16_t*>(ws + w.kc);
  P.vct = blocks ? nullptr : reinterpret_cast<const uint16_t*>(ws + w.vct);
  P.col_idx_pad = reinterpret_cast<const int32_t*>(ws + w.cidx);
  P.col_cnt = col_cnt;
  P.col_bits = reinterpret_cast<const uint32_t*>(ws + w.cbits);
  P.off_bits = reinterpret_cast<const uint32_t*>(ws + w.obits);
  P.dlist = reinterpret_cast<const int32_t*>(ws + w.dlist);
  P.dcnt = reinterpret_cast<const int32_t*>(ws + w.dcnt);
  P.cidx_stride = d.S_pad; P.cb_words = w.cb_words; P.rb_words = w.rb_words;
  P.dlist_stride = w.dlist_stride; P.off_max = w.off_max;
  Scope sc(SA_K_SPARSE_FLASH, st);
  return dev(sa::launch_flash(2, out_dtype == SA_OUT_F32, P, st));
}

// Argument checks, then the passes.  Chunks: the lists selected from chunk m mask the
// query rows of segment m (merge_index with itv = S / chunk_n); a single chunk is the
// whole matrix.  Partition (Sec. 5.4, long sequences): the heads are taken
// heads_per_pass at a time - the workspace holds the metadata and the gathered K / V
// of one pass only - and the query tiles of a chunk in n_segments consecutive launches.
// Every (head, query tile) is computed by one workgroup whatever the partition, so the
// result does not depend on it.
sa_status sparse_attn(const sa_shape* shape, int n_chunks, int granularity, const sa_partition* part,
                      const void* q, const void* k, const void* v,
                      const int32_t* col_idx_all, const int32_t* col_cnt_all,
                      const int32_t* slash_idx_all, const int32_t* slash_cnt_all,
                      int32_t local_window,
                      void* out, int out_dtype, float* out_lse, uint64_t* tiles,
                      void* workspace, size_t workspace_bytes, void* stream) {
  Dims d;
  sa_status s = check_shape(shape, &d);
  if (s != SA_OK) return s;
  s = check_chunks(d, n_chunks, granularity);
  if (s != SA_OK) return s;
  int heads_per_pass = d.n_bh, n_segments = 1;
  if (part != nullptr) {
    s = check_partition(part, d, &heads_per_pass, &n_segments);
    if (s != SA_OK) return s;
  }
  const bool blocks = granularity != 1;
  if (q == nullptr || k == nullptr || v == nullptr || out == nullptr || col_idx_all == nullptr ||
      col_cnt_all == nullptr || slash_idx_all == nullptr || slash_cnt_all == nullptr)
    return SA_ERR_INVALID_ARG;
  if (local_window < 1) return SA_ERR_INVALID_ARG;
  if (out_dtype != SA_OUT_BF16 && out_dtype != SA_OUT_F32) return SA_ERR_INVALID_ARG;
  BlockWs bw = block_ws(d, blocks ? granularity : 64, heads_per_pass);
  if (!blocks) bw.sp = sparse_ws(d, heads_per_pass, true);
  s = check_ws(workspace, workspace_bytes, blocks ? bw.total : bw.sp.total);
  if (s != SA_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  if (tiles != nullptr) {
    s = dev(sa::launch_fill_u32(reinterpret_cast<uint32_t*>(tiles), 2 * (size_t)d.n_bh, 0u, st));
    if (s != SA_OK) return s;
  }
  {
    // V^T for the contiguous (slash / window) tiles: once per call
    Scope sc(SA_K_TRANSPOSE_V, st);
    s = dev(transpose_v(d, v, reinterpret_cast<uint16_t*>(ws + bw.sp.vt), st));
    if (s != SA_OK) return s;
  }
  const size_t n_cand = (size_t)(d.S + granularity - 1) / granularity;   // list capacity per head
  for (int m = 0; m < n_chunks; ++m) {
    int row_lo, row_hi;
    segment_rows(d.S, n_chunks, m, &row_lo, &row_hi);
    const int qtile0 = row_lo / sa::kFlashBQ;
    const int qtile1 = (row_hi + sa::kFlashBQ - 1) / sa::kFlashBQ;    // one past the last tile with a row of the segment
    const size_t chunk_off = (size_t)m * d.n_bh;
    for (int h0 = 0; h0 < d.n_bh; h0 += heads_per_pass) {
      const int nh = (d.n_bh - h0 < heads_per_pass) ? d.n_bh - h0 : heads_per_pass;
      const int32_t* cnt_used = nullptr;
      s = prepare_heads(d, bw, granularity, h0, nh, n_cand, k, v,
                        col_idx_all + chunk_off * n_cand, col_cnt_all + chunk_off,
                        slash_idx_all + chunk_off * n_cand, slash_cnt_all + chunk_off,
                        local_window, row_hi, ws, st, &cnt_used);
      if (s != SA_OK) return s;
      const int segs = (n_segments < qtile1 - qtile0) ? n_segments : (qtile1 - qtile0);
      for (int g = 0; g < segs; ++g) {
        const int a0 = qtile0 + (int)((long long)(qtile1 - qtile0) * g / segs);
        const int a1 = qtile0 + (int)((long long)(qtile1 - qtile0) * (g + 1) / segs);
        s = launch_attend(d, bw.sp, blocks, h0, nh, a0, a1 - a0, row_lo, row_hi, q, k, cnt_used, out, out_dtype, out_lse,
                          tiles, ws, st);
        if (s != SA_OK) return s;
      }
    }
  }
  return SA_OK;
}
}  // namespace

extern "C" {

sa_status sa_sparse_attn(const sa_shape* shape, const void* q, const void* k, const void* v,
                         const int32_t* col_idx, const int32_t* col_cnt,
                         const int32_t* slash_idx, const int32_t* slash_cnt,
                         int32_t local_window,
                         void* out, int out_dtype, float* out_lse, uint64_t* tiles,
                         void* workspace, size_t workspace_bytes, void* stream) {
  return sparse_attn(shape, 1, 1, nullptr, q, k, v, col_idx, col_cnt, slash_idx, slash_cnt, local_window, out,
                     out_dtype, out_lse, tiles, workspace, workspace_bytes, stream);
}

size_t sa_partitioned_workspace_bytes(const sa_shape* shape, const sa_partition* partition) {
  Dims d;
  int hpp = 0, segs = 0;
  if (check_shape(shape, &d) != SA_OK || check_partition(partition, d, &hpp, &segs) != SA_OK) return 0;
  return sparse_ws(d, hpp).total;
}

sa_status sa_sparse_attn_partitioned(const sa_shape* shape, const sa_partition* partition,
                                     const void* q, const void* k, const void* v,
                                     const int32_t* col_idx, const int32_t* col_cnt,
                                     const int32_t* slash_idx, const int32_t* slash_cnt,
                                     int32_t local_window,
                                     void* out, int out_dtype, float* out_lse, uint64_t* tiles,
                                     void* workspace, size_t workspace_bytes, void* stream) {
  if (partition == nullptr) return SA_ERR_INVALID_ARG;
  return sparse_attn(shape, 1, 1, partition, q, k, v, col_idx, col_cnt, slash_idx, slash_cnt, local_window, out,
                     out_dtype, out_lse, tiles, workspace, workspace_bytes, stream);
}

sa_status sa_block_sparse_attn(const sa_shape* shape, int32_t granularity,
                               const void* q, const void* k, const void* v,
                               const int32_t* col_blocks, const int32_t* col_cnt,
                               const int32_t* slash_blocks, const int32_t* slash_cnt,
                               int32_t local_window,
                               void* out, int out_dtype, float* out_lse, uint64_t* tiles,
                               void* workspace, size_t workspace_bytes, void* stream) {
  if (granularity < 1) return SA_ERR_INVALID_ARG;
  if (granularity == 1) return SA_ERR_UNSUPPORTED;   // per-token strips are sa_sparse_attn
  return sparse_attn(shape, 1, granularity, nullptr, q, k, v, col_blocks, col_cnt, slash_blocks, slash_cnt, local_window, out,
                     out_dtype, out_lse, tiles, workspace, workspace_bytes, stream);
}

sa_status sa_sparse_attn_chunked(const sa_shape* shape, const sa_sampling* sampling,
                                 const void* q, const void* k, const void* v,
                                 const int32_t* col_idx, const int32_t* col_cnt,
                                 const int32_t* slash_idx, const int32_t* slash_cnt,
                                 int32_t local_window,
                                 void* out, int out_dtype, float* out_lse, uint64_t* tiles,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  if (sampling == nullptr) return SA_ERR_INVALID_ARG;
  return sparse_attn(shape, sampling->n_chunks, sampling->granularity, nullptr, q, k, v, col_idx, col_cnt,
                     slash_idx, slash_cnt, local_window, out, out_dtype, out_lse, tiles, workspace, workspace_bytes,
                     stream);
}

sa_status sa_dense_attn(const sa_shape* shape, const void* q, const void* k, const void* v,
                        void* out, int out_dtype, float* out_lse,
                        void* workspace, size_t workspace_bytes, void* stream) {
  Dims d;
  sa_status s = check_shape(shape, &d);
  if (s != SA_OK) return s;
  if (q == nullptr || k == nullptr || v == nullptr || out == nullptr) return SA_ERR_INVALID_ARG;
  if (out_dtype != SA_OUT_BF16 && out_dtype != SA_OUT_F32) return SA_ERR_INVALID_ARG;
  s = check_ws(workspace, workspace_bytes, dense_ws(d));
  if (s != SA_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint16_t* vt = static_cast<uint16_t*>(workspace);
  {
    Scope sc(SA_K_TRANSPOSE_V, st);
    s = dev(transpose_v(d, v, vt, st));
  }
  if (s != SA_OK) return s;
  sa::FlashParams P = base_flash(d, q, k);
  P.vt = vt; P.out = out; P.lse = out_lse;
  Scope sc(SA_K_DENSE_FLASH, st);
  return dev(sa::launch_flash(0, out_dtype == SA_OUT_F32, P, st));
}

sa_status sa_dense_attn_static(const sa_shape* shape, const void* q, const void* k, const void* v,
                               void* out, int out_dtype, float* out_lse, void* stream) {
  Dims d;
  sa_status s = check_shape(shape, &d);
  if (s != SA_OK) return s;
  if (q == nullptr || k == nullptr || v == nullptr || out == nullptr) return SA_ERR_INVALID_ARG;
  if (out_dtype != SA_OUT_BF16 && out_dtype != SA_OUT_F32) return SA_ERR_INVALID_ARG;
  if (dense_ws(d) > (size_t)SA_STATIC_SCRATCH_BYTES) return SA_ERR_TOO_LARGE;   // V^T must fit the static array
  void* ws = nullptr;
  s = static_scratch(&ws);
  if (s != SA_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint16_t* vt = static_cast<uint16_t*>(ws);
  // V^T is rewritten, zero padding included, up to the last key tile the kernel reads:
  // nothing of an earlier call's contents is used
  {
    Scope sc(SA_K_TRANSPOSE_V, st);
    s = dev(transpose_v(d, v, vt, st));
  }
  if (s != SA_OK) return s;
  sa::FlashParams P = base_flash(d, q, k);
  P.vt = vt; P.out = out; P.lse = out_lse;
  Scope sc(SA_K_DENSE_FLASH, st);
  return dev(sa::launch_flash(0, out_dtype == SA_OUT_F32, P, st));
}

sa_status sa_probe_mfma(int32_t iters, int32_t waves_per_simd, float* sink, void* stream) {
  if (iters < 1 || waves_per_simd < 1 || waves_per_simd > 8 || sink == nullptr) return SA_ERR_INVALID_ARG;
  return dev(sa::launch_probe_mfma(iters, waves_per_simd, sink, static_cast<hipStream_t>(stream)));
}

sa_status sa_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (src == nullptr || dst == nullptr || bytes % 16 != 0) return SA_ERR_INVALID_ARG;
  return dev(sa::launch_probe_copy(src, dst, bytes, static_cast<hipStream_t>(stream)));
}

sa_status sa_profile_enable(int enable) {
  if (enable && !g_prof.created) {
    for (int k = 0; k < SA_K_COUNT; ++k)
      for (int i = 0; i < SA_PROFILE_SLOTS; ++i) {
        if (hipEventCreate(&g_prof.start[k][i]) != hipSuccess) return SA_ERR_DEVICE;
        if (hipEventCreate(&g_prof.stop[k][i]) != hipSuccess) return SA_ERR_DEVICE;
      }
    g_prof.created = true;
  }
  for (int k = 0; k < SA_K_COUNT; ++k) g_prof.count[k] = 0;
  g_prof.on = (enable != 0);
  return SA_OK;
}

int sa_profile_read(int kernel, float* ms, int cap) {
  if (kernel < 0 || kernel >= SA_K_COUNT || ms == nullptr || cap < 0 || !g_prof.created) return -1;
  long long n = g_prof.count[kernel];
  long long first = (n > SA_PROFILE_SLOTS) ? n - SA_PROFILE_SLOTS : 0;
  int w = 0;
  for (long long i = first; i < n && w < cap; ++i) {
    int slot = (int)(i % SA_PROFILE_SLOTS);
    if (hipEventSynchronize(g_prof.stop[kernel][slot]) != hipSuccess) return -1;
    float t = 0.f;
    if (hipEventElapsedTime(&t, g_prof.start[kernel][slot], g_prof.stop[kernel][slot]) != hipSuccess) return -1;
    ms[w++] = t;
  }
  return w;
}

const char* sa_status_string(int status) {
  switch (status) {
    case SA_OK: return "ok";
    case SA_ERR_INVALID_ARG: return "invalid argument";
    case SA_ERR_UNSUPPORTED: return "unsupported configuration";
    case SA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SA_ERR_DEVICE: return "HIP runtime error";
    case SA_ERR_TOO_LARGE: return "problem exceeds the static scratch of the entry point that allocates nothing";
    default: return "unknown status";
  }
}

int sa_version(void) { return 130; }

}  // extern "C"
