// Stage 1, pass 2 (Algorithm 1 stage 1; Sec. 4.2): with the row log-sum-exp of
// every sampled query known, recompute p_ij = exp(q_i.k_j*scale - lse_i) tile by
// tile and accumulate it down the key columns and along the diagonals.
//
// One workgroup = 128 keys (4 waves x 32 keys, K resident in registers as the
// MFMA B operand) x one chunk of sampled rows.  S = Q K^T is formed 32 rows at
// a time, so one lane holds ONE key (lane % 32) and 16 query rows: the column
// sum is in-lane arithmetic.  Diagonal sums go to a per-wave LDS window with
// LDS float adds (each wave adds in its own program order), the four windows are
// combined in a fixed order and written as one partial per (key block, chunk);
// a second kernel adds the partials in a fixed order.  No global float atomics:
// repeated runs give identical bits.
#include "sa_device.h"
#include "sa_kernels.h"

namespace sa {

namespace {

constexpr int KB = 128;          // keys per workgroup
constexpr int QC = 2048;         // sampled rows per chunk
constexpr int WWIN = QC + 64;    // floats in one wave's diagonal window
constexpr int WIN = QC + 128;    // floats in the combined (key block, chunk) partial
constexpr int QROW_B = 272;      // bytes per staged Q row
constexpr int QSTAGE_B = 32 * QROW_B + 32 * 4;   // 32 rows + 32 lse values

__global__ __launch_bounds__(256) void score_accumulate_kernel(ScoreParams P) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  float* win = reinterpret_cast<float*>(smem);                  // [4][WWIN]
  char* qstage = smem + 4 * WWIN * 4;                           // [2][QSTAGE_B]

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int ql = lane & 31, hf = lane >> 5;
  const int kb = blockIdx.x, ch = blockIdx.y, bh = blockIdx.z;
  const int S = P.S;
  const int r0 = S - P.n_s;
  const int row0 = r0 + ch * QC;                    // first row of the chunk
  const int row_end = min(row0 + QC, S);            // one past the last row
  const int j0 = kb * KB;
  if (row_end - 1 < j0) return;                     // chunk entirely above these keys
  const int jw = j0 + 32 * wave;
  const int j_me = jw + ql;
  const int bkv = bh / P.group;
  const float c2 = P.scale_log2;

  // K^T operand of this wave's 32 keys (zero beyond the sequence end)
  bf16x8 kf[8];
  {
    const uint16_t* krow = P.k + ((size_t)bkv * S + min(j_me, S - 1)) * kHeadDim;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 v = *reinterpret_cast<const uint4*>(krow + ks * 16 + hf * 8);
      if (j_me >= S) v = make_uint4(0u, 0u, 0u, 0u);
      kf[ks] = as_bf16x8(v);
    }
  }
  for (int x = tid; x < 4 * WWIN; x += 256) win[x] = 0.f;

  // first 32-row block that reaches the keys of the workgroup
  const int nblk = (row_end - row0 + 31) / 32;
  int b_first = (j0 > row0) ? (j0 - row0) / 32 : 0;
  const uint16_t* qbase = P.q + (size_t)bh * S * kHeadDim;
  const float* lbase = P.lse + (size_t)bh * P.n_s;

  uint4 pq[2];
  float pl = 0.f;
  auto load_block = [&](int b) {
    int rb = row0 + 32 * b;
#pragma unroll
    for (int n = 0; n < 2; ++n) {
      int c = tid + 256 * n;
      int row = c >> 4, col = c & 15;
      int i = rb + row;
      pq[n] = (i < S) ? *reinterpret_cast<const uint4*>(qbase + (size_t)i * kHeadDim + col * 8)
                      : make_uint4(0u, 0u, 0u, 0u);
    }
    if (tid < 32) {
      int i = rb + tid;
      pl = (i < S) ? lbase[i - r0] * kLog2e : 0.f;
    }
  };
  auto store_block = [&](char* st) {
#pragma unroll
    for (int n = 0; n < 2; ++n) {
      int c = tid + 256 * n;
      int row = c >> 4, col = c & 15;
      *reinterpret_cast<uint4*>(st + row * QROW_B + col * 16) = pq[n];
    }
    if (tid < 32) reinterpret_cast<float*>(st + 32 * QROW_B)[tid] = pl;
  };

  if (b_first < nblk) {
    load_block(b_first);
    store_block(qstage + (b_first & 1) * QSTAGE_B);
  }
  __syncthreads();

  float colacc = 0.f;
  float* mywin = win + wave * WWIN;
  for (int b = b_first; b < nblk; ++b) {
    const char* st = qstage + (b & 1) * QSTAGE_B;
    const bool have_next = (b + 1 < nblk);
    if (have_next) load_block(b + 1);
    const int rb = row0 + 32 * b;
    if (rb + 31 >= jw) {          // some row of the block reaches this wave's keys
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
      const char* qp = st + ql * QROW_B + hf * 16;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        bf16x8 qf = as_bf16x8(*reinterpret_cast<const uint4*>(qp + ks * 32));
        s = mfma_32x32x16(qf, kf[ks], s);
      }
      // element r: query row rb + 8*(r/4) + 4*hf + r%4, key j_me
      const float* ls = reinterpret_cast<const float*>(st + 32 * QROW_B);
      const bool edge = (rb < jw + 32) || (rb + 32 > S);
      const int wbase = (rb - row0) - ql + 31;    // window slot of (row rb, key j_me)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4 l4 = *reinterpret_cast<const float4*>(ls + 8 * g + 4 * hf);
        float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          int m = 8 * g + 4 * hf + t;
          float p = fast_exp2(fmaf(s[4 * g + t], c2, -lv[t]));
          if (edge) {
            int i = rb + m;
            p = (i >= j_me && i < S) ? p : 0.f;
          }
          colacc += p;
          atomicAdd(mywin + wbase + m, p);
        }
      }
    }
    if (have_next) store_block(qstage + ((b + 1) & 1) * QSTAGE_B);
    __syncthreads();
  }

  // column sums of this chunk (both lane halves hold disjoint rows)
  float ctot = colacc + swap_half(colacc);
  if (hf == 0 && j_me < S) P.col[((size_t)bh * P.n_chunks + ch) * S + j_me] = ctot;

  // combine the four wave windows: slot x <-> offset x + (row0 - j0 - 127)
  float* out = P.partial + (((size_t)bh * P.n_kblocks + kb) * P.n_chunks + ch) * WIN;
  for (int x = tid; x < WIN; x += 256) {
    float acc = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      int y = x - 96 + 32 * w;
      if (y >= 0 && y < WWIN) acc += win[w * WWIN + y];
    }
    out[x] = acc;
  }
}

// col[h][j] = sum over chunks; slash[h][o] = sum over the (key block, chunk)
// partials that contain offset o, both in a fixed order with fp64 accumulation.
__global__ __launch_bounds__(256) void score_finalize_kernel(ScoreParams P, const float* colpart) {
  const int bh = blockIdx.y;
  const int x = blockIdx.x * 256 + threadIdx.x;
  const int S = P.S;
  if (x >= S) return;
  const int r0 = S - P.n_s;
  double c = 0.0, s = 0.0;
  for (int ch = 0; ch < P.n_chunks; ++ch) {
    int row0 = r0 + ch * QC;
    int row_end = min(row0 + QC, S);
    // column x
    if (row_end - 1 >= (x / KB) * KB) c += (double)colpart[((size_t)bh * P.n_chunks + ch) * S + x];
    // offset x: slot = x - row0 + 128 kb + 127 in [0, WIN)
    int kb_lo = row0 - x - 127;                       // 128 kb >= kb_lo
    kb_lo = (kb_lo <= 0) ? 0 : (kb_lo + KB - 1) / KB;
    int kb_hi_num = row0 - x + WIN - 1 - 127;         // 128 kb <= kb_hi_num
    if (kb_hi_num < 0) continue;
    int kb_hi = min(kb_hi_num / KB, P.n_kblocks - 1);
    for (int kb = kb_lo; kb <= kb_hi; ++kb) {
      if (row_end - 1 < kb * KB) break;               // block not live for this chunk
      int slot = x - row0 + KB * kb + 127;
      s += (double)P.partial[(((size_t)bh * P.n_kblocks + kb) * P.n_chunks + ch) * WIN + slot];
    }
  }
  P.col[(size_t)bh * S + x] = (float)c;
  P.slash[(size_t)bh * S + x] = (float)s;
}

}  // namespace

void score_geometry(int S, int n_s, int* n_kblocks, int* n_chunks, int* chunk_rows, int* win) {
  *n_kblocks = (S + KB - 1) / KB;
  *n_chunks = (n_s + QC - 1) / QC;
  *chunk_rows = QC;
  *win = WIN;
}

size_t score_partial_floats(int S, int n_s, int n_bh) {
  int nk, nc, cr, w;
  score_geometry(S, n_s, &nk, &nc, &cr, &w);
  // slash partials followed by per-chunk column sums
  return (size_t)n_bh * nk * nc * w + (size_t)n_bh * nc * S;
}

static ScoreParams with_geometry(const ScoreParams& P0) {
  ScoreParams P = P0;
  int cr;
  score_geometry(P.S, P.n_s, &P.n_kblocks, &P.n_chunks, &cr, &P.win);
  P.chunk_rows = cr;
  return P;
}

static float* column_partials(const ScoreParams& P) {
  return P.partial + (size_t)P.n_bh * P.n_kblocks * P.n_chunks * P.win;
}

hipError_t launch_score_accumulate(const ScoreParams& P0, hipStream_t st) {
  ScoreParams A = with_geometry(P0);
  A.col = column_partials(A);      // the accumulate kernel writes per-chunk column sums
  size_t shmem = 4 * WWIN * 4 + 2 * QSTAGE_B;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_accumulate_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  if (e != hipSuccess) return e;
  dim3 grid(A.n_kblocks, A.n_chunks, A.n_bh);
  hipLaunchKernelGGL(score_accumulate_kernel, grid, dim3(256), shmem, st, A);
  return hipGetLastError();
}

hipError_t launch_score_finalize(const ScoreParams& P0, hipStream_t st) {
  ScoreParams P = with_geometry(P0);
  dim3 g2((P.S + 255) / 256, P.n_bh);
  hipLaunchKernelGGL(score_finalize_kernel, g2, dim3(256), 0, st, P, column_partials(P));
  return hipGetLastError();
}

}  // namespace sa
