// Stage 1, pass 2 (Algorithm 1 stage 1; Sec. 4.2): with the row log-sum-exp of
// every sampled query known, recompute p_ij = exp(q_i.k_j*scale - lse_i) tile by
// tile and accumulate it down the key columns and along the diagonals.
//
// One workgroup = 256 keys (4 waves x 64 keys, K resident in registers as two
// MFMA B operands), taking the chunks of 1024 sampled rows one after the other.  S = Q K^T is formed 32 rows at
// a time, so one lane holds ONE key (lane % 32) and 16 query rows: the column
// sum is in-lane arithmetic.  For the diagonals, the tile (row block b, key
// sub-block kb) has exactly the lane/register -> diagonal mapping of every other
// tile with the same b - kb, so tiles of one diagonal class are first added up
// in registers.  A finished class (16 registers x 32 lanes per lane half, 59
// distinct diagonals) is first summed along its diagonals across lanes - register
// r is pulled from the lane e(r) positions on (one ds_bpermute each, all 16 in
// flight together), which leaves every lane with the totals of two diagonals - and
// then added into a window in LDS that is private to the wave and to the lane half
// with two read-add-writes per lane whose slots no other lane touches.
// The eight windows are combined in a fixed order into one partial per (key
// block, chunk) and a second kernel adds the partials in a fixed order.  No
// float atomics anywhere: repeated runs give identical bits.
#include <type_traits>

#include "sa_device.h"
#include "sa_kernels.h"

namespace sa {

namespace {

typedef __attribute__((address_space(3))) float lds_f32;   // LDS-qualified, keeps ds_ instructions

constexpr int KB = 256;          // keys per workgroup (4 waves x 2 sub-blocks x 32)
constexpr int QC = 1024;         // sampled rows per chunk
constexpr int WWIN = QC + 64;    // floats in one (wave, lane half) diagonal window
constexpr int WIN = QC + 256;    // floats in the combined (key block, chunk) partial
constexpr int QROW_B = 272;      // bytes per staged Q row
constexpr int QSTAGE_B = 32 * QROW_B + 32 * 4;   // 32 rows + 32 lse values

__global__ __launch_bounds__(256, 2) void score_accumulate_kernel(ScoreParams P) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  float* win = reinterpret_cast<float*>(smem);                  // [4 waves][2 halves][WWIN]
  char* qstage = smem + 8 * WWIN * 4;                           // [2][QSTAGE_B]

  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int ql = lane & 31, hf = lane >> 5;
  const int kb = blockIdx.x, bh = blockIdx.z;
  const int S = P.S;
  const int r0 = P.row_first;                       // sampled rows [r0, r_end)
  const int r_end = r0 + P.n_s;
  const int j0 = kb * KB;
  if (r_end - 1 < j0) return;                       // every sampled row lies above these keys
  const int jw = j0 + 64 * wave;
  const int bkv = bh / P.group;
  const float c2 = P.scale_log2;

  // K^T operands of this wave's 2 x 32 keys (zero beyond the sequence end)
  bf16x8 kf[2][8];
#pragma unroll
  for (int sb = 0; sb < 2; ++sb) {
    int j = jw + 32 * sb + ql;
    const uint16_t* krow = P.k + ((size_t)bkv * S + min(j, S - 1)) * kHeadDim;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 v = *reinterpret_cast<const uint4*>(krow + ks * 16 + hf * 8);
      if (j >= S) v = make_uint4(0u, 0u, 0u, 0u);
      kf[sb][ks] = as_bf16x8(v);
    }
  }
  const uint16_t* qbase = P.q + (size_t)bh * S * kHeadDim;
  const float* lbase = P.lse + (size_t)bh * P.n_s;
  const int qrow_t = tid >> 4, qcol_t = tid & 15;
  // slot of (row rb + m, key jw + 32 sb + ql) in this wave's window:
  //   32 (b - sb + 1) + (m - ql) + 31
  // The class sum.  Register r of lane ql holds the diagonal e(r) - ql, with e(r) =
  // 8 (r / 4) + r % 4, of 59 in all (-31 .. 27).  Lane L collects diagonal L - 31 (from
  // the registers with e(r) <= L, lane e(r) + 31 - L) and diagonal L + 1 (from the
  // others, lane e(r) - 1 - L): for each r one pull from lane (e(r) + 31 - L) mod 32 of
  // its own half, credited to the one or the other by 0/1 factors (the products are
  // exact).  Their window slots are 32 b' + L and 32 b' + 32 + L.
  float* mywin = win + (wave * 2 + hf) * WWIN + ql + 4 * hf;
  int pull[16];
  float first[16], second[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int e = 8 * (r >> 2) + (r & 3);
    pull[r] = 4 * (((e + 31 - ql) & 31) + 32 * hf);
    first[r] = (ql >= e) ? 1.f : 0.f;
    second[r] = 1.f - first[r];
  }

  // The keys stay in registers while the workgroup goes through the chunks of sampled
  // rows one after the other (each chunk has its own window and its own partial sums).
  for (int ch = 0; ch < P.n_chunks; ++ch) {
  const int row0 = r0 + ch * QC;                    // first row of the chunk
  const int row_end = min(row0 + QC, r_end);        // one past the last row
  if (row_end - 1 < j0) continue;                   // chunk entirely above these keys (uniform)
  for (int x = tid; x < 8 * WWIN; x += 256) win[x] = 0.f;

  // first 32-row block that reaches the keys of the workgroup, rounded down to even
  const int nblk = (row_end - row0 + 31) / 32;
  const int b_first = ((j0 > row0) ? (j0 - row0) / 32 : 0) & ~1;

  uint4 pq0, pq1;
  float pl = 0.f;
  auto load_block = [&](int b) {
    int rb = row0 + 32 * b;
    int i0 = rb + qrow_t, i1 = i0 + 16;
    pq0 = make_uint4(0u, 0u, 0u, 0u);
    pq1 = make_uint4(0u, 0u, 0u, 0u);
    if (i0 < S) pq0 = *reinterpret_cast<const uint4*>(qbase + (size_t)i0 * kHeadDim + qcol_t * 8);
    if (i1 < S) pq1 = *reinterpret_cast<const uint4*>(qbase + (size_t)i1 * kHeadDim + qcol_t * 8);
    if (tid < 32) {
      int i = rb + tid;
      pl = (i < r_end) ? lbase[i - r0] * kLog2e : 0.f;
    }
  };
  auto store_block = [&](char* st) {
    *reinterpret_cast<uint4*>(st + qrow_t * QROW_B + qcol_t * 16) = pq0;
    *reinterpret_cast<uint4*>(st + (qrow_t + 16) * QROW_B + qcol_t * 16) = pq1;
    if (tid < 32) reinterpret_cast<float*>(st + 32 * QROW_B)[tid] = pl;
  };

  if (b_first < nblk) {
    load_block(b_first);
    store_block(qstage + (b_first & 1) * QSTAGE_B);
  }
  __syncthreads();

  float colacc[2] = {0.f, 0.f};
  f32x16 dacc[2];                 // diagonal classes (b - sb) even / odd
#pragma unroll
  for (int r = 0; r < 16; ++r) { dacc[0][r] = 0.f; dacc[1][r] = 0.f; }
  // add class C (held in dacc[C]) into the window at block position bpos.  The
  // registers are not cleared: the first tile of the next class to use them (always a
  // sub-block-0 tile) assigns instead of adding.
  auto flush_class = [&](f32x16& acc, int bpos) {
    float a1 = 0.f, a2 = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float v = __int_as_float(__builtin_amdgcn_ds_bpermute(pull[r], __float_as_int(acc[r])));
      a1 = fmaf(v, first[r], a1);
      a2 = fmaf(v, second[r], a2);
    }
    volatile lds_f32* s1 = (volatile lds_f32*)(mywin + 32 * bpos);
    *s1 = *s1 + a1;
    if (ql < 27) {                                   // diagonals 28 .. 32 do not exist
      volatile lds_f32* s2 = (volatile lds_f32*)(mywin + 32 * bpos + 32);
      *s2 = *s2 + a2;
    }
  };

  // one 32-row block against both key sub-blocks; PAR = parity of b (compile time)
  auto do_block = [&](int b, auto par_tag) {
    constexpr int PAR = decltype(par_tag)::value;
    const char* st = qstage + (b & 1) * QSTAGE_B;
    const int rb = row0 + 32 * b;
    if (rb + 31 >= jw) {            // some row reaches this wave's first sub-block
      bf16x8 qf[8];
      const char* qp = st + ql * QROW_B + hf * 16;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(qp + ks * 32));
      const float* ls = reinterpret_cast<const float*>(st + 32 * QROW_B);
      float lv[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4 l4 = *reinterpret_cast<const float4*>(ls + 8 * g + 4 * hf);
        lv[4 * g] = l4.x; lv[4 * g + 1] = l4.y; lv[4 * g + 2] = l4.z; lv[4 * g + 3] = l4.w;
      }
      // both sub-blocks' products first (alternating accumulators), then their
      // exponentials and sums: the matrix pipe works through the second product while
      // the vector pipe starts on the first.  A sub-block that no row of the block
      // reaches yet is computed all the same and masked to zero by the edge path.
      f32x16 s2[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) { s2[0][r] = 0.f; s2[1][r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        s2[0] = mfma_32x32x16(qf[ks], kf[0][ks], s2[0]);
        s2[1] = mfma_32x32x16(qf[ks], kf[1][ks], s2[1]);
      }
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        const int jsb = jw + 32 * sb;
        // element r: query row rb + 8*(r/4) + 4*hf + r%4, key jsb + ql
        const bool edge = (rb < jsb + 32) || (rb + 32 > r_end);
        const int j_me = jsb + ql;
        // straight-line code: all exponentials first, the (rare) edge mask in one
        // wave-uniform branch, then the sums
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) p[r] = fast_exp2(fmaf(s2[sb][r], c2, -lv[r]));
        if (edge) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            int i = rb + 8 * (r >> 2) + 4 * hf + (r & 3);
            p[r] = (i >= j_me && i < r_end) ? p[r] : 0.f;
          }
        }
        float csum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          csum += p[r];
          // tile (b, 0) opens class b, tile (b, 1) completes class b - 1
          if (sb == 0) dacc[PAR & 1][r] = p[r]; else dacc[(PAR + 1) & 1][r] += p[r];
        }
        colacc[sb] += csum;
      }
    } else {
      // no row of the block reaches this wave's keys yet: class b opens empty
#pragma unroll
      for (int r = 0; r < 16; ++r) dacc[PAR & 1][r] = 0.f;
    }
    // class b - 1 (tiles (b-1, 0) and (b, 1)) is complete: add it into the window
    flush_class(dacc[(PAR + 1) & 1], b);       // window position 32 * ((b - 1) + 1)
  };

  for (int b = b_first; b < nblk; b += 2) {
    // even block
    if (b + 1 < nblk) load_block(b + 1);
    do_block(b, std::integral_constant<int, 0>{});
    if (b + 1 < nblk) store_block(qstage + ((b + 1) & 1) * QSTAGE_B);
    __syncthreads();
    if (b + 1 >= nblk) break;
    // odd block
    if (b + 2 < nblk) load_block(b + 2);
    do_block(b + 1, std::integral_constant<int, 1>{});
    if (b + 2 < nblk) store_block(qstage + ((b + 2) & 1) * QSTAGE_B);
    __syncthreads();
  }
  // the last class (only its sub-block-0 tile exists): b = nblk - 1
  if (((nblk - 1) & 1) == 0) flush_class(dacc[0], nblk); else flush_class(dacc[1], nblk);
  __syncthreads();

  // column sums of this chunk (both lane halves hold disjoint rows)
#pragma unroll
  for (int sb = 0; sb < 2; ++sb) {
    float ctot = colacc[sb] + swap_half(colacc[sb]);
    int j = jw + 32 * sb + ql;
    if (hf == 0 && j < S) P.col[((size_t)bh * P.n_chunks + ch) * S + j] = ctot;
  }

  // combine the eight windows: slot x <-> offset x + (row0 - j0 - 255);
  // wave w slot y <-> offset y + (row0 - j0 - 64 w - 63)
  float* out = P.partial + (((size_t)bh * P.n_kblocks + kb) * P.n_chunks + ch) * WIN;
  for (int x = tid; x < WIN; x += 256) {
    float acc = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      int y = x - 192 + 64 * w;
      if (y >= 0 && y < WWIN) acc += win[(w * 2) * WWIN + y] + win[(w * 2 + 1) * WWIN + y];
    }
    out[x] = acc;
  }
  __syncthreads();     // the windows are cleared for the next chunk only after everyone has read them
  }  // chunks
}

// col[h][j] = sum over chunks; slash[h][o] = sum over the (key block, chunk)
// partials that contain offset o, both in a fixed order with fp64 accumulation.
__global__ __launch_bounds__(256) void score_finalize_kernel(ScoreParams P, const float* colpart) {
  const int bh = blockIdx.y;
  const int x = blockIdx.x * 256 + threadIdx.x;
  const int S = P.S;
  if (x >= S) return;
  const int r0 = P.row_first;
  double c = 0.0, s = 0.0;
  for (int ch = 0; ch < P.n_chunks; ++ch) {
    int row0 = r0 + ch * QC;
    int row_end = min(row0 + QC, r0 + P.n_s);
    // column x
    if (row_end - 1 >= (x / KB) * KB) c += (double)colpart[((size_t)bh * P.n_chunks + ch) * S + x];
    // offset x: slot = x - row0 + KB kb + (KB - 1) in [0, WIN)
    int kb_lo = row0 - x - (KB - 1);                  // KB kb >= kb_lo
    kb_lo = (kb_lo <= 0) ? 0 : (kb_lo + KB - 1) / KB;
    int kb_hi_num = row0 - x + WIN - 1 - (KB - 1);    // KB kb <= kb_hi_num
    if (kb_hi_num < 0) continue;
    int kb_hi = min(kb_hi_num / KB, P.n_kblocks - 1);
    for (int kb = kb_lo; kb <= kb_hi; ++kb) {
      if (row_end - 1 < kb * KB) break;               // block not live for this chunk
      int slot = x - row0 + KB * kb + (KB - 1);
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
  size_t shmem = 8 * WWIN * 4 + 2 * QSTAGE_B;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_accumulate_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  if (e != hipSuccess) return e;
  dim3 grid(A.n_kblocks, 1, A.n_bh);       // a workgroup takes the row chunks in turn
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
