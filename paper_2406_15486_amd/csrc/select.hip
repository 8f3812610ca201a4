// Stage 2 (Algorithm 1 stage 2; Sec. 4.3): per head and direction, the fewest
// strips whose score mass reaches alpha * total, ties to the lower index.
//
// Sorting is not needed to find the cut.  With candidates ordered by (score
// descending, index ascending) the kept set is {score > v} plus the first m
// candidates with score == v, for the cut value v.  v is found by a most-
// significant-digit radix descent over the fp32 bit patterns (non-negative
// floats order like their bits): four passes of 8 bits, each building a
// 256-bin histogram of (count, fp64 score sum) of the candidates that match
// the digits fixed so far, then walking the bins from the top until the
// running fp64 sum reaches the target.  A last pass writes the kept indices in
// ascending order by stream compaction.  One workgroup per problem.
#include "sa_device.h"
#include "sa_kernels.h"

namespace sa {

namespace {

constexpr int NT = 1024;
constexpr int NW = NT / 64;

__global__ __launch_bounds__(NT) void select_kernel(SelectParams P) {
  __shared__ double hsum[256];
  __shared__ unsigned int hcnt[256];
  __shared__ double sh_above, sh_target;
  __shared__ unsigned int sh_prefix, sh_above_cnt, sh_m, sh_done;
  __shared__ unsigned int wtie[NW], wsel[NW];
  __shared__ unsigned int tie_base, sel_base;

  // workgroups [0, n_prob) take the first set of problems, [n_prob, 2 n_prob) the
  // second one (the two directions of a layer in one launch)
  const bool second = (int)blockIdx.x >= P.n_prob;
  const int prob = second ? (int)blockIdx.x - P.n_prob : (int)blockIdx.x;
  const int S = P.S;
  const float* sc = (second ? P.scores2 : P.scores) + (size_t)prob * S;
  int32_t* idx = (second ? P.idx2 : P.idx) + (size_t)prob * S;
  int32_t* cnt_out = (second ? P.cnt2 : P.cnt) + prob;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double alpha = (double)(second ? P.alpha2 : P.alpha);

  if (alpha >= 1.0) {                       // keep everything
    for (int i = tid; i < S; i += NT) idx[i] = i;
    if (tid == 0) *cnt_out = S;
    return;
  }

  if (tid == 0) { sh_above = 0.0; sh_prefix = 0u; sh_above_cnt = 0u; sh_done = 0u; sh_m = 0u; }
  unsigned int mask = 0u;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) { hsum[tid] = 0.0; hcnt[tid] = 0u; }
    __syncthreads();
    const unsigned int prefix = sh_prefix;
    for (int i = tid; i < S; i += NT) {
      float v = sc[i];
      unsigned int key = __float_as_uint(v) & 0x7FFFFFFFu;
      if ((key & mask) == prefix) {
        unsigned int b = (key >> shift) & 255u;
        atomicAdd(&hcnt[b], 1u);
        atomicAdd(&hsum[b], (double)__uint_as_float(key));
      }
    }
    __syncthreads();
    if (tid == 0) {
      if (pass == 0) {
        double total = 0.0;
        for (int b = 255; b >= 0; --b) total += hsum[b];
        sh_target = alpha * total;
        if (!(sh_target > 0.0)) sh_done = 1u;   // alpha == 0 or no mass: keep nothing
      }
      if (!sh_done) {
        double above = sh_above;
        unsigned int acnt = sh_above_cnt;
        int chosen = -1, last_b = 0;
        double last_above = above;
        unsigned int last_acnt = acnt;
        for (int b = 255; b >= 0; --b) {
          if (hcnt[b] == 0u) continue;
          if (above + hsum[b] >= sh_target) { chosen = b; break; }
          last_b = b; last_above = above; last_acnt = acnt;
          above += hsum[b];
          acnt += hcnt[b];
        }
        if (chosen < 0) {   // only by fp64 rounding of the bin sums: cut inside the lowest non-empty bin
          chosen = last_b; above = last_above; acnt = last_acnt;
        }
        sh_above = above;
        sh_above_cnt = acnt;
        sh_prefix = prefix | ((unsigned int)chosen << shift);
        if (pass == 3) {
          // all candidates left share the exact value v: how many are needed
          double v = (double)__uint_as_float(sh_prefix);
          unsigned int c = hcnt[chosen];
          unsigned int m = 1u;
          if (v > 0.0) {
            double need = (sh_target - above) / v;
            m = (need <= 1.0) ? 1u : (need >= (double)c ? c : (unsigned int)need);
            while (m > 1u && above + (double)(m - 1u) * v >= sh_target) --m;
            while (m < c && above + (double)m * v < sh_target) ++m;
          }
          sh_m = m;
        }
      }
    }
    mask |= 255u << shift;
    __syncthreads();
    if (sh_done) {
      if (tid == 0) *cnt_out = 0;
      return;
    }
  }

  const unsigned int vkey = sh_prefix;
  const unsigned int m = sh_m;
  if (tid == 0) { tie_base = 0u; sel_base = 0u; }
  __syncthreads();
  for (int i0 = 0; i0 < S; i0 += NT) {
    int i = i0 + tid;
    unsigned int key = (i < S) ? (__float_as_uint(sc[i]) & 0x7FFFFFFFu) : 0u;
    bool gt = (i < S) && key > vkey;
    bool tie = (i < S) && key == vkey;
    unsigned long long bt = __ballot(tie);
    if (lane == 0) wtie[wave] = __popcll(bt);
    __syncthreads();
    unsigned int trank = tie_base;
    for (int w = 0; w < wave; ++w) trank += wtie[w];
    trank += __popcll(bt & ((1ull << lane) - 1ull));
    bool sel = gt || (tie && trank < m);
    unsigned long long bs = __ballot(sel);
    if (lane == 0) wsel[wave] = __popcll(bs);
    __syncthreads();
    unsigned int pos = sel_base;
    for (int w = 0; w < wave; ++w) pos += wsel[w];
    pos += __popcll(bs & ((1ull << lane) - 1ull));
    if (sel) idx[pos] = i;
    __syncthreads();
    if (tid == 0) {
      unsigned int t = 0u, s = 0u;
      for (int w = 0; w < NW; ++w) { t += wtie[w]; s += wsel[w]; }
      tie_base += t;
      sel_base += s;
    }
    __syncthreads();
  }
  if (tid == 0) *cnt_out = (int)sel_base;
}

}  // namespace

hipError_t launch_select(const SelectParams& P, hipStream_t st) {
  if (P.n_prob <= 0) return hipSuccess;
  const int sets = (P.scores2 != nullptr) ? 2 : 1;
  hipLaunchKernelGGL(select_kernel, dim3(sets * P.n_prob), dim3(NT), 0, st, P);
  return hipGetLastError();
}

}  // namespace sa
