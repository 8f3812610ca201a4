// Stage 2 (Algorithm 1 stage 2; Sec. 4.3): per head and direction, the fewest
// strips whose score mass reaches alpha * total, ties to the lower index.
//
// Sorting is not needed to find the cut.  With candidates ordered by (score
// descending, index ascending) the kept set is {score > v} plus the first m
// candidates with score == v, for the cut value v.  v is found by a most-
// significant-digit radix descent over the fp32 bit patterns (non-negative
// floats order like their bits): the exponent first, then the mantissa in
// digits of 8, 8 and 7 bits.  Each pass builds a histogram, over the candidates
// that match the digits fixed so far, of (count, sum of the 23-bit mantissas);
// all candidates of a bin share their exponent, so the bin's score mass is
// (count * 2^23 + mantissa sum) * 2^(e - 150) EXACTLY, from integer sums whose
// order cannot matter.  One thread then walks the bins from the top, adding
// their masses in fp64 in that fixed order, until the running sum reaches the
// target.  Nothing in the kernel adds floating-point numbers atomically:
// repeated runs give identical lists.
//
// The histogram lives in LDS and is updated with one 64-bit integer atomic per
// candidate (count in the upper bits, mantissa sum below).  Scores of one head
// crowd into a few exponents, and atomics of one wave to one address are served
// one after the other; so every bin has kCopies copies, indexed by lane % kCopies
// (then a wave's atomics land on distinct addresses and banks), which are added
// up before the walk.
//
// A last double sweep writes the kept indices in ascending order: every wave owns
// a contiguous segment of the candidates, counts what it will keep, and after one
// exchange of the counts writes its part of the list.  One workgroup per problem.
#include "sa_device.h"
#include "sa_kernels.h"

namespace sa {

namespace {

constexpr int NT = 1024;
constexpr int NW = NT / 64;
constexpr int kCopies = 32;                 // copies of every histogram bin
constexpr int kCntShift = 43;               // packed bin: count << 43 | mantissa sum (2^24 candidates at most:
                                            // a copy sees 2^19 of them, mantissa sum < 2^42, count < 2^20)
constexpr int kBatch = 16;                  // scores a lane requests before it uses the first
constexpr size_t kSelectLds = 256 * kCopies * sizeof(unsigned long long);

// the bit pattern a score is ranked by: negative, infinite and NaN scores carry no
// mass and rank with the zeros
__device__ __forceinline__ unsigned int score_key(float v) {
  const unsigned int u = __float_as_uint(v);
  return (v > 0.0f && u < 0x7F800000u) ? u : 0u;
}

__global__ __launch_bounds__(NT) void select_kernel(SelectParams P) {
  extern __shared__ __attribute__((aligned(16))) unsigned long long hist[];   // [256 bins][kCopies]
  __shared__ unsigned long long hms[256];     // sum of the mantissas per bin
  __shared__ unsigned int hcnt[256];
  __shared__ double bsum[256];                // mass per bin
  __shared__ double sh_above, sh_target;
  __shared__ unsigned int sh_prefix, sh_m, sh_done;
  __shared__ unsigned int w_gt[NW], w_tie[NW];

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

  // every wave owns a contiguous run of whole 64-candidate groups
  const int n_groups = (S + 63) / 64;
  const int g_lo = (int)((long long)n_groups * wave / NW), g_hi = (int)((long long)n_groups * (wave + 1) / NW);

  if (tid == 0) { sh_above = 0.0; sh_prefix = 0u; sh_done = 0u; sh_m = 0u; }
  // digit p: bits [shift, shift + width) of the 31-bit key
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = (pass == 3) ? 0 : 23 - 8 * pass;
    const int above_shift = (pass == 0) ? 31 : 31 - 8 * pass;    // bits from here up are fixed
    const unsigned int dmask = (pass == 3) ? 127u : 255u;
    for (int x = tid; x < 256 * kCopies; x += NT) hist[x] = 0ull;
    __syncthreads();
    const unsigned int prefix = sh_prefix;
    unsigned long long* my_hist = hist + (lane & (kCopies - 1));
    // kBatch loads in flight per lane: a wave that waits for every score before it asks
    // for the next spends the pass waiting
    for (int g0 = g_lo; g0 < g_hi; g0 += kBatch) {
      float v[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int i = (g0 + u) * 64 + lane;
        v[u] = (g0 + u < g_hi && i < S) ? sc[i] : 0.0f;
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const unsigned int key = score_key(v[u]);
        const bool in = g0 + u < g_hi && (g0 + u) * 64 + lane < S;
        const bool live = in && (pass == 0 || (key >> above_shift) == (prefix >> above_shift));
        const unsigned int b = (key >> shift) & dmask;
        if (live) atomicAdd(my_hist + b * kCopies, (1ull << kCntShift) | (unsigned long long)(key & 0x7FFFFFu));
      }
    }
    __syncthreads();
    if (tid < 256) {
      // the copies of bin tid, each thread starting at another copy (spreads the LDS banks)
      unsigned long long c = 0ull, ms = 0ull;
      for (int x = 0; x < kCopies; ++x) {
        const unsigned long long v = hist[tid * kCopies + ((x + tid) & (kCopies - 1))];
        c += v >> kCntShift;
        ms += v & ((1ull << kCntShift) - 1ull);
      }
      hcnt[tid] = (unsigned int)c;
      hms[tid] = ms;
    }
    __syncthreads();
    if (tid < 256) {
      // exponent of the bin's candidates: the bin itself in the first pass
      const unsigned int e = (pass == 0) ? (unsigned int)tid : (prefix >> 23);
      const unsigned long long units = (e > 0u ? ((unsigned long long)hcnt[tid] << 23) : 0ull) + hms[tid];
      bsum[tid] = ldexp((double)units, e > 0u ? (int)e - 150 : -149);   // exact: units < 2^53
    }
    __syncthreads();
    if (tid == 0) {
      if (pass == 0) {
        double total = 0.0;
        for (int b = 255; b >= 0; --b) total += bsum[b];
        sh_target = alpha * total;
        if (!(sh_target > 0.0)) sh_done = 1u;   // alpha == 0 or no mass: keep nothing
      }
      if (!sh_done) {
        double above = sh_above;
        int chosen = -1, last_b = 0;
        double last_above = above;
        for (int b = (int)dmask; b >= 0; --b) {
          if (hcnt[b] == 0u) continue;
          if (above + bsum[b] >= sh_target) { chosen = b; break; }
          last_b = b; last_above = above;
          above += bsum[b];
        }
        if (chosen < 0) {   // only by fp64 rounding of the running sum: cut inside the lowest non-empty bin
          chosen = last_b; above = last_above;
        }
        sh_above = above;
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
    __syncthreads();
    if (sh_done) {
      if (tid == 0) *cnt_out = 0;
      return;
    }
  }

  // ---- ordered compaction: count per wave segment, exchange, write -------------
  const unsigned int vkey = sh_prefix;
  const unsigned int m = sh_m;
  const unsigned long long lt = (1ull << lane) - 1ull;
  unsigned int n_gt = 0u, n_tie = 0u;
  for (int g0 = g_lo; g0 < g_hi; g0 += kBatch) {
    float v[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int i = (g0 + u) * 64 + lane;
      v[u] = (g0 + u < g_hi && i < S) ? sc[i] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const unsigned int key = score_key(v[u]);
      const bool in = g0 + u < g_hi && (g0 + u) * 64 + lane < S;
      n_gt += (unsigned int)__popcll(__ballot(in && key > vkey));
      n_tie += (unsigned int)__popcll(__ballot(in && key == vkey));
    }
  }
  if (lane == 0) { w_gt[wave] = n_gt; w_tie[wave] = n_tie; }
  __syncthreads();
  unsigned int tie_run = 0u, pos_run = 0u;   // ties before this wave's segment; list position of its first kept index
  for (int w = 0; w < wave; ++w) {
    const unsigned int t = w_tie[w];
    const unsigned int kept_ties = (tie_run >= m) ? 0u : ((m - tie_run < t) ? m - tie_run : t);
    pos_run += w_gt[w] + kept_ties;
    tie_run += t;
  }
  for (int g0 = g_lo; g0 < g_hi; g0 += kBatch) {
    float v[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int i = (g0 + u) * 64 + lane;
      v[u] = (g0 + u < g_hi && i < S) ? sc[i] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int i = (g0 + u) * 64 + lane;
      const unsigned int key = score_key(v[u]);
      const bool in = g0 + u < g_hi && i < S;
      const bool gt = in && key > vkey;
      const bool tie = in && key == vkey;
      const unsigned long long bt = __ballot(tie);
      const unsigned int trank = tie_run + (unsigned int)__popcll(bt & lt);
      const bool sel = gt || (tie && trank < m);
      const unsigned long long bs = __ballot(sel);
      if (sel) idx[pos_run + (unsigned int)__popcll(bs & lt)] = i;
      tie_run += (unsigned int)__popcll(bt);
      pos_run += (unsigned int)__popcll(bs);
    }
  }
  if (wave == NW - 1 && lane == 0) *cnt_out = (int)pos_run;
}

}  // namespace

hipError_t launch_select(const SelectParams& P, hipStream_t st) {
  if (P.n_prob <= 0) return hipSuccess;
  const int sets = (P.scores2 != nullptr) ? 2 : 1;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSelectLds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(select_kernel, dim3(sets * P.n_prob), dim3(NT), kSelectLds, st, P);
  return hipGetLastError();
}

}  // namespace sa
