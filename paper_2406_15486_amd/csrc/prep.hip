// Small data-movement kernels around the attention kernels:
//  - gather_transpose: V -> V^T (so the PV product reads 16-byte MFMA operands)
//    and, for the strip-masked path, K/V rows gathered by selected column index
//    into compact per-head arrays (Algorithm 1, merge_index: column strips);
//  - mask_prep: the selected columns and offsets (plus the local window) as
//    bitmaps, and the list of 64-key tile diagonals that hold at least one kept
//    offset (Algorithm 1, merge_index: slash strips extended over the matrix);
//  - block granularity (Algorithm 1, block_reduction with blk > 1): token scores
//    summed over blocks, and the block lists turned into the same metadata.
#include "sa_device.h"
#include "sa_kernels.h"

namespace sa {

namespace {

constexpr int GT_ROW_B = 260;   // bytes per gathered row in LDS (256 + 4 pad)

__global__ __launch_bounds__(256) void gather_transpose_kernel(GatherParams P) {
  __shared__ __attribute__((aligned(16))) char tile[64 * GT_ROW_B];
  const int g = blockIdx.y;
  const int c0 = blockIdx.x * 64;
  const int cnt = P.cnt ? min(max(P.cnt[g], 0), P.S) : P.S;
  const int tid = threadIdx.x;
  if (P.idx_pad != nullptr) {
    // padded copy of the index list: INT_MAX marks "no column"
    if (tid < 64) {
      int c = c0 + tid;
      if (c < P.idx_pad_stride)
        P.idx_pad[(size_t)g * P.idx_pad_stride + c] = (c < cnt) ? P.idx[(size_t)g * P.idx_stride + c] : 0x7FFFFFFF;
    }
  }
  if (P.out_t == nullptr && P.out_rows == nullptr) return;   // only the padded index list was wanted
  if (c0 >= ((cnt + 63) & ~63)) return;   // nothing reads beyond the last partial tile
  // rows of an earlier segment see no key at or after their end: a tile of the ascending
  // list that starts there is left alone
  if (P.key_limit > 0 && P.idx != nullptr && P.idx[(size_t)g * P.idx_stride + c0] >= P.key_limit) return;
  const uint16_t* src = P.src + (size_t)((P.head0 + g) / P.group) * P.S * kHeadDim;
#pragma unroll
  for (int n = 0; n < 4; ++n) {
    int c = tid + 256 * n;
    int row = c >> 4, col = c & 15;
    int cc = c0 + row;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (cc < cnt) {
      int j = P.idx ? P.idx[(size_t)g * P.idx_stride + cc] : cc;
      j = min(max(j, 0), P.S - 1);   // a malformed list must not read out of bounds
      v = *reinterpret_cast<const uint4*>(src + (size_t)j * kHeadDim + col * 8);
    }
    if (P.out_rows != nullptr)
      *reinterpret_cast<uint4*>(P.out_rows + ((size_t)g * P.C_pad + cc) * kHeadDim + col * 8) = v;
    uint32_t* dst = reinterpret_cast<uint32_t*>(tile + row * GT_ROW_B + col * 16);
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
  }
  if (P.out_t == nullptr) return;   // rows-only gather
  __syncthreads();
#pragma unroll
  for (int n = 0; n < 4; ++n) {
    int c = tid + 256 * n;
    int drow = c >> 3, kc = c & 7;
    uint16_t e[8];
#pragma unroll
    for (int x = 0; x < 8; ++x)
      e[x] = *reinterpret_cast<const uint16_t*>(tile + (8 * kc + x) * GT_ROW_B + drow * 2);
    uint4 v;
    v.x = e[0] | ((uint32_t)e[1] << 16);
    v.y = e[2] | ((uint32_t)e[3] << 16);
    v.z = e[4] | ((uint32_t)e[5] << 16);
    v.w = e[6] | ((uint32_t)e[7] << 16);
    *reinterpret_cast<uint4*>(P.out_t + ((size_t)g * kHeadDim + drow) * P.C_pad + c0 + 8 * kc) = v;
  }
}

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}

__global__ __launch_bounds__(256) void set_bits_kernel(MaskPrepParams P) {
  const int h = blockIdx.y;
  const int c = blockIdx.x * 256 + threadIdx.x;
  uint32_t* cb = P.col_bits + (size_t)h * P.cb_words;
  uint32_t* ob = P.off_bits + (size_t)h * P.rb_words;
  if (c < P.S && c < P.col_cnt[h]) {
    int j = P.col_idx[(size_t)h * P.S + c];
    if (j >= 0 && j < P.S) atomicOr(cb + (j >> 5), 1u << (j & 31));
  }
  if (P.slash_idx != nullptr && c < P.S && c < P.slash_cnt[h]) {
    int o = P.slash_idx[(size_t)h * P.S + c];
    if (o >= 0 && o < P.S) {
      int x = P.off_max - o;
      atomicOr(ob + (x >> 5), 1u << (x & 31));
    }
  }
  if (c < P.window && c < P.S) {
    int x = P.off_max - c;
    atomicOr(ob + (x >> 5), 1u << (x & 31));
  }
}

// any kept offset in [lo, hi] (0 <= lo <= hi)?  offset o sits at bit off_max - o
__device__ bool any_offset(const uint32_t* ob, int off_max, int lo, int hi) {
  int x_lo = off_max - hi, x_hi = off_max - lo;
  for (int w = x_lo >> 5; w <= (x_hi >> 5); ++w) {
    uint32_t m = 0xFFFFFFFFu;
    if (w == (x_lo >> 5)) m &= 0xFFFFFFFFu << (x_lo & 31);
    if (w == (x_hi >> 5)) m &= 0xFFFFFFFFu >> (31 - (x_hi & 31));
    if (ob[w] & m) return true;
  }
  return false;
}

// Tile diagonal d pairs the 256-row query tile starting at row i0 with the
// 64-key tile starting at key i0 + 192 - 64 d: it spans offsets
// [64 d - 255, 64 d + 63], the 32 rows of wave w (of 8) the 95 offsets from
// 64 d - 255 + 32 w on.  dlist = ascending d with at least one kept offset; an
// entry is d | (mask << 24), bit w of mask set when wave w sees a kept offset.
__global__ __launch_bounds__(256) void dlist_kernel(MaskPrepParams P) {
  __shared__ int wave_cnt[4];
  __shared__ int base;
  const int h = blockIdx.x;
  const uint32_t* ob = P.off_bits + (size_t)h * P.rb_words;
  int32_t* dl = P.dlist + (size_t)h * P.dlist_stride;
  const int nd = (P.S + 63) / 64 + 3;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) base = 0;
  __syncthreads();
  for (int d0 = 0; d0 < nd; d0 += 256) {
    int d = d0 + tid;
    uint32_t mask = 0;
    if (d < nd) {
      for (int w = 0; w < 8; ++w) {
        int lo = max(0, 64 * d - 255 + 32 * w), hi = min(P.S - 1, 64 * d - 255 + 32 * w + 94);
        if (lo <= hi && any_offset(ob, P.off_max, lo, hi)) mask |= 1u << w;
      }
    }
    const bool f = mask != 0;
    unsigned long long b = __ballot(f);
    if (lane == 0) wave_cnt[wave] = __popcll(b);
    __syncthreads();
    int pre = base;
    for (int w = 0; w < wave; ++w) pre += wave_cnt[w];
    if (f) dl[pre + __popcll(b & ((1ull << lane) - 1ull))] = (int32_t)((uint32_t)d | (mask << 24));
    __syncthreads();
    if (tid == 0) base += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
    __syncthreads();
  }
  if (tid == 0) P.dcnt[h] = base;
}

// ---- block granularity ----------------------------------------------------------
// out[g][b] = sum of in[g][b*blk .. (b+1)*blk) (the last block may be short): one
// wave per block, lanes stride the block, fp64 partial sums combined in a fixed
// butterfly order, so the result does not depend on the launch.
__global__ __launch_bounds__(256) void block_reduce_kernel(const float* in, float* out, int S, int blk, int nb) {
  const int g = blockIdx.y;
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (b >= nb) return;
  const float* src = in + (size_t)g * S;
  const int lo = b * blk, hi = min(lo + blk, S);
  double acc = 0.0;
  for (int e = lo + lane; e < hi; e += 64) acc += (double)src[e];
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if (lane == 0) out[(size_t)g * nb + b] = (float)acc;
}

// every offset 0 .. S-1 kept: bits off_max - (S-1) .. off_max of each head's bitmap
__global__ void all_offsets_kernel(uint32_t* off_bits, int n_bh, int rb_words, int S, int off_max) {
  const int x_lo = off_max - (S - 1), x_hi = off_max;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)n_bh * rb_words) return;
  const int w = (int)(i % rb_words);
  uint32_t m = 0u;
  if (w >= (x_lo >> 5) && w <= (x_hi >> 5)) {
    m = 0xFFFFFFFFu;
    if (w == (x_lo >> 5)) m &= 0xFFFFFFFFu << (x_lo & 31);
    if (w == (x_hi >> 5)) m &= 0xFFFFFFFFu >> (31 - (x_hi & 31));
  }
  off_bits[i] = m;
}

__device__ __forceinline__ int floor_div(int x, int y) { return x >= 0 ? x / y : -((-x + y - 1) / y); }

// selected key blocks -> the token columns they hold (ascending, as the strip path
// wants them).  Only the last block of the sequence can be short, and an ascending
// list has it last, so token slot c belongs to list entry c / blk.
__global__ __launch_bounds__(256) void expand_blocks_kernel(BlockPrepParams P) {
  const int h = blockIdx.y;
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int cnt = min(max(P.col_bcnt[h], 0), P.nb);
  const int32_t* bl = P.col_blk + (size_t)h * P.nb;
  if (c == 0) {
    int n = 0;
    if (cnt > 0) {
      int last = min(max(bl[cnt - 1], 0), P.nb - 1);
      n = (cnt - 1) * P.blk + min(P.blk, P.S - last * P.blk);
    }
    P.tok_cnt[h] = min(n, P.S);
  }
  if (c >= P.S) return;
  const int r = c / P.blk;
  int j = 0x7FFFFFFF;
  if (r < cnt) {
    int J = min(max(bl[r], 0), P.nb - 1);   // a malformed list must not lead out of bounds
    j = min(J * P.blk + c % P.blk, P.S - 1);
  }
  P.tok_idx[(size_t)h * P.S + c] = j;
}

// kept block diagonals (block row minus block column): a full block on diagonal
// delta spans the offsets blk*delta - (blk-1) .. blk*delta + (blk-1), so a selected
// block b of offsets [blk*b, blk*b + blk) lies on diagonals b and b + 1, and the
// window [0, w) on every diagonal with blk*delta - (blk-1) <= w - 1.
__global__ __launch_bounds__(256) void diag_bits_kernel(BlockPrepParams P) {
  const int h = blockIdx.y;
  const int c = blockIdx.x * 256 + threadIdx.x;
  uint32_t* db = P.diag_bits + (size_t)h * P.db_words;
  const int cnt = min(max(P.slash_bcnt[h], 0), P.nb);
  if (c < cnt) {
    int b = P.slash_blk[(size_t)h * P.nb + c];
    if (b >= 0 && b < P.nb) {
      atomicOr(db + (b >> 5), 1u << (b & 31));
      atomicOr(db + ((b + 1) >> 5), 1u << ((b + 1) & 31));
    }
  }
  if (c <= P.nb && (long long)c * P.blk - (P.blk - 1) <= (long long)P.window - 1)
    atomicOr(db + (c >> 5), 1u << (c & 31));
}

// The tile-diagonal list of the block mask.  With 256-row query tiles, 64-key tiles
// and blk in {64, 128, 256}, the 32 rows of wave w lie in one row block and the key
// tile of tile diagonal d in one column block, floor(32 w / blk) - floor((192 - 64 d)
// / blk) block diagonals apart whatever the query tile: the entry format is that of
// dlist_kernel, the per-wave bit now saying "this wave's block is kept".
__global__ __launch_bounds__(256) void dlist_block_kernel(BlockPrepParams P) {
  __shared__ int wave_cnt[4];
  __shared__ int base;
  const int h = blockIdx.x;
  const uint32_t* db = P.diag_bits + (size_t)h * P.db_words;
  int32_t* dl = P.dlist + (size_t)h * P.dlist_stride;
  const int nd = (P.S + 63) / 64 + 3;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) base = 0;
  __syncthreads();
  for (int d0 = 0; d0 < nd; d0 += 256) {
    int d = d0 + tid;
    uint32_t mask = 0;
    if (d < nd) {
      const int kb = floor_div(192 - 64 * d, P.blk);
      for (int w = 0; w < 8; ++w) {
        const int delta = (32 * w) / P.blk - kb;
        const int o_lo = 64 * d - 255 + 32 * w, o_hi = o_lo + 94;   // offsets the wave meets on this tile
        if (delta >= 0 && delta <= P.nb && o_hi >= 0 && o_lo <= P.S - 1 && ((db[delta >> 5] >> (delta & 31)) & 1u))
          mask |= 1u << w;
      }
    }
    const bool f = mask != 0;
    unsigned long long b = __ballot(f);
    if (lane == 0) wave_cnt[wave] = __popcll(b);
    __syncthreads();
    int pre = base;
    for (int w = 0; w < wave; ++w) pre += wave_cnt[w];
    if (f) dl[pre + __popcll(b & ((1ull << lane) - 1ull))] = (int32_t)((uint32_t)d | (mask << 24));
    __syncthreads();
    if (tid == 0) base += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
    __syncthreads();
  }
  if (tid == 0) P.dcnt[h] = base;
}

}  // namespace

hipError_t launch_block_reduce(const float* in, float* out, int n_rows, int S, int blk, hipStream_t st) {
  const int nb = (S + blk - 1) / blk;
  if (n_rows == 0 || nb == 0) return hipSuccess;
  hipLaunchKernelGGL(block_reduce_kernel, dim3((nb + 3) / 4, n_rows), dim3(256), 0, st, in, out, S, blk, nb);
  return hipGetLastError();
}

// Block lists -> the metadata of the strip path: token columns of the selected key
// blocks (tok_idx / tok_cnt), their bitmap, every offset >= 0 kept inside a computed
// tile (the kept blocks are kept whole), and the tile-diagonal list.
hipError_t launch_block_prep(const BlockPrepParams& P, hipStream_t st) {
  size_t ncb = (size_t)P.n_bh * P.cb_words, nob = (size_t)P.n_bh * P.rb_words, ndb = (size_t)P.n_bh * P.db_words;
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1024), dim3(256), 0, st, P.col_bits, ncb, 0u);
  hipLaunchKernelGGL(all_offsets_kernel, dim3((unsigned)((nob + 255) / 256)), dim3(256), 0, st, P.off_bits, P.n_bh,
                     P.rb_words, P.S, P.off_max);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(64), dim3(256), 0, st, P.diag_bits, ndb, 0u);
  dim3 grid((P.S + 255) / 256, P.n_bh);
  hipLaunchKernelGGL(expand_blocks_kernel, grid, dim3(256), 0, st, P);
  hipLaunchKernelGGL(diag_bits_kernel, dim3((P.nb + 256) / 256, P.n_bh), dim3(256), 0, st, P);
  MaskPrepParams M;
  M.col_idx = P.tok_idx; M.col_cnt = P.tok_cnt; M.slash_idx = nullptr; M.slash_cnt = nullptr;
  M.col_bits = P.col_bits; M.off_bits = P.off_bits; M.dlist = P.dlist; M.dcnt = P.dcnt;
  M.n_bh = P.n_bh; M.S = P.S; M.window = 0;     // (the offset bitmap is already complete)
  M.cb_words = P.cb_words; M.rb_words = P.rb_words; M.dlist_stride = P.dlist_stride; M.off_max = P.off_max;
  hipLaunchKernelGGL(set_bits_kernel, grid, dim3(256), 0, st, M);
  hipLaunchKernelGGL(dlist_block_kernel, dim3(P.n_bh), dim3(256), 0, st, P);
  return hipGetLastError();
}

hipError_t launch_gather_transpose(const GatherParams& P, hipStream_t st) {
  dim3 grid(P.C_pad / 64, P.n_out);
  if (grid.x == 0 || grid.y == 0) return hipSuccess;
  hipLaunchKernelGGL(gather_transpose_kernel, grid, dim3(256), 0, st, P);
  return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t st) {
  if (n == 0) return hipSuccess;
  int blocks = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks), dim3(256), 0, st, p, n, v);
  return hipGetLastError();
}

hipError_t launch_mask_prep(const MaskPrepParams& P, hipStream_t st) {
  size_t ncb = (size_t)P.n_bh * P.cb_words, nob = (size_t)P.n_bh * P.rb_words;
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1024), dim3(256), 0, st, P.col_bits, ncb, 0u);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1024), dim3(256), 0, st, P.off_bits, nob, 0u);
  dim3 grid((P.S + 255) / 256, P.n_bh);
  hipLaunchKernelGGL(set_bits_kernel, grid, dim3(256), 0, st, P);
  hipLaunchKernelGGL(dlist_kernel, dim3(P.n_bh), dim3(256), 0, st, P);
  return hipGetLastError();
}

}  // namespace sa
