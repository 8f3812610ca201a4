// Flash-style attention kernels for gfx950: dense causal attention (Eq. 1-2),
// row log-sum-exp of the sampled queries (stage 1, pass 1) and attention under
// the merged column / slash / window mask (Eq. 3, Algorithm 1 last step).
//
// One workgroup = 4 waves = 128 query rows of one head; each wave owns 32
// queries.  Keys are visited in tiles of 32 (small tiles and <= 168 registers
// keep three workgroups, i.e. three waves per SIMD, resident).  For every tile the
// wave forms S^T = K Q^T (keys x queries) with 32x32x16 bf16 MFMAs, so that one
// lane holds scores of ONE query (lane % 32) for 16 keys of the tile: the
// row-wise online softmax is then in-lane arithmetic plus a single exchange
// between lanes l and l^32.  The probabilities, rounded to bf16, are directly
// the B operand of O^T += V^T P^T, so the accumulators (O^T, head_dim x
// queries) again keep one query per lane and the rescale is a per-lane scalar.
// K tiles live in LDS as [key][d]; V is read from a pre-transposed copy
// (V^T, [d][key]) so both MFMA A operands are 16-byte LDS reads.
#include "sa_device.h"
#include "sa_kernels.h"

namespace sa {

namespace {

constexpr int BQ = kFlashBQ;          // 128 query rows per workgroup
constexpr int BK = kFlashBK;          // 32 keys per tile
constexpr int NT = 256;
// LDS tiles are unpadded (the direct global->LDS loads write 1 KB runs); bank
// conflicts are avoided by XOR-swizzling the 16-byte chunk index with the row.
constexpr int KROW_B = 256;           // bytes per K row in LDS: 16 chunks, chunk c of row p stored at c ^ (p & 15)
constexpr int VROW_B = 64;            // bytes per V^T row in LDS: 4 chunks, chunk c of row d stored at c ^ ((d >> 2) & 3)
constexpr int KTILE_B = BK * KROW_B;
constexpr int VTILE_B = kHeadDim * VROW_B;
constexpr int IDX_B = 256;            // 64 dwords that travel with a tile (key indices or mask words)
constexpr int STAGE_B = KTILE_B + VTILE_B + IDX_B;
constexpr float kLazy = 8.0f;         // rescale only when a row maximum grows by more than 2^8

enum TileKind : int { TK_PLAIN = 0, TK_CAUSAL = 1, TK_COLIDX = 2, TK_RANGE = 3 };

struct Tile {
  const uint16_t* kb;   // K array the tile's rows come from (row stride 128 elements)
  const uint16_t* vt;   // &V^T[0][first key] (row stride vt_stride elements)
  const int32_t* idx;   // key index of each of the 64 rows (TK_COLIDX) or null
  int krow0;            // first row of the tile in kb
  int kmax;             // last row of kb that may be read (rows past it are clamped: they are masked anyway)
  int vt_stride;
  int rows;             // rows of the tile that are real keys
  int j0;               // first key index (contiguous tiles)
  int kind;
};

typedef __attribute__((address_space(3))) void lds_void;

}  // namespace

// MODE: 0 dense causal, 1 row log-sum-exp only (no V), 2 strip-masked sparse.
template <int MODE, bool OUT_F32>
__global__ __launch_bounds__(NT, 3) void flash_kernel(FlashParams P) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr bool WITH_V = (MODE != 1);

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in an SGPR
  const int lane = tid & 63;
  const int ql = lane & 31;   // query within the wave / row within a 32-row operand
  const int hf = lane >> 5;   // which half of the contraction block this lane feeds

  // ---- which (head, query tile) this workgroup owns ------------------------
  int bh, a;
  {
    const int bid = blockIdx.x;
    if (MODE == 2) {
      // heads are sliced over the 8 XCDs (workgroups go round-robin to XCDs) and an
      // XCD works through one head at a time, heavy (late) query tiles first: the
      // workgroups resident on it then stream the gathered columns of the same head,
      // a working set (tens of MB per XCD) that the memory-side cache can hold.
      if (P.n_bh >= 8) {
        int xcd = bid & 7, slot = bid >> 3;
        a = P.n_qtiles - 1 - slot % P.n_qtiles;
        bh = xcd + 8 * (slot / P.n_qtiles);
        if (bh >= P.n_bh) return;
      } else {
        a = P.n_qtiles - 1 - bid / P.n_bh;
        bh = bid % P.n_bh;
        if (a < 0) return;
      }
    } else {
      // a bundle = the query heads sharing one KV head at one query tile; the
      // bundle's workgroups land on one XCD so the K/V stream is shared in L2.
      int xcd = bid & 7, slot = bid >> 3;
      int bl = slot / P.group, hg = slot % P.group;
      int bundle = bl * 8 + xcd;
      if (bundle >= P.n_qtiles * P.n_bkv) return;
      a = P.n_qtiles - 1 - bundle / P.n_bkv;
      int bkv = bundle % P.n_bkv;
      bh = bkv * P.group + hg;
    }
  }
  const int bkv = bh / P.group;
  const int S = P.S;
  const int i0 = P.q_row0 + a * BQ;                     // first query row of the workgroup
  const int i_last_wg = min(i0 + BQ, P.q_row0 + P.n_qrows) - 1;  // last valid row
  const int iw0 = i0 + 32 * wave;                        // first query row of the wave
  const int i_me = iw0 + ql;                             // this lane's query row
  const bool row_ok = i_me <= i_last_wg;

  // ---- Q^T operand: 8 contraction steps of 16, resident in registers -------
  bf16x8 qf[8];
  {
    const uint16_t* qrow = P.q + ((size_t)bh * S + (row_ok ? i_me : i_last_wg)) * kHeadDim;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(qrow + ks * 16 + hf * 8));
  }

  f32x16 o[4];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[mb][r] = 0.f;
  float m_run = kNegBig;   // running max, in log2 units (score * scale * log2 e)
  float l_run = 0.f;       // running sum of exp2 for this lane's keys
  const float c2 = P.scale_log2;

  // ---- tile schedule --------------------------------------------------------
  const uint16_t* kbase = P.k + (size_t)bkv * S * kHeadDim;
  const uint16_t* vtbase = WITH_V ? P.vt + (size_t)bkv * kHeadDim * P.S_pad : nullptr;
  int n_col_tiles = 0, n_rng = 0;
  const int32_t* cidx = nullptr;
  const int32_t* dl = nullptr;
  const uint32_t* cbits = nullptr;
  const uint32_t* obits = nullptr;
  const uint16_t* kc = nullptr;
  const uint16_t* vct = nullptr;
  const int a32 = i0 / BK;   // index of the 32-key tile that holds row i0 (i0 % 128 == 0 in MODE 2)
  if (MODE == 2) {
    cidx = P.col_idx_pad + (size_t)bh * P.cidx_stride;
    int cnt = min(max(P.col_cnt[bh], 0), S);
    // number of selected columns j <= last row of the tile (ascending list)
    int lo = 0, hi = cnt;
    while (lo < hi) {
      int mid = (lo + hi) >> 1;
      if (cidx[mid] <= i_last_wg) lo = mid + 1; else hi = mid;
    }
    n_col_tiles = (lo + BK - 1) / BK;
    dl = P.dlist + (size_t)bh * P.dlist_stride;
    int dc = min(max(P.dcnt[bh], 0), P.dlist_stride);
    // entries d of the ascending list whose key tile a32 + 3 - d is >= 0
    lo = 0; hi = dc;
    while (lo < hi) {
      int mid = (lo + hi) >> 1;
      if (dl[mid] <= a32 + 3) lo = mid + 1; else hi = mid;
    }
    n_rng = lo;
    cbits = P.col_bits + (size_t)bh * P.cb_words;
    obits = P.off_bits + (size_t)bh * P.rb_words;
    kc = P.kc + (size_t)bh * P.S_pad * kHeadDim;
    vct = P.vct + (size_t)bh * kHeadDim * P.S_pad;
  }
  const int n_tiles = (MODE == 2) ? (n_col_tiles + n_rng) : (min(i_last_wg, S - 1) / BK + 1);

  auto get_tile = [&](int t) -> Tile {
    Tile T;
    if (MODE == 2 && t < n_col_tiles) {
      T.kb = kc;
      T.krow0 = t * BK;
      T.kmax = P.S_pad - 1;
      T.vt = vct + t * BK;
      T.vt_stride = P.S_pad;
      T.idx = cidx + t * BK;
      T.rows = BK;
      T.j0 = 0;
      T.kind = TK_COLIDX;
    } else {
      int j0;
      if (MODE == 2) {
        // tile diagonal d <-> key tile a32 + 3 - d; walk from far to near
        int d = dl[n_rng - 1 - (t - n_col_tiles)];
        j0 = (a32 + 3 - d) * BK;
        T.kind = TK_RANGE;
      } else {
        j0 = t * BK;
        T.kind = (j0 + BK - 1 > i0) ? TK_CAUSAL : TK_PLAIN;
      }
      T.kb = kbase;
      T.krow0 = j0;
      T.kmax = S - 1;
      T.vt = WITH_V ? vtbase + j0 : nullptr;
      T.vt_stride = P.S_pad;
      T.idx = nullptr;
      T.rows = min(BK, S - j0);
      T.j0 = j0;
    }
    return T;
  };

  // Staging of one tile with direct global -> LDS loads (no registers in between).
  // One wave instruction writes a 1 KB run of LDS, lane l its bytes [16 l, 16 l + 16):
  // for K that is 4 physical rows, for V^T 16 rows.  Each lane therefore fetches the
  // global chunk that belongs at its LDS position: the K row whose slot it is (bits 2
  // and 3 of the row index exchanged, see krow_slot) and the chunk that the XOR
  // swizzle maps there.  Wave w issues runs w and w+4 of either tile.
  int koff[2], voff[2];
#pragma unroll
  for (int n = 0; n < 2; ++n) {
    int run = wave + 4 * n;
    int p = 4 * run + (lane >> 4);                 // physical K row
    int c = (lane & 15) ^ (p & 15);                // logical 16-byte chunk stored there
    koff[n] = (krow_slot(p) << 16) | (c * 8);      // key row within the tile, element offset in the row
    int d = 16 * run + (lane >> 2);                // V^T row
    int cv = (lane & 3) ^ ((d >> 2) & 3);
    voff[n] = (d << 16) | (cv * 8);
  }
  auto tile_dma = [&](const Tile& T, char* stage) {
#pragma unroll
    for (int n = 0; n < 2; ++n) {
      int run = wave + 4 * n;
      int row = min(T.krow0 + (koff[n] >> 16), T.kmax);
      const uint16_t* g = T.kb + (size_t)row * kHeadDim + (koff[n] & 0xFFFF);
      __builtin_amdgcn_global_load_lds(g, (lds_void*)(stage + 1024 * run), 16, 0, 0);
    }
    if (WITH_V) {
#pragma unroll
      for (int n = 0; n < 2; ++n) {
        int run = wave + 4 * n;
        const uint16_t* g = T.vt + (size_t)(voff[n] >> 16) * T.vt_stride + (voff[n] & 0xFFFF);
        __builtin_amdgcn_global_load_lds(g, (lds_void*)(stage + KTILE_B + 1024 * run), 16, 0, 0);
      }
    }
    if (MODE == 2 && wave == 0) {
      // 64 dwords that travel with the tile: the key indices of a gathered tile (32, twice),
      // or for a range tile 16 words of the offset bitmap (covering every offset of the
      // 128 x 32 tile) followed by the word of the column bitmap
      const int32_t* g;
      if (T.idx != nullptr) {
        g = T.idx + (lane & 31);
      } else {
        int wb = (P.off_max - (i0 - T.j0 + BQ - 1)) >> 5;          // first offset-bitmap word needed
        g = reinterpret_cast<const int32_t*>(lane < 16 ? obits + wb + lane : cbits + (T.j0 >> 5));
      }
      __builtin_amdgcn_global_load_lds(g, (lds_void*)(stage + KTILE_B + VTILE_B), 4, 0, 0);
    }
  };
  auto tile_wait = [&]() { __builtin_amdgcn_s_waitcnt(0x0f70); };   // vmcnt(0): this wave's direct loads have landed

  unsigned long long tiles_done = 0;
  if (n_tiles > 0) tile_dma(get_tile(0), smem);
  tile_wait();
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    char* stage = smem + (t & 1) * STAGE_B;
    Tile T = get_tile(t);
    if (t + 1 < n_tiles) tile_dma(get_tile(t + 1), smem + ((t + 1) & 1) * STAGE_B);

    // nothing to do for this wave when every key of the tile lies after all its rows
    bool skip = (T.kind != TK_COLIDX) && (T.j0 > iw0 + 31);
    if (MODE == 2 && T.kind == TK_RANGE) {
      // every key of the tile already belongs to a selected column: the
      // column pass has covered it, nothing is left for the range pass
      // (the two column-bitmap words were staged with the tile)
      const uint32_t* mw = reinterpret_cast<const uint32_t*>(stage + KTILE_B + VTILE_B);
      skip = skip || (mw[16] == 0xFFFFFFFFu) || (T.rows <= 0);   // or the tile lies past the sequence end
    }

    if (!skip) {
      ++tiles_done;
      // ---- S^T = K Q^T ----------------------------------------------------------
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
      {
        // row p = ql; logical chunk 2 ks + hf lives at physical chunk (2 ks + hf) ^ (p & 15)
        const char* kp = stage + ql * KROW_B;
        const int ksw = ql & 15;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          bf16x8 kf = as_bf16x8(*reinterpret_cast<const uint4*>(kp + (((2 * ks + hf) ^ ksw) << 4)));
          s = mfma_32x32x16(kf, qf[ks], s);
        }
      }
      // element r of s is key  j0 + 16*(r/8) + 8*hf + r%8  vs query i_me

      // ---- mask ---------------------------------------------------------------
      const float ninf = -__builtin_inff();
      if (T.kind == TK_CAUSAL) {
        if (T.j0 + BK - 1 > iw0) {
          int tl = i_me - (T.j0 + 8 * hf);   // keep bit b iff b <= tl
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            int b = 16 * (r >> 3) + (r & 7);
            s[r] = (b <= tl) ? s[r] : ninf;
          }
        }
      } else if (MODE == 2 && T.kind == TK_COLIDX) {
        const int32_t* il = reinterpret_cast<const int32_t*>(stage + KTILE_B + VTILE_B);
        if (il[BK - 1] > iw0) {
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const int4* ip = reinterpret_cast<const int4*>(il + 16 * u + 8 * hf);
            int4 x0 = ip[0], x1 = ip[1];
            int jj[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) s[8 * u + e] = (jj[e] <= i_me) ? s[8 * u + e] : ninf;
          }
        }
      } else if (MODE == 2 && T.kind == TK_RANGE) {
        const uint32_t* mw = reinterpret_cast<const uint32_t*>(stage + KTILE_B + VTILE_B);
        const int wb = (P.off_max - (i0 - T.j0 + BQ - 1)) >> 5;
        int tl = i_me - (T.j0 + 8 * hf);
        int x0 = P.off_max - tl;                       // >= 0 by construction of the bitmap
        int k = (x0 >> 5) - wb;                        // word of the staged window
        uint32_t lo = mw[k], hi = mw[k + 1];
        uint32_t ow = __builtin_amdgcn_alignbit(hi, lo, x0 & 31);  // bit b <-> offset tl - b
        uint32_t cw = mw[16] >> (8 * hf);                          // bit 16u+e <-> key is a selected column
        uint32_t km = ow & ~cw;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int b = 16 * (r >> 3) + (r & 7);
          // all-ones where the pair is kept; then a bitwise select between score and -inf
          uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe(km, b, 1);
          s[r] = __uint_as_float((__float_as_uint(s[r]) & keep) | (0xFF800000u & ~keep));
        }
      }

      // ---- online softmax (one query per lane) -------------------------------
      float mx = s[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
      mx = fmaxf(mx, swap_half(mx));
      // lazy rescale: keep the old reference maximum unless it grew by more than
      // 2^kLazy (probabilities then stay <= 2^kLazy, exact in fp32 and bf16 alike)
      const float m_cand = mx * c2;
      const bool grow = m_cand > m_run + kLazy;
      if (__any(grow)) {
        float m_new = grow ? m_cand : m_run;
        float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        l_run *= alpha;
        if (WITH_V) {
#pragma unroll
          for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[mb][r] *= alpha;
        }
      }
      float rs = 0.f;
      uint32_t pk[8];
      {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = fast_exp2(fmaf(s[r], c2, -m_run));
          rs += p[r];
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) pk[r] = pack_bf16x2(p[2 * r], p[2 * r + 1]);
      }
      l_run += rs;

      if (WITH_V) {
        // ---- O^T += V^T P^T ---------------------------------------------------
        // row d = 32 mb + ql; logical chunk 2 u + hf lives at physical chunk (2 u + hf) ^ ((d >> 2) & 3)
        const char* vp = stage + KTILE_B + ql * VROW_B;
        const int vsw = (ql >> 2) & 3;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          uint4 pw = {pk[4 * u], pk[4 * u + 1], pk[4 * u + 2], pk[4 * u + 3]};
          bf16x8 pb = as_bf16x8(pw);
#pragma unroll
          for (int mb = 0; mb < 4; ++mb) {
            bf16x8 vf = as_bf16x8(*reinterpret_cast<const uint4*>(vp + mb * 32 * VROW_B + (((2 * u + hf) ^ vsw) << 4)));
            o[mb] = mfma_32x32x16(vf, pb, o[mb]);
          }
        }
      }
    }

    tile_wait();
    __syncthreads();
  }

  // ---- epilogue -------------------------------------------------------------
  float l_tot = l_run + swap_half(l_run);
  if (MODE == 2 && P.tiles != nullptr && lane == 0) atomicAdd(P.tiles + bh, tiles_done);
  if (!row_ok) return;
  if (P.lse != nullptr && hf == 0) {
    size_t at = (MODE == 1) ? ((size_t)bh * P.n_qrows + (i_me - P.q_row0)) : ((size_t)bh * S + i_me);
    P.lse[at] = m_run * kLn2 + __logf(l_tot);
  }
  if (WITH_V) {
    float inv = 1.0f / l_tot;
    size_t rowoff = ((size_t)bh * S + i_me) * kHeadDim;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        int d = 32 * mb + 8 * g + 4 * hf;
        float x0 = o[mb][4 * g] * inv, x1 = o[mb][4 * g + 1] * inv;
        float x2 = o[mb][4 * g + 2] * inv, x3 = o[mb][4 * g + 3] * inv;
        if (OUT_F32) {
          float4 v4 = {x0, x1, x2, x3};
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(P.out) + rowoff + d) = v4;
        } else {
          uint2 v2 = {pack_bf16x2(x0, x1), pack_bf16x2(x2, x3)};
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(P.out) + rowoff + d) = v2;
        }
      }
  }
}

template <int MODE, bool OUT_F32>
static hipError_t launch_one(const FlashParams& P, int grid, hipStream_t st) {
  size_t shmem = 2 * STAGE_B;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&flash_kernel<MODE, OUT_F32>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((flash_kernel<MODE, OUT_F32>), dim3(grid), dim3(NT), shmem, st, P);
  return hipGetLastError();
}

hipError_t launch_flash(int mode, bool out_f32, const FlashParams& P, hipStream_t st) {
  int grid;
  if (mode == 2) {
    grid = (P.n_bh >= 8) ? 8 * P.n_qtiles * ((P.n_bh + 7) / 8) : P.n_qtiles * P.n_bh;
  } else {
    int bundles = P.n_qtiles * P.n_bkv;
    grid = ((bundles + 7) / 8) * 8 * P.group;
  }
  if (grid <= 0) return hipSuccess;
  switch (mode) {
    case 0: return out_f32 ? launch_one<0, true>(P, grid, st) : launch_one<0, false>(P, grid, st);
    case 1: return launch_one<1, false>(P, grid, st);
    default: return out_f32 ? launch_one<2, true>(P, grid, st) : launch_one<2, false>(P, grid, st);
  }
}

}  // namespace sa
