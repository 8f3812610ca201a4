// Flash-style attention kernels for gfx950: dense causal attention (Eq. 1-2),
// row log-sum-exp of the sampled queries (stage 1, pass 1) and attention under
// the merged column / slash / window mask (Eq. 3, Algorithm 1 last step).
//
// A workgroup owns 256 query rows of one head; each of its 8 waves owns 32 of
// them.  Keys are visited in tiles of 64, one K/V stream per workgroup.  For every
// tile a wave forms S^T = K Q^T (keys x queries) with 32x32x16 bf16 MFMAs, so that
// one lane holds scores of ONE query (lane % 32) for 16 keys per 32-key half
// tile: the row-wise online softmax is then in-lane arithmetic plus a single
// exchange between lanes l and l^32.  The probabilities, rounded to bf16, are
// directly the B operand of O^T += V^T P^T, so the accumulators (O^T, head_dim x
// queries) again keep one query per lane and the rescale is a per-lane scalar.
// K tiles live in LDS as [key][d]; V is read from a pre-transposed copy
// (V^T, [d][key]) so both MFMA A operands are 16-byte LDS reads.
//
// Schedule.  The waves form two groups of four (rows 0..127 and 128..255); waves
// w and w+4 share a SIMD.  Left alone, two waves that alternate an MFMA section
// and a vector-ALU (softmax) section fall into step - both on the matrix pipe,
// then both on the vector pipe - and each pipe idles half the time.  Here the
// groups run the two phases of a tile in opposite order - group 0 the MFMAs of
// P V(t-1) and K Q^T(t) and then the softmax of tile t, group 1 the softmax of
// tile t-1 and then the same MFMAs - and one workgroup barrier per tile re-aligns
// them, so every SIMD always has one wave feeding the matrix pipe and one feeding
// the vector pipe.  Both groups read the same K/V tiles; four stages of each are
// resident in LDS, filled by direct global->LDS loads two and three tiles ahead.
// The log-sum-exp sweep stages no V and needs half the registers: two of its
// workgroups share a CU.
#include <type_traits>

#include "sa_device.h"
#include "sa_kernels.h"

namespace sa {

namespace {

constexpr int BQ = kFlashBQ;          // 256 query rows per workgroup
constexpr int BK = kFlashBK;          // 64 keys per tile
constexpr int NT = 512;               // two groups of four waves
constexpr int NSTAGE = 4;             // K and V^T tiles resident in LDS
constexpr int NAUX = 8;               // ring of aux-word slots
constexpr int kDiagMask = 0x00FFFFFF;  // a tile-diagonal list entry: diagonal in bits 0..23, one bit per wave above
// LDS tiles are unpadded (the direct global->LDS loads write 1 KB runs); bank
// conflicts are avoided by XOR-swizzling the 16-byte chunk index with the row.
constexpr int KROW_B = 256;           // bytes per K row in LDS: 16 chunks, chunk c of row p stored at c ^ (p & 15)
constexpr int VROW_B = 128;           // bytes per V^T row in LDS: 8 chunks, chunk c of row d stored at c ^ ((d >> 1) & 7)
constexpr int KTILE_B = BK * KROW_B;
constexpr int VTILE_B = kHeadDim * VROW_B;
constexpr int AUX_B = 256;            // 64 dwords per tile: key indices or mask words
constexpr int OFF_K = 0;
constexpr int OFF_V = OFF_K + NSTAGE * KTILE_B;
constexpr int OFF_A = OFF_V + NSTAGE * VTILE_B;
constexpr int OFF_DUMP = OFF_A + NAUX * AUX_B;      // 1 KB per wave: where loads of tiles past the end go
constexpr int LDS_B = OFF_DUMP + 8 * 1024;          // 141312 bytes
// The log-sum-exp sweep stages K only: its dump area follows the K stages, and with
// 72 KB of LDS and at most 128 registers per lane two of its workgroups share a CU.
constexpr int OFF_DUMP_LSE = OFF_V;
constexpr int LDS_B_LSE = OFF_DUMP_LSE + 8 * 1024;  // 73728 bytes
constexpr float kSumBound = 256.0f;    // a tile's exponentials may sum to 2^8 per lane before the reference maximum moves

enum TileKind : int { TK_PLAIN = 0, TK_CAUSAL = 1, TK_COLIDX = 2, TK_RANGE = 3 };
// What a stretch of the tile loop knows at compile time about the tiles it touches
// (the tile of an iteration, the one before and the four ahead).  KIND: nothing (0),
// all of them gathered-column tiles (1), or none of them (2); REAL: all of them lie
// inside the schedule; INTERIOR: the tiles up to the next one hold only keys before the
// workgroup's first row, so every wave works on them and nothing is masked.  The loop
// runs in stretches, so that the long ones carry no per-tile choice between the two kinds
// of addressing, aux words and activity tests, and no stand-ins for tiles past the end.
template <int KIND_, bool REAL_, bool INTERIOR_ = false>
struct Stretch {
  static constexpr int KIND = KIND_;
  static constexpr bool REAL = REAL_;
  static constexpr bool INTERIOR = INTERIOR_;
};
using AnyTiles = Stretch<0, false>;
using PlainTiles = Stretch<0, true, true>;       // dense / log-sum-exp sweep below the diagonal
using ColTiles = Stretch<1, true, true>;
using RngTiles = Stretch<2, false>;
using RngRealTiles = Stretch<2, true>;

// a wave-uniform 64-bit value / pointer, forced into scalar registers (the inline
// assembly below takes its base address in a scalar register pair; left alone, the
// compiler may do wave-uniform address arithmetic in vector registers)
__device__ __forceinline__ uint64_t scalar_u64(uint64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t scalar_ptr(const void* p) { return scalar_u64(reinterpret_cast<uint64_t>(p)); }
// Direct global -> LDS load: lane l of the wave moves N bytes from global address
// `base` + `off` (base wave-uniform, in scalar registers; off per lane) to LDS
// address `lds` + N * l (`lds` wave-uniform, passed in M0).  It is written as inline
// assembly so that the waits on it are the explicit vm_wait calls below: the
// compiler, when it issues this instruction itself, makes every later LDS read wait
// for all of them (it cannot tell the buffers apart), which serialises the prefetch
// with the arithmetic.  The loads of a wave complete in order.
// The wave-uniform operands are forced into scalar registers here, whatever the
// compiler made of the address arithmetic (free when they already are scalar).
__device__ __forceinline__ void dma16(uint64_t base, uint32_t off, uint32_t lds) {
  const uint64_t sbase = scalar_u64(base);
  const uint32_t slds = __builtin_amdgcn_readfirstlane(lds);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(sbase), "s"(slds)
               : "memory", "m0");
}
__device__ __forceinline__ void dma4(uint64_t base, uint32_t off, uint32_t lds) {
  const uint64_t sbase = scalar_u64(base);
  const uint32_t slds = __builtin_amdgcn_readfirstlane(lds);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(sbase), "s"(slds)
               : "memory", "m0");
}
// wait until at most N of this wave's vector-memory loads are still in flight
template <int N>
__device__ __forceinline__ void vm_wait() {
  static_assert(N >= 0 && N < 16, "vmcnt immediate");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// workgroup barrier; LDS reads issued before it have returned
__device__ __forceinline__ void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0), as the builtin: the compiler's own counters see it too
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

}  // namespace

// MODE: 0 dense causal, 1 row log-sum-exp only (no V), 2 strip-masked sparse.
// IN_PLACE (strip-masked mode, block lists): the gathered-column tiles are runs of 64
// consecutive keys (blocks of 64, 128 or 256 keys), so they are read from K and V^T
// themselves instead of from gathered copies; the padded index list still travels with
// every tile (causal edge, short last block).
template <int MODE, bool OUT_F32, bool IN_PLACE = false>
__global__ __launch_bounds__(NT, (MODE == 1) ? 4 : 1) void flash_kernel(FlashParams P) {
  static_assert(!IN_PLACE || MODE == 2, "in-place column tiles belong to the strip-masked mode");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr bool WITH_V = (MODE != 1);
  // Where a wave issues its share of the tile loads.  Each direct load stalls the wave
  // 40-100 cycles; the two MFMA phases of a SIMD hardly overlap, so a stall there costs
  // the iteration, while the softmax phase is the shorter one and has room.  The
  // log-sum-exp sweep is the other way round (short MFMA phase, no P V).
  constexpr bool kLoadsInSoftmax = (MODE != 1);
  constexpr int kOffDump = WITH_V ? OFF_DUMP : OFF_DUMP_LSE;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // 0..7, wave-uniform, kept in an SGPR
  const int grp = wave >> 2;           // phase group
  const int lane = tid & 63;
  const int ql = lane & 31;   // query within the wave / row within a 32-row operand
  const int hf = lane >> 5;   // which half of the contraction block this lane feeds
  const uint32_t smem_lds = __builtin_amdgcn_readfirstlane((int)(uintptr_t)(__attribute__((address_space(3))) char*)smem);

  // ---- which (head, query tile) this workgroup owns ------------------------
  // (the log-sum-exp sweep may also cut the keys of a query tile into k_splits
  // equal parts, one workgroup each, to even out the last round of the launch)
  int bh, a, split = 0;
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
      a += P.qtile0;
    } else {
      // a bundle = the query heads sharing one KV head at one query tile; the
      // bundle's workgroups land on one XCD so the K/V stream is shared in L2.
      int xcd = bid & 7, slot = bid >> 3;
      int bl = slot / P.group, hg = slot % P.group;
      int bundle = bl * 8 + xcd;
      const int ks = (MODE == 1) ? P.k_splits : 1;
      if (bundle >= P.n_qtiles * ks * P.n_bkv) return;
      const int av = P.n_qtiles * ks - 1 - bundle / P.n_bkv;
      a = av / ks;
      split = av % ks;
      int bkv = bundle % P.n_bkv;
      bh = bkv * P.group + hg;
    }
  }
  const int bkv = ((MODE == 2 ? P.head0 : 0) + bh) / P.group;
  const int S = P.S;
  const int i0 = P.q_row0 + a * BQ;                     // first query row of the workgroup
  const int i_last_wg = min(i0 + BQ, P.q_row0 + P.n_qrows) - 1;  // last valid row
  const int iw0 = i0 + 32 * wave;                        // first query row of the wave
  const int i_me = iw0 + ql;                             // this lane's query row
  const bool row_ok = i_me <= i_last_wg && (MODE != 2 || i_me >= P.row_lo);
  const int a64 = i0 / BK;   // index of the 64-key tile that holds row i0 (i0 % 256 == 0 in MODE 2)
  const uint16_t* kbase = P.k + (size_t)bkv * S * kHeadDim;
  const uint16_t* vtbase = WITH_V ? P.vt + (size_t)bkv * kHeadDim * P.S_pad : nullptr;

  // ---- tile schedule: gathered-column tiles, then range tiles (sparse), or the
  //      causal sweep (dense / log-sum-exp) ------------------------------------------
  const int32_t* cidx = nullptr;
  const int32_t* dl = nullptr;
  const uint32_t* cbits = nullptr;
  const uint32_t* obits = nullptr;
  const uint16_t* kc = nullptr;
  const uint16_t* vct = nullptr;
  int n_col_tiles = 0, n_rng = 0;
  if (MODE == 2) {
    cidx = P.col_idx_pad + (size_t)bh * P.cidx_stride;
    int cnt = min(max(P.col_cnt[bh], 0), S);
    int lo = 0, hi = cnt;          // selected columns j <= last row of the tile (ascending list)
    while (lo < hi) {
      int mid = (lo + hi) >> 1;
      if (cidx[mid] <= i_last_wg) lo = mid + 1; else hi = mid;
    }
    n_col_tiles = (lo + BK - 1) / BK;
    dl = P.dlist + (size_t)bh * P.dlist_stride;
    int dc = min(max(P.dcnt[bh], 0), P.dlist_stride);
    lo = 0; hi = dc;               // tile diagonals d whose key tile a64 + 3 - d is >= 0
    while (lo < hi) {
      int mid = (lo + hi) >> 1;
      if ((dl[mid] & kDiagMask) <= a64 + 3) lo = mid + 1; else hi = mid;
    }
    n_rng = lo;
    cbits = P.col_bits + (size_t)bh * P.cb_words;
    obits = P.off_bits + (size_t)bh * P.rb_words;
    kc = P.kc + (size_t)bh * P.S_pad * kHeadDim;
    vct = P.vct + (size_t)bh * kHeadDim * P.S_pad;
  }
  n_col_tiles = __builtin_amdgcn_readfirstlane(n_col_tiles);
  n_rng = __builtin_amdgcn_readfirstlane(n_rng);
  int t_base = 0;                        // first key tile of this workgroup's share of the causal sweep
  int n_sweep = min(i_last_wg, S - 1) / BK + 1;
  if (MODE == 1 && P.k_splits > 1) {
    t_base = (int)((long long)n_sweep * split / P.k_splits);
    n_sweep = (int)((long long)n_sweep * (split + 1) / P.k_splits) - t_base;
  }
  t_base = __builtin_amdgcn_readfirstlane(t_base);
  const int n_tiles = __builtin_amdgcn_readfirstlane((MODE == 2) ? (n_col_tiles + n_rng) : n_sweep);

  // Kind of tile t (wave-uniform; no memory access), and whether t lies inside the schedule.
  // `kc` is the Stretch the calling iteration belongs to: what it knows at compile time.
  auto is_col = [&](auto kc, int t) __attribute__((always_inline)) -> bool {
    constexpr int KIND = decltype(kc)::KIND;
    return MODE == 2 && (KIND == 1 || (KIND == 0 && t < n_col_tiles));
  };
  auto is_real = [&](auto kc, int t) __attribute__((always_inline)) -> bool { return decltype(kc)::REAL || t < n_tiles; };
  // Descriptor of tile t.  A range tile is named by its tile diagonal d: key tile
  // a64 + 3 - d, which the 256 rows meet at offsets [64 d - 255, 64 d + 63].  The d
  // values come from a list in global memory; they are fetched (fetch_d) four tiles
  // ahead of their first use and handed on in scalar registers, so that no phase
  // waits on a scalar load.
  auto fetch_d = [&](auto kc, int t) __attribute__((always_inline)) -> int {
    // read through the constant address space: the list is not written while the kernel
    // runs, and only so does the load stay a scalar one (tracked apart from the vector
    // loads in flight) behind the barriers and inline assembly of the loop
    typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
    if (IN_PLACE && is_col(kc, t))
      return ((const_i32_ptr)(uintptr_t)cidx)[BK * t];                       // first key of the tile's block
    if (MODE == 2 && !is_col(kc, t) && is_real(kc, t))
      return ((const_i32_ptr)(uintptr_t)dl)[n_rng - 1 - (t - n_col_tiles)];   // far to near
    return 0;
  };
  // first key of tile t
  auto first_key = [&](auto kc, int t, int d) __attribute__((always_inline)) -> int {  // contiguous tiles only; d = list entry
    if (IN_PLACE && is_col(kc, t)) return d;         // the entry of an in-place column tile is its first key
    return (MODE == 2) ? (a64 + 3 - (d & kDiagMask)) * BK : (t + (MODE == 1 ? t_base : 0)) * BK;
  };
  // array bases as scalars, once
  const uint64_t s_kbase = scalar_ptr(kbase), s_vtbase = scalar_ptr(vtbase);
  const uint64_t s_kc = scalar_ptr(kc), s_vct = scalar_ptr(vct), s_cidx = scalar_ptr(cidx);
  const uint64_t s_cbits = scalar_ptr(cbits), s_obits = scalar_ptr(obits);

  // ---- Q^T operand: 8 contraction steps of 16, resident in registers -------
  bf16x8 qf[8];
  {
    int qr = row_ok ? i_me : max(min(i_last_wg, S - 1), 0);
    const uint16_t* qrow = P.q + ((size_t)bh * S + qr) * kHeadDim;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      qf[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(qrow + ks * 16 + hf * 8));
  }

  f32x16 o[4];
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[mb][r] = 0.f;
  float m_run = kNegBig;   // reference maximum, in log2 units (score * scale * log2 e)
  float l_run = 0.f;       // running sum of exp2 for this lane's keys
  const float c2 = P.scale_log2;

  // ---- staging ---------------------------------------------------------------------
  // One wave instruction writes a 1 KB run of LDS, lane l its bytes [16 l, 16 l + 16):
  // for K that is 4 physical rows, for V^T 8 rows.  Each lane therefore fetches the
  // global chunk that belongs at its LDS position: the K row whose slot it is (bits 2
  // and 3 of the row index exchanged, see krow_slot) and the chunk that the XOR
  // swizzle maps there.  A tile is 16 runs of K and 16 of V^T; wave w issues runs w
  // and w + 8 of each.  The lane's byte offset inside a run is fixed for the whole
  // kernel, and run w + 8 lies a constant 32 K rows / 64 V^T rows after run w
  // (neither the swizzle nor the slot permutation sees that step): per tile and per
  // load only the scalar base address changes, so issuing costs no vector arithmetic.
  uint32_t koff0, voff0;
  {
    int p = 4 * wave + (lane >> 4);                // physical K row of run `wave`
    int c = (lane & 15) ^ (p & 15);                // logical 16-byte chunk stored there
    koff0 = krow_slot(p) * KROW_B + c * 16;        // key row within the tile, byte in the row
    int d = 8 * wave + (lane >> 3);                // V^T row
    int cv = (lane & 7) ^ ((d >> 1) & 7);
    voff0 = (uint32_t)d * (uint32_t)P.S_pad * 2u + cv * 16;
  }
  // The loads are issued one at a time (load_v_one / load_k_one, n = 0, 1), so the
  // caller can spread them between its exponentials (or its MFMAs): a wave that issues
  // them back to back stalls on each.  Loads of a tile past the end of the schedule still go out (to a
  // stand-in address and the wave's dump area), which keeps the number of loads per
  // phase, and with it the vmcnt arithmetic, constant.
  uint64_t ld_vbase = 0, ld_vbase1 = 0, ld_kbase = 0;
  uint32_t ld_vdst = 0, ld_kdst = 0, ld_vstep = 0, ld_kstep = 0, ld_klim = 0;   // step: LDS distance of run w + 8
  // A tile past the end of the schedule is replaced by a stand-in: the first tile of
  // K / V^T, always readable, loaded into the wave's dump kilobyte.
  auto load_v_begin = [&](auto kc, int t, int d) __attribute__((always_inline)) {
    if (!WITH_V) return;
    const bool real = is_real(kc, t), col = !IN_PLACE && real && is_col(kc, t);   // col: from the gathered copy
    const uint32_t off = !real ? 0u : (col ? (uint32_t)t : (uint32_t)first_key(kc, t, d)) * 2u;   // bytes into a V^T row; t * 64 keys for a gathered tile
    ld_vbase = col ? s_vct + (uint64_t)((uint32_t)t * (BK * 2u)) : s_vtbase + off;
    ld_vbase1 = ld_vbase + 128ull * (uint32_t)P.S_pad;            // run w + 8: 64 rows of V^T further on
    ld_vdst = smem_lds + 1024 * wave + (real ? OFF_V + (t & (NSTAGE - 1)) * VTILE_B : kOffDump);
    ld_vstep = real ? 8192 : 0;                    // a stand-in tile writes both runs to the same dump kilobyte
  };
  auto load_k_begin = [&](auto kc, int t, int d) __attribute__((always_inline)) {
    const bool real = is_real(kc, t), col = !IN_PLACE && real && is_col(kc, t);
    const int kmax = col ? P.S_pad - 1 : S - 1;    // last row of the array that may be read
    // a range tile may start past the last key (all of it masked): the base row is
    // clamped, and so is each lane's byte offset, to the last row that exists
    const int row0 = min(!real ? 0 : (col ? t * BK : first_key(kc, t, d)), kmax);
    ld_kbase = (col ? s_kc : s_kbase) + ((uint64_t)(uint32_t)row0 << 8);
    ld_klim = (uint32_t)(kmax - row0) * KROW_B + (koff0 & (KROW_B - 1));
    ld_kdst = smem_lds + 1024 * wave + (real ? OFF_K + (t & (NSTAGE - 1)) * KTILE_B : kOffDump);
    ld_kstep = real ? 8192 : 0;
  };
  auto load_v_one = [&](int n) {
    if (!WITH_V) return;
    dma16(n == 0 ? ld_vbase : ld_vbase1, voff0, ld_vdst + ld_vstep * n);
  };
  auto load_k_one = [&](int n) {
    dma16(ld_kbase, min(koff0 + 32 * KROW_B * n, ld_klim), ld_kdst + ld_kstep * n);
  };
  // the 64 dwords that go with a tile: the key indices of a gathered tile, or for a
  // range tile 16 words of the offset bitmap (covering every offset of the 256 x 64
  // tile) followed by the 2 words of the column bitmap.  One load, by wave t % 8.
  const uint32_t aux_lane = lane < 16 ? 4u * lane : 4u * (lane & 1);
  auto dma_aux = [&](auto kc, int t, int d) __attribute__((always_inline)) {
    if (MODE != 2 || wave != (t & 7)) return;
    const bool real = is_real(kc, t);
    const uint32_t dst = smem_lds + (real ? OFF_A + (t & (NAUX - 1)) * AUX_B : kOffDump);
    if (real && is_col(kc, t)) {
      dma4(s_cidx + (uint64_t)((uint32_t)t * (BK * 4u)), 4u * lane, dst);
    } else {
      const int j0 = real ? first_key(kc, t, d) : 0;
      const int wb = (P.off_max - (i0 - j0 + BQ - 1)) >> 5;          // first offset-bitmap word needed
      // lanes 0..15: offset words wb ..; lanes 16..63: the two column words, alternating.
      // The column bitmaps lie below the offset bitmaps in the workspace (and within
      // 4 GB of them), so offsets from the column word are non-negative 32-bit values.
      const uint64_t cw = s_cbits + (uint64_t)((uint32_t)(j0 >> 5) * 4u);
      const uint32_t gap = (uint32_t)(s_obits + (uint64_t)((uint32_t)wb * 4u) - cw);
      dma4(cw, aux_lane + (lane < 16 ? gap : 0u), dst);
    }
  };

  // Whether this wave has anything to do on tile t.
  //  - gathered tile: its first key index (an aux word) must not lie after the wave's rows;
  //  - range tile: one of the 95 offsets between the wave's 32 rows and the tile's 64
  //    keys must be kept.  That depends on the tile diagonal and the wave only, not on
  //    the query tile, so the list entry carries it as a bit per wave (bits 24..31; a
  //    key after a row gives a negative offset, never kept).  Also not all 64 keys may
  //    be selected columns (the column pass covered those: two aux words), and the
  //    tile must start before the sequence end.
  // The aux words are read early (act_words) and looked at later (tile_active), so
  // that the wait for them hides behind MFMAs.
  auto act_words = [&](auto kc, int t, uint32_t& w0, uint32_t& w1) __attribute__((always_inline)) {
    if (MODE != 2 || decltype(kc)::INTERIOR) return;
    const uint32_t* ax = reinterpret_cast<const uint32_t*>(smem + OFF_A + (t & (NAUX - 1)) * AUX_B);
    if (is_col(kc, t)) {
      w0 = ax[0];
    } else {
      w0 = ax[16];
      w1 = ax[17];
    }
  };
  auto tile_active = [&](auto kc, int t, int d, uint32_t w0, uint32_t w1) __attribute__((always_inline)) -> bool {
    if (decltype(kc)::INTERIOR) return true;
    bool act;
    const int j0 = first_key(kc, t, d);
    if (is_col(kc, t)) {
      act = (int)w0 <= iw0 + 31;
    } else if (MODE == 2) {
      act = (((uint32_t)d >> (24 + wave)) & 1u) && ((w0 & w1) != 0xFFFFFFFFu) && (j0 < S);
    } else {
      act = j0 <= iw0 + 31;                        // else every key of the tile lies after the wave's rows
    }
    return __builtin_amdgcn_readfirstlane((int)act) != 0;
  };

  // ---- operand ring and the MFMA phase -------------------------------------------
  // A phase issues up to 32 MFMAs: 16 of P V(t-1) (keys in groups of 16, head-dim
  // blocks 0..3 within a group) and 16 of K Q^T(t) (8 contraction steps for each
  // of two 32-key halves).  Their A operands come from LDS through a ring of 8
  // registers x 16 bytes: after MFMA i has consumed slot i % 8, the operand of MFMA
  // i + 8 is read into it, so every read has 7 MFMAs (~250 cycles) to return and the
  // matrix pipe does not wait on LDS round trips.  sched_barrier pins the order: the
  // compiler would otherwise sink each read down to its use.
  f32x16 s[2];
  uint32_t pk[2][8];
  uint4 R[8];
#define SA_PIN() __builtin_amdgcn_sched_barrier(0)
  // K operand i = 2 ks + sb: contraction step ks, 32-key half sb (the halves alternate
  // so that consecutive MFMAs of the sweep accumulate into different registers)
  auto ld_k = [&](int slot, int i, int buf) {
    // row p = 32 sb + ql; logical chunk 2 ks + hf lives at physical chunk (2 ks + hf) ^ (p & 15)
    const int sb = i & 1, ks = i >> 1;
    const char* kp = smem + OFF_K + buf * KTILE_B + (32 * sb + ql) * KROW_B;
    R[slot] = *reinterpret_cast<const uint4*>(kp + (((2 * ks + hf) ^ (ql & 15)) << 4));
  };
  // V^T operand i = 8 sb + 4 u + mb: keys 32 sb + 16 u .., head-dim block mb
  auto ld_v = [&](int slot, int i, int buf) {
    // row d = 32 mb + ql; logical chunk 4 sb + 2 u + hf lives at physical chunk (..) ^ ((d >> 1) & 7)
    const int sb = i >> 3, u = (i >> 2) & 1, mb = i & 3;
    const char* vp = smem + OFF_V + buf * VTILE_B + (32 * mb + ql) * VROW_B;
    R[slot] = *reinterpret_cast<const uint4*>(vp + (((4 * sb + 2 * u + hf) ^ ((ql >> 1) & 7)) << 4));
  };
  // P V: on entry the ring holds V operands 0..7 (read during the softmax phase);
  // the second half of the sweep re-fills it with the first 8 K operands of the next
  // tile (read even when that tile turns out to need no work from this wave).  The
  // loads of the tiles further ahead go out under the MFMAs, one per 3 MFMAs.
  auto mm_pv = [&](int bufp, int bufq, auto&& setup_a, auto&& setup_v, auto&& setup_k, auto&& look, auto&& decide) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      // scalar bookkeeping in small pieces, so that no gap between two MFMAs grows long
      if (!kLoadsInSoftmax) {
        if (i == 1) setup_a();
        if (i == 2) setup_v();
        if (i == 4) load_v_one(0);
        if (i == 5) setup_k();
        if (i == 7) load_v_one(1);
        if (i == 10) load_k_one(0);
        if (i == 13) load_k_one(1);
      }
      if (i == 3) look();                          // read the words that say whether the next tile needs this wave
      if (i == 9) decide();                        // ... and decide, under the MFMAs
      const int sb = i >> 3, u = (i >> 2) & 1, mb = i & 3;
      uint4 pw = {pk[sb][4 * u], pk[sb][4 * u + 1], pk[sb][4 * u + 2], pk[sb][4 * u + 3]};
      o[mb] = mfma_32x32x16(as_bf16x8(R[i & 7]), as_bf16x8(pw), o[mb]);      // O^T += V^T P^T
      SA_PIN();
      if (i + 8 < 16) ld_v(i & 7, i + 8, bufp); else ld_k(i & 7, i - 8, bufq);
      SA_PIN();
    }
  };
  // first 8 K operands of a tile into the ring (when no P V sweep did it)
  auto warm_k = [&](int bufq) {
#pragma unroll
    for (int i = 0; i < 8; ++i) ld_k(i, i, bufq);
    SA_PIN();
  };
  // K Q^T: the ring holds K operands 0..7.  `with_loads`: no P V sweep went before,
  // so this sweep issues the loads of the tiles further ahead.
  // Element r of s[sb] is key j0 + 32*sb + 16*(r/8) + 8*hf + r%8 against query i_me.
  auto mm_qk = [&](int bufq, bool with_loads) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (with_loads && !kLoadsInSoftmax) {
        if (i == 2) load_v_one(0);
        if (i == 5) load_v_one(1);
        if (i == 8) load_k_one(0);
        if (i == 11) load_k_one(1);
      }
      const int sb = i & 1, ks = i >> 1;
      if (ks == 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[sb][r] = 0.f;
      }
      s[sb] = mfma_32x32x16(as_bf16x8(R[i & 7]), qf[ks], s[sb]);
      SA_PIN();
      if (i + 8 < 16) ld_k(i & 7, i + 8, bufq);
      SA_PIN();
    }
  };

  // ---- the softmax phase: mask, online softmax (one query per lane), bf16 --------
  auto step_softmax = [&](auto kc, int t, int d) __attribute__((always_inline)) {
    const int j0 = first_key(kc, t, d);
    constexpr bool INTERIOR = decltype(kc)::INTERIOR;
    const int kind = is_col(kc, t) ? TK_COLIDX : (MODE == 2) ? TK_RANGE : (!INTERIOR && j0 + BK - 1 > i0) ? TK_CAUSAL : TK_PLAIN;
    const int buf = t & (NSTAGE - 1);
    // Mask: one 32-bit pattern per lane and 32-key half, bit b <-> key
    // j0 + 32 sb + 8 hf + b of the lane's 16 (b = 0..7, 16..23), set = keep.  The
    // pattern is built per tile kind; one loop applies it (a 1-bit signed extract and
    // a bitwise select between the score and -inf per element).
    bool masked = false;                   // wave-uniform
    uint32_t km[2] = {0xFFFFFFFFu, 0xFFFFFFFFu};
    if (kind == TK_CAUSAL) {
      if (j0 + BK - 1 > iw0) {             // keep key <= query, i.e. b <= tl
        masked = true;
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
          const int tl = i_me - (j0 + 32 * sb + 8 * hf);
          km[sb] = tl < 0 ? 0u : (tl >= 31 ? 0xFFFFFFFFu : (2u << tl) - 1u);
        }
      }
    } else if (MODE == 2 && kind == TK_COLIDX) {
      const int32_t* il = reinterpret_cast<const int32_t*>(smem + OFF_A + (t & (NAUX - 1)) * AUX_B);
      if (!INTERIOR && il[BK - 1] > iw0) {   // only the last gathered tiles reach past a row: keep index <= query
        masked = true;
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
          uint32_t m = 0;
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const int4* ip = reinterpret_cast<const int4*>(il + 32 * sb + 16 * u + 8 * hf);
            int4 x0 = ip[0], x1 = ip[1];
            int jj[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) m |= (jj[e] <= i_me ? 1u : 0u) << (16 * u + e);
          }
          km[sb] = m;
        }
      }
    } else if (MODE == 2 && kind == TK_RANGE) {
      masked = true;
      const uint32_t* mw = reinterpret_cast<const uint32_t*>(smem + OFF_A + (t & (NAUX - 1)) * AUX_B);
      const int wb = (P.off_max - (i0 - j0 + BQ - 1)) >> 5;
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        int tl = i_me - (j0 + 32 * sb + 8 * hf);
        int x0 = P.off_max - tl;                       // >= 0 by construction of the bitmap
        int k = (x0 >> 5) - wb;                        // 0 .. 10: word of the staged window
        uint32_t lo = mw[k], hi = mw[k + 1];
        uint32_t ow = __builtin_amdgcn_alignbit(hi, lo, x0 & 31);  // bit b <-> offset tl - b
        uint32_t cw = mw[16 + sb] >> (8 * hf);                     // bit 16u+e <-> key is a selected column
        km[sb] = ow & ~cw;
      }
      // a tile that keeps every pair (a whole block of the block mask, the inside of a
      // band of offsets) needs no masking at all
      masked = __builtin_amdgcn_ballot_w64((km[0] & km[1]) != 0xFFFFFFFFu) != 0ull;
    }
    if (masked) {
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int bit = 16 * (r >> 3) + (r & 7);
          const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe(km[sb], bit, 1);   // all-ones where kept
          s[sb][r] = __uint_as_float((__float_as_uint(s[sb][r]) & keep) | (0xFF800000u & ~keep));
        }
    }

    // the operand ring is idle: fetch the first 8 V operands of this tile's P V now,
    // so that the reads return under the exponentials
    if (WITH_V) {
      SA_PIN();
#pragma unroll
      for (int i = 0; i < 8; ++i) ld_v(i, i, buf);
      SA_PIN();
    }
    // Online softmax, optimistic: the exponentials are taken against the reference
    // maximum the row already has, and only their sum is looked at.  A sum within
    // 2^8 means that no probability exceeds 2^8, which is all the reference is
    // for (exact in fp32 and bf16 alike); then the tile costs no maximum at all.
    // Otherwise (first tiles of a row, or a score far above what the row has seen: the
    // sum is large, inf or NaN) the row maximum of the tile is formed, the reference
    // moved up to it, the accumulators rescaled and the exponentials taken again.
    float rs = 0.f;
    auto exponentials = [&](auto first_tag) {
      constexpr bool FIRST = decltype(first_tag)::value;
      rs = 0.f;
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          if (kLoadsInSoftmax && FIRST) {          // the loads of the tiles ahead, spread over the exponentials
            if (sb == 0 && r == 4) load_v_one(0);
            if (sb == 0 && r == 12) load_v_one(1);
            if (sb == 1 && r == 4) load_k_one(0);
            if (sb == 1 && r == 12) load_k_one(1);
          }
          p[r] = fast_exp2(fmaf(s[sb][r], c2, -m_run));
          rs += p[r];
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) pk[sb][r] = pack_bf16x2(p[2 * r], p[2 * r + 1]);
      }
    };
    exponentials(std::true_type{});
    if (__any(!(rs <= kSumBound))) {
      // (the maximum starts from a value the compiler cannot see through: otherwise it
      // forms the whole maximum ahead of the branch, on every tile)
      float mx = s[0][0];
      asm volatile("" : "+v"(mx));
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sb][r]);
      mx = half_max(mx);                     // the two lanes of a row agree on its reference
      const float m_cand = mx * c2;
      const float m_new = (m_cand > m_run) ? m_cand : m_run;
      const float alpha = fast_exp2(m_run - m_new);
      m_run = m_new;
      l_run *= alpha;
      if (WITH_V) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[mb][r] *= alpha;
      }
      exponentials(std::false_type{});
    }
    l_run += rs;
  };

  // ---- the two-phase pipeline --------------------------------------------------------
  // MFMA phase(u):    P V(u-1), K Q^T(u)
  // softmax phase(u): softmax(u)
  // Iteration u also issues the loads of aux(u+3), V(u+2), K(u+3): from its softmax phase
  // (dense and strip-masked kernels) or from its MFMA phase (log-sum-exp sweep).
  // Group 0 runs MFMA phase u in the first half of iteration u, group 1 in the second.
  // Slot t % 4 of the K (V^T) ring is re-filled with tile t + 4 only after the barrier
  // that follows its last reader - K Q^T(t) (P V(t)) of group 1; a load is waited for
  // by the wave that issued it before the barrier that precedes its first reader.  Loads complete
  // in order, so "at most n in flight" means everything but the last n has landed: at
  // the end of iteration u the loads of iteration u - 1 that feed the next softmax and
  // K Q^T (V(u+1), and K(u+1) from iteration u - 2) must be in, the rest may still fly.
  unsigned long long tiles_done = 0;
  bool act_t = false;                        // this wave has work on the tile whose softmax comes next
  bool pre_done = false, pre_act = false;    // the next tile was already looked at (and the ring warmed for it)
  int dq0 = fetch_d(AnyTiles{}, 0), dq1 = fetch_d(AnyTiles{}, 1), dq2 = fetch_d(AnyTiles{}, 2), dq3 = fetch_d(AnyTiles{}, 3);   // tile diagonals of tiles u .. u+3
  // The scores, the probabilities and the operand ring are written on some paths only
  // (a wave may have no work on a tile).  An empty asm that "defines" them where their
  // old contents are dead tells the compiler so; without it every path that skips a
  // write carries the old value along, and the register allocator copies whole arrays
  // between two homes inside the loop.
  auto forget_ring_and_p = [&]() {
#pragma unroll
    for (int i = 0; i < 8; ++i) asm volatile("" : "=v"(R[i]));
#pragma unroll
    for (int i = 0; i < 8; ++i) asm volatile("" : "=v"(pk[0][i]), "=v"(pk[1][i]));
  };
  auto forget_scores = [&]() { asm volatile("" : "=v"(s[0]), "=v"(s[1])); };
  auto softmax_phase = [&](auto kc, int u, int d_u, int d_next, int it) __attribute__((always_inline)) {   // tile diagonals of tiles u and u + 1; iteration
    forget_ring_and_p();                     // consumed by the MFMA phase before
    if (kLoadsInSoftmax) {
      // the loads of iteration `it`: aux(it + 3), V(it + 2), K(it + 3)
      dma_aux(kc, it + 3, dq3);
      load_v_begin(kc, it + 2, dq2);
      load_k_begin(kc, it + 3, dq3);
      if (!act_t) { load_v_one(0); load_v_one(1); load_k_one(0); load_k_one(1); }
    }
    if (act_t) step_softmax(kc, u, d_u);
    // A wave with nothing to do here looks at the next tile now, so that its next MFMA
    // phase knows at once whether it has work.
    if (!act_t && is_real(kc, u + 1)) {
      uint32_t w0 = 0, w1 = 0;
      act_words(kc, u + 1, w0, w1);
      pre_act = tile_active(kc, u + 1, d_next, w0, w1);
      pre_done = true;
    }
  };
  auto mfma_phase = [&](auto kc, int u) __attribute__((always_inline)) {
    forget_scores();                         // consumed by the softmax phase before
    const bool have = is_real(kc, u);
    auto setup_a = [&]() { dma_aux(kc, u + 3, dq3); };
    auto setup_v = [&]() { load_v_begin(kc, u + 2, dq2); };
    auto setup_k = [&]() { load_k_begin(kc, u + 3, dq3); };
    auto ahead_setup = [&]() { setup_a(); setup_v(); setup_k(); };
    __builtin_amdgcn_s_setprio(1);
    const bool pv = WITH_V && act_t;
    bool act_n = false;
    if (pv) {
      uint32_t aw0 = 0, aw1 = 0;
      auto look = [&]() { if (have) act_words(kc, u, aw0, aw1); };
      auto decide = [&]() { act_n = have && tile_active(kc, u, dq0, aw0, aw1); };
      mm_pv((u - 1) & (NSTAGE - 1), u & (NSTAGE - 1), setup_a, setup_v, setup_k, look, decide);
    } else {
      if (!kLoadsInSoftmax) ahead_setup();
      if (MODE == 1) {
        // one call site for the warm-up: with two, the ring gets two homes in the
        // log-sum-exp kernel and 32 register copies per tile (-6 % there; the other
        // two kernels measured 1 % slower with this form, so they keep the one below)
        if (pre_done) {
          act_n = pre_act;
        } else if (have) {
          uint32_t aw0 = 0, aw1 = 0;
          act_words(kc, u, aw0, aw1);
          act_n = tile_active(kc, u, dq0, aw0, aw1);
        }
        if (act_n) warm_k(u & (NSTAGE - 1));
      } else if (pre_done) {
        act_n = pre_act;
        if (act_n) warm_k(u & (NSTAGE - 1));
      } else if (have) {
        uint32_t aw0 = 0, aw1 = 0;
        act_words(kc, u, aw0, aw1);
        act_n = tile_active(kc, u, dq0, aw0, aw1);
        if (act_n) warm_k(u & (NSTAGE - 1));
      }
    }
    pre_done = false;
    if (act_n) mm_qk(u & (NSTAGE - 1), !pv);
    __builtin_amdgcn_s_setprio(0);
    if (!kLoadsInSoftmax && !pv && !act_n) {
      load_v_one(0); load_v_one(1); load_k_one(0); load_k_one(1);
    }
    tiles_done += act_n ? 1 : 0;
    act_t = act_n;
    // everything but this phase's loads and the K loads of the one before has landed
    // (the wave that also fetched aux words waits for one load more than it must)
    if (!kLoadsInSoftmax) { if (WITH_V) vm_wait<6>(); else vm_wait<4>(); }
  };
  // before the barrier that ends an iteration everything has landed but that iteration's
  // loads and the K loads of the one before
  auto end_of_iteration_wait = [&]() {
    if (kLoadsInSoftmax) { if (WITH_V) vm_wait<6>(); else vm_wait<4>(); }
  };
#undef SA_PIN

  // prologue: K(0..2), V(0..1) and the aux words of tiles 0..2
  {
    const AnyTiles any{};
    dma_aux(any, 0, dq0); dma_aux(any, 1, dq1); dma_aux(any, 2, dq2);
    load_k_begin(any, 0, dq0); load_k_one(0); load_k_one(1);
    load_k_begin(any, 1, dq1); load_k_one(0); load_k_one(1);
    load_k_begin(any, 2, dq2); load_k_one(0); load_k_one(1);
    load_v_begin(any, 0, dq0); load_v_one(0); load_v_one(1);
    load_v_begin(any, 1, dq1); load_v_one(0); load_v_one(1);
  }
  // vmcnt(0), as the builtin: the compiler then also knows that the Q loads above have
  // landed and places no waits of its own for them inside the loop, where they would
  // wait for the loads in flight there as well
  __builtin_amdgcn_s_waitcnt(0x0f70);
  wg_barrier();
  // Iteration n: group 0 runs MFMA phase n, then softmax phase n; group 1 runs softmax
  // phase n - 1, then MFMA phase n; one workgroup barrier ends the iteration.  The
  // barrier is all the LDS traffic needs (a stage is re-filled, and a landed tile is
  // first read, at least one iteration after the other side touched it - see above);
  // starting the two groups on opposite phases after each barrier is what keeps one
  // wave of every SIMD on the matrix pipe while the other is on the vector pipe.
  // (The loop is written out once per group: one loop that picks the phase at run
  // time keeps the registers of both phases alive everywhere and spills.)
  // Iteration n touches tiles n - 1 .. n + 4 and decides on the work of tiles n and n + 1.
  // Strip-masked kernel: the selected keys that are not before the workgroup's first row
  // (at most 256) lie in the last five gathered tiles, so the iterations n + 1 <
  // n_col_tiles - 5 see gathered tiles only, with work for every wave and nothing to mask;
  // the iterations n > n_col_tiles see range tiles only; the few in between take the
  // general form.  Dense and log-sum-exp sweeps: the tiles below key tile a64 (the one
  // that holds the first row) are interior.  The iterations n + 4 < n_tiles see no tile
  // past the end of the schedule.
  const int n_gen0 = (MODE == 2) ? max(n_col_tiles - 6, 0)                 // first iteration of the general form
                                 : max(min(a64 - t_base - 1, n_tiles - 4), 0);
  const int n_gen1 = (MODE == 2) ? min(n_col_tiles, n_tiles) : n_tiles;    // its last
  const int n_real = n_tiles - 4;                                          // first iteration that may see a tile past the end
  if (grp == 0) {
    auto iteration = [&](auto kc, int n) __attribute__((always_inline)) {
      // the scalar load is issued here and collected by the barrier's lgkmcnt(0): waited
      // for anywhere else, it would drain the LDS reads in flight as well
      const int dq4 = fetch_d(kc, n + 4);
      mfma_phase(kc, n);                     // n = 0: K Q^T(0) only; n = n_tiles: the last P V
      softmax_phase(kc, n, dq0, dq1, n);
      end_of_iteration_wait();
      wg_barrier();
      dq0 = dq1; dq1 = dq2; dq2 = dq3; dq3 = dq4;
    };
    int n = 0;
    if (MODE == 2) {
      for (; n < n_gen0; ++n) iteration(ColTiles{}, n);
      for (; n <= n_gen1; ++n) iteration(AnyTiles{}, n);
      for (; n < n_real; ++n) iteration(RngRealTiles{}, n);
      for (; n <= n_tiles; ++n) iteration(RngTiles{}, n);
    } else {
      for (; n < n_gen0; ++n) iteration(PlainTiles{}, n);
      for (; n <= n_gen1; ++n) iteration(AnyTiles{}, n);
    }
  } else {
    int dprev = 0;                           // tile diagonal of tile n - 1
    auto iteration = [&](auto kc, int n) __attribute__((always_inline)) {
      const int dq4 = fetch_d(kc, n + 4);
      softmax_phase(kc, n - 1, dprev, dq0, n);
      mfma_phase(kc, n);
      end_of_iteration_wait();
      wg_barrier();
      dprev = dq0; dq0 = dq1; dq1 = dq2; dq2 = dq3; dq3 = dq4;
    };
    int n = 0;
    if (MODE == 2) {
      for (; n < n_gen0; ++n) iteration(ColTiles{}, n);
      for (; n <= n_gen1; ++n) iteration(AnyTiles{}, n);
      for (; n < n_real; ++n) iteration(RngRealTiles{}, n);
      for (; n <= n_tiles; ++n) iteration(RngTiles{}, n);
    } else {
      for (; n < n_gen0; ++n) iteration(PlainTiles{}, n);
      for (; n <= n_gen1; ++n) iteration(AnyTiles{}, n);
    }
  }
  vm_wait<0>();                              // nothing may still be writing LDS when the workgroup ends

  // ---- epilogue -------------------------------------------------------------
  float l_tot = half_sum(l_run);
  if (MODE == 2 && P.tiles != nullptr && lane == 0 && tiles_done > 0) atomicAdd(P.tiles + bh, tiles_done);
  if (!row_ok) return;
  if (P.lse != nullptr && hf == 0) {
    size_t at = (MODE == 1) ? (((size_t)split * P.n_bh + bh) * P.n_qrows + (i_me - P.q_row0)) : ((size_t)bh * S + i_me);
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

// out[i] = log sum_s exp(part[s][i]): the key splits of the log-sum-exp sweep, in fixed order
__global__ void lse_combine_kernel(const float* part, float* out, size_t n, int k) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float m = part[i];
  for (int s = 1; s < k; ++s) m = fmaxf(m, part[(size_t)s * n + i]);
  float z = 0.f;
  for (int s = 0; s < k; ++s) z += __expf(part[(size_t)s * n + i] - m);
  out[i] = m + __logf(z);
}

hipError_t launch_lse_combine(const float* part, float* out, size_t n, int k, hipStream_t st) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(lse_combine_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part, out, n, k);
  return hipGetLastError();
}

// How many key splits even out the log-sum-exp launch: W workgroups of equal length cut
// k ways take ceil(W k / 512) / k rounds on 256 CUs x 2 workgroups; a split keeps at least 64 tiles, and
// every row must see a key in every split (the sampled rows start at row_first).
int lse_key_splits(int row_first, int n_s, int n_bh) {
  const int n_qtiles = (n_s + kFlashBQ - 1) / kFlashBQ;
  const long long W = (long long)n_qtiles * n_bh;
  const int min_tiles = row_first / kFlashBK;       // key tiles the first sampled row sees, at least
  int best = 1;
  double best_t = (double)((W + 511) / 512);
  for (int k = 2; k <= 8; k *= 2) {
    if (min_tiles / k < 64) break;
    double t = (double)((W * k + 511) / 512) / k;
    if (t < best_t - 1e-9) { best_t = t; best = k; }
  }
  return best;
}

template <int MODE, bool OUT_F32, bool IN_PLACE = false>
static hipError_t launch_one(const FlashParams& P, int grid, hipStream_t st) {
  size_t shmem = (MODE == 1) ? LDS_B_LSE : LDS_B;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&flash_kernel<MODE, OUT_F32, IN_PLACE>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((flash_kernel<MODE, OUT_F32, IN_PLACE>), dim3(grid), dim3(NT), shmem, st, P);
  return hipGetLastError();
}

hipError_t launch_flash(int mode, bool out_f32, const FlashParams& P, hipStream_t st) {
  int grid;
  if (mode == 2) {
    grid = (P.n_bh >= 8) ? 8 * P.n_qtiles * ((P.n_bh + 7) / 8) : P.n_qtiles * P.n_bh;
  } else {
    int bundles = P.n_qtiles * (mode == 1 ? P.k_splits : 1) * P.n_bkv;
    grid = ((bundles + 7) / 8) * 8 * P.group;
  }
  if (grid <= 0) return hipSuccess;
  switch (mode) {
    case 0: return out_f32 ? launch_one<0, true>(P, grid, st) : launch_one<0, false>(P, grid, st);
    case 1: return launch_one<1, false>(P, grid, st);
    default:
      if (P.cols_in_place)
        return out_f32 ? launch_one<2, true, true>(P, grid, st) : launch_one<2, false, true>(P, grid, st);
      return out_f32 ? launch_one<2, true>(P, grid, st) : launch_one<2, false>(P, grid, st);
  }
}

}  // namespace sa
