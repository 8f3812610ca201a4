// Flash-style attention kernels for gfx950: dense causal attention (Eq. 1-2),
// row log-sum-exp of the sampled queries (stage 1, pass 1) and attention under
// the merged column / slash / window mask (Eq. 3, Algorithm 1 last step).
//
// A wave owns 32 query rows.  Keys are visited in tiles of 64.  For every tile
// the wave forms S^T = K Q^T (keys x queries) with 32x32x16 bf16 MFMAs, so that
// one lane holds scores of ONE query (lane % 32) for 16 keys per 32-key half
// tile: the row-wise online softmax is then in-lane arithmetic plus a single
// exchange between lanes l and l^32.  The probabilities, rounded to bf16, are
// directly the B operand of O^T += V^T P^T, so the accumulators (O^T, head_dim x
// queries) again keep one query per lane and the rescale is a per-lane scalar.
// K tiles live in LDS as [key][d]; V is read from a pre-transposed copy
// (V^T, [d][key]) so both MFMA A operands are 16-byte LDS reads.
//
// Schedule.  A workgroup is two groups of four waves; each group owns one
// 128-row query tile (two neighbouring tiles of one head) with its own K/V
// stream.  Waves w and w+4 share a SIMD.  Left alone, two waves that alternate
// an MFMA section and a vector-ALU (softmax) section fall into step - both on
// the matrix pipe, then both on the vector pipe - and each pipe idles half the
// time.  Here the groups are held one phase apart by two workgroup barriers per
// tile: while group 0 does the softmax of its tile t, group 1 issues the MFMAs of
// P V(t-1) and K Q^T(t), and vice versa, so every SIMD always has one wave
// feeding the matrix pipe and one feeding the vector pipe.
#include "sa_device.h"
#include "sa_kernels.h"

namespace sa {

namespace {

constexpr int BQ = kFlashBQ;          // 128 query rows per group
constexpr int BK = kFlashBK;          // 64 keys per tile
constexpr int NT = 512;               // two groups of four waves
// LDS tiles are unpadded (the direct global->LDS loads write 1 KB runs); bank
// conflicts are avoided by XOR-swizzling the 16-byte chunk index with the row.
constexpr int KROW_B = 256;           // bytes per K row in LDS: 16 chunks, chunk c of row p stored at c ^ (p & 15)
constexpr int VROW_B = 128;           // bytes per V^T row in LDS: 8 chunks, chunk c of row d stored at c ^ ((d >> 1) & 7)
constexpr int KTILE_B = BK * KROW_B;
constexpr int VTILE_B = kHeadDim * VROW_B;
constexpr int AUX_B = 256;            // 64 dwords per tile: key indices or mask words
constexpr int OFF_K = 0;                       // per group: K tiles, double buffered
constexpr int OFF_V = 2 * KTILE_B;             //            V^T tiles, double buffered
constexpr int OFF_A = OFF_V + 2 * VTILE_B;     //            aux words, ring of four
constexpr int GROUP_B = OFF_A + 4 * AUX_B;     // 66560 bytes per group
constexpr float kLazy = 8.0f;         // rescale only when a row maximum grows by more than 2^8

enum TileKind : int { TK_PLAIN = 0, TK_CAUSAL = 1, TK_COLIDX = 2, TK_RANGE = 3 };

struct Tile {
  const uint16_t* kb;   // K array the tile's rows come from (row stride 128 elements)
  const uint16_t* vt;   // &V^T[0][first key] (row stride S_pad elements)
  const int32_t* idx;   // key index of each of the 64 rows (TK_COLIDX) or null
  int krow0;            // first row of the tile in kb
  int kmax;             // last row of kb that may be read (rows past it are clamped: they are masked anyway)
  int j0;               // first key index (contiguous tiles)
  int kind;
};

// Direct global -> LDS load: lane l of the wave moves N bytes from global address
// `base` + `off` (base wave-uniform, in scalar registers; off per lane) to LDS
// address `lds` + N * l (`lds` wave-uniform, passed in M0).  It is written as inline
// assembly so that the waits on it are the explicit vm_wait calls below: the
// compiler, when it issues this instruction itself, makes every later LDS read wait
// for all of them (it cannot tell the buffers apart), which serialises the prefetch
// of tile t+1 with the arithmetic on tile t.  The loads of a wave complete in order.
// a wave-uniform pointer, forced into scalar registers
__device__ __forceinline__ uint64_t scalar_ptr(const void* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ void dma16(uint64_t base, uint32_t off, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds)
               : "memory", "m0");
}
__device__ __forceinline__ void dma4(uint64_t base, uint32_t off, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(base), "s"(lds)
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
template <int MODE, bool OUT_F32>
__global__ __launch_bounds__(NT, 1) void flash_kernel(FlashParams P) {
  extern __shared__ __attribute__((aligned(16))) char smem_all[];
  constexpr bool WITH_V = (MODE != 1);

  const int tid = threadIdx.x;
  const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in an SGPR
  const int grp = wave8 >> 2;          // phase group
  const int wave = wave8 & 3;          // wave within the group
  const int lane = tid & 63;
  const int ql = lane & 31;   // query within the wave / row within a 32-row operand
  const int hf = lane >> 5;   // which half of the contraction block this lane feeds
  char* smem = smem_all + grp * GROUP_B;
  const uint32_t smem_lds = __builtin_amdgcn_readfirstlane(
      (int)(uintptr_t)(__attribute__((address_space(3))) char*)smem_all + grp * GROUP_B);

  // ---- which head and pair of query tiles this workgroup owns ----------------
  const int n_pairs = (P.n_qtiles + 1) >> 1;
  int bh, ap;
  {
    const int bid = blockIdx.x;
    if (MODE == 2) {
      // heads are sliced over the 8 XCDs (workgroups go round-robin to XCDs) and an
      // XCD works through one head at a time, heavy (late) query tiles first: the
      // workgroups resident on it then stream the gathered columns of the same head,
      // a working set (tens of MB per XCD) that the memory-side cache can hold.
      if (P.n_bh >= 8) {
        int xcd = bid & 7, slot = bid >> 3;
        ap = n_pairs - 1 - slot % n_pairs;
        bh = xcd + 8 * (slot / n_pairs);
        if (bh >= P.n_bh) return;
      } else {
        ap = n_pairs - 1 - bid / P.n_bh;
        bh = bid % P.n_bh;
        if (ap < 0) return;
      }
    } else {
      // a bundle = the query heads sharing one KV head at one pair of query tiles; the
      // bundle's workgroups land on one XCD so the K/V stream is shared in L2.
      int xcd = bid & 7, slot = bid >> 3;
      int bl = slot / P.group, hg = slot % P.group;
      int bundle = bl * 8 + xcd;
      if (bundle >= n_pairs * P.n_bkv) return;
      ap = n_pairs - 1 - bundle / P.n_bkv;
      int bkv = bundle % P.n_bkv;
      bh = bkv * P.group + hg;
    }
  }
  const int bkv = bh / P.group;
  const int S = P.S;
  const uint16_t* kbase = P.k + (size_t)bkv * S * kHeadDim;
  const uint16_t* vtbase = WITH_V ? P.vt + (size_t)bkv * kHeadDim * P.S_pad : nullptr;
  const int32_t* cidx = nullptr;
  const int32_t* dl = nullptr;
  const uint32_t* cbits = nullptr;
  const uint32_t* obits = nullptr;
  int col_cnt = 0, d_cnt = 0;
  if (MODE == 2) {
    cidx = P.col_idx_pad + (size_t)bh * P.cidx_stride;
    col_cnt = min(max(P.col_cnt[bh], 0), S);
    dl = P.dlist + (size_t)bh * P.dlist_stride;
    d_cnt = min(max(P.dcnt[bh], 0), P.dlist_stride);
    cbits = P.col_bits + (size_t)bh * P.cb_words;
    obits = P.off_bits + (size_t)bh * P.rb_words;
  }

  // tile schedule of query tile `qt`: gathered-column tiles, then range tiles
  // (sparse), or the causal sweep (dense / log-sum-exp)
  auto schedule = [&](int qt, int& nct, int& nrg) -> int {
    nct = 0; nrg = 0;
    if (qt >= P.n_qtiles) return 0;
    const int first = P.q_row0 + qt * BQ;
    const int last = min(first + BQ, P.q_row0 + P.n_qrows) - 1;
    if (MODE == 2) {
      int lo = 0, hi = col_cnt;      // selected columns j <= last row of the tile (ascending list)
      while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (cidx[mid] <= last) lo = mid + 1; else hi = mid;
      }
      nct = (lo + BK - 1) / BK;
      lo = 0; hi = d_cnt;            // tile diagonals d with key tile first/64 + 1 - d >= 0
      while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (dl[mid] <= first / BK + 1) lo = mid + 1; else hi = mid;
      }
      nrg = lo;
      return nct + nrg;
    }
    return min(last, S - 1) / BK + 1;
  };
  const int a = 2 * ap + (1 - grp);          // group 0 takes the later (heavier) tile of the pair
  int n_col_tiles, n_rng, pn_col, pn_rng;
  const int n_tiles = __builtin_amdgcn_readfirstlane(schedule(a, n_col_tiles, n_rng));
  const int n_partner = schedule(2 * ap + grp, pn_col, pn_rng);
  const int n_iter = __builtin_amdgcn_readfirstlane(max(n_tiles, n_partner));   // both groups pass the same barriers
  n_col_tiles = __builtin_amdgcn_readfirstlane(n_col_tiles);
  n_rng = __builtin_amdgcn_readfirstlane(n_rng);

  const int i0 = P.q_row0 + a * BQ;                     // first query row of the group
  const int i_last_g = min(i0 + BQ, P.q_row0 + P.n_qrows) - 1;   // last valid row (< i0 for an empty group)
  const int iw0 = i0 + 32 * wave;                        // first query row of the wave
  const int i_me = iw0 + ql;                             // this lane's query row
  const bool row_ok = i_me <= i_last_g;
  const int a64 = i0 / BK;   // index of the 64-key tile that holds row i0 (i0 % 128 == 0 in MODE 2)
  const uint16_t* kc = (MODE == 2) ? P.kc + (size_t)bh * P.S_pad * kHeadDim : nullptr;
  const uint16_t* vct = (MODE == 2) ? P.vct + (size_t)bh * kHeadDim * P.S_pad : nullptr;

  // Descriptor of tile t.  A range tile is named by its tile diagonal d: key tile
  // a64 + 1 - d.  The d values come from a list in global memory; they are fetched
  // (fetch_d) two tiles ahead of their first use and handed on in scalar registers,
  // so that no phase waits on a scalar load.
  auto fetch_d = [&](int t) -> int {
    // read through the constant address space: the list is not written while the kernel
    // runs, and only so does the load stay a scalar one (tracked apart from the vector
    // loads in flight) behind the barriers and inline assembly of the loop
    typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
    if (MODE == 2 && t >= n_col_tiles && t < n_tiles)
      return ((const_i32_ptr)(uintptr_t)dl)[n_rng - 1 - (t - n_col_tiles)];   // far to near
    return 0;
  };
  auto get_tile = [&](int t, int d) -> Tile {
    Tile T;
    if (MODE == 2 && t < n_col_tiles) {
      T.kb = kc;
      T.krow0 = t * BK;
      T.kmax = P.S_pad - 1;
      T.vt = vct + t * BK;
      T.idx = cidx + t * BK;
      T.j0 = 0;
      T.kind = TK_COLIDX;
    } else {
      int j0;
      if (MODE == 2) {
        j0 = (a64 + 1 - d) * BK;
        T.kind = TK_RANGE;
      } else {
        j0 = t * BK;
        T.kind = (j0 + BK - 1 > i0) ? TK_CAUSAL : TK_PLAIN;
      }
      T.kb = kbase;
      T.krow0 = j0;
      T.kmax = S - 1;
      T.vt = WITH_V ? vtbase + j0 : nullptr;
      T.idx = nullptr;
      T.j0 = j0;
    }
    return T;
  };

  // ---- Q^T operand: 8 contraction steps of 16, resident in registers -------
  bf16x8 qf[8];
  {
    int qr = row_ok ? i_me : max(min(i_last_g, S - 1), 0);
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
  // swizzle maps there.  Wave w of the group issues runs w, w+4, w+8, w+12.
  // The lane's byte offset inside a run is fixed for the whole kernel, and run n of
  // a wave lies a constant 16 K rows / 32 V^T rows after run 0 (neither the swizzle
  // nor the slot permutation sees that step): per tile and per load only the scalar
  // base address changes, so issuing a tile costs no vector arithmetic.
  uint32_t koff0, voff0;
  {
    int p = 4 * wave + (lane >> 4);                // physical K row of run `wave`
    int c = (lane & 15) ^ (p & 15);                // logical 16-byte chunk stored there
    koff0 = krow_slot(p) * KROW_B + c * 16;        // key row within the tile, byte in the row
    int d = 8 * wave + (lane >> 3);                // V^T row
    int cv = (lane & 7) ^ ((d >> 1) & 7);
    voff0 = (uint32_t)d * (uint32_t)P.S_pad * 2u + cv * 16;
  }
  // The 4 loads of a V^T tile and the 4 of a K tile are issued one at a time
  // (load_v_one / load_k_one), so the callers can spread them between their other
  // instructions: a wave that issues them back to back stalls ~40 cycles on each.
  bool ld_v_on = false, ld_k_on = false;
  uint64_t ld_vbase = 0, ld_kbase = 0;
  uint32_t ld_vdst = 0, ld_kdst = 0, ld_klim = 0;
  auto load_v_begin = [&](int t, int d, bool on) {
    ld_v_on = WITH_V && on;
    if (ld_v_on) {
      const Tile T = get_tile(t, d);
      ld_vbase = scalar_ptr(T.vt);
      ld_vdst = smem_lds + OFF_V + (t & 1) * VTILE_B + 1024 * wave;
    }
  };
  auto load_k_begin = [&](int t, int d, bool on) {
    ld_k_on = on;
    if (ld_k_on) {
      const Tile T = get_tile(t, d);
      // a range tile may start past the last key (all of it masked): the base row is
      // clamped, and so is each lane's byte offset, to the last row that exists
      const int row0 = min(T.krow0, T.kmax);
      ld_kbase = scalar_ptr(T.kb + (size_t)row0 * kHeadDim);
      ld_klim = (uint32_t)(T.kmax - row0) * KROW_B + (koff0 & (KROW_B - 1));
      ld_kdst = smem_lds + OFF_K + (t & 1) * KTILE_B + 1024 * wave;
    }
  };
  auto load_v_one = [&](int n) {
    if (ld_v_on) dma16(ld_vbase + (uint64_t)(64 * n) * (uint64_t)P.S_pad, voff0, ld_vdst + 4096 * n);
  };
  auto load_k_one = [&](int n) {
    if (ld_k_on) dma16(ld_kbase, min(koff0 + 16 * KROW_B * n, ld_klim), ld_kdst + 4096 * n);
  };
  // the 64 dwords that go with a tile: the key indices of a gathered tile, or for a
  // range tile 16 words of the offset bitmap (covering every offset of the 128 x 64
  // tile) followed by the 2 words of the column bitmap.  One load, by wave 0.
  auto dma_aux = [&](int t, int d) {
    if (MODE != 2 || wave != 0) return;
    const Tile T = get_tile(t, d);
    const uint32_t dst = smem_lds + OFF_A + (t & 3) * AUX_B;
    if (T.idx != nullptr) {
      dma4(scalar_ptr(T.idx), 4u * lane, dst);
    } else {
      int wb = (P.off_max - (i0 - T.j0 + BQ - 1)) >> 5;          // first offset-bitmap word needed
      // lanes 0..15: offset words wb ..; lanes 16..63: the two column words, alternating.
      // The column bitmaps lie below the offset bitmaps in the workspace (and within
      // 4 GB of them), so offsets from the column word are non-negative 32-bit values.
      const uint32_t* cw = cbits + (T.j0 >> 5);
      const uint32_t gap = (uint32_t)((const char*)(obits + wb) - (const char*)cw);
      dma4(scalar_ptr(cw), lane < 16 ? gap + 4u * lane : 4u * (lane & 1), dst);
    }
  };
  const bool aux_wave = (MODE == 2) && (wave == 0);

  // Whether this wave has anything to do on tile t.  For the sparse kernel the answer
  // needs two of the tile's aux words from LDS; they are read early (act_words) and
  // looked at later (tile_active), so that the wait for them hides behind MFMAs.
  auto act_words = [&](int t, uint32_t& w0, uint32_t& w1) {
    if (MODE != 2) return;
    const uint32_t* ax = reinterpret_cast<const uint32_t*>(smem + OFF_A + (t & 3) * AUX_B);
    w0 = ax[t < n_col_tiles ? 0 : 16];             // first key index, or first column-bitmap word
    w1 = ax[17];                                   // second column-bitmap word (range tiles)
  };
  auto tile_active = [&](int t, int d, uint32_t w0, uint32_t w1) -> bool {
    const Tile T = get_tile(t, d);
    bool act;
    if (MODE == 2 && T.kind == TK_COLIDX) {
      act = (int)w0 <= iw0 + 31;                   // else every column of the tile lies after the wave's rows
    } else {
      act = T.j0 <= iw0 + 31;                      // else every key of the tile lies after the wave's rows
      // a range tile whose keys all belong to selected columns was covered by the
      // column pass; one that starts past the sequence end holds no key at all
      if (MODE == 2) act = act && ((w0 & w1) != 0xFFFFFFFFu) && (T.j0 < S);
    }
    return __builtin_amdgcn_readfirstlane((int)act) != 0;
  };

  // ---- operand ring and the MFMA phase -------------------------------------------
  // A phase issues up to 32 MFMAs: 16 of P V(t) (keys in groups of 16, head-dim
  // blocks 0..3 within a group) and 16 of K Q^T(t+1) (two 32-key halves, 8
  // contraction steps each).  Their A operands come from LDS through a ring of 8
  // registers x 16 bytes: after MFMA i has consumed slot i % 8, the operand of MFMA
  // i + 8 is read into it, so every read has 7 MFMAs (~250 cycles) to return and the
  // matrix pipe does not wait on LDS round trips.  sched_barrier pins the order: the
  // compiler would otherwise sink each read down to its use.
  f32x16 s[2];
  uint32_t pk[2][8];
  uint4 R[8];
#define SA_PIN() __builtin_amdgcn_sched_barrier(0)
  // K operand i = 8 sb + ks: 32-key half sb, contraction step ks
  auto ld_k = [&](int slot, int i, int buf) {
    // row p = 32 sb + ql; logical chunk 2 ks + hf lives at physical chunk (2 ks + hf) ^ (p & 15)
    const int sb = i >> 3, ks = i & 7;
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
  // P V(t): on entry the ring holds V operands 0..7 (read during the softmax phase);
  // the second half of the sweep re-fills it with the first 8 K operands of tile t+1
  // (read even when that tile turns out to need no work from this wave)
  auto mm_pv = [&](int bufp, int bufq, auto&& next_tile_setup) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      // the loads of the tile after next go out under the MFMAs: set-up after the
      // first MFMA has been issued, then one load per 3 MFMAs
      if (i == 1) next_tile_setup();
      if (i >= 4 && (i - 4) % 3 == 0) load_k_one((i - 4) / 3);
      const int sb = i >> 3, u = (i >> 2) & 1, mb = i & 3;
      uint4 pw = {pk[sb][4 * u], pk[sb][4 * u + 1], pk[sb][4 * u + 2], pk[sb][4 * u + 3]};
      o[mb] = mfma_32x32x16(as_bf16x8(R[i & 7]), as_bf16x8(pw), o[mb]);      // O^T += V^T P^T
      SA_PIN();
      if (i + 8 < 16) ld_v(i & 7, i + 8, bufp); else ld_k(i & 7, i - 8, bufq);
      SA_PIN();
    }
  };
  // K Q^T(t+1): the ring holds K operands 0..7 unless `cold`.
  // Element r of s[sb] is key j0 + 32*sb + 16*(r/8) + 8*hf + r%8 against query i_me.
  auto mm_qk = [&](int bufq, bool cold) {
    if (cold) {
#pragma unroll
      for (int i = 0; i < 8; ++i) ld_k(i, i, bufq);
    }
    SA_PIN();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (cold && (i & 3) == 2) load_k_one(i >> 2);   // not issued by a P V sweep before
      const int sb = i >> 3, ks = i & 7;
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
  auto step_softmax = [&](int t, int d) {
    const Tile T = get_tile(t, d);
    const int buf = t & 1;
    const float ninf = -__builtin_inff();
    if (T.kind == TK_CAUSAL) {
      if (T.j0 + BK - 1 > iw0) {
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
          int tl = i_me - (T.j0 + 32 * sb + 8 * hf);   // keep bit b iff b <= tl
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            int b = 16 * (r >> 3) + (r & 7);
            s[sb][r] = (b <= tl) ? s[sb][r] : ninf;
          }
        }
      }
    } else if (MODE == 2 && T.kind == TK_COLIDX) {
      const int32_t* il = reinterpret_cast<const int32_t*>(smem + OFF_A + (t & 3) * AUX_B);
      if (il[BK - 1] > iw0) {
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const int4* ip = reinterpret_cast<const int4*>(il + 32 * sb + 16 * u + 8 * hf);
            int4 x0 = ip[0], x1 = ip[1];
            int jj[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e)
              s[sb][8 * u + e] = (jj[e] <= i_me) ? s[sb][8 * u + e] : ninf;
          }
      }
    } else if (MODE == 2 && T.kind == TK_RANGE) {
      const uint32_t* mw = reinterpret_cast<const uint32_t*>(smem + OFF_A + (t & 3) * AUX_B);
      const int wb = (P.off_max - (i0 - T.j0 + BQ - 1)) >> 5;
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        int tl = i_me - (T.j0 + 32 * sb + 8 * hf);
        int x0 = P.off_max - tl;                       // >= 0 by construction of the bitmap
        int k = (x0 >> 5) - wb;                        // 0 .. 8: word of the staged window
        uint32_t lo = mw[k], hi = mw[k + 1];
        uint32_t ow = __builtin_amdgcn_alignbit(hi, lo, x0 & 31);  // bit b <-> offset tl - b
        uint32_t cw = mw[16 + sb] >> (8 * hf);                     // bit 16u+e <-> key is a selected column
        uint32_t km = ow & ~cw;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int b = 16 * (r >> 3) + (r & 7);
          // all-ones where the pair is kept; then a bitwise select between score and -inf
          uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe(km, b, 1);
          s[sb][r] = __uint_as_float((__float_as_uint(s[sb][r]) & keep) | (0xFF800000u & ~keep));
        }
      }
    }

    float mx = s[0][0];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sb][r]);
    mx = half_max(mx);
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
    // the operand ring is idle: fetch the first 8 V operands of this tile's P V now,
    // so that the reads return under the exponentials
    if (WITH_V) {
      SA_PIN();
#pragma unroll
      for (int i = 0; i < 8; ++i) ld_v(i, i, buf);
      SA_PIN();
    }
    float rs = 0.f;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      float p[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[r] = fast_exp2(fmaf(s[sb][r], c2, -m_run));
        rs += p[r];
        if ((r & 7) == 7) {                  // one load of the next V^T tile every 8 keys
          SA_PIN();
          load_v_one(2 * sb + (r >> 3));
          SA_PIN();
        }
      }
#pragma unroll
      for (int r = 0; r < 8; ++r) pk[sb][r] = pack_bf16x2(p[2 * r], p[2 * r + 1]);
    }
    l_run += rs;
  };

  // ---- the two-phase pipeline --------------------------------------------------------
  // Per group and tile t:
  //   softmax phase(t): issue V(t+1); softmax(t);               wait for K(t+1), aux(t+1)
  //   MFMA phase(t):    issue aux(t+2), K(t+2); P V(t), K Q^T(t+1);   wait for V(t+1)
  // The two groups run the same sequence half an iteration apart.  A buffer is
  // re-filled only after the barrier that follows its last reader; a load is waited
  // for by the wave that issued it before the barrier that precedes its first reader
  // (loads complete in order, so "at most n in flight" means everything but the last n
  // has landed).  The K loads go out between the MFMAs, whose issue slots are mostly
  // idle, the V loads between the exponentials.
  unsigned long long tiles_done = 0;
  bool act_t = false;                        // this wave has work on the tile whose softmax comes next
  int d0 = fetch_d(0), d1 = fetch_d(1), d2 = 0;   // tile diagonals of tiles t, t+1 and (in flight) t+2
  auto softmax_phase = [&](int t) {          // window: d0 = tile t, d1 = tile t+1
    load_v_begin(t + 1, d1, t + 1 < n_tiles);
    if (act_t) {
      step_softmax(t, d0);                   // issues the V loads between its exponentials
    } else {
#pragma unroll
      for (int n = 0; n < 4; ++n) load_v_one(n);
    }
    if (ld_v_on) vm_wait<4>(); else vm_wait<0>();
  };
  auto mfma_phase = [&](int t) {             // window: d0 = tile t+1, d1 = tile t+2; t = -1: only K Q^T(0)
    const bool have_next = t + 1 < n_tiles;
    const bool more = t + 2 < n_tiles;
    uint32_t aw0 = 0, aw1 = 0;
    if (have_next) act_words(t + 1, aw0, aw1);
    auto next_tile_setup = [&]() {
      if (more) dma_aux(t + 2, d1);
      load_k_begin(t + 2, d1, more);
    };
    __builtin_amdgcn_s_setprio(1);
    const bool pv = WITH_V && act_t;
    if (pv) mm_pv(t & 1, (t + 1) & 1, next_tile_setup); else next_tile_setup();
    const bool act_n = have_next && tile_active(t + 1, d0, aw0, aw1);
    if (act_n) mm_qk((t + 1) & 1, !pv);
    __builtin_amdgcn_s_setprio(0);
    if (!pv && !act_n) {
#pragma unroll
      for (int n = 0; n < 4; ++n) load_k_one(n);
    }
    tiles_done += act_n ? 1 : 0;
    act_t = act_n;
    if (WITH_V) {                            // V(t+1) went out before the loads of this phase
      if (!more) vm_wait<0>();
      else if (aux_wave) vm_wait<5>();
      else vm_wait<4>();
    }
  };
#undef SA_PIN

  // prologue: K(0), V(0) and the aux words of tile 0
  if (n_tiles > 0) {
    dma_aux(0, d0);
    load_k_begin(0, d0, true);
    load_v_begin(0, d0, true);
#pragma unroll
    for (int n = 0; n < 4; ++n) { load_k_one(n); load_v_one(n); }
  }
  // vmcnt(0), as the builtin: the compiler then also knows that the Q loads above have
  // landed and places no waits of its own for them inside the loop, where they would
  // wait for the loads in flight there as well
  __builtin_amdgcn_s_waitcnt(0x0f70);
  wg_barrier();
  // group 1 starts one barrier late and group 0 passes one more at the end, so the
  // MFMA phase of one group always coincides with the softmax phase of the other
  if (grp == 1) wg_barrier();
  for (int t = 0; t < n_iter; ++t) {
    mfma_phase(t - 1);                       // t = 0: K Q^T(0) only
    wg_barrier();
    d2 = fetch_d(t + 2);                     // in flight during the softmax phase
    softmax_phase(t);
    wg_barrier();
    d0 = d1; d1 = d2;
  }
  mfma_phase(n_iter - 1);                    // the last P V
  if (grp == 0) wg_barrier();

  // ---- epilogue -------------------------------------------------------------
  float l_tot = half_sum(l_run);
  if (MODE == 2 && P.tiles != nullptr && lane == 0 && tiles_done > 0) atomicAdd(P.tiles + bh, tiles_done);
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
  size_t shmem = 2 * GROUP_B;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&flash_kernel<MODE, OUT_F32>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((flash_kernel<MODE, OUT_F32>), dim3(grid), dim3(NT), shmem, st, P);
  return hipGetLastError();
}

hipError_t launch_flash(int mode, bool out_f32, const FlashParams& P, hipStream_t st) {
  int grid;
  const int n_pairs = (P.n_qtiles + 1) / 2;
  if (mode == 2) {
    grid = (P.n_bh >= 8) ? 8 * n_pairs * ((P.n_bh + 7) / 8) : n_pairs * P.n_bh;
  } else {
    int bundles = n_pairs * P.n_bkv;
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
