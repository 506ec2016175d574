// Tree-masked verification attention, bf16 inputs, MFMA path (gfx950).
//
// What it computes (Section 2.1 step 2 of the paper: the target model scores
// all draft candidates in one pass; Section 3.1.2: candidates form a tree and
// are verified through a tree attention mask): every tree node attends to the
// committed KV prefix, to itself and to its tree ancestors.
//
// Mapping.  The G query heads that share one KV head and the T tree nodes are
// packed into one matrix of M = T*G query rows (row m = node m/G, head m%G), so
// a KV head's K/V stream is read once for all of them.  One workgroup of
// WM x WN waves owns 32*WM query rows of one (sequence, KV head) and one split
// of the key range; the key range (prefix tiles, then tree tiles, 32 keys each)
// is cut into `splits` contiguous pieces.  Wave (wm, wn) holds query rows
// [32*wm, 32*wm+32) and processes every WN-th tile.  Workgroups have 4 waves
// (4x1 or 2x2) and two of them fit a CU: a single wave per SIMD is bound by its
// own in-order instruction issue (MFMA chain, exponentials, transfer
// bookkeeping), which a second workgroup on the CU overlaps.  (8-wave 2x4
// workgroups measured no better: they start later and their wider epilogue
// merge costs what the shorter tile loop gains.)
//
// Per tile and wave, with everything transposed so that a lane owns one query
// row:   S^T = K . Q^T   (v_mfma_f32_32x32x16_bf16, A = K rows from LDS,
// B = Q rows held in registers), masking, online softmax (running max and sum,
// max exchanged between the two half-waves with v_permlane32_swap), then
// O^T += V^T . P^T with V^T operands fetched by LDS transpose reads
// (ds_read_b64_tr_b16) from the row-major V tile.  The tree mask is a 128-bit
// ancestor set per node, built in LDS by the workgroups that own tree tiles.
//
// K/V travel HBM -> LDS directly (global_load_lds_dwordx4: 16 bytes per lane,
// 16 lanes per 256-byte row) into a ring of tiles, rounds ahead in flight;
// each lane fetches the 16-byte chunk that the XOR swizzle maps to its LDS
// slot, so that both the 128-bit K reads and the transpose V reads are free of
// bank conflicts.
#include <type_traits>

#include "jk_device.h"
#include "jk_internal.h"

namespace jk {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // native vector: plain loads/stores, no struct copies
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;
typedef __attribute__((address_space(3))) shortx4 lds_shortx4;

// LDS reads by byte address.  Tile bases are multiples of 256 bytes, so the XOR swizzles can
// be applied to the finished address: one address register per operand stream plus an
// immediate per read, instead of a register per read.
__device__ __forceinline__ bf16x8 lds_read128(unsigned addr) { return *(lds_bf16x8*)(size_t)addr; }
__device__ __forceinline__ bf16x8 lds_read_tr2(unsigned addr, unsigned second) {
  const shortx4 x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)(size_t)addr);
  const shortx4 x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)(size_t)(addr + second));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(x0, x1, 0, 1, 2, 3, 4, 5, 6, 7));
}

constexpr int kWaveRows = 32;   // query rows per wave
#ifndef JK_SPREAD
#define JK_SPREAD 1
#endif
constexpr int kSpread = JK_SPREAD;  // score phases of a pipelined tile pair that carry the next round's transfers (0: none)

struct KParams {
  const uint16_t *q, *kc, *vc, *kt, *vt;
  const int32_t *parent, *prefix_len;
  uint16_t* out;
  float* part_o;
  float2* part_ml;
  int B, T, Hkv, G, M, m_pad, max_prefix, splits, n_qtiles, total_wgs;
  unsigned long long mg_qtiles, mg_splits, mg_hkv, mg_g;  // floor(2^32 / d) + 1: n / d == (n * mg) >> 32 for n * d < 2^32
  unsigned long long mg_splits_m1;                        // the same for max(splits - 1, 1)
  long long q_sb, q_st, q_sh, kc_sb, kc_sl, kc_sh, kt_sb, kt_st, kt_sh, o_sb, o_st, o_sh;
  float scale_log2;
  // paged cache (block_table != nullptr): kc / vc are page pools, token t of sequence b lives in page
  // block_table[b * max_blocks + t / page_size], slot t % page_size; tpp = 32-key tiles per page
  const int32_t* block_table;
  int max_blocks, tpp, n_pages;
  int through;  // bit 0: outputs and partials, bit 1: the partials' (max, sum) pairs go through to memory (see the epilogue)
  long long page_stride;
  unsigned long long mg_tpp;
  // split merge inside this kernel (fused != 0; see merge_slice and the end of the kernel): sync = one
  // 64-byte line of words per (unit, row tile) group in the workspace header, spin_limit = polls a
  // workgroup spends waiting for its group before it leaves its slice to the group's last arriver
  unsigned* sync;
  unsigned* err;  // the workspace's sticky device error word
  int fused;
  unsigned spin_limit;
  int merge_rows, merge_shift;  // rows per slice = ceil(tile rows / splits); splits padded to 2^merge_shift
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// n / d by multiplication with the host-made constant mg = floor(2^32 / d) + 1 (exact while n * d < 2^32)
__device__ __forceinline__ int div_mg(int n, unsigned long long mg) {
  return (int)(((unsigned long long)(unsigned)n * mg) >> 32);
}

// max over the two half-waves (lane l and lane l^32)
__device__ __forceinline__ float half_swap_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int D>
struct Geo {
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int TILE_BYTES = kTileKeys * ROW_BYTES;
  static constexpr int CPR = D / 8;               // 16-byte chunks per row
  static constexpr int DK = D / 16;               // k-steps of Q.K^T
  static constexpr int DB = D / 32;               // 32-wide d blocks of the output
  static constexpr int O_LD = D + 4;              // padded row of the epilogue buffer (floats)
  static constexpr int NB = TILE_BYTES / 1024;    // 1 KB transfers per tile and tensor
  __device__ static __forceinline__ int kswz(int row) { return (row / (16 / CPR)) % CPR; }
  __device__ static __forceinline__ int vswz(int row) { return (row / (4 / DB)) % DB; }
  // K operand of k-step ks (A of S^T = K . Q^T; lane = key row c32, half g): chunk
  // (2*ks + g) ^ kswz of its row = byte address (tile + k_lane(lane)) ^ (ks << 5)
  __device__ static __forceinline__ unsigned k_lane(int lane) {
    const int c32 = lane & 31, g = lane >> 5;
    return (unsigned)(c32 * ROW_BYTES + ((kswz(c32) ^ g) << 4));
  }
  // V^T operand (transpose read: the 16 lanes of a group address 4 keys x 32 bytes, lane i of
  // the group receives d-column i of those 4 keys; contraction index 4*q'+r of MFMA j is key
  // 16*j + 8*q' + 4*g + r): 64-byte block db ^ vswz of key row 4*g + (lane%16)/4 = byte
  // address ((tile + v_lane(lane)) ^ (db << 6)) + 16*j*ROW_BYTES, second half 8 rows further
  __device__ static __forceinline__ unsigned v_lane(int lane) {
    const int g = lane >> 5, jj = (lane & 15) >> 2, cc = lane & 3, h16 = (lane & 31) >> 4;
    const int key_lo = 4 * g + jj;
    return (unsigned)(key_lo * ROW_BYTES + 32 * h16 + 8 * cc + (vswz(key_lo) << 6));
  }
};

using dev::dma16;
using dev::uniform_ptr;

// Wait until at most `rounds_behind` rounds of this wave's transfers are still in flight
// (they complete in issue order).  The count must be an immediate, hence the switch.
template <int STEP>
__device__ __forceinline__ void wait_dma(int rounds_behind) {
#define JK_VM(n) __builtin_amdgcn_s_waitcnt(dev::vmcnt_imm(n))
  switch (rounds_behind) {
    case 0: JK_VM(0); break;
    case 1: JK_VM(STEP); break;
    case 2: JK_VM(2 * STEP); break;
    case 3: JK_VM(3 * STEP); break;
    case 4: JK_VM(4 * STEP); break;
    case 5: JK_VM(5 * STEP); break;
    default: JK_VM(6 * STEP); break;
  }
#undef JK_VM
}

// The K/V streams of this (sequence, KV head) and the tile range of this split.
struct TileSrc {
  long long kc_sl, kt_st;  // row strides (elements)
  int L, T, n_ptiles, t_begin, t_end;
  // paged cache: page ids of the split's prefix tiles (LDS), index of the first one, tiles per page
  const int* pg_s;
  int pg_first, tpp;
  unsigned long long mg_tpp;
  long long page_stride;
};

constexpr int kMaxPagesPerSplit = 1024;  // page ids a workgroup keeps in LDS (the host keeps splits within it)

// Where a lane's 16-byte chunks sit inside a tile.  A wave-level transfer fills 1 KB =
// 64/CPR consecutive tile rows; lane l writes physical chunk l%CPR of row blk*(64/CPR) +
// l/CPR and fetches the logical chunk that the swizzle maps there, so the tile arrives
// already swizzled.  The 2*NB transfers of a tile (NB for K, then NB for V) are dealt to
// the NW waves in order, N to each: a wave therefore fetches only K or only V chunks.
template <int D, int NW>
struct LaneChunks {
  static constexpr int N = 2 * Geo<D>::NB / NW;
  static_assert(N >= 1 && Geo<D>::NB % N == 0, "a wave's transfers stay within K or within V");
  unsigned off[N];        // byte offset of the chunk from the first row of a full cache tile
  unsigned lds[N];        // byte offset inside the K+V tile pair
  const uint16_t* cache;  // K or V cache of this (sequence, KV head), wave-uniform
  const uint16_t* tree;   // K or V of the tree
  int wave, lane;
  // tile row and byte offset inside the row of chunk i: recomputed where the rare clamped
  // transfers need them rather than held in registers across the tile loop
  __device__ __forceinline__ void where(int i, int& row, unsigned& col_b) const {
    using G_ = Geo<D>;
    constexpr int RPB = 64 / G_::CPR;
    const int is_v = (wave * N) / G_::NB;
    const int blk = (wave * N + i) % G_::NB;
    row = blk * RPB + lane / G_::CPR;
    const int pc = lane % G_::CPR;
    const int kcol = pc ^ G_::kswz(row);                                  // K: 16-byte chunks swizzled
    const int vcol = (((pc >> 2) ^ G_::vswz(row)) << 2) | (pc & 3);       // V: 64-byte blocks swizzled
    col_b = (unsigned)(is_v ? vcol : kcol) * 16u;
  }
};

template <int D, int NW>
__device__ __forceinline__ void lane_chunks(LaneChunks<D, NW>& lc, int wave, int lane, const TileSrc& ts,
                                            const uint16_t* kc, const uint16_t* vc, const uint16_t* kt,
                                            const uint16_t* vt) {
  using G_ = Geo<D>;
  constexpr int N = LaneChunks<D, NW>::N;
  const int is_v = (wave * N) / G_::NB;
  lc.cache = uniform_ptr(is_v ? vc : kc);
  lc.tree = uniform_ptr(is_v ? vt : kt);
  lc.wave = wave;
  lc.lane = lane;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const int blk = (wave * N + i) % G_::NB;
    int row;
    unsigned col_b;
    lc.where(i, row, col_b);
    lc.off[i] = (unsigned)row * (unsigned)ts.kc_sl * 2u + col_b;  // < 2^31: strides are bounded by the host
    lc.lds[i] = is_v * G_::TILE_BYTES + blk * 1024;
  }
}

// First row of prefix tile t of this (sequence, KV head): contiguous cache, or looked up in the
// split's page list (the tile never straddles pages: a page holds whole tiles).
template <bool PAGED>
__device__ __forceinline__ const uint16_t* prefix_tile_base(const TileSrc& ts, const uint16_t* cache, int t) {
  if (!PAGED) return cache + (long long)t * kTileKeys * ts.kc_sl;
  const int pi = div_mg(t, ts.mg_tpp);
  const int page = __builtin_amdgcn_readfirstlane(ts.pg_s[pi - ts.pg_first]);
  return cache + (long long)page * ts.page_stride + (long long)(t - pi * ts.tpp) * kTileKeys * ts.kc_sl;
}

// Issue the transfers of round r (TPR tiles, K and V) into ring slot `slot` (byte address).
template <int D, int NW, int TPR, bool PAGED>
__device__ __forceinline__ void dma_round(int r, const TileSrc& ts, const LaneChunks<D, NW>& lc, unsigned slot) {
  using G_ = Geo<D>;
  constexpr int N = LaneChunks<D, NW>::N;
  const int t0 = ts.t_begin + r * TPR;
  if ((t0 + TPR) * kTileKeys <= ts.L) {
    // every tile of the round is a full prefix tile: a scalar base per tile plus the lane's
    // precomputed offsets
    if (!PAGED) {
      const long long tile_elems = (long long)kTileKeys * ts.kc_sl;
      const uint16_t* base = lc.cache + (long long)t0 * tile_elems;
#pragma unroll
      for (int w = 0; w < TPR; ++w) {
#pragma unroll
        for (int i = 0; i < N; ++i) dma16(base, lc.off[i], slot + w * 2 * G_::TILE_BYTES + lc.lds[i]);
        base += tile_elems;
      }
    } else {
#pragma unroll
      for (int w = 0; w < TPR; ++w) {
        const uint16_t* base = prefix_tile_base<true>(ts, lc.cache, t0 + w);
#pragma unroll
        for (int i = 0; i < N; ++i) dma16(base, lc.off[i], slot + w * 2 * G_::TILE_BYTES + lc.lds[i]);
      }
    }
    return;
  }
#pragma unroll 1
  for (int w = 0; w < TPR; ++w) {
    int t = t0 + w;
    if (t >= ts.t_end) t = ts.t_end - 1;  // duplicate of a real tile, never consumed
    const unsigned dst = slot + w * 2 * G_::TILE_BYTES;
    // ragged last prefix tile or tree tile: rows past the end re-read the last valid row
    const bool tree = t >= ts.n_ptiles;
    const int key0 = (tree ? t - ts.n_ptiles : t) * kTileKeys;
    const int last = (tree ? ts.T : ts.L) - 1 - key0;  // >= 0 (and >= 31 for a full prefix tile)
    const long long rs = tree ? ts.kt_st : ts.kc_sl;
    const uint16_t* base = tree ? lc.tree + (long long)key0 * rs : prefix_tile_base<PAGED>(ts, lc.cache, t);
#pragma unroll
    for (int i = 0; i < N; ++i) {
      int row;
      unsigned col_b;
      lc.where(i, row, col_b);
      const int rr = row < last ? row : last;
      dma16(base, (unsigned)rr * (unsigned)rs * 2u + col_b, dst + lc.lds[i]);
    }
  }
}

// The transfers of a round of full prefix tiles of a contiguous cache, one at a time: piece
// k = chunk k % N of tile k / N of the round.  Issued between the MFMAs of the tile loop: all
// waves of a workgroup leave the barrier together, and a burst of transfers from every wave
// queues up in front of the CU's one address unit (1 KB = 16 cycles each) while the waves
// wait to get rid of them with nothing else issued.
template <int D, int NW, int TPR>
struct RoundPieces {
  static constexpr int N = LaneChunks<D, NW>::N;
  static constexpr int PIECES = TPR * N;
  const uint16_t* base;  // first tile of the round
  long long tile_elems;
  unsigned slot;
  const LaneChunks<D, NW>* lc;
  __device__ __forceinline__ void issue(int k) const {
    const int w = k / N, i = k % N;
    dma16(base + w * tile_elems, lc->off[i], slot + w * 2 * Geo<D>::TILE_BYTES + lc->lds[i]);
  }
  // pieces [P * step / steps, P * (step + 1) / steps): an even share for each of `steps` places
  __device__ __forceinline__ void share(int step, int steps) const {
    // (fenced: left alone, the compiler gathers the MFMAs in front of the transfers)
    if (PIECES * step / steps < PIECES * (step + 1) / steps) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < PIECES; ++k)
      if (k >= PIECES * step / steps && k < PIECES * (step + 1) / steps) issue(k);
    if (PIECES * step / steps < PIECES * (step + 1) / steps) __builtin_amdgcn_sched_barrier(0);
  }
};

// Largest of a lane's 16 scores of a tile, as a tree three levels deep: a chain of fifteen
// dependent maxima would spend its latency with nothing else to issue.
__device__ __forceinline__ float max16(const floatx16& s) {
  const float a = fmaxf(fmaxf(s[0], s[1]), s[2]), b = fmaxf(fmaxf(s[3], s[4]), s[5]);
  const float c = fmaxf(fmaxf(s[6], s[7]), s[8]), d = fmaxf(fmaxf(s[9], s[10]), s[11]);
  const float e = fmaxf(fmaxf(s[12], s[13]), s[14]);
  return fmaxf(fmaxf(fmaxf(a, b), c), fmaxf(fmaxf(d, e), s[15]));
}

// Per-wave state of the online softmax and the output accumulation (32 query rows).
template <int D>
struct WaveState {
  bf16x8 q[Geo<D>::DK];
  floatx16 o[Geo<D>::DB];
  float m, l;
};

// S^T = K . Q^T of KT consecutive 32-key tiles (K tiles 2*TILE_BYTES apart in LDS) against
// the wave's 32 query rows.  A chain of MFMAs into one accumulator issues only every other
// MFMA slot (each waits for its predecessor's result), so two independent chains are kept in
// flight: the two tiles' (KT = 2), or the even and odd k-steps of the one tile, summed at
// the end (KT = 1).
template <int D, int KT>
__device__ __forceinline__ void qk_tiles(const WaveState<D>& st, unsigned k_addr, floatx16& s0, floatx16& s1) {
  using G_ = Geo<D>;
  floatx16 a0, a1;
#pragma unroll
  for (int i = 0; i < 16; ++i) a0[i] = a1[i] = 0.f;
  if (KT == 2) {
#pragma unroll
    for (int ks = 0; ks < G_::DK; ++ks) {
      const bf16x8 k0 = lds_read128(k_addr ^ (ks << 5));
      const bf16x8 k1 = lds_read128((k_addr ^ (ks << 5)) + 2 * G_::TILE_BYTES);
      a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, st.q[ks], a0, 0, 0, 0);
      a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, st.q[ks], a1, 0, 0, 0);
    }
    s0 = a0;
    s1 = a1;
  } else {
#pragma unroll
    for (int ks = 0; ks < G_::DK; ks += 2) {
      const bf16x8 k0 = lds_read128(k_addr ^ (ks << 5));
      const bf16x8 k1 = lds_read128(k_addr ^ ((ks + 1) << 5));
      a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, st.q[ks], a0, 0, 0, 0);
      a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, st.q[ks + 1], a1, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) s0[i] = a0[i] + a1[i];
  }
}

// Hide the masked keys of one tile's scores.  mask_mode: 0 none, 1 ragged prefix tail (keys
// >= nvalid hidden), 2 tree tile (bits = visibility of the tile's 32 keys; 0 for a tile
// past the end of the split).  Register i of a lane is key 8*(i/4) + 4*g + i%4 of the tile.
__device__ __forceinline__ void mask_tile(floatx16& sacc, int mask_mode, int nvalid, unsigned int bits, int g) {
  if (mask_mode == 0) return;
  // masked tiles are rare: keep their per-register key indices out of the loop-invariant
  // registers (the compiler would otherwise hold 32 of them across the whole tile loop)
  asm volatile("" : "+v"(g));
  if (mask_mode == 2) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int kk = 8 * (i / 4) + 4 * g + (i % 4);
      if (!((bits >> kk) & 1u)) sacc[i] = -INFINITY;
    }
  } else if (mask_mode == 1) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int kk = 8 * (i / 4) + 4 * g + (i % 4);
      if (kk >= nvalid) sacc[i] = -INFINITY;
    }
  }
}

// Online softmax and O^T += V^T . P^T for the KT tiles of a round whose (masked) scores are
// in s0 (and s1); v0 / v1 are their V tiles in LDS.  Two tiles share one running-maximum
// update, and their independent MFMA chains fill each other's latencies.
template <int D, int KT>
__device__ __forceinline__ void softmax_probs(WaveState<D>& st, const floatx16& s0, const floatx16& s1,
                                              float scale_log2, bf16x8 (&pb)[2 * KT]) {
  using G_ = Geo<D>;
  constexpr int DB = G_::DB;
  // The reference maximum m of a row moves only when the round's maximum exceeds it by more
  // than kLazy (in log2 units): weights then stay below 2^kLazy, harmless in fp32/bf16, and
  // the rescale of the accumulators becomes rare.  The result is unchanged: weights, their
  // sum and the accumulators all carry the same reference.
  constexpr float kLazy = 8.f;
  float tmax = max16(s0);
  if (KT == 2) tmax = fmaxf(tmax, max16(s1));
  tmax = half_swap_max(tmax) * scale_log2;
  const float m_old = st.m;
  const bool up = tmax > m_old + kLazy;  // false for tmax = -inf; true for the first visible key
  const float m_ref = up ? tmax : m_old;
  const float m_use = (m_ref == -INFINITY) ? 0.f : m_ref;
  const float alpha = up ? fast_exp2(m_old - m_use) : 1.f;
  const bool moved = up && (m_old != -INFINITY);  // accumulators are still zero before the first key
  st.m = m_ref;
  // probabilities become bf16 B operands of the value product
  float lsum = 0.f;
#pragma unroll
  for (int kt = 0; kt < KT; ++kt)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float sc = kt == 0 ? s0[8 * j + e] : s1[8 * j + e];
        const float pr = fast_exp2(fmaf(sc, scale_log2, -m_use));
        lsum += pr;
        pb[2 * kt + j][e] = (__bf16)pr;
      }
  st.l = fmaf(st.l, alpha, lsum);
  if (__any(moved)) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) st.o[db][i] *= alpha;
  }
}

template <int D, int KT>
__device__ __forceinline__ void softmax_pv(WaveState<D>& st, const floatx16& s0, const floatx16& s1,
                                           unsigned v_addr, float scale_log2) {
  using G_ = Geo<D>;
  constexpr int DB = G_::DB;
  bf16x8 pb[2 * KT];
  softmax_probs<D, KT>(st, s0, s1, scale_log2, pb);
  // ---- O^T += V^T . P^T
#pragma unroll
  for (int kt = 0; kt < KT; ++kt)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 vf = lds_read_tr2((v_addr ^ (db << 6)) + kt * 2 * G_::TILE_BYTES + 16 * j * G_::ROW_BYTES,
                                       8 * G_::ROW_BYTES);
        st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[2 * kt + j], st.o[db], 0, 0, 0);
      }
}

// Two unmasked tiles A, B of a round, software-pipelined by hand.  Within one tile the score
// product (MFMA), the softmax (vector ALU, a quarter-rate exponential per score) and the
// value product (MFMA) depend on each other, and a lone wave on its SIMD issues in order: it
// would use the two units one after the other.  Here the vector work of one tile is written
// between the MFMAs of the other:
//   S(A) | softmax(A) with S(B) | softmax(B) with O += P(A) V(A) | O += P(B) V(B)
template <int D>
struct PairPipe {
  using G_ = Geo<D>;
  static constexpr int DK = G_::DK, DB = G_::DB;
  // The pipelined pair never rescales the accumulators.  A row's reference m is fixed by the
  // first tile it sees (its maximum) or by the general path (which moves it, lazily, with a
  // rescale), and probabilities 2^(s - m) are allowed to grow: bf16 and fp32 have eight
  // exponent bits, so weights up to 2^kFrame lose no precision, and sums over 2^24 keys stay
  // far below 2^127.  A conditional rescale of the 64 accumulator registers inside the pair
  // costs the path that skips it a copy of all of them per tile pair (the compiler gives the
  // rescaled block new registers) and 64 registers of pressure where it sits.  A score more
  // than 2^kFrame above the reference (about 44 nats: a degenerate softmax) raises `left`;
  // the workgroup then repeats its whole split on the general path (see the tile loop).
  static constexpr float kFrame = 64.f;
  // The reference of a row: the maximum of the first tile its split sees (FIRST: nothing has been
  // accumulated for any row of the wave yet), kept from then on.  Later tiles do not even look for
  // their maximum: a weight beyond 2^kFrame shows in the row's sum, which the tile loop tests once,
  // after the last tile (left_frame below).
  static __device__ __forceinline__ float reference(WaveState<D>& st, const floatx16& s, float scale_log2, bool first) {
    if (!first) return st.m;  // (uniform)
    const float tmax = half_swap_max(max16(s)) * scale_log2;  // (an unmasked tile of finite scores: finite)
    const float m = (st.m == -INFINITY) ? tmax : st.m;
    st.m = m;
    return m;
  }
  // whether a weight of this lane's row went beyond 2^kFrame (or was NaN): its sum tells
  static __device__ __forceinline__ bool left_frame(const WaveState<D>& st) { return !(st.l < 1.8446744e19f); }

  // two scores -> probabilities (elements 2*i, 2*i+1 of the tile) into their bf16 operand slot; the
  // row sum takes the rounded probabilities (one dot product with (1, 1) instead of two additions,
  // and numerator and denominator of the softmax then carry the same rounding)
  static __device__ __forceinline__ void two_probs(const floatx16& s, int i, float scale_log2, float m_use,
                                                   float& lsum, bf16x8 (&pb)[2]) {
    const float p0 = fast_exp2(fmaf(s[2 * i], scale_log2, -m_use));
    const float p1 = fast_exp2(fmaf(s[2 * i + 1], scale_log2, -m_use));
    bf16x2 pk, one;
    pk[0] = (__bf16)p0;
    pk[1] = (__bf16)p1;
    one[0] = one[1] = (__bf16)1.f;
    lsum = __builtin_amdgcn_fdot2_f32_bf16(pk, one, lsum, false);
    pb[(2 * i) / 8][(2 * i) % 8] = pk[0];
    pb[(2 * i) / 8][(2 * i) % 8 + 1] = pk[1];
  }

  // k_addr / v_addr: LDS byte address of tile A's K / V tile plus the lane's Geo::k_lane / v_lane
  // `next`: the transfers of the round that refills the ring (SPREAD > 0), issued between the
  // MFMAs of the first SPREAD score phases
  // `first`: the wave's first tiles of its split (uniform)
  template <int SPREAD, class Pieces>
  static __device__ __forceinline__ void run(WaveState<D>& st, unsigned k_addr, unsigned v_addr, float scale_log2,
                                             const Pieces& next, bool first) {
    static_assert(DK == 8 || DK == 4, "head_dim 128 or 64");
    constexpr unsigned kNextTile = 2 * G_::TILE_BYTES;  // tile B's K (V) tile follows tile A's K and V
    auto v_frag = [&](unsigned tile_off, int j, int db) {
      return lds_read_tr2((v_addr ^ (db << 6)) + tile_off + 16 * j * G_::ROW_BYTES, 8 * G_::ROW_BYTES);
    };
    // LDS operands are fetched a whole phase ahead of the MFMAs that use them: a read issued
    // just before its MFMA would expose the LDS latency eight times per phase
    bf16x8 kf[DK], vfA[2 * DB], vfB[2 * DB];

    // ---- S(A), and between its MFMAs the transfers of the next round
    floatx16 sA, sB;
#pragma unroll
    for (int i = 0; i < 16; ++i) sA[i] = sB[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) kf[ks] = lds_read128(k_addr ^ (ks << 5));
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) {
      sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], st.q[ks], sA, 0, 0, 0);
      if (SPREAD > 0) next.share(ks, DK * SPREAD);
    }
    // (scheduling fences between the phases: left alone, the compiler hoists the next phase's
    // LDS reads above this phase and runs out of registers)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) kf[ks] = lds_read128((k_addr ^ (ks << 5)) + kNextTile);  // lands while the chain drains

    // ---- softmax(A) between the MFMAs of S(B).  The first half of S(B) is issued ahead of
    // the running-maximum update of A (a chain of dependent vector instructions that waits
    // for the last MFMA of S(A)): the matrix unit works through them meanwhile.
    bf16x8 pA[2], pB[2];
    float lsum = 0.f;
#pragma unroll
    for (int ks = 0; ks < DK / 2; ++ks) {
      sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], st.q[ks], sB, 0, 0, 0);
      if (SPREAD > 1) next.share(DK + ks, DK * SPREAD);
    }
    __builtin_amdgcn_sched_barrier(0);
    const float mA = reference(st, sA, scale_log2, first);
#pragma unroll
    for (int ks = DK / 2; ks < DK; ++ks) {
      sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], st.q[ks], sB, 0, 0, 0);
      if (SPREAD > 1) next.share(DK + ks, DK * SPREAD);
#pragma unroll
      for (int i = (ks - DK / 2) * (16 / DK); i < (ks - DK / 2 + 1) * (16 / DK); ++i)
        two_probs(sA, i, scale_log2, mA, lsum, pA);
    }
    st.l += lsum;
    __builtin_amdgcn_sched_barrier(0);

    // ---- softmax(B) between the MFMAs of O += V(A)^T . P(A)^T, in the same way.  The V
    // fragments of B are requested with those of A and arrive under this phase.
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int db = 0; db < DB; ++db) vfA[j * DB + db] = v_frag(0, j, db);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int db = 0; db < DB; ++db) vfB[j * DB + db] = v_frag(kNextTile, j, db);
#pragma unroll
    for (int db = 0; db < DB; ++db)
      st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfA[db], pA[0], st.o[db], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    lsum = 0.f;
    const float mB = mA;  // (the reference is fixed by now)
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfA[DB + db], pA[1], st.o[db], 0, 0, 0);
#pragma unroll
      for (int i = db * (8 / DB); i < (db + 1) * (8 / DB); ++i) two_probs(sB, i, scale_log2, mB, lsum, pB);
    }
    st.l += lsum;
    __builtin_amdgcn_sched_barrier(0);

    // ---- O += V(B)^T . P(B)^T
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int db = 0; db < DB; ++db)
        st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfB[j * DB + db], pB[j], st.o[db], 0, 0, 0);
  }
};

// One unmasked tile on its own: the odd last tile of a split of the 4x1 arrangement (everybody
// else waits for the splits that have one).  All LDS operands are requested before the first
// MFMA, the K fragments first: the V fragments then arrive under the score product and the
// softmax instead of in front of the value product.  Same fixed reference frame as the
// pipelined pair: no rescale of the accumulators here.  (For the one-tile rounds of the 2x2
// arrangement this path measured slower than the general one - 63 registers more, and those
// shapes are not bound by the tile arithmetic.)
template <int D>
__device__ __forceinline__ void lone_tile(WaveState<D>& st, unsigned k_addr, unsigned v_addr, float scale_log2,
                                          bool first) {
  using G_ = Geo<D>;
  constexpr int DK = G_::DK, DB = G_::DB;
  bf16x8 kf[DK], vf[2 * DB];
#pragma unroll
  for (int ks = 0; ks < DK; ++ks) kf[ks] = lds_read128(k_addr ^ (ks << 5));
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int db = 0; db < DB; ++db)
      vf[j * DB + db] = lds_read_tr2((v_addr ^ (db << 6)) + 16 * j * G_::ROW_BYTES, 8 * G_::ROW_BYTES);
  __builtin_amdgcn_sched_barrier(0);
  floatx16 a0, a1, s0;
#pragma unroll
  for (int i = 0; i < 16; ++i) a0[i] = a1[i] = 0.f;
#pragma unroll
  for (int ks = 0; ks < DK; ks += 2) {  // two chains: a dependent MFMA issues only every other slot
    a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], st.q[ks], a0, 0, 0, 0);
    a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks + 1], st.q[ks + 1], a1, 0, 0, 0);
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) s0[i] = a0[i] + a1[i];
  const float m = PairPipe<D>::reference(st, s0, scale_log2, first);
  bf16x8 pb[2];
  float lsum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) PairPipe<D>::two_probs(s0, i, scale_log2, m, lsum, pb);
  st.l += lsum;
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int db = 0; db < DB; ++db)
      st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[j * DB + db], pb[j], st.o[db], 0, 0, 0);
}

// Profiling build only (-DJK_TIMING, not part of the shipped library): thread 0 of every
// workgroup records the 100 MHz wall clock at points of the kernel (entry, speculative
// transfers issued, prefix length known, transfers issued, first round landed, loop done,
// columns parked, partials stored, arrived at the group word, group complete, end); jk_debug_read_timing copies the table of the last launch to the host
// (grids of at most 4096 workgroups).  Phase times of the kernel are measured with it.
#ifdef JK_TIMING
__device__ unsigned long long g_jk_ts[4096 * 16];
#define JK_TS(i) do { if (threadIdx.x == 0) g_jk_ts[blockIdx.x * 16 + (i)] = wall_clock64(); } while (0)
#else
#define JK_TS(i) do { } while (0)
#endif

// ---------------------------------------------------------------- split merge inside the kernel
// The workgroups that hold the S key splits of one (unit, row tile) group all run on one XCD
// (the host only asks for this path when its workgroup numbering guarantees it and the
// device's round-robin placement has been verified), so they can meet in that XCD's L2
// without the whole-cache write-back an agent-scope release costs on a part with eight L2s:
// partials are written with ordinary stores (a CU's vector cache writes through to L2; a
// store is acknowledged, and counted off vmcnt, once L2 has it), arrivals are counted with
// atomics that carry no device scope and therefore execute in that L2, and the partials are
// read back with loads that miss the reader's vector cache (invalidated first).  This is the
// hardware's own recipe for workgroup-scope synchronisation between CUs that share an L2.
__device__ __forceinline__ unsigned l2_atomic_add(unsigned* p, unsigned x) {
  unsigned v;
  asm volatile("global_atomic_add %0, %1, %2, off sc0\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p), "v"(x) : "memory");
  return v;
}
__device__ __forceinline__ unsigned l2_atomic_or(unsigned* p, unsigned x) {
  unsigned v;
  asm volatile("global_atomic_or %0, %1, %2, off sc0\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p), "v"(x) : "memory");
  return v;
}
__device__ __forceinline__ unsigned l2_atomic_swap(unsigned* p, unsigned x) {
  unsigned v;
  asm volatile("global_atomic_swap %0, %1, %2, off sc0\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p), "v"(x) : "memory");
  return v;
}
__device__ __forceinline__ void l2_atomic_add_noret(unsigned* p, unsigned x) {
  asm volatile("global_atomic_add %0, %1, off" ::"v"(p), "v"(x) : "memory");
}

// Group word: bits 0-7 arrivals of this call, bits 8-15 workgroups that gave up waiting, bits
// 16-31 call number (epoch).  The last arriver adds 2^16 - S - (give-ups << 8): count and
// give-ups return to zero and the epoch moves on, which is what the waiting workgroups look for.
constexpr unsigned kSyncCountMask = 0xffu, kSyncGaveUpOne = 0x100u, kSyncEpochOne = 0x10000u;

// Merge of rows [slice * R, (slice + 1) * R) of the group's row tile over all S splits, written to
// the output.  16 bytes (8 columns) of a row per thread; the arithmetic per element is that of the
// stand-alone merge kernel (splits in chunks of 8, running maximum), so both give the same bits.
struct MergeArgs {
  const float* part_o;
  const float2* part_ml;
  uint16_t* out;
  int M, m_pad, splits, G;
  unsigned long long mg_g;
  long long o_sb, o_st, o_sh;
};
// Reductions over aligned groups of 2^sh lanes (sh uniform): within a row of 16 lanes by DPP
// (quad permutes, then the mirrors of 8 and of 16 lanes: after the quads every lane of a quad
// holds the quad's value, so a mirror pairs quads as well as an exchange would), across rows by shuffles.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float group_max(float x, int sh) {
  if (sh >= 1) x = fmaxf(x, dpp_f<0xB1>(x));   // quad_perm [1,0,3,2]
  if (sh >= 2) x = fmaxf(x, dpp_f<0x4E>(x));   // quad_perm [2,3,0,1]
  if (sh >= 3) x = fmaxf(x, dpp_f<0x141>(x));  // row_half_mirror
  if (sh >= 4) x = fmaxf(x, dpp_f<0x140>(x));  // row_mirror
  if (sh >= 5) x = fmaxf(x, __shfl_xor(x, 16));
  if (sh >= 6) x = fmaxf(x, __shfl_xor(x, 32));
  return x;
}
__device__ __forceinline__ float group_sum(float x, int sh) {
  if (sh >= 1) x += dpp_f<0xB1>(x);
  if (sh >= 2) x += dpp_f<0x4E>(x);
  if (sh >= 3) x += dpp_f<0x141>(x);
  if (sh >= 4) x += dpp_f<0x140>(x);
  if (sh >= 5) x += __shfl_xor(x, 16);
  if (sh >= 6) x += __shfl_xor(x, 32);
  return x;
}

// Merge of one slice (R consecutive rows of a row tile) over all S splits, written to the output:
//   m = max_s m_s,  l = sum_s l_s 2^(m_s - m),  out = sum_s O_s 2^(m_s - m) / l.
// What limits it is the issue rate of a lone wave per SIMD (about eight cycles an instruction)
// and the CU's one path to L2, so: everything that does not depend on the partials (row numbers,
// byte offsets, the output address) is worked out by merge_prepare while the workgroup still
// waits for its partners; then (A) one thread per (row, split) fetches that pair's (max, sum)
// once, the 2^sh lanes of a row find the row's maximum and sum and park the normalised weight
// 2^(m_s - m) / l in LDS, while (B) one thread per (row, 4 columns) has its 8 bytes of every
// split's partial in flight and afterwards only multiplies and adds.  At most THREADS (row, split)
// pairs exist per slice (R = ceil(tile rows / S), S padded to 2^sh), one per thread.
struct MergeThread {
  unsigned raw_off;   // byte offset of this thread's 8 bytes in split 0's partial (rows of the first pass)
  unsigned ml_off;    // byte offset of this thread's (row, split) pair
  unsigned dst_off;   // element offset of this thread's 4 output columns in `out` (first pass)
  int r_b, row_lo, row_hi;
  bool live_a, live_b;
};

template <int D, int THREADS, int QROWS>
__device__ __forceinline__ MergeThread merge_prepare(const MergeArgs& p, int unit_id, int b, int kv, int slice, int R,
                                                     int sh, int tile_row0, int tid) {
  constexpr int CPR = D / 4;
  MergeThread t;
  const int S = p.splits;
  t.row_lo = slice * R;
  t.row_hi = min(QROWS, t.row_lo + R);
  const int chunk = tid % CPR;
  t.r_b = t.row_lo + tid / CPR;
  const unsigned unit_row0 = (unsigned)(unit_id * S) * (unsigned)p.m_pad + (unsigned)tile_row0;  // (the host keeps the
  t.live_b = t.r_b < t.row_hi && tile_row0 + t.r_b < p.M;                                        // partials below 2^31 bytes)
  t.raw_off = ((unit_row0 + (unsigned)t.r_b) * (unsigned)D + (unsigned)chunk * 4u) * 2u;
  const int ra = t.row_lo + (tid >> sh), sa = tid & ((1 << sh) - 1);
  t.live_a = ra < t.row_hi && tile_row0 + ra < p.M && sa < S;
  t.ml_off = (unit_row0 + (unsigned)ra + (unsigned)sa * (unsigned)p.m_pad) * 8u;
  const int m = tile_row0 + (t.live_b ? t.r_b : 0);
  const int node = div_mg(m, p.mg_g);
  t.dst_off = (unsigned)(b * p.o_sb + node * p.o_st + (long long)(kv * p.G + (m - node * p.G)) * p.o_sh) + chunk * 4;
  return t;
}

template <int D, int THREADS, int QROWS>
__device__ __forceinline__ void merge_run(const MergeArgs& p, const MergeThread& t, int sh, int b, int kv, int tile_row0,
                                          int tid, float* wbuf) {
  constexpr int CPR = D / 4, RPP = THREADS / CPR;
  if (t.row_lo >= t.row_hi) return;  // (uniform)
  const int S = p.splits;
  const unsigned char* part = reinterpret_cast<const unsigned char*>(p.part_o);
  const unsigned po_step = (unsigned)p.m_pad * D * 2;  // bytes from one split's partial to the next
  // ---- the (max, sum) pair of this thread's (row, split) first, then (B), first half: this thread's
  // bytes of up to 16 splits go out (32-bit offsets from one base: an add per load)
  float2 ml = make_float2(-INFINITY, 0.f);
  if (t.live_a) ml = *reinterpret_cast<const float2*>(reinterpret_cast<const unsigned char*>(p.part_ml) + t.ml_off);
  u32x2 raw[16];
  {
    unsigned off = t.raw_off;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      raw[u] = u32x2{0u, 0u};
      if (t.live_b && u < S) raw[u] = *reinterpret_cast<const u32x2*>(part + off);
      off += po_step;
    }
  }
  JK_TS(11);
  // ---- (A): pair (row, split) of this thread
  {
    if (!(ml.y > 0.f)) ml = make_float2(-INFINITY, 0.f);  // an empty split carries no weight
    const float mx = group_max(ml.x, sh);
    const float w = fast_exp2(ml.x - ((mx == -INFINITY) ? 0.f : mx));  // exp2(-inf) = 0
    const float l = group_sum(ml.y * w, sh);
    // (l > 0 for a live row: it sees at least its own tree key; dead rows are not stored.  A row's
    // weights start at a multiple of four floats, for the 16-byte reads below)
    const int wsh = sh < 2 ? 2 : sh;
    wbuf[((tid >> sh) << wsh) | (tid & ((1 << sh) - 1))] = w / l;
  }
  JK_TS(12);
  __syncthreads();
#ifdef JK_TIMING
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  JK_TS(13);
#endif
  // ---- (B), second half
  for (int r = t.r_b, pass = 0; r < t.row_hi; r += RPP, ++pass) {
    const bool live = tile_row0 + r < p.M;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const float* wrow = wbuf + ((r - t.row_lo) << (sh < 2 ? 2 : sh));
    for (int s0 = 0; s0 < S; s0 += 16) {
      if (pass > 0 || s0 > 0) {  // (beyond the first 16 splits of the first row: fetched here)
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          raw[u] = u32x2{0u, 0u};
          if (live && s0 + u < S)
            raw[u] = *reinterpret_cast<const u32x2*>(part + ((unsigned)(s0 + u) * po_step + t.raw_off + (unsigned)(pass * RPP * D * 2)));
        }
      }
      float w[16];
#pragma unroll
      for (int u = 0; u < 16; u += 4) {  // (slots beyond S hold zeros or other rows' weights; their data are zeros)
        const float4 w4 = *reinterpret_cast<const float4*>(wrow + s0 + u);
        w[u] = w4.x; w[u + 1] = w4.y; w[u + 2] = w4.z; w[u + 3] = w4.w;
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const float wu = s0 + u < S ? w[u] : 0.f;
        acc[0] = fmaf(__uint_as_float(raw[u][0] << 16), wu, acc[0]);
        acc[1] = fmaf(__uint_as_float(raw[u][0] & 0xffff0000u), wu, acc[1]);
        acc[2] = fmaf(__uint_as_float(raw[u][1] << 16), wu, acc[2]);
        acc[3] = fmaf(__uint_as_float(raw[u][1] & 0xffff0000u), wu, acc[3]);
      }
    }
    if (!live) continue;
    u32x2 pk;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      bf16x2 o;
      o[0] = (__bf16)acc[2 * h];
      o[1] = (__bf16)acc[2 * h + 1];
      pk[h] = __builtin_bit_cast(unsigned, o);
    }
    uint16_t* dst;
    if (pass == 0) {
      dst = p.out + t.dst_off;
    } else {
      const int m = tile_row0 + r;
      const int node = div_mg(m, p.mg_g);
      dst = p.out + b * p.o_sb + node * p.o_st + (long long)(kv * p.G + (m - node * p.G)) * p.o_sh + (tid % CPR) * 4;
    }
    *reinterpret_cast<u32x2*>(dst) = pk;  // (an ordinary store measured no slower than one through to memory here)
  }
  __syncthreads();  // wbuf is free again (another slice may follow)
}

// LDS plan of one workgroup, shared by the kernel and its launcher.
template <int D, int WM, int WN, int KT, bool PAGED = false, bool DEEP = false>
struct Plan {
  using G_ = Geo<D>;
  static constexpr int NW = WM * WN;                    // waves
  static constexpr int THREADS = 64 * NW;
  static constexpr int TPR = WN * KT;                   // tiles per round: KT consecutive ones per key column
  // (deeper rings measured slower: with six tiles c3 +0.9 us per call, with eight +4.6 - more transfers in
  // flight at once delay the first round's data by more than the later rounds gain)
  // DEEP (2x2 only): six tiles, two rounds in flight.  For a lone workgroup per CU that does nothing but stream a
  // long prefix (few query rows, no splits: c6) 64 KB in flight instead of 32 measured 59.3 -> 56.1 us; where two
  // workgroups share a CU they have that much in flight between them, and the deeper ring, which lets only one
  // fit, measured slower (c7 23.3 -> 30.6 us, c2 12.1 -> 12.4)
  static constexpr int RING_TILES = TPR >= 4 ? 2 * TPR : (DEEP ? 6 : 4);  // K+V tile pairs resident in LDS
  static constexpr int NR = RING_TILES / TPR;           // rounds resident in the ring
  static constexpr int QROWS = kWaveRows * WM;
  static constexpr int STAGE_BYTES = TPR * 2 * G_::TILE_BYTES;  // one round: TPR tiles of K and V
  static constexpr int RING_BYTES = NR * STAGE_BYTES;
  static constexpr int OBUF_BYTES = (WN - 1) * QROWS * G_::O_LD * 4;  // epilogue: O^T of key columns 1..WN-1
  static constexpr int PATCH_LD = D * 2 + 16;                         // padded bf16 row of the store patches
  static constexpr int PATCH_BYTES = kWaveRows * PATCH_LD;            // one owner wave's 32 finished rows
  static constexpr int EPI_BYTES = OBUF_BYTES + WM * PATCH_BYTES;
  static constexpr int UNION_BYTES = RING_BYTES > EPI_BYTES ? RING_BYTES : EPI_BYTES;
  static constexpr int ML_BYTES = NW * kWaveRows * 8;
  static constexpr int PAGES_BYTES = PAGED ? kMaxPagesPerSplit * 4 : 0;
  static constexpr int SMEM = UNION_BYTES + ML_BYTES + JK_MAX_TREE * 16 + JK_MAX_TREE * 4 + 16 + PAGES_BYTES;
  static constexpr int WGS_PER_CU = 2 * SMEM <= 160 * 1024 && NW <= 4 ? 2 : 1;
  static constexpr int REG_WGS = NW <= 4 ? 2 : 1;  // register budget: at most 256 VGPRs, no detour through AGPRs
  static_assert(SMEM <= 160 * 1024, "LDS budget");
  static_assert(THREADS >= JK_MAX_TREE, "one thread per tree node in the prologue");
};

template <int D, int WM, int WN, int KT, bool PAGED, bool DEEP>
__global__ __launch_bounds__((Plan<D, WM, WN, KT, PAGED, DEEP>::THREADS), (Plan<D, WM, WN, KT, PAGED, DEEP>::REG_WGS)) void tva_bf16_kernel(
    const KParams p) {
  using G_ = Geo<D>;
  using P_ = Plan<D, WM, WN, KT, PAGED, DEEP>;
  constexpr int TPR = P_::TPR;
  constexpr int DK = G_::DK, DB = G_::DB;
  constexpr int NW = P_::NW, THREADS = P_::THREADS, NR = P_::NR, QROWS = P_::QROWS;
  constexpr int TILE_BYTES = G_::TILE_BYTES;
  constexpr int STAGE_BYTES = P_::STAGE_BYTES;
  constexpr int DMA_PER_ROUND = TPR * LaneChunks<D, NW>::N;  // transfers a wave issues per round
  static_assert(NR >= 2 && (NR - 2) * DMA_PER_ROUND <= 63, "wave arrangement");

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];  // the kernel has no other LDS: offset 0
  unsigned char* ring = smem;
  float* obuf = reinterpret_cast<float*>(smem);                                   // [WN-1][QROWS][O_LD], after the loop
  float2* mlbuf = reinterpret_cast<float2*>(smem + P_::UNION_BYTES);              // [WN-1][QROWS]
  unsigned long long* anc = reinterpret_cast<unsigned long long*>(smem + P_::UNION_BYTES + P_::ML_BYTES);  // [128][2]
  int* par_s = reinterpret_cast<int*>(smem + P_::UNION_BYTES + P_::ML_BYTES + JK_MAX_TREE * 16);           // [128]
  int* repeat_s = par_s + JK_MAX_TREE;  // set by a wave whose scores left the pipelined pairs' fixed reference frame
  int* pg_s = repeat_s + 4;             // [1024], paged caches only

  JK_TS(0);
  // ---- touch every 64-byte line of the kernel arguments at once: the compiler fetches them
  // in several dependent batches, and this way only the first batch pays a trip to memory
  {
    typedef __attribute__((address_space(4))) const unsigned kernarg_word;
    kernarg_word* ka = (kernarg_word*)__builtin_amdgcn_kernarg_segment_ptr();
    static_assert(sizeof(KParams) > 320 && sizeof(KParams) <= 384, "six lines of kernel arguments");
    const unsigned a0 = ka[0], a1 = ka[16], a2 = ka[32], a3 = ka[48], a4 = ka[64], a5 = ka[80];
    asm volatile("" ::"s"(a0), "s"(a1), "s"(a2), "s"(a3), "s"(a4), "s"(a5));
  }
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WM;
  const int wn = wave / WM;
  const int c32 = lane & 31;
  const int g = lane >> 5;
  const int T = p.T, G = p.G, M = p.M, splits = p.splits;
  const float scale_log2 = p.scale_log2;

  // ---- which piece of work: consecutive hardware workgroup ids alternate between the 8
  // XCDs, so give each XCD a contiguous range of logical ids; q-tiles of one (b, kv, split)
  // are adjacent logical ids and therefore share that XCD's L2 for their common K/V.
  int wid;
  {
    const int n = blockIdx.x;
    const int per = p.total_wgs >> 3;  // total_wgs is padded to a multiple of 8
    wid = (n & 7) * per + (n >> 3);
  }
  int rest = div_mg(wid, p.mg_qtiles);
  const int qtile = wid - rest * p.n_qtiles;
  const int unit_id = div_mg(rest, p.mg_splits);  // b * Hkv + kv
  if (unit_id >= p.B * p.Hkv) return;             // padding workgroup
  const int split = rest - unit_id * splits;
  const int b = div_mg(unit_id, p.mg_hkv);
  const int kv = unit_id - b * p.Hkv;

  // ---- the prefix length first, as a per-lane vector load (an atomic load is never turned
  // into a scalar one, and the compiler must not see that the address is uniform, or it
  // moves the value to a scalar register at once and waits for it): scalar loads share one
  // counter with the kernel-argument loads, so waiting for an argument would wait for this
  // trip to memory as well.  Then the query rows and the
  // parent array, none of which depends on it.  All ordinary loads are older than the K/V
  // transfers: the compiler's waits for them then never include a transfer.
  int lane_zero = 0;
  asm volatile("" : "+v"(lane_zero));  // hides from the compiler that the address is uniform
  const int L_raw = __hip_atomic_load(p.prefix_len + b + lane_zero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  WaveState<D> st;
  const int m_row = qtile * QROWS + wm * kWaveRows + c32;  // this lane's query row
  const bool row_ok = m_row < M;
  const int mm = row_ok ? m_row : M - 1;
  const int my_node = div_mg(mm, p.mg_g);
  u32x4 q_raw[DK];
  {
    const uint16_t* src =
        p.q + b * p.q_sb + my_node * p.q_st + (long long)(kv * G + (mm - my_node * G)) * p.q_sh + 8 * g;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) q_raw[ks] = *reinterpret_cast<const u32x4*>(src + ks * 16);  // clamped row: in bounds
  }
  // (the first wave builds the ancestor sets, nodes lane and lane + 64)
  int parent_lo = -1, parent_hi = -1;
  if (wave == 0) {
    if (lane < T) parent_lo = p.parent[(long long)b * T + lane];
    if (lane + 64 < T) parent_hi = p.parent[(long long)b * T + lane + 64];
  }

  // ---- tile range of this split.  The prefix length is still on its way: start the K/V
  // stream on the assumption that it equals the host's upper bound (the usual case); if it
  // turns out shorter, the speculative transfers are waited for and everything is redone.
  TileSrc ts;
  ts.T = T;
  ts.kc_sl = p.kc_sl;
  ts.kt_st = p.kt_st;
  ts.pg_s = pg_s;
  ts.pg_first = 0;
  ts.tpp = p.tpp;
  ts.mg_tpp = p.mg_tpp;
  ts.page_stride = p.page_stride;
  const int n_ttiles = (T + kTileKeys - 1) / kTileKeys;
  // Splits are dealt whole rounds (TPR tiles).  The rounds at the end of the key range that
  // hold the ragged prefix tile or masked tree tiles are slower (per-lane clamped transfers,
  // mask arithmetic, ancestor sets first), so each of them counts double when the rounds are
  // shared out (up to half of a split's share), the surplus going to the first splits: the
  // split that ends the range then finishes with the others instead of after them.
  auto set_range = [&](int len) {
    ts.L = len;
    ts.n_ptiles = (len + kTileKeys - 1) / kTileKeys;
    const int nt = ts.n_ptiles + n_ttiles;
    const int R = (nt + TPR - 1) / TPR;
    const int slow = R - (len / kTileKeys) / TPR;  // rounds that are not all full prefix tiles
    const int share = div_mg(R, p.mg_splits);
    const int extra = slow < share / 2 ? slow : share / 2;
    const int Rv = R + extra;
    const int base = div_mg(Rv, p.mg_splits);
    const int rem = Rv - base * splits;
    int rb = split * base + (split < rem ? split : rem);
    int re = rb + base + (split < rem ? 1 : 0);
    rb = rb < R ? rb : R;
    re = re < R ? re : R;
    ts.t_begin = rb * TPR < nt ? rb * TPR : nt;
    ts.t_end = re * TPR < nt ? re * TPR : nt;
    if (KT == 2 && WN == 1) {
      // One wave column taking tile pairs.  Everybody waits for the slowest split (the merge needs all
      // partials), so the shares are dealt in tiles of what the loop is fast at: full prefix tiles,
      // evenly (a split with an odd number ends on a lone tile, which costs about half a pair).  What
      // is left - the ragged tile, the masked tree tiles, all of them on the slower general path - goes
      // to the last split, priced at two full tiles a tile (measured: two tree tiles 2.8 us, a pair of
      // full tiles 1.31), and that split gets correspondingly fewer full tiles (none at all if the tail
      // is worth a whole share: the host may add a split for it, whose workgroups are short and share
      // a CU with a regular one).
      const int F = len / kTileKeys;  // full prefix tiles
      const int tail = nt - F;
      int tb = 0, te = nt;
      if (splits > 1) {
        const int per = div_mg(F + 2 * tail + splits - 1, p.mg_splits);  // ceil((F + 2 tail) / splits)
        int f_last = per - 2 * tail;
        f_last = f_last < 0 ? 0 : (f_last > F ? F : f_last);
        f_last &= ~1;  // (whole pairs: the general path takes the tail two tiles at a time, and a full tile must not split one of its rounds)
        const int rest = F - f_last;  // full tiles of the other splits
        const int base_t = div_mg(rest, p.mg_splits_m1), rem_t = rest - base_t * (splits - 1);
        if (split == splits - 1) {
          tb = rest;
        } else {
          tb = split * base_t + (split < rem_t ? split : rem_t);
          te = tb + base_t + (split < rem_t ? 1 : 0);
        }
      }
      ts.t_begin = tb;
      ts.t_end = te;
    }
  };
  const unsigned ring_addr = (unsigned)(size_t)LDS_PTR(unsigned char, ring);  // a multiple of 1024
  const unsigned k_lane = G_::k_lane(lane), v_lane = G_::v_lane(lane);
  LaneChunks<D, NW> lc;
  lane_chunks<D, NW>(lc, wave, lane, ts, p.kc + (PAGED ? 0 : b * p.kc_sb) + (long long)kv * p.kc_sh,
                     p.vc + (PAGED ? 0 : b * p.kc_sb) + (long long)kv * p.kc_sh, p.kt + b * p.kt_sb + (long long)kv * p.kt_sh,
                     p.vt + b * p.kt_sb + (long long)kv * p.kt_sh);

  set_range(p.max_prefix);
  int n_rounds = (ts.t_end - ts.t_begin + TPR - 1) / TPR;
  // Paged cache: page ids of the prefix tiles this split will fetch (whole rounds), clamped into the pool, so
  // that a transfer stays inside the pool whatever the table holds: the first rounds can then be asked for on
  // the same assumption as with a contiguous cache (entries past a sequence's pages may hold anything; if the
  // length turns out shorter, the list is made again).  An id outside the pool is reported once the list is final.
  bool bad_page = false;
  auto fill_pages = [&]() {
    bad_page = false;
    const int te = min(ts.n_ptiles, ts.t_begin + n_rounds * TPR);
    if (te > ts.t_begin) {
      ts.pg_first = div_mg(ts.t_begin, p.mg_tpp);
      const int n_pg = div_mg(te - 1, p.mg_tpp) - ts.pg_first + 1;  // <= kMaxPagesPerSplit by the host's plan
      for (int i = tid; i < n_pg && i < kMaxPagesPerSplit; i += THREADS) {
        const int pi = ts.pg_first + i;
        const int id = pi < p.max_blocks ? p.block_table[(long long)b * p.max_blocks + pi] : 0;
        bad_page = bad_page || id < 0 || id >= p.n_pages;
        pg_s[i] = id < 0 ? 0 : (id >= p.n_pages ? p.n_pages - 1 : id);
      }
    }
    __syncthreads();
  };
  if (PAGED) fill_pages();
  const bool spec_any = n_rounds > 0 && (ts.t_begin + TPR) * kTileKeys <= p.max_prefix;  // same for every wave
  int n_spec = 0;  // rounds already issued, all of them full prefix tiles under the assumption
#pragma unroll
  for (int r = 0; r < NR - 1; ++r)
    if (n_spec == r && r < n_rounds && (ts.t_begin + (r + 1) * TPR) * kTileKeys <= p.max_prefix) {
      dma_round<D, NW, TPR, PAGED>(r, ts, lc, ring_addr + r * STAGE_BYTES);
      n_spec = r + 1;
    }
  JK_TS(1);

  int L = __builtin_amdgcn_readfirstlane(L_raw);
  L = L < 0 ? 0 : (L > p.max_prefix ? p.max_prefix : L);
  JK_TS(2);
  if (L != p.max_prefix) {  // uniform over the workgroup
    if (spec_any) {
      wait_dma<DMA_PER_ROUND>(0);  // the ring must be quiet before the same slots are filled again
      __syncthreads();
    }
    n_spec = 0;
    set_range(L);
    n_rounds = (ts.t_end - ts.t_begin + TPR - 1) / TPR;
    if (PAGED) fill_pages();
  }
  const bool has_tree = ts.t_end > ts.n_ptiles;
  if (PAGED && bad_page) __hip_atomic_fetch_or(p.err, kDevErrBadPage, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
  for (int r = 0; r < NR - 1; ++r)
    if (r >= n_spec && r < n_rounds) dma_round<D, NW, TPR, PAGED>(r, ts, lc, ring_addr + r * STAGE_BYTES);

  JK_TS(3);
  // ---- ancestor sets (only workgroups that reach tree tiles need them), by pointer
  // doubling: after k steps a node knows its nearest 2^k ancestors-or-self and its 2^k-th
  // ancestor, so the number of steps is logarithmic in the depth of the tree rather than
  // the depth itself (every step is a round trip through LDS).  One wave does it alone, two
  // nodes per lane: the LDS operations of a wave complete in program order, so the steps
  // need no barrier (as rounds of the whole workgroup, with two or three barriers each, the
  // same steps took three times as long, and the split that owns the tree tiles is the one
  // the others wait for).  The barrier of the first round publishes the sets: tree tiles
  // are masked inside the loop only.
  if (has_tree && wave == 0) {
    const int n_lo = lane, n_hi = lane + 64;
    int up_lo = (parent_lo >= -1 && parent_lo < n_lo) ? parent_lo : -1;  // indices strictly decrease towards the root
    int up_hi = (parent_hi >= -1 && parent_hi < n_hi) ? parent_hi : -1;  // (-1 as well for lanes past the tree)
    // an entry that breaks -1 <= parent[i] < i was just replaced by -1: say so in the workspace's error word
    if (up_lo != parent_lo || up_hi != parent_hi) {
      typedef __attribute__((address_space(4))) const KParams KArgs;
      KArgs* late = (KArgs*)__builtin_amdgcn_kernarg_segment_ptr();
      asm volatile("" : "+s"(late));  // (fetched here: not worth a scalar register pair across the kernel)
      __hip_atomic_fetch_or(late->err, kDevErrBadTree, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    unsigned long long lo_lo = n_lo < T ? 1ull << n_lo : 0ull, hi_lo = 0ull;  // node lane: bit < 64
    unsigned long long lo_hi = 0ull, hi_hi = n_hi < T ? 1ull << lane : 0ull;  // node lane + 64: bit >= 64
    const bool two = T > 64;  // uniform
    for (;;) {
      par_s[n_lo] = up_lo;
      anc[2 * n_lo] = lo_lo;
      anc[2 * n_lo + 1] = hi_lo;
      if (two) {
        par_s[n_hi] = up_hi;
        anc[2 * n_hi] = lo_hi;
        anc[2 * n_hi + 1] = hi_hi;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      if (!__any(up_lo >= 0 || up_hi >= 0)) break;  // nobody has an ancestor left to fold in: LDS holds the sets
      if (up_lo >= 0) {
        lo_lo |= anc[2 * up_lo];
        hi_lo |= anc[2 * up_lo + 1];
        up_lo = par_s[up_lo];
      }
      if (two && up_hi >= 0) {
        lo_hi |= anc[2 * up_hi];
        hi_hi |= anc[2 * up_hi + 1];
        up_hi = par_s[up_hi];
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // every read of this step precedes the next step's writes
      __builtin_amdgcn_wave_barrier();
    }
  }

#pragma unroll
  for (int ks = 0; ks < DK; ++ks) {
    u32x4 v = q_raw[ks];
    if (!row_ok) v = u32x4{0u, 0u, 0u, 0u};
    st.q[ks] = __builtin_bit_cast(bf16x8, v);
  }
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.o[db][i] = 0.f;
  st.m = -INFINITY;
  st.l = 0.f;

  // mask of tile t: mode (see mask_tile), valid keys of a ragged prefix tile, visibility bits
  auto mask_of = [&](int t, int& mode, int& nvalid, unsigned int& bits) {
    mode = 0;
    nvalid = kTileKeys;
    bits = 0;
    if (t >= ts.t_end) {
      mode = 2;  // past the split: every key hidden (its LDS tile holds a copy of real data)
    } else if (t >= ts.n_ptiles) {
      const int tt = t - ts.n_ptiles;
      mode = 2;
      bits = (unsigned int)(anc[2 * my_node + (tt >> 1)] >> ((tt & 1) * 32));
    } else {
      nvalid = L - t * kTileKeys;
      mode = nvalid < kTileKeys ? 1 : 0;
    }
  };

  // ---- main loop.  Round r lives in ring slot r % NR; wave column wn takes tiles
  // (r*WN + wn)*KT .. +KT-1 of the split.  Before the barrier a wave waits for its own
  // transfers of round r; after the barrier every wave's have landed, and every wave has
  // finished round r-1, whose slot is therefore free for round r+NR-1.
  //
  // The pipelined pairs work in a fixed reference frame (see PairPipe).  If a score leaves it,
  // the wave says so in LDS after the loop, and the workgroup runs the loop once more, from
  // its first round, on the general path only (lazy rescale): rare, and the pairs stay free
  // of any conditional touch of the accumulators.
  bool left = false;     // a weight of this lane's row went beyond the frame (see PairPipe::reference)
  bool general = false;  // uniform: the repeat
  if (KT == 2 && tid == 0) *repeat_s = 0;  // (read behind the barrier that follows the loop)
  for (;;) {
  for (int r = 0; r < n_rounds; ++r) {
    // (what the round will do is worked out in front of the barrier: scalar arithmetic that
    // would otherwise stand between the barrier and the round's first LDS reads)
    const int tb = ts.t_begin + (r * WN + wn) * KT;
    const unsigned tile_a = ring_addr + (r % NR) * STAGE_BYTES + wn * KT * 2 * TILE_BYTES;  // K of the first tile
    const bool pair = KT == 2 && !general && (tb + 2) * kTileKeys <= L && tb + 2 <= ts.t_end;  // two full prefix tiles
    // the refill of the ring: on its own, or (full prefix tiles behind a pipelined pair)
    // piece by piece between the pair's MFMAs
    RoundPieces<D, NW, TPR> next;
    const int t_next = ts.t_begin + (r + NR - 1) * TPR;
    const bool refill = r + NR - 1 < n_rounds;
    // (paged caches refill in one go: with a base pointer per tile the interleaved refill measured slower)
    const bool spread = kSpread > 0 && !PAGED && WN == 1 && refill && pair && (t_next + TPR) * kTileKeys <= L;
    next.tile_elems = (long long)kTileKeys * ts.kc_sl;
    next.base = lc.cache + (long long)t_next * next.tile_elems;
    next.slot = ring_addr + ((r + NR - 1) % NR) * STAGE_BYTES;
    next.lc = &lc;
    const int ahead = n_rounds - 1 - r;  // rounds issued after r: min(NR-2, ahead)
    wait_dma<DMA_PER_ROUND>(ahead < NR - 2 ? ahead : NR - 2);
    __syncthreads();
    if (r == 0) JK_TS(4);
    if (refill && !spread) dma_round<D, NW, TPR, PAGED>(r + NR - 1, ts, lc, ring_addr + ((r + NR - 1) % NR) * STAGE_BYTES);
    if (pair && spread) {
      PairPipe<D>::template run<kSpread>(st, tile_a + k_lane, tile_a + TILE_BYTES + v_lane, scale_log2, next, r == 0);
    } else if (pair) {
      PairPipe<D>::template run<0>(st, tile_a + k_lane, tile_a + TILE_BYTES + v_lane, scale_log2, next, r == 0);
    } else if (KT == 2 && WN == 1 && !general && tb + 1 == ts.t_end && (tb + 1) * kTileKeys <= L) {
      lone_tile<D>(st, tile_a + k_lane, tile_a + TILE_BYTES + v_lane, scale_log2, r == 0);  // no mask, half the work
    } else if (tb < ts.t_end) {
      int mode, nvalid;
      unsigned int bits;
      floatx16 s0, s1;
      // (the general path may rescale the sums: what the fast paths left in them is tested first)
      if (KT == 2 && !general) left = left || PairPipe<D>::left_frame(st);
      qk_tiles<D, KT>(st, tile_a + k_lane, s0, s1);
      mask_of(tb, mode, nvalid, bits);
      mask_tile(s0, mode, nvalid, bits, g);
      if (KT == 2) {
        mask_of(tb + 1, mode, nvalid, bits);
        mask_tile(s1, mode, nvalid, bits, g);
      }
      softmax_pv<D, KT>(st, s0, s1, tile_a + TILE_BYTES + v_lane, scale_log2);
    }
  }
  if (KT == 2 && !general && (left || PairPipe<D>::left_frame(st))) *repeat_s = 1;
  JK_TS(5);
  __syncthreads();  // every wave is done with the ring before it becomes the epilogue buffer (or is filled again)
  if (KT != 2 || general || __builtin_amdgcn_readfirstlane(*repeat_s) == 0) break;
  general = true;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.o[db][i] = 0.f;
  st.m = -INFINITY;
  st.l = 0.f;
#pragma unroll
  for (int r = 0; r < NR - 1; ++r)
    if (r < n_rounds) dma_round<D, NW, TPR, PAGED>(r, ts, lc, ring_addr + r * STAGE_BYTES);
  }

  // ---- epilogue: the waves of key column 0 own the result of their 32 rows.  The other
  // columns park their O^T and (max, sum) in LDS (the ring is dead by now); the owners fold
  // them into their own accumulators, register for register (all waves share one layout),
  // and store straight from that layout: lane (row, g) holds, per 32-wide block db and
  // quarter q4, the 4 columns 32*db + 8*q4 + 4*g .. +3 of its row.
  // (the lane's indices are worked out afresh, from the execution mask: kept in registers
  // across the tile loop, which has none to spare, they - or the thread id they come from -
  // are spilled to memory and read back here)
  const int lane_e = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  const int c32_e = lane_e & 31, g_e = lane_e >> 5;
  const bool row_ok_e = qtile * QROWS + wm * kWaveRows + c32_e < M;
  const float l_own = half_swap_sum(st.l);
  const int row = wm * kWaveRows + c32_e;
  if (wn != 0) {
    float* orow = obuf + ((size_t)(wn - 1) * QROWS + row) * G_::O_LD;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        float4 v = make_float4(st.o[db][4 * q4], st.o[db][4 * q4 + 1], st.o[db][4 * q4 + 2], st.o[db][4 * q4 + 3]);
        *reinterpret_cast<float4*>(orow + 32 * db + 8 * q4 + 4 * g_e) = v;
      }
    if (g_e == 0) mlbuf[(wn - 1) * QROWS + row] = make_float2(st.m, l_own);
  }
  if (WN > 1) __syncthreads();
  JK_TS(6);
  if (wn == 0) {
    float mx = st.m;
#pragma unroll
    for (int w = 1; w < WN; ++w) mx = fmaxf(mx, mlbuf[(w - 1) * QROWS + row].x);
    const float mx_use = (mx == -INFINITY) ? 0.f : mx;
    float lsum = l_own;
    if (WN > 1) {
      const float w0 = fast_exp2(st.m - mx_use);
      lsum *= w0;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) st.o[db][i] *= w0;
#pragma unroll
      for (int w = 1; w < WN; ++w) {
        const float2 ml = mlbuf[(w - 1) * QROWS + row];
        const float wgt = fast_exp2(ml.x - mx_use);
        lsum = fmaf(ml.y, wgt, lsum);
        const float* orow = obuf + ((size_t)(w - 1) * QROWS + row) * G_::O_LD;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const float4 v = *reinterpret_cast<const float4*>(orow + 32 * db + 8 * q4 + 4 * g_e);
            st.o[db][4 * q4] = fmaf(v.x, wgt, st.o[db][4 * q4]);
            st.o[db][4 * q4 + 1] = fmaf(v.y, wgt, st.o[db][4 * q4 + 1]);
            st.o[db][4 * q4 + 2] = fmaf(v.z, wgt, st.o[db][4 * q4 + 2]);
            st.o[db][4 * q4 + 3] = fmaf(v.w, wgt, st.o[db][4 * q4 + 3]);
          }
      }
    }
    // ---- store.  The accumulator layout gives a lane 4 columns here and 4 there of one row:
    // stored as it is, every instruction would touch 32 rows with 16 bytes each.  So the wave
    // first lays its 32 finished rows out in LDS as bf16 (a private patch behind the parked
    // columns) and reads them back row-wise: 16 lanes x 16 bytes per row, whole 128-byte lines
    // per store.  Holds the final result (no splits) or the split's partial in bf16 (the
    // running max and sum stay fp32): partials are written, flushed and read back once per
    // split, and are the largest avoidable traffic of a call.
    const float mul = splits == 1 ? 1.f / lsum : 1.f;  // lsum > 0: every row sees at least its own tree key
    const long long prow0 = ((long long)unit_id * splits + split) * p.m_pad + qtile * QROWS + wm * kWaveRows;
    if (splits > 1 && row_ok_e && g_e == 0) {
      if (p.through & 2) dev::store_through(p.part_ml + prow0 + c32_e, dev::store_u32x2{__float_as_uint(mx), __float_as_uint(lsum)});
      else p.part_ml[prow0 + c32_e] = make_float2(mx, lsum);
    }
    unsigned char* patch = smem + P_::OBUF_BYTES + wm * P_::PATCH_BYTES;
    {
      unsigned char* prow = patch + c32_e * P_::PATCH_LD;
      // (a lone wave per SIMD issues an instruction every five to eight cycles: this part of the
      // kernel is bound by its instruction count, hence the uniform branches around whole loops
      // rather than conditions inside them)
      auto to_patch = [&](auto scaled) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            bf16x2 lo, hi;
            lo[0] = (__bf16)(decltype(scaled)::value ? st.o[db][4 * q4] * mul : st.o[db][4 * q4]);
            lo[1] = (__bf16)(decltype(scaled)::value ? st.o[db][4 * q4 + 1] * mul : st.o[db][4 * q4 + 1]);
            hi[0] = (__bf16)(decltype(scaled)::value ? st.o[db][4 * q4 + 2] * mul : st.o[db][4 * q4 + 2]);
            hi[1] = (__bf16)(decltype(scaled)::value ? st.o[db][4 * q4 + 3] * mul : st.o[db][4 * q4 + 3]);
            uint2 pk;
            pk.x = __builtin_bit_cast(unsigned int, lo);
            pk.y = __builtin_bit_cast(unsigned int, hi);
            *reinterpret_cast<uint2*>(prow + (32 * db + 8 * q4 + 4 * g_e) * 2) = pk;
          }
      };
      if (splits == 1) to_patch(std::true_type{});
      else to_patch(std::false_type{});
    }
    // (same wave wrote and reads: LDS operations of a wave complete in order)
    constexpr int CPR = G_::CPR;             // 16-byte chunks per row
    constexpr int RPI = 64 / CPR;            // rows per store instruction
    const int chunk = lane_e % CPR, rsub = lane_e / CPR;
    const int rows_valid = M - (qtile * QROWS + wm * kWaveRows);  // rows of this wave that exist (32 or more: all)
    if (splits == 1) {
#pragma unroll
      for (int k = 0; k < kWaveRows / RPI; ++k) {
        const int rr = k * RPI + rsub;                               // row of the wave
        const int m = qtile * QROWS + wm * kWaveRows + rr;           // query row
        const u32x4 v = *reinterpret_cast<const u32x4*>(patch + rr * P_::PATCH_LD + chunk * 16);
        if (rr < rows_valid) {
          const int node = div_mg(m, p.mg_g);
          uint16_t* dst = p.out + b * p.o_sb + node * p.o_st + (long long)(kv * G + (m - node * G)) * p.o_sh;
          if (p.through & 1) dev::store_through(dst + chunk * 8, v);
          else *reinterpret_cast<u32x4*>(dst + chunk * 8) = v;
        }
      }
    } else {
      // partial rows are D elements apart: one address, constant steps
      unsigned char* dst0 = reinterpret_cast<unsigned char*>(p.part_o) + ((prow0 + rsub) * D + chunk * 8) * 2;
      const unsigned char* src0 = patch + rsub * P_::PATCH_LD + chunk * 16;
      auto store_rows = [&](auto through, auto guarded) {
#pragma unroll
        for (int k = 0; k < kWaveRows / RPI; ++k) {
          const u32x4 v = *reinterpret_cast<const u32x4*>(src0 + k * RPI * P_::PATCH_LD);
          if (!decltype(guarded)::value || k * RPI + rsub < rows_valid) {
            if (decltype(through)::value) dev::store_through(dst0 + k * RPI * D * 2, v);
            else *reinterpret_cast<u32x4*>(dst0 + k * RPI * D * 2) = v;
          }
        }
      };
      const bool thr = p.through & 1;
      if (rows_valid >= kWaveRows) {
        if (thr) store_rows(std::true_type{}, std::false_type{});
        else store_rows(std::false_type{}, std::false_type{});
      } else {
        if (thr) store_rows(std::true_type{}, std::true_type{});
        else store_rows(std::false_type{}, std::true_type{});
      }
    }
  }
  if (splits > 1) {
    // ---- merge of the group's splits in this kernel.  Every workgroup of the group owns the slice
    // of R = ceil(QROWS / splits) rows numbered like its split and merges it once all partials are
    // in L2.  Waiting is bounded: a workgroup that gives up records its slice in the group's mask
    // and leaves; the group's last arriver, which never waits, then merges those slices as well,
    // so the result is complete whenever every workgroup of the group runs, however late.
    // (The arguments this part needs are fetched from the kernel-argument segment here rather than
    // held in scalar registers across the tile loop, which has none to spare.)
    typedef __attribute__((address_space(4))) const KParams KArgs;
    KArgs* late = (KArgs*)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(late));
    const int tid_e = wave * 64 + lane_e;  // (the thread id, rebuilt: see the note on lane_e above)
    if (late->fused) {
      int* mode_s = repeat_s + 1;  // 0 leave, 1 merge own slice, 2 also the slices in mode_s[1..2]
      // (what the merge of this workgroup's own slice needs besides the partials: computed now, while
      // the partial stores travel and before the wait for the group)
      MergeArgs ma;
      ma.part_o = p.part_o; ma.part_ml = p.part_ml; ma.out = p.out;
      ma.M = M; ma.m_pad = p.m_pad; ma.splits = splits; ma.G = G; ma.mg_g = p.mg_g;
      ma.o_sb = p.o_sb; ma.o_st = p.o_st; ma.o_sh = p.o_sh;
      const int merge_rows = late->merge_rows, merge_shift = late->merge_shift;
      const int tile_row0 = qtile * QROWS;
      const MergeThread mt = merge_prepare<D, THREADS, QROWS>(ma, unit_id, b, kv, split, merge_rows, merge_shift, tile_row0, tid_e);
      JK_TS(7);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's partial stores have reached L2
      __syncthreads();
      JK_TS(8);
      if (tid_e == 0) {
        unsigned* word = late->sync + (size_t)(unit_id * late->n_qtiles + qtile) * 16;
        const unsigned S = (unsigned)splits;
        const unsigned old = l2_atomic_add(word, 1u);
        const unsigned epoch = old >> 16;
        int mode = 1;
        unsigned m_lo = 0u, m_hi = 0u;
        if ((old & kSyncCountMask) == S - 1) {
          const unsigned gave_up = (old >> 8) & 0xffu;
          l2_atomic_add_noret(word, kSyncEpochOne - S - gave_up * kSyncGaveUpOne);
          if (gave_up) {
            mode = 2;
            m_lo = l2_atomic_swap(word + 1, 0u);
            m_hi = l2_atomic_swap(word + 2, 0u);
          }
        } else {
          const unsigned limit = late->spin_limit;
          unsigned polls = 0;
          for (;;) {
            const unsigned v = l2_atomic_add(word, 0u);
            if ((v >> 16) != epoch || (v & kSyncCountMask) == S) break;
            if (++polls > limit) {
              l2_atomic_or(word + 1 + (split >> 5), 1u << (split & 31));
              const unsigned v2 = l2_atomic_add(word, kSyncGaveUpOne);
              // (complete after all, between the last poll and the mark: the last arriver has not seen
              // the mark, so this slice is still ours; the stray mark only costs a later call a repeat)
              if (!((v2 >> 16) != epoch || (v2 & kSyncCountMask) == S)) mode = 0;
              __hip_atomic_fetch_or(late->err, kDevErrMergeWait, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              break;
            }
            __builtin_amdgcn_s_sleep(1);
          }
        }
        mode_s[0] = mode;
        mode_s[1] = (int)m_lo;
        mode_s[2] = (int)m_hi;
      }
      __syncthreads();
      JK_TS(9);
      const int mode = __builtin_amdgcn_readfirstlane(mode_s[0]);
      if (mode != 0) {
        // (No line of the partials can sit in this CU's vector cache: the cache starts every kernel
        // empty, this kernel reads partials nowhere else, and no partial is rewritten after the group
        // is complete.  The loads below therefore go to L2 without an invalidate in front of them.)
        asm volatile("" ::: "memory");
        float* wbuf = reinterpret_cast<float*>(smem);  // (ring and epilogue buffers are dead: every wave is past its stores)
        merge_run<D, THREADS, QROWS>(ma, mt, merge_shift, b, kv, tile_row0, tid_e, wbuf);
        if (mode == 2) {
          const unsigned long long left_over =
              ((unsigned long long)(unsigned)mode_s[2] << 32) | (unsigned long long)(unsigned)mode_s[1];
          for (int j = 0; j < splits; ++j)
            if (j != split && ((left_over >> j) & 1ull)) {
              const MergeThread mj = merge_prepare<D, THREADS, QROWS>(ma, unit_id, b, kv, j, merge_rows, merge_shift, tile_row0, tid_e);
              merge_run<D, THREADS, QROWS>(ma, mj, merge_shift, b, kv, tile_row0, tid_e, wbuf);
            }
        }
      }
    }
  }
#ifdef JK_TIMING
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // (so that the last stamp includes the result stores)
#endif
  JK_TS(10);
}

template <int D, int WM, int WN, int KT, bool PAGED, bool DEEP = false>
hipError_t launch_one(const KParams& kp, hipStream_t stream) {
  using P_ = Plan<D, WM, WN, KT, PAGED, DEEP>;
  auto kern = tva_bf16_kernel<D, WM, WN, KT, PAGED, DEEP>;
  static LdsLimitRaised raised;
  if (hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), P_::SMEM, raised); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(kp.total_wgs), dim3(P_::THREADS), P_::SMEM, stream, kp);
  return hipGetLastError();
}

}  // namespace

#ifdef JK_TIMING
extern "C" int jk_debug_read_timing(unsigned long long* host, size_t n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_jk_ts), n * sizeof(unsigned long long));
}
#endif

hipError_t launch_tva_bf16(const AttnArgs& a, const AttnPlan& pl, hipStream_t stream) {
  KParams kp;
  kp.q = static_cast<const uint16_t*>(a.q);
  kp.kc = static_cast<const uint16_t*>(a.k_cache);
  kp.vc = static_cast<const uint16_t*>(a.v_cache);
  kp.kt = static_cast<const uint16_t*>(a.k_tree);
  kp.vt = static_cast<const uint16_t*>(a.v_tree);
  kp.parent = a.parent;
  kp.prefix_len = a.prefix_len;
  kp.out = static_cast<uint16_t*>(a.out);
  kp.part_o = a.part_o;
  kp.part_ml = a.part_ml;
  const jk_attn_desc& d = a.d;
  kp.B = d.batch; kp.T = d.n_tree; kp.Hkv = d.n_kv_heads; kp.G = d.n_q_heads / d.n_kv_heads;
  kp.M = pl.m_rows; kp.m_pad = pl.m_pad; kp.max_prefix = a.max_prefix_len;
  kp.splits = pl.splits; kp.n_qtiles = pl.n_qtiles;
  const long long work = (long long)d.batch * d.n_kv_heads * pl.splits * pl.n_qtiles;
  kp.total_wgs = (int)((work + 7) / 8 * 8);
  kp.q_sb = d.q_stride_b; kp.q_st = d.q_stride_t; kp.q_sh = d.q_stride_h;
  kp.kc_sb = d.kc_stride_b; kp.kc_sl = d.kc_stride_l; kp.kc_sh = d.kc_stride_h;
  kp.kt_sb = d.kt_stride_b; kp.kt_st = d.kt_stride_t; kp.kt_sh = d.kt_stride_h;
  kp.o_sb = d.o_stride_b; kp.o_st = d.o_stride_t; kp.o_sh = d.o_stride_h;
  kp.scale_log2 = a.scale_log2;
  auto magic = [](int d) { return (1ull << 32) / (unsigned long long)d + 1ull; };
  kp.mg_qtiles = magic(pl.n_qtiles);
  kp.mg_splits = magic(pl.splits);
  kp.mg_splits_m1 = magic(pl.splits > 1 ? pl.splits - 1 : 1);
  kp.mg_hkv = magic(d.n_kv_heads);
  kp.mg_g = magic(kp.G);

  kp.block_table = a.block_table;
  kp.max_blocks = a.max_blocks;
  kp.n_pages = a.n_pages;
  kp.tpp = a.block_table ? a.page_size / kTileKeys : 1;
  kp.page_stride = a.page_stride;
  kp.mg_tpp = magic(kp.tpp);
  // Results written with ordinary stores stay dirty in the XCDs' L2s until the end of the
  // kernel writes them back.  When the whole grid is resident at once (every workgroup ends
  // within the same microsecond) that write-back is exposed, and stores that go through to
  // memory at once measured faster (c3 -0.2 us, c2 -0.65 us per call); with several
  // workgroups per CU in turn, dirty lines of finished workgroups drain while the others
  // compute, and ordinary stores measured faster (c4 +0.8 us with write-through).  The small
  // (max, sum) pairs: through only for the 2x2 arrangement (c2 -0.35 us; c3, 4x1: +0.25 us).
  const bool one_wave = work <= (long long)device_cu_count();
  kp.through = (one_wave ? 1 : 0) | (one_wave && pl.wn > 1 ? 2 : 0);
  // merged in the kernel: ordinary stores (measured: the L2 passes them on and keeps no line of them, but they are
  // acknowledged after 0.7 us and read back in 0.4; stores through to memory take 1.3 and 1.0)
  kp.fused = pl.fused;
  if (pl.fused && pl.splits > 1) kp.through = 0;
  kp.sync = a.sync;
  kp.err = a.err;
  kp.spin_limit = tuning().spin_limit >= 0 ? (unsigned)tuning().spin_limit : 4096u;  // about 2 ms of polling
  kp.merge_rows = (pl.q_rows + pl.splits - 1) / pl.splits;
  kp.merge_shift = 0;
  while ((1 << kp.merge_shift) < pl.splits) ++kp.merge_shift;
  const int key = (d.head_dim * 1000 + pl.wm * 100 + pl.wn * 10 + pl.kt) * 2 + (a.block_table ? 1 : 0);
  if (pl.deep && pl.wm == 2 && pl.wn == 2 && pl.kt == 1) {
    if (d.head_dim == 128) return a.block_table ? launch_one<128, 2, 2, 1, true, true>(kp, stream) : launch_one<128, 2, 2, 1, false, true>(kp, stream);
    if (d.head_dim == 64) return a.block_table ? launch_one<64, 2, 2, 1, true, true>(kp, stream) : launch_one<64, 2, 2, 1, false, true>(kp, stream);
  }
#define JK_CASE(D_, WM_, WN_, KT_)                                                                  \
  case ((D_) * 1000 + (WM_) * 100 + (WN_) * 10 + (KT_)) * 2: return launch_one<D_, WM_, WN_, KT_, false>(kp, stream); \
  case ((D_) * 1000 + (WM_) * 100 + (WN_) * 10 + (KT_)) * 2 + 1: return launch_one<D_, WM_, WN_, KT_, true>(kp, stream);
  switch (key) {
    JK_CASE(128, 4, 1, 2)
    JK_CASE(128, 2, 2, 1)
    JK_CASE(64, 4, 1, 2)
    JK_CASE(64, 2, 2, 1)
    default: return hipErrorInvalidValue;
  }
#undef JK_CASE
}

}  // namespace jk
