// Tree-masked verification attention, bf16 inputs, MFMA path (gfx950).
//
// What it computes (Section 2.1 step 2 of the paper: the target model scores
// all draft candidates in one pass; Section 3.1.2: candidates form a tree and
// are verified through a tree attention mask): every tree node attends to the
// committed KV prefix, to itself and to its tree ancestors.
//
// Mapping.  The G query heads that share one KV head and the T tree nodes are
// packed into one matrix of M = T*G query rows (row m = node m/G, head m%G), so
// a KV head's K/V stream is read once for all of them.  One workgroup (4
// waves) owns 64*WM query rows of one (sequence, KV head) and one split of the
// key range; the key range (prefix tiles, then tree tiles, 32 keys each) is
// cut into `splits` contiguous pieces.  Waves are arranged WM x WN: wave
// (wm, wn) holds query rows [64*wm, 64*wm+64) and processes every WN-th tile.
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
// 16 lanes per 256-byte row) into a ring of 8 tiles, several rounds in flight;
// each lane fetches the 16-byte chunk that the XOR swizzle maps to its LDS
// slot, so that both the 128-bit K reads and the transpose V reads are free of
// bank conflicts.
#include "jk_internal.h"

namespace jk {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // native vector: plain loads/stores, no struct copies

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

struct KParams {
  const uint16_t *q, *kc, *vc, *kt, *vt;
  const int32_t *parent, *prefix_len;
  uint16_t* out;
  float* part_o;
  float2* part_ml;
  int B, T, Hkv, G, M, m_pad, max_prefix, splits, n_qtiles, total_wgs;
  long long q_sb, q_st, q_sh, kc_sb, kc_sl, kc_sh, kt_sb, kt_st, kt_sh, o_sb, o_st, o_sh;
  float scale_log2;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

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
  static constexpr int NCH = kTileKeys * CPR / 256;  // chunks per thread per tile and tensor
  static constexpr int DK = D / 16;               // k-steps of Q.K^T
  static constexpr int DB = D / 32;               // 32-wide d blocks of the output
  static constexpr int O_LD = D + 4;              // padded row of the epilogue buffer (floats)
  __device__ static __forceinline__ int kswz(int row) { return (row / (16 / CPR)) % CPR; }
  __device__ static __forceinline__ int vswz(int row) { return (row / (4 / DB)) % DB; }
  // byte offset inside a K tile of logical 16-byte chunk c of row r
  __device__ static __forceinline__ int koff(int r, int c) { return r * ROW_BYTES + ((c ^ kswz(r)) << 4); }
  // V tile: 64-byte blocks are swizzled, the 4 chunks inside a block keep their order
  __device__ static __forceinline__ int voff(int r, int c) {
    return r * ROW_BYTES + ((((c >> 2) ^ vswz(r)) << 2 | (c & 3)) << 4);
  }
};

// 16 bytes per lane straight from global memory into LDS (global_load_lds_dwordx4): lane l
// of the wave lands at lds_base + 16*l.  Written as inline assembly so that the compiler
// does not know about the transfer: its own bookkeeping would make every later LDS read
// wait for ALL outstanding transfers, which would serialise the multi-stage ring.  The
// kernel orders transfers and reads itself (wait_dma + __syncthreads).
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_base) {
  const unsigned base = __builtin_amdgcn_readfirstlane(lds_base);  // wave-uniform by construction
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(base), "v"(gptr)
               : "memory", "m0");
}

// Wait until at most n of this wave's transfers are still in flight (they complete in
// issue order).  The count must be an immediate, hence the switch.
template <int STEP>
__device__ __forceinline__ void wait_dma(int rounds_behind) {
  // s_waitcnt immediate on gfx9: vmcnt in bits [3:0] and [15:14]; expcnt/lgkmcnt left at their maxima
#define JK_VM(n) __builtin_amdgcn_s_waitcnt((((n) & 0xF) | (((n) >> 4) << 14)) | 0x0F70)
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

// Everything a thread needs to fetch its chunks of a tile.
struct TileSrc {
  const uint16_t *kc, *vc, *kt, *vt;  // bases of this (sequence, KV head)
  long long kc_sl, kt_st;             // row strides (elements)
  int L, T, n_ptiles, t_begin, t_end;
};

// Where a lane's 16-byte chunks sit inside a tile.  A wave-level transfer fills 1 KB =
// 64/CPR consecutive tile rows; lane l writes physical chunk l%CPR of row blk*(64/CPR) +
// l/CPR and fetches the logical chunk that the swizzle maps there, so the tile arrives
// already swizzled.
template <int D>
struct LaneChunks {
  static constexpr int NIK = Geo<D>::TILE_BYTES / 1024 / 4;  // transfers per wave, tile and tensor
  int row[NIK];         // tile row
  int kcol[NIK];        // element offset of the K chunk inside the row
  int vcol[NIK];        // element offset of the V chunk inside the row
  long long koff[NIK];  // row * cache row stride + kcol: offset inside a full prefix tile
  long long voff[NIK];
  unsigned lds[NIK];    // byte offset of the 1 KB block inside a tile
};

template <int D>
__device__ __forceinline__ void lane_chunks(LaneChunks<D>& lc, int wave, int lane, long long kc_sl) {
  using G_ = Geo<D>;
  constexpr int RPB = 64 / G_::CPR;
#pragma unroll
  for (int i = 0; i < LaneChunks<D>::NIK; ++i) {
    const int blk = wave * LaneChunks<D>::NIK + i;
    const int row = blk * RPB + lane / G_::CPR;
    const int pc = lane % G_::CPR;
    lc.row[i] = row;
    lc.kcol[i] = (pc ^ G_::kswz(row)) * 8;
    lc.vcol[i] = ((((pc >> 2) ^ G_::vswz(row)) << 2) | (pc & 3)) * 8;
    lc.koff[i] = (long long)row * kc_sl + lc.kcol[i];
    lc.voff[i] = (long long)row * kc_sl + lc.vcol[i];
    lc.lds[i] = blk * 1024;
  }
}

// Issue the transfers of round r (WN tiles, K and V) into ring slot `slot` (byte address).
template <int D, int WN>
__device__ __forceinline__ void dma_round(int r, const TileSrc& ts, const LaneChunks<D>& lc, unsigned slot) {
  using G_ = Geo<D>;
  constexpr int NIK = LaneChunks<D>::NIK;
#pragma unroll
  for (int w = 0; w < WN; ++w) {
    int t = ts.t_begin + r * WN + w;
    if (t >= ts.t_end) t = ts.t_end - 1;  // duplicate of a real tile, never consumed
    const unsigned kdst = slot + (w * 2 + 0) * G_::TILE_BYTES, vdst = slot + (w * 2 + 1) * G_::TILE_BYTES;
    if ((t + 1) * kTileKeys <= ts.L) {
      // full prefix tile: one scalar tile offset plus the lane's precomputed offsets
      const long long tile_off = (long long)t * kTileKeys * ts.kc_sl;
#pragma unroll
      for (int i = 0; i < NIK; ++i) {
        dma16(ts.kc + tile_off + lc.koff[i], kdst + lc.lds[i]);
        dma16(ts.vc + tile_off + lc.voff[i], vdst + lc.lds[i]);
      }
    } else {
      // ragged last prefix tile or tree tile: rows past the end re-read the last valid row
      const bool tree = t >= ts.n_ptiles;
      const int key0 = (tree ? t - ts.n_ptiles : t) * kTileKeys;
      const int last = (tree ? ts.T : ts.L) - 1 - key0;  // >= 0
      const uint16_t* kb = tree ? ts.kt : ts.kc;
      const uint16_t* vb = tree ? ts.vt : ts.vc;
      const long long rs = tree ? ts.kt_st : ts.kc_sl;
#pragma unroll
      for (int i = 0; i < NIK; ++i) {
        const int rr = lc.row[i] < last ? lc.row[i] : last;
        const long long rowoff = (long long)(key0 + rr) * rs;
        dma16(kb + rowoff + lc.kcol[i], kdst + lc.lds[i]);
        dma16(vb + rowoff + lc.vcol[i], vdst + lc.lds[i]);
      }
    }
  }
}

// Per-wave state of the online softmax and the output accumulation.
template <int D>
struct WaveState {
  bf16x8 q[2][Geo<D>::DK];
  floatx16 o[2][Geo<D>::DB];
  float m[2], l[2];
};

// One 32-key tile against the wave's 64 query rows.  mask_mode: 0 none, 1 ragged prefix
// tail (keys >= nvalid hidden), 2 tree tile (bits[qb] = visibility of the tile's 32 keys).
template <int D>
__device__ __forceinline__ void compute_tile(WaveState<D>& st, const unsigned char* kt_s,
                                             const unsigned char* vt_s, int mask_mode, int nvalid,
                                             unsigned int bits0, unsigned int bits1, float scale_log2,
                                             int lane) {
  using G_ = Geo<D>;
  constexpr int DK = G_::DK, DB = G_::DB;
  // The lane id is laundered through an empty asm so that the two dozen LDS addresses below
  // are recomputed per tile (a few ALU operations) instead of being hoisted out of the tile
  // loop, where they would push the register demand past the 256 directly usable vector
  // registers and force the Q operands out into accumulation registers.
  asm volatile("" : "+v"(lane));
  const int c32 = lane & 31, g = lane >> 5;
  // ---- S^T = K . Q^T
  floatx16 sacc[2];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[qb][i] = 0.f;
#pragma unroll
  for (int ks = 0; ks < DK; ++ks) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(kt_s + G_::koff(c32, 2 * ks + g));
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
      sacc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st.q[qb][ks], sacc[qb], 0, 0, 0);
  }
  // ---- masks: register i of a lane is key 8*(i/4) + 4*g + i%4 of the tile
  if (mask_mode == 2) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const unsigned int bits = qb ? bits1 : bits0;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int kk = 8 * (i / 4) + 4 * g + (i % 4);
        if (!((bits >> kk) & 1u)) sacc[qb][i] = -INFINITY;
      }
    }
  } else if (mask_mode == 1) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int kk = 8 * (i / 4) + 4 * g + (i % 4);
        if (kk >= nvalid) sacc[qb][i] = -INFINITY;
      }
  }
  // ---- online softmax; probabilities become bf16 B operands of the value product.
  // The reference maximum m of a row moves only when the tile's maximum exceeds it by more
  // than kLazy (in log2 units): weights then stay below 2^kLazy, harmless in fp32/bf16, and
  // the rescale of the 64x128 accumulators (which live in accumulation registers and are
  // costly to touch from the vector ALU) becomes rare.  The result is unchanged: weights,
  // their sum and the accumulators all carry the same reference.
  constexpr float kLazy = 8.f;
  bf16x8 pb[2][2];
  float alpha[2];
  bool moved = false;
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    float tmax = sacc[qb][0];
#pragma unroll
    for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, sacc[qb][i]);
    tmax = half_swap_max(tmax) * scale_log2;
    const float m_old = st.m[qb];
    const bool up = tmax > m_old + kLazy;  // false for tmax = -inf; true for the first visible key
    const float m_ref = up ? tmax : m_old;
    const float m_use = (m_ref == -INFINITY) ? 0.f : m_ref;
    alpha[qb] = up ? fast_exp2(m_old - m_use) : 1.f;
    moved |= up && (m_old != -INFINITY);   // accumulators are still zero before the first key
    st.m[qb] = m_ref;
    float lsum = 0.f;
    float pr[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      pr[i] = fast_exp2(fmaf(sacc[qb][i], scale_log2, -m_use));
      lsum += pr[i];
    }
    st.l[qb] = fmaf(st.l[qb], alpha[qb], lsum);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) pb[qb][j][e] = (__bf16)pr[8 * j + e];
  }
  if (__any(moved)) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) st.o[qb][db][i] *= alpha[qb];
  }
  // ---- O^T += V^T . P^T ; contraction index 4*q'+r of MFMA j is key 16*j + 8*q' + 4*g + r
  const int jj = (lane & 15) >> 2, cc = lane & 3, h16 = (lane & 31) >> 4;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      shortx4 v0, v1;
      {
        const int key = 16 * j + 4 * g + jj;
        const unsigned char* ad = vt_s + key * G_::ROW_BYTES + ((db ^ G_::vswz(key)) << 6) + 32 * h16 + 8 * cc;
        v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(shortx4, ad));
      }
      {
        const int key = 16 * j + 8 + 4 * g + jj;
        const unsigned char* ad = vt_s + key * G_::ROW_BYTES + ((db ^ G_::vswz(key)) << 6) + 32 * h16 + 8 * cc;
        v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(shortx4, ad));
      }
      const shortx8 v01 = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
      const bf16x8 a = __builtin_bit_cast(bf16x8, v01);
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
        st.o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb][j], st.o[qb][db], 0, 0, 0);
    }
  }
}

template <int D, int WM, int WN, int NR>
__global__ __launch_bounds__(256, 1) void tva_bf16_kernel(const KParams p) {
  using G_ = Geo<D>;
  constexpr int NCH = G_::NCH, DK = G_::DK, DB = G_::DB;
  constexpr int QROWS = 64 * WM;
  constexpr int TILE_BYTES = G_::TILE_BYTES;
  constexpr int STAGE_BYTES = WN * 2 * TILE_BYTES;   // one round: WN tiles of K and V
  constexpr int RING_BYTES = NR * STAGE_BYTES;
  constexpr int DMA_PER_ROUND = WN * 2 * (TILE_BYTES / 1024 / 4);  // transfers a wave issues per round
  constexpr int OBUF_BYTES = 4 * 64 * G_::O_LD * 4;
  constexpr int UNION_BYTES = RING_BYTES > OBUF_BYTES ? RING_BYTES : OBUF_BYTES;
  static_assert(NR >= 2 && NR <= 8 && (NR - 2) * DMA_PER_ROUND <= 63, "ring depth");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* ring = smem;
  float* obuf = reinterpret_cast<float*>(smem);                            // [WN][QROWS][O_LD], after the loop
  float2* mlbuf = reinterpret_cast<float2*>(smem + UNION_BYTES);           // [WN][QROWS]
  unsigned long long* anc = reinterpret_cast<unsigned long long*>(smem + UNION_BYTES + 4 * 64 * 8);  // [128][2]
  int* par_s = reinterpret_cast<int*>(smem + UNION_BYTES + 4 * 64 * 8 + JK_MAX_TREE * 16);           // [128]

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
  const int qtile = wid % p.n_qtiles;
  int rest = wid / p.n_qtiles;
  const int split = rest % splits;
  rest /= splits;
  if (rest >= p.B * p.Hkv) return;  // padding workgroup
  const int kv = rest % p.Hkv;
  const int b = rest / p.Hkv;

  int L = p.prefix_len[b];
  L = L < 0 ? 0 : (L > p.max_prefix ? p.max_prefix : L);
  TileSrc ts;
  ts.L = L;
  ts.T = T;
  ts.n_ptiles = (L + kTileKeys - 1) / kTileKeys;
  const int nt = ts.n_ptiles + (T + kTileKeys - 1) / kTileKeys;
  ts.t_begin = (int)((long long)split * nt / splits);
  ts.t_end = (int)((long long)(split + 1) * nt / splits);
  ts.kc = p.kc + b * p.kc_sb + (long long)kv * p.kc_sh;
  ts.vc = p.vc + b * p.kc_sb + (long long)kv * p.kc_sh;
  ts.kt = p.kt + b * p.kt_sb + (long long)kv * p.kt_sh;
  ts.vt = p.vt + b * p.kt_sb + (long long)kv * p.kt_sh;
  ts.kc_sl = p.kc_sl;
  ts.kt_st = p.kt_st;
  const int n_rounds = (ts.t_end - ts.t_begin + WN - 1) / WN;

  // ---- ancestor sets (only workgroups that reach tree tiles need them)
  const bool has_tree = ts.t_end > ts.n_ptiles;
  int my_parent = -1;
  if (has_tree && tid < T) my_parent = p.parent[(long long)b * T + tid];

  // ---- this wave's 64 query rows as MFMA B operands (lane: row c32, 8 consecutive d)
  WaveState<D> st;
  const int row_base = qtile * QROWS + wm * 64;  // first row (within the KV head's M rows)
  int node_of[2];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int m = row_base + qb * 32 + c32;
    const bool ok = m < M;
    const int mm = ok ? m : M - 1;
    const int node = mm / G, hg = mm % G;
    node_of[qb] = node;
    const uint16_t* src = p.q + b * p.q_sb + node * p.q_st + (long long)(kv * G + hg) * p.q_sh + 8 * g;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) {
      u32x4 v = *reinterpret_cast<const u32x4*>(src + ks * 16);  // clamped row: always in bounds
      if (!ok) v = u32x4{0u, 0u, 0u, 0u};
      st.q[qb][ks] = __builtin_bit_cast(bf16x8, v);
    }
  }
  // ---- start the K/V stream: NR-1 rounds in flight.  The ordinary loads above (Q, parent)
  // are older than every transfer, so the compiler's waits for them never wait for a transfer
  // that was issued later... but a wait placed after this point does: hence they come first.
  const unsigned ring_addr = (unsigned)(size_t)LDS_PTR(unsigned char, ring);
  LaneChunks<D> lc;
  lane_chunks<D>(lc, wave, lane, ts.kc_sl);
#pragma unroll
  for (int r = 0; r < NR - 1; ++r)
    if (r < n_rounds) dma_round<D, WN>(r, ts, lc, ring_addr + r * STAGE_BYTES);

  if (has_tree) {
    if (tid < T) par_s[tid] = (my_parent >= -1 && my_parent < tid) ? my_parent : -1;
    __syncthreads();
    if (tid < T) {
      unsigned long long lo = 0, hi = 0;
      int a = tid;
      while (a >= 0) {  // parent indices strictly decrease, so at most tid+1 steps
        if (a < 64) lo |= 1ull << a; else hi |= 1ull << (a - 64);
        a = par_s[a];
      }
      anc[2 * tid] = lo;
      anc[2 * tid + 1] = hi;
    }
    // visibility to the other threads is ordered by the first __syncthreads of the tile loop
  }

#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) st.o[qb][db][i] = 0.f;
    st.m[qb] = -INFINITY;
    st.l[qb] = 0.f;
  }

  // ---- main loop.  Round r lives in ring slot r % NR.  Before the barrier a wave waits for
  // its own transfers of round r; after the barrier every wave's have landed, and every wave
  // has finished round r-1, whose slot is therefore free for round r+NR-1.
  for (int r = 0; r < n_rounds; ++r) {
    const int ahead = n_rounds - 1 - r;  // rounds issued after r: min(NR-2, ahead)
    wait_dma<DMA_PER_ROUND>(ahead < NR - 2 ? ahead : NR - 2);
    __syncthreads();
    if (r + NR - 1 < n_rounds)
      dma_round<D, WN>(r + NR - 1, ts, lc, ring_addr + ((r + NR - 1) % NR) * STAGE_BYTES);
    const int t = ts.t_begin + r * WN + wn;
    if (t < ts.t_end) {
      int mode = 0, nvalid = kTileKeys;
      unsigned int bits0 = 0, bits1 = 0;
      if (t >= ts.n_ptiles) {
        const int tt = t - ts.n_ptiles;
        mode = 2;
        bits0 = (unsigned int)(anc[2 * node_of[0] + (tt >> 1)] >> ((tt & 1) * 32));
        bits1 = (unsigned int)(anc[2 * node_of[1] + (tt >> 1)] >> ((tt & 1) * 32));
      } else {
        nvalid = L - t * kTileKeys;
        mode = nvalid < kTileKeys ? 1 : 0;
      }
      const unsigned char* kt_s = ring + (r % NR) * STAGE_BYTES + wn * 2 * TILE_BYTES;
      compute_tile<D>(st, kt_s, kt_s + TILE_BYTES, mode, nvalid, bits0, bits1, scale_log2, lane);
    }
  }
  __syncthreads();  // every wave is done with the ring before it becomes the epilogue buffer

  // ---- epilogue: O^T and (max, sum) of each wave into LDS
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const float l_tot = half_swap_sum(st.l[qb]);
    const int row = wm * 64 + qb * 32 + c32;
    float* orow = obuf + ((size_t)wn * QROWS + row) * G_::O_LD;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        float4 v = make_float4(st.o[qb][db][4 * q4], st.o[qb][db][4 * q4 + 1], st.o[qb][db][4 * q4 + 2],
                               st.o[qb][db][4 * q4 + 3]);
        *reinterpret_cast<float4*>(orow + 32 * db + 8 * q4 + 4 * g) = v;
      }
    if (g == 0) mlbuf[wn * QROWS + row] = make_float2(st.m[qb], l_tot);
  }
  __syncthreads();

  // ---- merge the WN key-interleaved waves, then write the split's partial (or the result)
  constexpr int D4 = D / 4;
  const long long unit = (long long)(b * p.Hkv + kv);
  for (int it = tid; it < QROWS * D4; it += 256) {
    const int row = it / D4, d4 = it % D4;
    const int m = qtile * QROWS + row;
    if (m >= M) continue;
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < WN; ++w) mx = fmaxf(mx, mlbuf[w * QROWS + row].x);
    const float mx_use = (mx == -INFINITY) ? 0.f : mx;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float lsum = 0.f;
#pragma unroll
    for (int w = 0; w < WN; ++w) {
      const float2 ml = mlbuf[w * QROWS + row];
      const float wgt = fast_exp2(ml.x - mx_use);
      const float4 o = *reinterpret_cast<const float4*>(obuf + ((size_t)w * QROWS + row) * G_::O_LD + 4 * d4);
      acc.x = fmaf(o.x, wgt, acc.x);
      acc.y = fmaf(o.y, wgt, acc.y);
      acc.z = fmaf(o.z, wgt, acc.z);
      acc.w = fmaf(o.w, wgt, acc.w);
      lsum = fmaf(ml.y, wgt, lsum);
    }
    if (splits == 1) {
      const float inv = 1.f / lsum;  // lsum > 0: every row sees at least its own tree key
      const int node = m / G, hg = m % G;
      uint16_t* dst = p.out + b * p.o_sb + node * p.o_st + (long long)(kv * G + hg) * p.o_sh + 4 * d4;
      bf16x2 lo, hi;
      lo[0] = (__bf16)(acc.x * inv);
      lo[1] = (__bf16)(acc.y * inv);
      hi[0] = (__bf16)(acc.z * inv);
      hi[1] = (__bf16)(acc.w * inv);
      uint2 pk;
      pk.x = __builtin_bit_cast(unsigned int, lo);
      pk.y = __builtin_bit_cast(unsigned int, hi);
      *reinterpret_cast<uint2*>(dst) = pk;
    } else {
      const long long prow = (unit * splits + split) * p.m_pad + m;
      *reinterpret_cast<float4*>(p.part_o + prow * D + 4 * d4) = acc;
      if (d4 == 0) p.part_ml[prow] = make_float2(mx, lsum);
    }
  }
}

template <int D, int WM, int WN, int NR>
hipError_t launch_one(const KParams& kp, hipStream_t stream) {
  using G_ = Geo<D>;
  constexpr int RING_BYTES = NR * WN * 2 * G_::TILE_BYTES;
  constexpr int OBUF_BYTES = 4 * 64 * G_::O_LD * 4;
  constexpr int UNION_BYTES = RING_BYTES > OBUF_BYTES ? RING_BYTES : OBUF_BYTES;
  constexpr int SMEM = UNION_BYTES + 4 * 64 * 8 + JK_MAX_TREE * 16 + JK_MAX_TREE * 4;
  static_assert(SMEM <= 160 * 1024, "LDS budget");
  auto kern = tva_bf16_kernel<D, WM, WN, NR>;
  static bool lds_limit_raised = false;  // idempotent, so a race between host threads is harmless
  if (!lds_limit_raised) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMEM);
    if (e != hipSuccess) return e;
    lds_limit_raised = true;
  }
  hipLaunchKernelGGL(kern, dim3(kp.total_wgs), dim3(256), SMEM, stream, kp);
  return hipGetLastError();
}

}  // namespace

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

  const int key = d.head_dim * 100 + pl.wm * 10 + pl.wn;
  switch (key) {
    // ring depth: 8 tiles of K+V (128 KB at head_dim 128) whatever the wave arrangement
    case 12841: return launch_one<128, 4, 1, 8>(kp, stream);
    case 12822: return launch_one<128, 2, 2, 4>(kp, stream);
    case 12814: return launch_one<128, 1, 4, 2>(kp, stream);
    case 6441: return launch_one<64, 4, 1, 8>(kp, stream);
    case 6422: return launch_one<64, 2, 2, 4>(kp, stream);
    case 6414: return launch_one<64, 1, 4, 2>(kp, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace jk
