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
// K/V travel HBM -> registers (128-bit loads, 16 lanes per 256-byte row,
// several tiles in flight) -> LDS (XOR-swizzled 16-byte chunks so both the
// 128-bit K reads and the transpose V reads are bank-conflict free).
#include "jk_internal.h"

namespace jk {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));

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

template <int D, int WM, int WN, int PD>
__global__ __launch_bounds__(256, 1) void tva_bf16_kernel(KParams p) {
  using G_ = Geo<D>;
  constexpr int NCH = G_::NCH, DK = G_::DK, DB = G_::DB;
  constexpr int QROWS = 64 * WM;
  constexpr int TILE_BYTES = G_::TILE_BYTES;
  constexpr int RING_BYTES = 2 * WN * 2 * TILE_BYTES;
  constexpr int OBUF_BYTES = 4 * 64 * G_::O_LD * 4;
  constexpr int UNION_BYTES = RING_BYTES > OBUF_BYTES ? RING_BYTES : OBUF_BYTES;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* ring = smem;
  float* obuf = reinterpret_cast<float*>(smem);                            // [WN][QROWS][O_LD], after the loop
  float2* mlbuf = reinterpret_cast<float2*>(smem + UNION_BYTES);           // [WN][QROWS]
  unsigned long long* anc = reinterpret_cast<unsigned long long*>(smem + UNION_BYTES + 4 * 64 * 8);  // [128][2]
  int* par_s = reinterpret_cast<int*>(smem + UNION_BYTES + 4 * 64 * 8 + JK_MAX_TREE * 16);           // [128]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave % WM;
  const int wn = wave / WM;
  const int c32 = lane & 31;
  const int g = lane >> 5;

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
  const int split = rest % p.splits;
  rest /= p.splits;
  if (rest >= p.B * p.Hkv) return;  // padding workgroup
  const int kv = rest % p.Hkv;
  const int b = rest / p.Hkv;

  int L = p.prefix_len[b];
  L = L < 0 ? 0 : (L > p.max_prefix ? p.max_prefix : L);
  const int n_ptiles = (L + kTileKeys - 1) / kTileKeys;
  const int n_ttiles = (p.T + kTileKeys - 1) / kTileKeys;
  const int nt = n_ptiles + n_ttiles;
  const int t_begin = (int)((long long)split * nt / p.splits);
  const int t_end = (int)((long long)(split + 1) * nt / p.splits);
  const int n_rounds = (t_end - t_begin + WN - 1) / WN;

  // ---- ancestor sets (only workgroups that reach tree tiles need them)
  const bool has_tree = t_end > n_ptiles;
  if (has_tree) {
    if (tid < p.T) {
      int pa = p.parent[(long long)b * p.T + tid];
      par_s[tid] = (pa >= -1 && pa < tid) ? pa : -1;
    }
    __syncthreads();
    if (tid < p.T) {
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

  // ---- this wave's 64 query rows as MFMA B operands (lane: row c32, 8 consecutive d)
  const int row_base = qtile * QROWS + wm * 64;  // first row (within the KV head's M rows)
  bf16x8 qreg[2][DK];
  int node_of[2];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int m = row_base + qb * 32 + c32;
    const bool ok = m < p.M;
    const int mm = ok ? m : p.M - 1;
    const int node = mm / p.G, hg = mm % p.G;
    node_of[qb] = node;
    const uint16_t* src = p.q + b * p.q_sb + node * p.q_st + (long long)(kv * p.G + hg) * p.q_sh + 8 * g;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) {
      uint4 v = ok ? *reinterpret_cast<const uint4*>(src + ks * 16) : make_uint4(0, 0, 0, 0);
      qreg[qb][ks] = __builtin_bit_cast(bf16x8, v);
    }
  }

  floatx16 oacc[2][DB];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[qb][db][i] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY};
  float l_run[2] = {0.f, 0.f};

  // ---- tile sources
  const uint16_t* kc_base = p.kc + b * p.kc_sb + (long long)kv * p.kc_sh;
  const uint16_t* vc_base = p.vc + b * p.kc_sb + (long long)kv * p.kc_sh;
  const uint16_t* kt_base = p.kt + b * p.kt_sb + (long long)kv * p.kt_sh;
  const uint16_t* vt_base = p.vt + b * p.kt_sb + (long long)kv * p.kt_sh;

  // per-thread chunk coordinates inside a tile (same for K and V)
  int ch_row[NCH], ch_col[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int cid = tid + j * 256;
    ch_row[j] = cid / G_::CPR;
    ch_col[j] = cid % G_::CPR;
  }

  uint4 pf[PD][WN][2][NCH];

  auto issue_round = [&](int r, uint4 (&dst)[WN][2][NCH]) {
#pragma unroll
    for (int w = 0; w < WN; ++w) {
      int t = t_begin + r * WN + w;
      if (t >= t_end) t = t_end - 1;  // duplicate of a real tile, never consumed
      const bool tree = t >= n_ptiles;
      const int key0 = (tree ? t - n_ptiles : t) * kTileKeys;
      const int last = (tree ? p.T : L) - 1 - key0;  // last valid row of the tile (>= 0)
      const uint16_t* kb = tree ? kt_base : kc_base;
      const uint16_t* vb = tree ? vt_base : vc_base;
      const long long rs = tree ? p.kt_st : p.kc_sl;
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        const int rr = ch_row[j] < last ? ch_row[j] : last;
        const long long off = (long long)(key0 + rr) * rs + ch_col[j] * 8;
        dst[w][0][j] = *reinterpret_cast<const uint4*>(kb + off);
        dst[w][1][j] = *reinterpret_cast<const uint4*>(vb + off);
      }
    }
  };
  auto store_round = [&](int r, const uint4 (&src)[WN][2][NCH]) {
    unsigned char* st = ring + (r & 1) * (WN * 2 * TILE_BYTES);
#pragma unroll
    for (int w = 0; w < WN; ++w) {
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        *reinterpret_cast<uint4*>(st + (w * 2 + 0) * TILE_BYTES + G_::koff(ch_row[j], ch_col[j])) = src[w][0][j];
        *reinterpret_cast<uint4*>(st + (w * 2 + 1) * TILE_BYTES + G_::voff(ch_row[j], ch_col[j])) = src[w][1][j];
      }
    }
  };

  auto compute_tile = [&](int t, const unsigned char* kt_s, const unsigned char* vt_s) {
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
        sacc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][ks], sacc[qb], 0, 0, 0);
    }
    // ---- masks: register i of a lane is key 8*(i/4) + 4*g + i%4 of the tile
    const bool tree = t >= n_ptiles;
    if (tree) {
      const int tt = t - n_ptiles;
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const unsigned long long w64 = anc[2 * node_of[qb] + (tt >> 1)];
        const unsigned int bits = (unsigned int)(w64 >> ((tt & 1) * 32));
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kk = 8 * (i / 4) + 4 * g + (i % 4);
          if (!((bits >> kk) & 1u)) sacc[qb][i] = -INFINITY;
        }
      }
    } else {
      const int nvalid = L - t * kTileKeys;
      if (nvalid < kTileKeys) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int kk = 8 * (i / 4) + 4 * g + (i % 4);
            if (kk >= nvalid) sacc[qb][i] = -INFINITY;
          }
      }
    }
    // ---- online softmax; probabilities become bf16 B operands of the value product
    bf16x8 pb[2][2];
    float alpha[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      float tmax = sacc[qb][0];
#pragma unroll
      for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, sacc[qb][i]);
      tmax = half_swap_max(tmax);
      const float m_new = fmaxf(m_run[qb], tmax * p.scale_log2);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      alpha[qb] = fast_exp2(m_run[qb] - m_use);
      m_run[qb] = m_new;
      float lsum = 0.f;
      float pr[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        pr[i] = fast_exp2(fmaf(sacc[qb][i], p.scale_log2, -m_use));
        lsum += pr[i];
      }
      l_run[qb] = fmaf(l_run[qb], alpha[qb], lsum);
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[qb][j][e] = (__bf16)pr[8 * j + e];
    }
    // rescale the accumulators only when some row's maximum moved
    if (__any((alpha[0] != 1.f) || (alpha[1] != 1.f))) {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[qb][db][i] *= alpha[qb];
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
          oacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb][j], oacc[qb][db], 0, 0, 0);
      }
    }
  };

  // ---- main loop: PD rounds of loads in flight in registers, double-buffered LDS
  if (n_rounds > 0) {
#pragma unroll
    for (int u = 0; u < PD; ++u)
      if (u < n_rounds) issue_round(u, pf[u]);
  }
  for (int r0 = 0; r0 < n_rounds; r0 += PD) {
#pragma unroll
    for (int u = 0; u < PD; ++u) {
      const int r = r0 + u;
      if (r < n_rounds) {
        store_round(r, pf[u]);
        if (r + PD < n_rounds) issue_round(r + PD, pf[u]);
        __syncthreads();
        const int t = t_begin + r * WN + wn;
        if (t < t_end) {
          const unsigned char* st = ring + (r & 1) * (WN * 2 * TILE_BYTES) + wn * 2 * TILE_BYTES;
          compute_tile(t, st, st + TILE_BYTES);
        }
      }
    }
  }
  __syncthreads();  // every wave is done with the ring before it becomes the epilogue buffer

  // ---- epilogue: O^T and (max, sum) of each wave into LDS
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const float l_tot = half_swap_sum(l_run[qb]);
    const int row = wm * 64 + qb * 32 + c32;
    float* orow = obuf + ((size_t)wn * QROWS + row) * G_::O_LD;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        float4 v = make_float4(oacc[qb][db][4 * q4], oacc[qb][db][4 * q4 + 1], oacc[qb][db][4 * q4 + 2],
                               oacc[qb][db][4 * q4 + 3]);
        *reinterpret_cast<float4*>(orow + 32 * db + 8 * q4 + 4 * g) = v;
      }
    if (g == 0) mlbuf[wn * QROWS + row] = make_float2(m_run[qb], l_tot);
  }
  __syncthreads();

  // ---- merge the WN key-interleaved waves, then write the split's partial (or the result)
  constexpr int D4 = D / 4;
  const long long unit = (long long)(b * p.Hkv + kv);
  for (int it = tid; it < QROWS * D4; it += 256) {
    const int row = it / D4, d4 = it % D4;
    const int m = qtile * QROWS + row;
    if (m >= p.M) continue;
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
    if (p.splits == 1) {
      const float inv = 1.f / lsum;  // lsum > 0: every row sees at least its own tree key
      const int node = m / p.G, hg = m % p.G;
      uint16_t* dst = p.out + b * p.o_sb + node * p.o_st + (long long)(kv * p.G + hg) * p.o_sh + 4 * d4;
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
      const long long prow = (unit * p.splits + split) * p.m_pad + m;
      *reinterpret_cast<float4*>(p.part_o + prow * D + 4 * d4) = acc;
      if (d4 == 0) p.part_ml[prow] = make_float2(mx, lsum);
    }
  }
}

template <int D, int WM, int WN, int PD>
hipError_t launch_one(const KParams& kp, hipStream_t stream) {
  using G_ = Geo<D>;
  constexpr int RING_BYTES = 2 * WN * 2 * G_::TILE_BYTES;
  constexpr int OBUF_BYTES = 4 * 64 * G_::O_LD * 4;
  constexpr int UNION_BYTES = RING_BYTES > OBUF_BYTES ? RING_BYTES : OBUF_BYTES;
  constexpr int SMEM = UNION_BYTES + 4 * 64 * 8 + JK_MAX_TREE * 16 + JK_MAX_TREE * 4;
  static_assert(SMEM <= 160 * 1024, "LDS budget");
  auto kern = tva_bf16_kernel<D, WM, WN, PD>;
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
    case 12841: return launch_one<128, 4, 1, 4>(kp, stream);
    case 12822: return launch_one<128, 2, 2, 2>(kp, stream);
    case 12814: return launch_one<128, 1, 4, 1>(kp, stream);
    case 6441: return launch_one<64, 4, 1, 4>(kp, stream);
    case 6422: return launch_one<64, 2, 2, 2>(kp, stream);
    case 6414: return launch_one<64, 1, 4, 1>(kp, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace jk
