// Merge of the KV splits of tree-verification attention: the partial states
// (m_s, l_s, O_s) of one query row combine as
//   m = max_s m_s,  l = sum_s l_s e^(m_s - m),  out = sum_s O_s e^(m_s - m) / l,
// which is the same softmax-weighted sum the unsplit definition gives
// (Section 2.1 step 2 of the paper defines the result; the split is an
// implementation device of this library).
#include "jk_device.h"
#include "jk_internal.h"

namespace jk {
namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct CParams {
  const float* part_o;
  const float2* part_ml;
  void* out;
  int B, Hkv, G, M, m_pad, D, splits;
  unsigned long long mg_hkv, mg_g;  // floor(2^32 / d) + 1: n / d == (n * mg) >> 32 while n * d < 2^32
  long long o_sb, o_st, o_sh;
};

__device__ __forceinline__ int div_mg(int n, unsigned long long mg) {
  return (int)(((unsigned long long)(unsigned)n * mg) >> 32);
}

// Four consecutive columns of a partial output row: fp32 partials (fp32 path) or bf16 (bf16 path).
template <bool BF16>
__device__ __forceinline__ float4 load_part4(const float* part_o, long long row, int D, int d4) {
  if (BF16) {
    const uint2 v = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(part_o) + row * D + 4 * d4);
    return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16),
                       __uint_as_float(v.y & 0xffff0000u));
  }
  return *reinterpret_cast<const float4*>(part_o + row * D + 4 * d4);
}

// A workgroup merges up to 4 consecutive query rows.  A row is
// covered by two groups of D/4 threads; each thread sums every other split for four output
// columns with up to four loads in flight, and the two halves meet in LDS.  LOG2: running
// maxima are in log2 units (bf16 path) rather than natural units (fp32 path).
template <bool LOG2, bool OUT_BF16>
__global__ __launch_bounds__(256) void tva_combine_kernel(CParams p) {
  __shared__ float s_w[256];      // [row in workgroup][split] weights, splits padded to a power of two
  __shared__ float s_l[256];
  __shared__ float4 s_acc[256];
  const int tid = threadIdx.x;
  const int d4n = p.D / 4;
  const int tpr = 2 * d4n;                          // threads per row
  const int rpw = 256 / (tpr > 64 ? tpr : 64);      // rows per workgroup (at most 4)
  const int spad = 256 / rpw;                       // weight slots per row: 64 or more, >= splits
  const long long n_rows = (long long)p.B * p.Hkv * p.M;

  // this thread's output columns; its first four partial loads go out before anything else,
  // so that their latency overlaps the weight computation below
  const int rr = tid / tpr, half = (tid % tpr) / d4n, d4 = tid % d4n;
  const long long r = (long long)blockIdx.x * rpw + rr;
  const bool live = rr < rpw && r < n_rows;
  const long long unit = live ? r / p.M : 0;
  const int m = live ? (int)(r % p.M) : 0;
  const long long row0 = unit * p.splits * p.m_pad + m;
  float4 pre[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int sp = half + 2 * u;
    pre[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live && sp < p.splits)
      pre[u] = load_part4<OUT_BF16>(p.part_o, row0 + (long long)sp * p.m_pad, p.D, d4);
  }

  // weights of every (row, split) of this workgroup: one thread each
  {
    const int wr = tid / spad, sp = tid % spad;
    const long long r2 = (long long)blockIdx.x * rpw + wr;
    float mv = -INFINITY, l = 0.f;
    if (r2 < n_rows && sp < p.splits) {
      const long long unit2 = r2 / p.M;
      const float2 ml = p.part_ml[(unit2 * p.splits + sp) * p.m_pad + (r2 % p.M)];
      if (ml.y > 0.f) { mv = ml.x; l = ml.y; }  // an empty split carries no weight
    }
    float mx = mv;
    // the (at most 64) real splits of a row sit in one wave: slots are 64-aligned
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    const float mx_use = (mx == -INFINITY) ? 0.f : mx;
    const float w = LOG2 ? __builtin_amdgcn_exp2f(mv - mx_use) : expf(mv - mx_use);
    float lw = l * w;
    for (int o = 32; o > 0; o >>= 1) lw += __shfl_xor(lw, o);
    s_w[tid] = w;
    if (sp == 0) s_l[wr] = lw;
  }
  __syncthreads();

  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (live) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int sp = half + 2 * u;
      const float w = sp < p.splits ? s_w[rr * spad + sp] : 0.f;
      if (w != 0.f) {  // an unused split may hold anything
        acc.x = fmaf(pre[u].x, w, acc.x);
        acc.y = fmaf(pre[u].y, w, acc.y);
        acc.z = fmaf(pre[u].z, w, acc.z);
        acc.w = fmaf(pre[u].w, w, acc.w);
      }
    }
    for (int s0 = half + 8; s0 < p.splits; s0 += 8) {
      float4 o[4];
      float w[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int sp = s0 + 2 * u;
        w[u] = sp < p.splits ? s_w[rr * spad + sp] : 0.f;
        o[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (w[u] != 0.f)
          o[u] = load_part4<OUT_BF16>(p.part_o, row0 + (long long)sp * p.m_pad, p.D, d4);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        acc.x = fmaf(o[u].x, w[u], acc.x);
        acc.y = fmaf(o[u].y, w[u], acc.y);
        acc.z = fmaf(o[u].z, w[u], acc.z);
        acc.w = fmaf(o[u].w, w[u], acc.w);
      }
    }
  }
  s_acc[tid] = acc;
  __syncthreads();
  if (!live || half != 0) return;
  {
    const float4 o = s_acc[tid + d4n];
    acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
  }
  const float inv = 1.f / s_l[rr];
  const int kv = (int)(unit % p.Hkv);
  const int b = (int)(unit / p.Hkv);
  const int node = m / p.G, hg = m % p.G;
  const long long off = b * p.o_sb + node * p.o_st + (long long)(kv * p.G + hg) * p.o_sh + 4 * d4;
  if (OUT_BF16) {
    bf16x2 lo, hi;
    lo[0] = (__bf16)(acc.x * inv);
    lo[1] = (__bf16)(acc.y * inv);
    hi[0] = (__bf16)(acc.z * inv);
    hi[1] = (__bf16)(acc.w * inv);
    uint2 pk;
    pk.x = __builtin_bit_cast(unsigned int, lo);
    pk.y = __builtin_bit_cast(unsigned int, hi);
    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out) + off) = pk;
  } else {
    *reinterpret_cast<float4*>(static_cast<float*>(p.out) + off) =
        make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
  }
}

// bf16 path: one wave per query row, a lane per CPL = D/64 output columns, no LDS and no
// barrier.  The row is wave-uniform, so the (max, sum) pairs of its splits are uniform
// (scalar) loads and every lane derives the same weights; splits go by in chunks of 8 with
// all of a chunk's loads in flight together, merged with a running maximum.  Grid: x = unit
// (sequence, KV head), y = blocks of 4 rows.
template <int D>
__global__ __launch_bounds__(256) void tva_combine_bf16_kernel(CParams p) {
  constexpr int CPL = D / 64;
  static_assert(CPL == 1 || CPL == 2, "head_dim 64 or 128");
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int unit = blockIdx.x;
  const int m = blockIdx.y * 4 + wave;
  if (m >= p.M) return;
  const int S = p.splits;
  const long long prow0 = (long long)unit * S * p.m_pad + m;
  const uint16_t* po = reinterpret_cast<const uint16_t*>(p.part_o) + prow0 * D + CPL * lane;
  const float2* pml = p.part_ml + prow0;
  const long long po_step = (long long)p.m_pad * D;  // one split further

  float m_run = -INFINITY, l_run = 0.f, acc0 = 0.f, acc1 = 0.f;
  for (int s0 = 0; s0 < S; s0 += 8) {
    float2 ml[8];
    unsigned raw[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const bool ok = s0 + u < S;
      ml[u] = ok ? pml[(long long)(s0 + u) * p.m_pad] : make_float2(-INFINITY, 0.f);
      if (!(ml[u].y > 0.f)) ml[u] = make_float2(-INFINITY, 0.f);  // an empty split carries no weight
      raw[u] = 0u;
      if (ok) {
        const uint16_t* src = po + (long long)(s0 + u) * po_step;
        raw[u] = CPL == 2 ? *reinterpret_cast<const unsigned*>(src) : (unsigned)*src;
      }
    }
    float cm = ml[0].x;
#pragma unroll
    for (int u = 1; u < 8; ++u) cm = fmaxf(cm, ml[u].x);
    const float m_new = fmaxf(m_run, cm);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float a = __builtin_amdgcn_exp2f(m_run - m_use);  // 0 while nothing has been merged yet
    acc0 *= a;
    acc1 *= a;
    l_run *= a;
    m_run = m_new;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float w = __builtin_amdgcn_exp2f(ml[u].x - m_use);  // exp2(-inf) = 0 for empty or absent splits
      l_run = fmaf(ml[u].y, w, l_run);
      if (w != 0.f) {  // an unused split may hold anything
        const float v0 = __uint_as_float(raw[u] << 16);  // the lane's first (or only) column sits in the low half
        const float v1 = __uint_as_float(raw[u] & 0xffff0000u);
        acc0 = fmaf(v0, w, acc0);
        if (CPL == 2) acc1 = fmaf(v1, w, acc1);
      }
    }
  }
  const float inv = 1.f / l_run;  // > 0: every row sees at least its own tree key
  const int b = div_mg(unit, p.mg_hkv), kv = unit - b * p.Hkv;
  const int node = div_mg(m, p.mg_g), hg = m - node * p.G;
  uint16_t* dst = static_cast<uint16_t*>(p.out) + b * p.o_sb + node * p.o_st + (long long)(kv * p.G + hg) * p.o_sh +
                  CPL * lane;
  if (CPL == 2) {
    bf16x2 o;
    o[0] = (__bf16)(acc0 * inv);
    o[1] = (__bf16)(acc1 * inv);
    dev::store_through(dst, __builtin_bit_cast(unsigned, o));  // through to memory: nothing here reads it again
  } else {
    const __bf16 o = (__bf16)(acc0 * inv);
    *dst = __builtin_bit_cast(uint16_t, o);
  }
}

}  // namespace

hipError_t launch_tva_combine(const AttnArgs& a, const AttnPlan& pl, hipStream_t stream) {
  CParams cp;
  cp.part_o = a.part_o;
  cp.part_ml = a.part_ml;
  cp.out = a.out;
  const jk_attn_desc& d = a.d;
  cp.B = d.batch; cp.Hkv = d.n_kv_heads; cp.G = d.n_q_heads / d.n_kv_heads;
  cp.M = pl.m_rows; cp.m_pad = pl.m_pad; cp.D = d.head_dim; cp.splits = pl.splits;
  cp.o_sb = d.o_stride_b; cp.o_st = d.o_stride_t; cp.o_sh = d.o_stride_h;
  auto magic = [](int v) { return (1ull << 32) / (unsigned long long)v + 1ull; };
  cp.mg_hkv = magic(cp.Hkv);
  cp.mg_g = magic(cp.G);
  if (d.dtype == JK_BF16) {
    const dim3 grid((unsigned)(d.batch * d.n_kv_heads), (unsigned)((pl.m_rows + 3) / 4));
    if (d.head_dim == 128)
      hipLaunchKernelGGL((tva_combine_bf16_kernel<128>), grid, dim3(256), 0, stream, cp);
    else
      hipLaunchKernelGGL((tva_combine_bf16_kernel<64>), grid, dim3(256), 0, stream, cp);
  } else {
    const int tpr = 2 * (d.head_dim / 4);
    const int rpw = 256 / (tpr > 64 ? tpr : 64);
    const unsigned grid = (unsigned)(((long long)d.batch * d.n_kv_heads * pl.m_rows + rpw - 1) / rpw);
    hipLaunchKernelGGL((tva_combine_kernel<false, false>), dim3(grid), dim3(256), 0, stream, cp);
  }
  return hipGetLastError();
}

}  // namespace jk
