// Merge of the KV splits of tree-verification attention: the partial states
// (m_s, l_s, O_s) of one query row combine as
//   m = max_s m_s,  l = sum_s l_s e^(m_s - m),  out = sum_s O_s e^(m_s - m) / l,
// which is the same softmax-weighted sum the unsplit definition gives
// (Section 2.1 step 2 of the paper defines the result; the split is an
// implementation device of this library).
#include "jk_internal.h"

namespace jk {
namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct CParams {
  const float* part_o;
  const float2* part_ml;
  void* out;
  int B, Hkv, G, M, m_pad, D, splits;
  long long o_sb, o_st, o_sh;
};

// One workgroup per query row.  Thread (sg, d4) sums every NG-th split for four output
// columns, so the loads of a row's splits are all in flight together; the NG partial sums
// meet in LDS.  LOG2: running maxima are in log2 units (bf16 path) rather than natural
// units (fp32 path).
template <bool LOG2, bool OUT_BF16>
__global__ __launch_bounds__(256) void tva_combine_kernel(CParams p) {
  __shared__ float s_m[kMaxSplits], s_w[kMaxSplits];
  __shared__ float4 s_acc[256];
  __shared__ float s_l;
  const int tid = threadIdx.x;
  const int d4n = p.D / 4;        // 16..64 threads cover a row
  const int ng = 256 / d4n;       // split groups
  const int d4 = tid % d4n, sg = tid / d4n;
  const long long r = blockIdx.x;  // (b * Hkv + kv) * M + m
  const int m = (int)(r % p.M);
  const long long unit = r / p.M;
  const int kv = (int)(unit % p.Hkv);
  const int b = (int)(unit / p.Hkv);
  const long long row0 = unit * p.splits * p.m_pad + m;

  float my_l = 0.f;
  if (tid < p.splits) {
    const float2 ml = p.part_ml[row0 + (long long)tid * p.m_pad];
    s_m[tid] = ml.y > 0.f ? ml.x : -INFINITY;  // an empty split carries no weight
    my_l = ml.y;
  }
  __syncthreads();
  float mx = -INFINITY;
  for (int s = 0; s < p.splits; ++s) mx = fmaxf(mx, s_m[s]);
  const float mx_use = (mx == -INFINITY) ? 0.f : mx;
  float lw = 0.f;
  if (tid < p.splits) {
    const float w = LOG2 ? __builtin_amdgcn_exp2f(s_m[tid] - mx_use) : expf(s_m[tid] - mx_use);
    s_w[tid] = w;
    lw = my_l * w;
  }
  if (tid < 64) {  // splits <= 64 all live in the first wave
    for (int o = 32; o > 0; o >>= 1) lw += __shfl_xor(lw, o);
    if (tid == 0) s_l = lw;
  }
  __syncthreads();

  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (sg < ng) {
    for (int s = sg; s < p.splits; s += ng) {
      const float w = s_w[s];
      if (w == 0.f) continue;
      const float4 o = *reinterpret_cast<const float4*>(p.part_o + (row0 + (long long)s * p.m_pad) * p.D + 4 * d4);
      acc.x = fmaf(o.x, w, acc.x);
      acc.y = fmaf(o.y, w, acc.y);
      acc.z = fmaf(o.z, w, acc.z);
      acc.w = fmaf(o.w, w, acc.w);
    }
  }
  s_acc[tid] = acc;
  __syncthreads();
  if (sg != 0) return;
  for (int g2 = 1; g2 < ng; ++g2) {
    const float4 o = s_acc[g2 * d4n + d4];
    acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
  }
  const float inv = 1.f / s_l;
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
  const unsigned grid = (unsigned)((long long)d.batch * d.n_kv_heads * pl.m_rows);
  if (d.dtype == JK_BF16)
    hipLaunchKernelGGL((tva_combine_kernel<true, true>), dim3(grid), dim3(256), 0, stream, cp);
  else
    hipLaunchKernelGGL((tva_combine_kernel<false, false>), dim3(grid), dim3(256), 0, stream, cp);
  return hipGetLastError();
}

}  // namespace jk
