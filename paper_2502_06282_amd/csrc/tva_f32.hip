// Tree-masked verification attention, fp32 inputs, plain-ALU path.
//
// Same definition as the bf16 kernel (Section 2.1 step 2; Section 3.1.2 tree
// mask), kept in fp32 end to end for small, accuracy-critical shapes: one
// workgroup per (sequence, query row, key split) computes the scores of its
// keys, a two-pass softmax over them (max, then exp and sum) and the weighted
// value sum, and writes one partial (max, sum, unnormalised output) that the
// combine kernel merges.
#include "jk_internal.h"

namespace jk {
namespace {

constexpr int kF32Chunk = 1024;  // keys per workgroup

struct FParams {
  const float *q, *kc, *vc, *kt, *vt;
  const int32_t *parent, *prefix_len;
  float* part_o;
  float2* part_ml;
  unsigned* err;  // the workspace's sticky device error word
  int B, T, Hkv, G, M, m_pad, D, max_prefix, splits;
  long long q_sb, q_st, q_sh, kc_sb, kc_sl, kc_sh, kt_sb, kt_st, kt_sh;
  float scale;
};

__device__ float block_reduce_max(float v, float* red) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
  for (int w = 1; w < 4; ++w) r = fmaxf(r, red[w]);
  __syncthreads();
  return r;
}
__device__ float block_reduce_sum(float v, float* red) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0] + red[1] + red[2] + red[3];
  __syncthreads();
  return r;
}

__global__ __launch_bounds__(256) void tva_f32_kernel(FParams p) {
  __shared__ float qs[256];
  __shared__ float sc[kF32Chunk];
  __shared__ float red[4];
  __shared__ float osum[256];
  __shared__ int par_s[JK_MAX_TREE];
  __shared__ unsigned long long anc_me[2];

  const int tid = threadIdx.x;
  const int split = blockIdx.x;
  const int m = blockIdx.y;
  const int kv = blockIdx.z % p.Hkv;
  const int b = blockIdx.z / p.Hkv;
  const int node = m / p.G, hg = m % p.G;
  const int D = p.D;

  int L = p.prefix_len[b];
  L = L < 0 ? 0 : (L > p.max_prefix ? p.max_prefix : L);
  const int ktot = L + p.T;
  const int k_begin = (int)((long long)split * ktot / p.splits);
  const int k_end = (int)((long long)(split + 1) * ktot / p.splits);

  if (tid < p.T) {
    int pa = p.parent[(long long)b * p.T + tid];
    const bool ok = pa >= -1 && pa < tid;
    par_s[tid] = ok ? pa : -1;
    if (!ok && split == 0 && m == 0 && kv == 0)  // reported once per sequence
      __hip_atomic_fetch_or(p.err, kDevErrBadTree, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (tid < D) qs[tid] = p.q[b * p.q_sb + node * p.q_st + (long long)(kv * p.G + hg) * p.q_sh + tid];
  __syncthreads();
  if (tid == 0) {
    unsigned long long lo = 0, hi = 0;
    int a = node;
    while (a >= 0) {
      if (a < 64) lo |= 1ull << a; else hi |= 1ull << (a - 64);
      a = par_s[a];
    }
    anc_me[0] = lo;
    anc_me[1] = hi;
  }
  __syncthreads();

  const float* kc = p.kc + b * p.kc_sb + (long long)kv * p.kc_sh;
  const float* vc = p.vc + b * p.kc_sb + (long long)kv * p.kc_sh;
  const float* kt = p.kt + b * p.kt_sb + (long long)kv * p.kt_sh;
  const float* vt = p.vt + b * p.kt_sb + (long long)kv * p.kt_sh;

  // the host guarantees k_end - k_begin <= kF32Chunk
  float lmax = -INFINITY;
  for (int j = k_begin + tid; j < k_end; j += 256) {
    float s;
    bool vis = true;
    const float* krow;
    if (j < L) {
      krow = kc + (long long)j * p.kc_sl;
    } else {
      const int tj = j - L;
      vis = (anc_me[tj >> 6] >> (tj & 63)) & 1ull;
      krow = kt + (long long)tj * p.kt_st;
    }
    if (vis) {
      float acc = 0.f;
      for (int d = 0; d < D; d += 4) {
        const float4 kk = *reinterpret_cast<const float4*>(krow + d);
        acc = fmaf(qs[d], kk.x, acc);
        acc = fmaf(qs[d + 1], kk.y, acc);
        acc = fmaf(qs[d + 2], kk.z, acc);
        acc = fmaf(qs[d + 3], kk.w, acc);
      }
      s = acc * p.scale;
    } else {
      s = -INFINITY;
    }
    sc[j - k_begin] = s;
    lmax = fmaxf(lmax, s);
  }
  const float mx = block_reduce_max(lmax, red);
  const float mx_use = (mx == -INFINITY) ? 0.f : mx;
  float lsum = 0.f;
  for (int j = k_begin + tid; j < k_end; j += 256) {
    const float e = expf(sc[j - k_begin] - mx_use);
    sc[j - k_begin] = e;
    lsum += e;
  }
  const float tot = block_reduce_sum(lsum, red);  // also orders the sc[] writes

  // weighted value sum: thread (kg, d) adds every ngroups-th key for output column d
  const int ngroups = 256 / D;  // >= 1 because D <= 256
  const int d = tid % D, kg = tid / D;
  float acc = 0.f;
  if (kg < ngroups) {
    for (int j = k_begin + kg; j < k_end; j += ngroups) {
      const float w = sc[j - k_begin];
      if (w != 0.f) {  // skips masked tree rows entirely
        const float* vrow = (j < L) ? vc + (long long)j * p.kc_sl : vt + (long long)(j - L) * p.kt_st;
        acc = fmaf(w, vrow[d], acc);
      }
    }
  }
  osum[tid] = acc;
  __syncthreads();
  if (tid < D) {
    float o = 0.f;
    for (int g2 = 0; g2 < ngroups; ++g2) o += osum[g2 * D + tid];
    const long long prow = ((long long)(b * p.Hkv + kv) * p.splits + split) * p.m_pad + m;
    p.part_o[prow * D + tid] = o;
    if (tid == 0) p.part_ml[prow] = make_float2(mx, tot);
  }
}

}  // namespace

hipError_t launch_tva_f32(const AttnArgs& a, const AttnPlan& pl, hipStream_t stream) {
  FParams fp;
  fp.q = static_cast<const float*>(a.q);
  fp.kc = static_cast<const float*>(a.k_cache);
  fp.vc = static_cast<const float*>(a.v_cache);
  fp.kt = static_cast<const float*>(a.k_tree);
  fp.vt = static_cast<const float*>(a.v_tree);
  fp.parent = a.parent;
  fp.prefix_len = a.prefix_len;
  fp.part_o = a.part_o;
  fp.part_ml = a.part_ml;
  fp.err = a.err;
  const jk_attn_desc& d = a.d;
  fp.B = d.batch; fp.T = d.n_tree; fp.Hkv = d.n_kv_heads; fp.G = d.n_q_heads / d.n_kv_heads;
  fp.M = pl.m_rows; fp.m_pad = pl.m_pad; fp.D = d.head_dim; fp.max_prefix = a.max_prefix_len;
  fp.splits = pl.splits;
  fp.q_sb = d.q_stride_b; fp.q_st = d.q_stride_t; fp.q_sh = d.q_stride_h;
  fp.kc_sb = d.kc_stride_b; fp.kc_sl = d.kc_stride_l; fp.kc_sh = d.kc_stride_h;
  fp.kt_sb = d.kt_stride_b; fp.kt_st = d.kt_stride_t; fp.kt_sh = d.kt_stride_h;
  fp.scale = a.scale_log2;  // for this path the host passes the plain softmax scale here
  hipLaunchKernelGGL(tva_f32_kernel, dim3(pl.splits, pl.m_rows, d.batch * d.n_kv_heads), dim3(256), 0,
                     stream, fp);
  return hipGetLastError();
}

}  // namespace jk
