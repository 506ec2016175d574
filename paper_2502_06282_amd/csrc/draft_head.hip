// Draft head step of the MoE draft model (gfx950): the two feature rows that the shared output
// embedding sees (Section 3.1.2 Eq. 4: the two selected experts' features scaled by their router
// scores; Section 3.2 Eq. 6-8: their weighted sum and their weighted difference), the logits of
// both heads, the draft distributions q = softmax(logits / temperature) that the acceptance test
// divides by, and each head's top-k candidates.
//
// Three kernels:
//   head_inputs_kernel     X[2R (padded to 32), d] bf16 from f_top, s_top (elementwise, tiny)
//   skinny_gemm_kernel     Y[M, N] fp32 = X[M, K] . W[N, K]^T with M <= 256: the weight matrix
//                          (gigabytes for an output embedding) is streamed from HBM exactly once,
//                          straight into MFMA operand registers; X is small, is shared by all
//                          workgroups through L2 and staged per 64-wide k block in LDS.
//   draft_softmax_topk_kernel  per logits row: maximum, normaliser, top-k by value (ties to the
//                          lower token id), probabilities.
#include <climits>

#include "jk_internal.h"

namespace jk {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned bf16_bits_rne(float f) {
  const unsigned u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xFFFF0000u); }

// ------------------------------------------------------------------ head inputs (Eq. 4 / Eq. 6, 7)
struct MixParams {
  const unsigned short* f_top;  // [rows][2][d] bf16
  const float* s_top;           // [rows][2]
  unsigned short* x;            // [m_pad][d] bf16, row 2r + h
  int rows, d, mode;
  float alpha, beta;
};

__global__ __launch_bounds__(256) void head_inputs_kernel(MixParams p) {
  const int row = blockIdx.x, r = row >> 1, h = row & 1;
  u32x4* dst = reinterpret_cast<u32x4*>(p.x + (long long)row * p.d);
  if (r >= p.rows) {  // padding rows of the last 32-row block
    for (int c = threadIdx.x; c < p.d / 8; c += 256) dst[c] = u32x4{0u, 0u, 0u, 0u};
    return;
  }
  const u32x4* f1 = reinterpret_cast<const u32x4*>(p.f_top + ((long long)r * 2 + 0) * p.d);
  const u32x4* f2 = reinterpret_cast<const u32x4*>(p.f_top + ((long long)r * 2 + 1) * p.d);
  const float s1 = p.s_top[2 * r], s2 = p.s_top[2 * r + 1];
  // x = c1 f1 + c2 f2
  float c1, c2;
  if (p.mode == JK_HEADS_DECOUPLED) {
    c1 = h == 0 ? s1 : 0.f;
    c2 = h == 0 ? 0.f : s2;
  } else {
    c1 = h == 0 ? s1 : p.beta;
    c2 = h == 0 ? s2 : -p.alpha;
  }
  for (int c = threadIdx.x; c < p.d / 8; c += 256) {
    const u32x4 a = f1[c], b = f2[c];
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // a term whose coefficient is zero is left out, so that a NaN in the other expert's
      // feature cannot leak into a decoupled head
      const float lo = (c1 != 0.f ? c1 * bf16_lo(a[i]) : 0.f) + (c2 != 0.f ? c2 * bf16_lo(b[i]) : 0.f);
      const float hi = (c1 != 0.f ? c1 * bf16_hi(a[i]) : 0.f) + (c2 != 0.f ? c2 * bf16_hi(b[i]) : 0.f);
      o[i] = bf16_bits_rne(lo) | (bf16_bits_rne(hi) << 16);
    }
    dst[c] = o;
  }
}

// ------------------------------------------------------------------ skinny GEMM
constexpr int kGemmThreads = 256;
constexpr int kStripRows = 128;  // weight rows (output columns) per workgroup: 32 per wave
constexpr int kKB = 64;          // k extent of one main-loop step (four MFMA k steps)
constexpr int kSlabLd = 144;     // bytes per X row in the LDS slab: 128 of data + 16 of padding

struct GemmParams {
  const unsigned short* x;  // [MB*32][k] bf16, rows >= m are readable (zero or anything: not stored)
  const unsigned short* w;  // [n][ldw] bf16
  float* y;                 // [m][ldy]
  int m, n, k;
  long long ldw, ldy;
};

// v_mfma_f32_32x32x16_bf16 computes D[i][j] += sum_k A[i][k] B[k][j] with lane l holding
// A[l % 32][8 (l / 32) .. + 8], B[.. same k ..][l % 32], and D[8 (v / 4) + 4 (l / 32) + v % 4][l % 32]
// in accumulator register v.  Here i runs over weight rows (output columns n) and j over X rows
// (output rows m): a lane's four consecutive accumulator registers are four consecutive n of
// one output row, i.e. one 16-byte store.  Which sixteen k of the 64-wide block a given MFMA
// sums over is free as long as A and B agree: lane half h takes k = 32 h + 8 step .. + 8, so
// that each lane's four weight loads of a block are 64 contiguous bytes.
template <int MB>
__global__ __launch_bounds__(kGemmThreads, 2) void skinny_gemm_kernel(GemmParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char slab[2][MB * 32 * kSlabLd];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;
  const int n_base = blockIdx.x * kStripRows + wave * 32;
  // weight rows past the end re-read the last row; their results are never stored
  const int n_row = min(n_base + r, p.n - 1);
  const u32x4* wp = reinterpret_cast<const u32x4*>(p.w + (long long)n_row * p.ldw + h * 32);
  const int nkb = p.k / kKB;

  floatx16 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;

  u32x4 wa[4], wb[4], xs[MB];
  auto load_w = [&](u32x4(&dst)[4], int kb) {
#pragma unroll
    for (int j = 0; j < 4; ++j) dst[j] = __builtin_nontemporal_load(wp + kb * 8 + j);
  };
  // X slab: MB*32 rows of 128 bytes, 16 bytes per thread and pass
  auto load_x = [&](int kb) {
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const int q = tid + kGemmThreads * i;
      xs[i] = *reinterpret_cast<const u32x4*>(p.x + (long long)(q >> 3) * p.k + kb * kKB + (q & 7) * 8);
    }
  };
  auto park_x = [&](int buf) {
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const int q = tid + kGemmThreads * i;
      *reinterpret_cast<u32x4*>(&slab[buf][(q >> 3) * kSlabLd + (q & 7) * 16]) = xs[i];
    }
  };
  auto step = [&](const u32x4(&cur)[4], u32x4(&nxt)[4], int kb, int buf) {
    const bool more = kb + 1 < nkb;
    if (more) {
      load_w(nxt, kb + 1);
      load_x(kb + 1);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, cur[j]);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(&slab[buf][(mb * 32 + r) * kSlabLd + h * 64 + j * 16]);
        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[mb], 0, 0, 0);
      }
    }
    if (more) park_x(buf ^ 1);
    __syncthreads();
  };

  load_w(wa, 0);
  load_x(0);
  park_x(0);
  __syncthreads();
  for (int kb = 0; kb < nkb; kb += 2) {  // k is a multiple of 128: an even number of steps
    step(wa, wb, kb, 0);
    step(wb, wa, kb + 1, 1);
  }

  // epilogue: lane (r, h) holds, for output row mb*32 + r, columns n_base + 8 q + 4 h + (0..3)
  const bool vec_ok = (p.ldy & 3) == 0 && (reinterpret_cast<size_t>(p.y) & 15) == 0;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int m = mb * 32 + r;
    if (m >= p.m) continue;
    float* yrow = p.y + (long long)m * p.ldy;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int n = n_base + 8 * q + 4 * h;
      if (vec_ok && n + 3 < p.n) {
        *reinterpret_cast<floatx4*>(yrow + n) =
            floatx4{acc[mb][4 * q], acc[mb][4 * q + 1], acc[mb][4 * q + 2], acc[mb][4 * q + 3]};
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t)
          if (n + t < p.n) yrow[n + t] = acc[mb][4 * q + t];
      }
    }
  }
}

template <int MB>
hipError_t launch_gemm_mb(const GemmParams& p, hipStream_t stream) {
  const unsigned grid = (unsigned)((p.n + kStripRows - 1) / kStripRows);
  hipLaunchKernelGGL(skinny_gemm_kernel<MB>, dim3(grid), dim3(kGemmThreads), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_gemm(const GemmParams& p, hipStream_t stream) {
  switch ((p.m + 31) / 32) {
    case 1: return launch_gemm_mb<1>(p, stream);
    case 2: return launch_gemm_mb<2>(p, stream);
    case 3: return launch_gemm_mb<3>(p, stream);
    case 4: return launch_gemm_mb<4>(p, stream);
    case 5: return launch_gemm_mb<5>(p, stream);
    case 6: return launch_gemm_mb<6>(p, stream);
    case 7: return launch_gemm_mb<7>(p, stream);
    case 8: return launch_gemm_mb<8>(p, stream);
    default: return hipErrorInvalidValue;
  }
}

// ------------------------------------------------------------------ softmax + top-k per logits row
constexpr int kSoftThreads = 1024;
constexpr int kSoftWaves = kSoftThreads / 64;
constexpr int kCandCap = 4096;

struct SoftParams {
  const float* logits;  // [n_rows][vocab]
  float* probs;         // [n_rows][vocab] or nullptr
  int* tk_ids;          // [n_rows][k]
  float* tk_probs;      // [n_rows][k]
  int n_rows, vocab, k;
  float inv_temp;
};

// order of candidates: larger value first, equal values by increasing token id
__device__ __forceinline__ bool better(float av, int ai, float bv, int bi) {
  return av > bv || (av == bv && ai < bi);
}

struct Best {
  float v;
  int id;
};

// best (value, id) pair of the block, for every thread
__device__ __forceinline__ Best block_best(float v, int id, float* sv, int* si) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(v, o);
    const int oi = __shfl_xor(id, o);
    if (better(ov, oi, v, id)) {
      v = ov;
      id = oi;
    }
  }
  __syncthreads();  // the previous round's readers are done with sv, si
  if ((threadIdx.x & 63) == 0) {
    sv[threadIdx.x >> 6] = v;
    si[threadIdx.x >> 6] = id;
  }
  __syncthreads();
  Best b{sv[0], si[0]};
#pragma unroll
  for (int i = 1; i < kSoftWaves; ++i)
    if (better(sv[i], si[i], b.v, b.id)) b = Best{sv[i], si[i]};
  return b;
}

// One workgroup per row.  Top-k: the k-th largest of the threads' own maxima is a lower bound of
// the row's k-th largest value, so only elements at or above it can be among the top k; they
// are collected in LDS during the normaliser pass (few, unless the row is full of ties) and the
// k winners are picked from that list.  A row with more such elements than the list holds is
// handled by k selection passes over the whole row instead.
__global__ __launch_bounds__(kSoftThreads) void draft_softmax_topk_kernel(SoftParams p) {
  __shared__ float sv[kSoftWaves];
  __shared__ int si[kSoftWaves];
  __shared__ double sd[kSoftWaves];
  __shared__ float cand_v[kCandCap];
  __shared__ int cand_i[kCandCap];
  __shared__ int n_cand;
  __shared__ float win_v[16];
  __shared__ int win_i[16];
  const int tid = threadIdx.x, V = p.vocab, K = p.k;
  const float* x = p.logits + (long long)blockIdx.x * V;
  const bool vec = (V & 3) == 0 && (reinterpret_cast<size_t>(p.logits) & 15) == 0;
  const int n4 = vec ? V / 4 : 0;
  const floatx4* x4 = reinterpret_cast<const floatx4*>(x);

  // every element once, ids increasing within a thread
  auto for_each = [&](auto&& fn) {
    for (int i = tid; i < n4; i += kSoftThreads) {
      const floatx4 q = x4[i];
      fn(4 * i, q[0]);
      fn(4 * i + 1, q[1]);
      fn(4 * i + 2, q[2]);
      fn(4 * i + 3, q[3]);
    }
    for (int i = 4 * n4 + tid; i < V; i += kSoftThreads) fn(i, x[i]);
  };

  // pass 1: each thread's maximum
  float tv = -INFINITY;
  int ti = INT_MAX;
  for_each([&](int i, float v) {
    if (v > tv) {
      tv = v;
      ti = i;
    }
  });
  if (tid == 0) n_cand = 0;
  float row_max = -INFINITY, tau = -INFINITY;
  for (int i = 0; i < K; ++i) {
    const Best b = block_best(tv, ti, sv, si);
    if (i == 0) row_max = b.v;
    tau = b.id == INT_MAX ? -INFINITY : b.v;
    if (b.id == ti) {  // (ids are distinct, INT_MAX marks "none")
      tv = -INFINITY;
      ti = INT_MAX;
    }
  }
  if (!(row_max > -INFINITY)) row_max = 0.f;  // a row of -inf (or NaN): nothing sensible to subtract
  __syncthreads();

  // pass 2: normaliser and candidates
  float lsum = 0.f;
  for_each([&](int i, float v) {
    lsum += expf((v - row_max) * p.inv_temp);
    if (v >= tau) {
      const int slot = atomicAdd(&n_cand, 1);
      if (slot < kCandCap) {
        cand_v[slot] = v;
        cand_i[slot] = i;
      }
    }
  });
  double ds = (double)lsum;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ds += __shfl_xor(ds, o);
  if ((tid & 63) == 0) sd[tid >> 6] = ds;
  __syncthreads();
  double z = 0.0;
#pragma unroll
  for (int i = 0; i < kSoftWaves; ++i) z += sd[i];
  const float inv_z = (float)(1.0 / z);
  const int nc = n_cand;

  if (nc <= kCandCap) {
    for (int i = 0; i < K; ++i) {
      float bv = -INFINITY;
      int bi = INT_MAX, bj = -1;
      for (int j = tid; j < nc; j += kSoftThreads)
        if (better(cand_v[j], cand_i[j], bv, bi)) {
          bv = cand_v[j];
          bi = cand_i[j];
          bj = j;
        }
      const Best b = block_best(bv, bi, sv, si);
      if (bj >= 0 && b.id == bi) {  // mine: take it out of the list
        cand_v[bj] = -INFINITY;
        cand_i[bj] = INT_MAX;
      }
      if (tid == 0) {
        win_v[i] = b.v;
        win_i[i] = b.id;
      }
      // (the next round's first barrier inside block_best orders the removal before the scans)
      __syncthreads();
    }
  } else {
    float pv = INFINITY;
    int pi = -1;
    for (int i = 0; i < K; ++i) {
      float bv = -INFINITY;
      int bi = INT_MAX;
      for_each([&](int id, float v) {
        const bool after = pi < 0 || v < pv || (v == pv && id > pi);
        if (after && better(v, id, bv, bi)) {
          bv = v;
          bi = id;
        }
      });
      const Best b = block_best(bv, bi, sv, si);
      pv = b.v;
      pi = b.id == INT_MAX ? V : b.id;
      if (tid == 0) {
        win_v[i] = b.v;
        win_i[i] = b.id;
      }
    }
    __syncthreads();
  }
  if (tid < K) {
    const int id = win_i[tid];
    const bool ok = id >= 0 && id < V;
    p.tk_ids[(long long)blockIdx.x * K + tid] = ok ? id : 0;
    p.tk_probs[(long long)blockIdx.x * K + tid] = ok ? expf((win_v[tid] - row_max) * p.inv_temp) * inv_z : 0.f;
  }

  // pass 3: the distribution itself
  if (p.probs) {
    float* q = p.probs + (long long)blockIdx.x * V;
    floatx4* q4 = reinterpret_cast<floatx4*>(q);
    const bool qvec = vec && (reinterpret_cast<size_t>(p.probs) & 15) == 0;
    if (qvec) {
      for (int i = tid; i < n4; i += kSoftThreads) {
        const floatx4 s = x4[i];
        floatx4 o;
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = expf((s[t] - row_max) * p.inv_temp) * inv_z;
        q4[i] = o;
      }
    } else {
      for (int i = tid; i < V; i += kSoftThreads) q[i] = expf((x[i] - row_max) * p.inv_temp) * inv_z;
    }
  }
}

}  // namespace

size_t draft_heads_workspace_bytes(int rows, int d_model) {
  const size_t m_pad = (size_t)((2 * rows + 31) / 32) * 32;
  return (m_pad * (size_t)d_model * 2 + 255) / 256 * 256;
}

hipError_t launch_draft_heads(const DraftHeadsArgs& a, hipStream_t stream) {
  const int m = 2 * a.rows, m_pad = (m + 31) / 32 * 32;
  MixParams mp;
  mp.f_top = static_cast<const unsigned short*>(a.f_top);
  mp.s_top = a.s_top;
  mp.x = static_cast<unsigned short*>(a.workspace);
  mp.rows = a.rows; mp.d = a.d_model; mp.mode = a.mode; mp.alpha = a.alpha; mp.beta = a.beta;
  hipLaunchKernelGGL(head_inputs_kernel, dim3(m_pad), dim3(256), 0, stream, mp);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  GemmParams gp;
  gp.x = mp.x;
  gp.w = static_cast<const unsigned short*>(a.w_head);
  gp.y = a.logits;
  gp.m = m; gp.n = a.vocab; gp.k = a.d_model;
  gp.ldw = a.d_model; gp.ldy = a.vocab;
  e = launch_gemm(gp, stream);
  if (e != hipSuccess) return e;

  SoftParams sp;
  sp.logits = a.logits; sp.probs = a.draft_probs; sp.tk_ids = a.topk_tokens; sp.tk_probs = a.topk_probs;
  sp.n_rows = m; sp.vocab = a.vocab; sp.k = a.top_k; sp.inv_temp = 1.0f / a.temperature;
  hipLaunchKernelGGL(draft_softmax_topk_kernel, dim3(m), dim3(kSoftThreads), 0, stream, sp);
  return hipGetLastError();
}

}  // namespace jk
