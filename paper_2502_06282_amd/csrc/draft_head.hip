// Draft head step of the MoE draft model (gfx950): the two feature rows that the shared output
// embedding sees (Section 3.1.2 Eq. 4: the two selected experts' features scaled by their router
// scores; Section 3.2 Eq. 6-8: their weighted sum and their weighted difference), the logits of
// both heads, the draft distributions q = softmax(logits / temperature) that the acceptance test
// divides by, and each head's top-k candidates.
//
// Kernels:
//   head_inputs_kernel     X[2R (padded to 32), d] bf16 from f_top, s_top (elementwise, tiny)
//   skinny_gemm_kernel     Y[M, N] fp32 = X[M, K] . W[N, K]^T with M <= 256: the weight matrix
//                          (gigabytes for an output embedding) is streamed from HBM exactly once;
//                          both operands are staged HBM/L2 -> LDS in swizzled 64-byte row segments
//                          and read from there in MFMA layout.  Batched over experts and split
//                          along k where a projection alone would not fill the chip.
//   row_parts_kernel, row_finish_kernel   per logits row: maximum, normaliser,
//                          top-k by value (ties to the lower token id), probabilities.
//   router_kernel, gated_act_kernel, select_kernel   the draft layer's router (Eq. 2, 5) and what
//                          surrounds the experts' three projections (Eq. 3).
#include <climits>

#include "jk_device.h"
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
constexpr int kGemmThreads = 512;  // 8 waves
constexpr int kKB = 32;            // k extent of one main-loop step (two MFMA k steps): 64 bytes per row

struct GemmParams {
  const uint16_t* x;  // [m][k] bf16
  const uint16_t* w;  // [n][ldw] bf16
  float* y;           // [m][ldy]
  int m, n, k;
  long long ldw, ldy;
  // batch (blockIdx.y): element offsets between consecutive problems; `sel` (device, may be null):
  // n_sel problem numbers, a problem that none of them names is switched off (the experts no
  // row selected; every workgroup scans the list itself: at most 256 entries, and no flag array
  // that a launch of its own would have to clear first)
  int batch;
  long long x_batch, w_batch, y_batch;
  const int* sel;
  int n_sel;
  // a second weight tensor over the same X (the experts' gate and up projections in one launch):
  // blockIdx.y in [batch, 2 batch) takes w2 / y2
  const uint16_t* w2;
  float* y2;
  // split of the k range (blockIdx.z): every part writes its own partial output, y_split elements
  // apart; whoever reads y adds them up in a fixed order
  int ksplit;
  long long y_split;
};

typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8_t;
__device__ __forceinline__ bf16x8 lds_read16(unsigned addr) { return *(lds_bf16x8_t*)(size_t)addr; }

using dev::dma16;
using dev::uniform_ptr;
using dev::wait_vm;

// Plan of one workgroup (one per CU, 8 waves).  Every wave owns NBW 32-row blocks of the weight
// strip and all MB 32-row blocks of X: NBW * MB accumulator tiles of 16 registers.  LDS holds a
// ring of DW steps of weight fragments per wave (private to the wave that loads and reads them)
// and a ring of DX steps of X slabs (shared by the workgroup).
template <int MB>
struct GemmCfg {
  static constexpr int NBW = MB <= 6 ? 2 : 1;
  static constexpr int STRIP = 8 * 32 * NBW;       // weight rows (output columns) per workgroup
  static constexpr int DW = NBW == 1 ? 6 : 4;
  static constexpr int DX = MB <= 3 ? 4 : (MB <= 5 ? 3 : (MB == 6 ? 2 : 3));
  static constexpr int W_STEP = NBW * 2048;        // bytes per wave and step: NBW*32 rows of 64 bytes
  static constexpr int W_WAVE = DW * W_STEP;
  static constexpr int X_STEP = MB * 2048;         // MB*32 rows of 64 bytes
  static constexpr int X_BASE = 8 * W_WAVE;
  static constexpr int SMEM = X_BASE + DX * X_STEP;
  static constexpr int NXI = 2 * MB;               // X transfers per step (1 KB = 16 rows each), dealt out to the waves
  static constexpr int NWI = 2 * NBW;              // weight transfers per wave and step
  static_assert(SMEM <= 160 * 1024, "LDS plan");
  // Transfers complete in issue order; a wave issues, per step, its cx X transfers, then NWI of
  // weights.  At the top of step kb the data of step kb must have landed: X(kb) was asked for
  // DX - 1 steps ago, W(kb) DW - 1 steps ago.
  static constexpr int wait_count(int cx) {
    const int per = cx + NWI;
    const int wx = NWI + (DX - 2) * per, ww = (DW - 2) * per;
    return cx == 0 ? ww : (wx < ww ? wx : ww);
  }
};

// v_mfma_f32_32x32x16_bf16 computes D[i][j] += sum_k A[i][k] B[k][j] with lane l holding
// A[l % 32][8 (l / 32) .. + 8], B[.. same k ..][l % 32], and D[8 (v / 4) + 4 (l / 32) + v % 4][l % 32]
// in accumulator register v.  Here i runs over weight rows (output columns n) and j over X rows
// (output rows m): a lane's four consecutive accumulator registers are four consecutive n of
// one output row, i.e. one 16-byte store.
//
// Both operands go HBM/L2 -> LDS in 64-byte row segments, four lanes per row (an MFMA operand
// read straight from global memory would touch 32 cache lines per instruction and use 32 bytes
// of each).  The strip is wide (up to 512 weight rows) because every workgroup has to pull all
// of X through the same path as its weights: X traffic is (m / strip) of the weight traffic.
// A row's four 16-byte pieces are stored XOR-swizzled with key(row) = (row >> 2) & 3 (the transfer
// fetches piece s ^ key into slot s).  Measured with SQ_LDS_BANK_CONFLICT: this key (like bits 3-4 of
// the row) gives no conflict cycles at all for an operand read (32 rows, one piece of each), bits
// 0-1 or 1-2 cost four cycles per read.
template <int MB>
__global__ __launch_bounds__(kGemmThreads, 1) void skinny_gemm_kernel(GemmParams p) {
  using C = GemmCfg<MB>;
  constexpr int NBW = C::NBW;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];  // the kernel's only LDS: offset 0
  int e = blockIdx.y;
  if (e >= p.batch) {
    e -= p.batch;
    p.w = p.w2;
    p.y = p.y2;
  }
  if (p.sel) {  // every wave scans the whole list itself: the same answer in all of them, no LDS, no barrier
    int mine = 0;
    for (int i = threadIdx.x & 63; i < p.n_sel; i += 64) mine |= (int)(p.sel[i] == e);
    if (!__any(mine)) return;  // (the whole workgroup: nobody waits at a later barrier)
  }
  p.x += (long long)e * p.x_batch;
  p.w += (long long)e * p.w_batch;
  p.y += (long long)e * p.y_batch + (long long)blockIdx.z * p.y_split;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;
  const long long strip0 = (long long)blockIdx.x * C::STRIP;
  const int n_base = (int)strip0 + wave * 32 * NBW;
  const int nkb = p.k / kKB / p.ksplit;  // k blocks of this part
  const int k_first = (int)blockIdx.z * nkb * kKB;
  // Workgroups start at different k blocks and wrap around, so that at any moment they ask for
  // different columns of the weight matrix and of X.
  const int kb0 = (int)((blockIdx.x * 5u) % (unsigned)nkb);
  auto rot = [&](int kb) {
    const int t = (kb < nkb ? kb : nkb - 1) + kb0;  // past the end: the last block again (unused, keeps the counts exact)
    return t >= nkb ? t - nkb : t;
  };

  // transfer geometry: one instruction covers 16 rows, lane l -> row l / 4 of them, slot l % 4
  const int sub = lane >> 2, slot = lane & 3;
  // slot `slot` of a row holds piece slot ^ key(row), key(row) = (row >> 2) & 3 (the same for every 16-row transfer)
  const unsigned piece = (unsigned)((slot ^ ((sub >> 2) & 3)) << 4);
  unsigned voff_w[C::NWI], voff_x[2];
#pragma unroll
  for (int i = 0; i < C::NWI; ++i) {
    const int row = min(n_base + 16 * i + sub, p.n - 1);  // rows past the end repeat the last one; never stored
    voff_w[i] = (unsigned)((row - strip0) * p.ldw * 2) + piece;
  }
  // X transfer q (16 rows) belongs to wave q % 8: at most two per wave (MB <= 8)
  const int cx = (wave < C::NXI ? 1 : 0) + (wave + 8 < C::NXI ? 1 : 0);
#pragma unroll
  for (int t = 0; t < 2; ++t)  // rows past the end repeat the last one (their results are never stored)
    voff_x[t] = (unsigned)((long long)min(16 * (wave + 8 * t) + sub, p.m - 1) * p.k * 2) + piece;
  const uint16_t* w_strip = uniform_ptr(p.w + strip0 * p.ldw);
  const unsigned w_ring = (unsigned)(wave * C::W_WAVE);

  auto issue_x = [&](int kb) {
    const uint16_t* xb = uniform_ptr(p.x + k_first + rot(kb) * kKB);
    const unsigned xs = (unsigned)(C::X_BASE + (kb % C::DX) * C::X_STEP);
    if (cx > 0) dma16(xb, voff_x[0], xs + (unsigned)(wave * 1024));
    if (cx > 1) dma16(xb, voff_x[1], xs + (unsigned)((wave + 8) * 1024));
  };
  auto issue_w = [&](int kb) {
    const uint16_t* wb = uniform_ptr(w_strip + k_first + rot(kb) * kKB);
    const unsigned ws = w_ring + (unsigned)((kb % C::DW) * C::W_STEP);
#pragma unroll
    for (int i = 0; i < C::NWI; ++i) dma16(wb, voff_w[i], ws + (unsigned)(i * 1024));
  };

  floatx16 acc[NBW][MB];
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.f;

  // operand read addresses within a slab: row r of a 32-row block (64 bytes per row), piece
  // 2 j + h of MFMA k step j, swizzled
  const unsigned rd = (unsigned)(r * 64);
  const unsigned key = (unsigned)((r >> 2) & 3);

#pragma unroll
  for (int s = 0; s < C::DX - 1; ++s) issue_x(s);
#pragma unroll
  for (int s = 0; s < C::DW - 1; ++s) issue_w(s);

  for (int kb = 0; kb < nkb; ++kb) {
    if (kb < (C::DW > C::DX ? C::DW : C::DX)) {
      wait_vm<0>();  // (the prologue's order differs from the steady state's)
    } else if (cx == 2) {
      wait_vm<C::wait_count(2)>();
    } else if (cx == 1) {
      wait_vm<C::wait_count(1)>();
    } else {
      wait_vm<C::wait_count(0)>();
    }
    __syncthreads();  // every wave's part of X(kb) has landed; everybody is done with step kb - 1
    issue_x(kb + C::DX - 1);
    issue_w(kb + C::DW - 1);
    const unsigned xa = (unsigned)(C::X_BASE + (kb % C::DX) * C::X_STEP) + rd;
    const unsigned wa = w_ring + (unsigned)((kb % C::DW) * C::W_STEP) + rd;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const unsigned pc = ((unsigned)(2 * j + h) ^ key) << 4;
      bf16x8 a[NBW];
#pragma unroll
      for (int nb = 0; nb < NBW; ++nb) a[nb] = lds_read16(wa + (unsigned)(nb * 2048) + pc);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const bf16x8 b = lds_read16(xa + (unsigned)(mb * 2048) + pc);
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
          acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[nb], b, acc[nb][mb], 0, 0, 0);
      }
    }
  }
  wait_vm<0>();  // the redundant transfers of the last steps must not outlive the workgroup's LDS

  // epilogue: lane (r, h) holds, for output row mb*32 + r, columns block + 8 q + 4 h + (0..3)
  const bool vec_ok = (p.ldy & 3) == 0 && (reinterpret_cast<size_t>(p.y) & 15) == 0;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int m = mb * 32 + r;
    if (m >= p.m) continue;
    float* yrow = p.y + (long long)m * p.ldy;
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n_base + 32 * nb + 8 * q + 4 * h;
        if (vec_ok && n + 3 < p.n) {
          *reinterpret_cast<floatx4*>(yrow + n) = floatx4{acc[nb][mb][4 * q], acc[nb][mb][4 * q + 1],
                                                          acc[nb][mb][4 * q + 2], acc[nb][mb][4 * q + 3]};
        } else {
#pragma unroll
          for (int t = 0; t < 4; ++t)
            if (n + t < p.n) yrow[n + t] = acc[nb][mb][4 * q + t];
        }
      }
  }
}

template <int MB>
hipError_t launch_gemm_mb(const GemmParams& p, hipStream_t stream) {
  static LdsLimitRaised raised;
  if (hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(skinny_gemm_kernel<MB>), GemmCfg<MB>::SMEM, raised);
      e != hipSuccess)
    return e;
  const unsigned grid = (unsigned)((p.n + GemmCfg<MB>::STRIP - 1) / GemmCfg<MB>::STRIP);
  hipLaunchKernelGGL(skinny_gemm_kernel<MB>, dim3(grid, (unsigned)(p.batch * (p.w2 ? 2 : 1)), (unsigned)p.ksplit), dim3(kGemmThreads),
                     GemmCfg<MB>::SMEM, stream, p);
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
// A row (a vocabulary of 10^5 entries) is cut into parts of at most 8 192 entries so that the
// work spreads over all CUs:
//   row_parts_kernel   per (row, part): maximum, sum of exp((x - max) / T), the part's k best
//   row_finish_kernel  per (row, part): the row's maximum and normaliser from the parts' pairs (every
//                      workgroup for itself), q = exp((x - max) / T) / Z of the part (if asked for);
//                      a row's first workgroup: the k best of the parts' candidates, their probabilities
constexpr int kPartThreads = 256;
constexpr int kPartPerThread = 32;                             // entries a thread holds in registers
constexpr int kPartMax = kPartThreads * kPartPerThread;        // 8 192
constexpr int kMaxTopK = 16;

struct SoftParams {
  const float* logits;  // [n_rows][vocab]
  float* probs;         // [n_rows][vocab] or nullptr
  int* tk_ids;          // [n_rows][k]
  float* tk_probs;      // [n_rows][k]
  float* part_ms;       // [n_rows][parts][2]   max, sum
  float* part_cv;       // [n_rows][parts][k]   candidate values
  int* part_ci;         // [n_rows][parts][k]   candidate ids (INT_MAX: none)
  int n_rows, vocab, k, parts, part_len;  // part_len: entries per part, a multiple of 4
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
// the same order without short-circuit evaluation: both operands are always read, so that a
// counting loop over LDS stays free of branches and its reads can be batched
__device__ __forceinline__ int beats(float av, int ai, float bv, int bi) {
  return (int)(av > bv) | ((int)(av == bv) & (int)(ai < bi));
}

__device__ __forceinline__ Best wave_best(float v, int id) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(v, o);
    const int oi = __shfl_xor(id, o);
    if (better(ov, oi, v, id)) {
      v = ov;
      id = oi;
    }
  }
  return Best{v, id};
}

constexpr int kCandCap = 512;

// best (value, id) pair of a 4-wave workgroup, for every thread.  `buf` alternates between
// consecutive calls, so that one barrier per call is enough.
__device__ __forceinline__ Best block_best4(float v, int id, float (*sv)[4], int (*si)[4], int buf) {
  const Best w = wave_best(v, id);
  if ((threadIdx.x & 63) == 0) {
    sv[buf][threadIdx.x >> 6] = w.v;
    si[buf][threadIdx.x >> 6] = w.id;
  }
  __syncthreads();
  Best b{sv[buf][0], si[buf][0]};
#pragma unroll
  for (int i = 1; i < 4; ++i)
    if (better(sv[buf][i], si[buf][i], b.v, b.id)) b = Best{sv[buf][i], si[buf][i]};
  return b;
}

// Top-k of a part: the k-th largest of 64 disjoint groups' maxima is a lower bound of the part's
// k-th largest value, so only entries at or above it can be among the k best; they are put on a
// short list in LDS (few, unless the part is full of ties) and each listed entry finds its place
// by counting the entries that beat it.  A part with more such entries than the list holds
// takes k passes over the registers instead.
__global__ __launch_bounds__(kPartThreads) void row_parts_kernel(SoftParams p) {
  __shared__ float sv[2][4];
  __shared__ int si[2][4];
  __shared__ float sf[4];
  __shared__ float cand_v[kCandCap];
  __shared__ int cand_i[kCandCap];
  __shared__ int n_cand;
  __shared__ float lane_max[kPartThreads];
  __shared__ float s_tau;
  const int tid = threadIdx.x, V = p.vocab, K = p.k;
  const int row = blockIdx.x / p.parts, part = blockIdx.x % p.parts;
  const int lo = part * p.part_len, hi = min(V, lo + p.part_len);
  const float* x = p.logits + (long long)row * V;
  const bool vec = (V & 3) == 0 && (reinterpret_cast<size_t>(p.logits) & 15) == 0;
  if (tid == 0) {
    n_cand = 0;
    s_tau = -INFINITY;
  }

  // entry (u, c) of this thread is vocabulary id lo + 4 (tid + 256 u) + c: ids increase with (u, c)
  auto id_of = [&](int i) { return lo + 4 * (tid + kPartThreads * (i >> 2)) + (i & 3); };
  float val[kPartPerThread];
#pragma unroll
  for (int u = 0; u < kPartPerThread / 4; ++u) {
    const int e = lo + 4 * (tid + kPartThreads * u);
    if (vec && e + 3 < hi) {
      const floatx4 q = *reinterpret_cast<const floatx4*>(x + e);
#pragma unroll
      for (int c = 0; c < 4; ++c) val[4 * u + c] = q[c];
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) val[4 * u + c] = e + c < hi ? x[e + c] : -INFINITY;
    }
  }
  // the thread's own maximum
  float tv = -INFINITY;
#pragma unroll
  for (int i = 0; i < kPartPerThread; ++i) tv = fmaxf(tv, val[i]);
  float m = tv;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  if ((tid & 63) == 0) sf[tid >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(sf[0], sf[1]), fmaxf(sf[2], sf[3]));
  const float m_use = m > -INFINITY ? m : 0.f;  // a part of -inf only: nothing sensible to subtract
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kPartPerThread; ++i) s += expf((val[i] - m_use) * p.inv_temp);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
  __syncthreads();
  if ((tid & 63) == 0) sf[tid >> 6] = s;
  __syncthreads();
  const long long slot = (long long)row * p.parts + part;
  if (tid == 0) {
    p.part_ms[2 * slot] = m;
    p.part_ms[2 * slot + 1] = (sf[0] + sf[1]) + (sf[2] + sf[3]);
  }

  // threshold: the k-th largest of the 64 per-lane maxima (maximum over the four waves of the
  // threads' own maxima), found by ranking: no rounds, no reductions
  lane_max[tid] = tv;
  __syncthreads();
  if (tid < 64) {
    const float v = fmaxf(fmaxf(lane_max[tid], lane_max[tid + 64]), fmaxf(lane_max[tid + 128], lane_max[tid + 192]));
    lane_max[tid] = v;  // (wave 0 only reads and writes its own column here)
  }
  __syncthreads();
  if (tid < 64) {
    const float mine = lane_max[tid];
    int rank = 0;
#pragma unroll 8
    for (int j = 0; j < 64; ++j) {
      rank += beats(lane_max[j], j, mine, tid);
    }
    if (rank == K - 1) s_tau = mine;
  }
  __syncthreads();
  const float tau = s_tau;
#pragma unroll
  for (int i = 0; i < kPartPerThread; ++i)
    if (val[i] >= tau && id_of(i) < hi) {
      const int at = atomicAdd(&n_cand, 1);
      if (at < kCandCap) {
        cand_v[at] = val[i];
        cand_i[at] = id_of(i);
      }
    }
  __syncthreads();
  const int nc = n_cand;
  int round_no = 0;
  if (nc <= kCandCap) {
    // rank every listed entry among the list; ranks below k are the winners' places
    if (tid < K && tid >= nc) {  // (a part with fewer than k entries)
      p.part_cv[slot * K + tid] = -INFINITY;
      p.part_ci[slot * K + tid] = INT_MAX;
    }
    for (int j = tid; j < nc; j += kPartThreads) {
      const float v = cand_v[j];
      const int id = cand_i[j];
      int rank = 0;
#pragma unroll 8
      for (int i = 0; i < nc; ++i) rank += beats(cand_v[i], cand_i[i], v, id);
      if (rank < K) {
        p.part_cv[slot * K + rank] = v;
        p.part_ci[slot * K + rank] = id;
      }
    }
  } else {
    // one winner per pass: every thread offers its best entry that comes after the previous
    // winner in the candidate order
    float pv = INFINITY;
    int pi = -1;
    for (int round = 0; round < K; ++round) {
      float bv = -INFINITY;
      int bi = INT_MAX;
#pragma unroll
      for (int i = 0; i < kPartPerThread; ++i) {
        const int id = id_of(i);
        const float v = val[i];
        const bool after = v < pv || (v == pv && id > pi);
        // ids increase with i, so among equal values the first one seen is the one to keep
        if (after && id < hi && v > bv) {
          bv = v;
          bi = id;
        }
      }
      const Best b = block_best4(bv, bi, sv, si, (round_no++) & 1);
      if (tid == 0) {
        p.part_cv[slot * K + round] = b.v;
        p.part_ci[slot * K + round] = b.id;
      }
      pv = b.v;
      pi = b.id;  // INT_MAX once the part is exhausted: nothing comes after it
    }
  }
}

// The row's maximum and 1 / normaliser from the parts' (max, sum) pairs: every wave of every workgroup that
// needs them reduces the pairs for itself, the same operations in the same order everywhere.
__device__ __forceinline__ void row_max_and_norm(const SoftParams& p, int row, float& m_use, float& inv_z) {
  const int lane = threadIdx.x & 63, P = p.parts;
  const float* ms = p.part_ms + (long long)row * P * 2;
  float m = -INFINITY;
  for (int i = lane; i < P; i += 64) m = fmaxf(m, ms[2 * i]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  m_use = m > -INFINITY ? m : 0.f;
  double z = 0.0;
  for (int i = lane; i < P; i += 64) {
    const float mp = ms[2 * i];
    if (mp > -INFINITY) z += (double)ms[2 * i + 1] * (double)expf((mp - m_use) * p.inv_temp);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) z += __shfl_xor(z, o);
  inv_z = (float)(1.0 / z);
}

// the k best of the parts' candidates and their probabilities (one workgroup of four waves per row)
__device__ __forceinline__ void row_top_k(const SoftParams& p, int row, float m_use, float inv_z) {
  const int tid = threadIdx.x, lane = tid & 63, K = p.k, P = p.parts;
  const float* cv = p.part_cv + (long long)row * P * K;
  const int* ci = p.part_ci + (long long)row * P * K;
  const int n = P * K;
  if (n <= 1024) {  // the usual case: every candidate finds its place by counting those that beat it
    __shared__ float mv[1024];
    __shared__ int mi[1024];
    for (int i = tid; i < n; i += 256) {
      mv[i] = cv[i];
      mi[i] = ci[i];
    }
    // places that no candidate claims (fewer than k candidates in the whole row) read "none";
    // the barrier orders these stores before the winners'
    if (tid < K) {
      p.tk_ids[(long long)row * K + tid] = 0;
      p.tk_probs[(long long)row * K + tid] = 0.f;
    }
    __syncthreads();
    for (int j = tid; j < n; j += 256) {
      const float v = mv[j];
      const int id = mi[j];
      if (id < 0 || id >= p.vocab) continue;  // an exhausted part's filler
      int rank = 0;
#pragma unroll 8
      for (int i = 0; i < n; ++i) rank += beats(mv[i], mi[i], v, id);
      if (rank < K) {
        p.tk_ids[(long long)row * K + rank] = id;
        p.tk_probs[(long long)row * K + rank] = expf((v - m_use) * p.inv_temp) * inv_z;
      }
    }
    return;
  }
  if (tid >= 64) return;  // very many parts: one wave, k selection passes over the candidates in memory
  float pv = INFINITY;
  int pi = -1;
  for (int round = 0; round < K; ++round) {
    float bv = -INFINITY;
    int bi = INT_MAX;
    for (int i = lane; i < n; i += 64) {
      const float v = cv[i];
      const int id = ci[i];
      const bool after = v < pv || (v == pv && id > pi);
      if (after && better(v, id, bv, bi)) {
        bv = v;
        bi = id;
      }
    }
    const Best b = wave_best(bv, bi);
    if (lane == 0) {
      const bool ok = b.id >= 0 && b.id < p.vocab;
      p.tk_ids[(long long)row * K + round] = ok ? b.id : 0;
      p.tk_probs[(long long)row * K + round] = ok ? expf((b.v - m_use) * p.inv_temp) * inv_z : 0.f;
    }
    pv = b.v;
    pi = b.id;
  }
}

// One workgroup per (row, part): q = exp((x - max) / T) / Z for the part (if the distributions are asked for:
// otherwise one workgroup per row); the workgroup of a row's first part also merges the parts' candidates
// into the row's k best.  One launch where a merge kernel and a probabilities kernel used to follow each other.
__global__ __launch_bounds__(kPartThreads) void row_finish_kernel(SoftParams p) {
  const int tid = threadIdx.x, V = p.vocab;
  const bool with_probs = p.probs != nullptr;
  const int row = with_probs ? blockIdx.x / p.parts : blockIdx.x, part = with_probs ? blockIdx.x % p.parts : 0;
  float m, inv_z;
  row_max_and_norm(p, row, m, inv_z);
  if (with_probs) {
    const int lo = part * p.part_len, hi = min(V, lo + p.part_len);
    const float* x = p.logits + (long long)row * V;
    float* q = p.probs + (long long)row * V;
    const bool vec = (V & 3) == 0 && (reinterpret_cast<size_t>(p.logits) & 15) == 0 &&
                     (reinterpret_cast<size_t>(p.probs) & 15) == 0;
#pragma unroll 4
    for (int u = 0; u < kPartPerThread / 4; ++u) {
      const int e = lo + 4 * (tid + kPartThreads * u);
      if (vec && e + 3 < hi) {
        const floatx4 s = *reinterpret_cast<const floatx4*>(x + e);
        floatx4 o;
#pragma unroll
        for (int c = 0; c < 4; ++c) o[c] = expf((s[c] - m) * p.inv_temp) * inv_z;
        *reinterpret_cast<floatx4*>(q + e) = o;
      } else {
        for (int c = 0; c < 4; ++c)
          if (e + c < hi) q[e + c] = expf((x[e + c] - m) * p.inv_temp) * inv_z;
      }
    }
  }
  if (part == 0) row_top_k(p, row, m, inv_z);
}

// ------------------------------------------------------------------ router and experts (Eq. 2, 3, 5)
constexpr int kMaxExperts = 64;

struct RouterParams {
  const uint16_t* u;          // [rows][d] bf16
  const uint16_t* centroids;  // [n_experts][d] bf16
  uint16_t* x;                // [rows padded to 32][d] bf16: copy of u, zero rows behind it
  float* s_top;               // [rows][2]
  int* idx;                   // [rows][2]
  int rows, d, n_experts;
};

// One workgroup per (padded) row: copies the row into the GEMM's padded input, and for real rows
// computes the router scores s_j = softmax_j(u . e_j) (Eq. 2; fp32), picks the two largest (Eq. 5,
// K = 2, ties to the lower expert).
__global__ __launch_bounds__(256) void router_kernel(RouterParams p) {
  __shared__ float score[kMaxExperts];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  u32x4* dst = reinterpret_cast<u32x4*>(p.x + (long long)row * p.d);
  if (row >= p.rows) {
    for (int c = tid; c < p.d / 8; c += 256) dst[c] = u32x4{0u, 0u, 0u, 0u};
    return;
  }
  const u32x4* src = reinterpret_cast<const u32x4*>(p.u + (long long)row * p.d);
  for (int c = tid; c < p.d / 8; c += 256) dst[c] = src[c];
  for (int j0 = wave; j0 < p.n_experts; j0 += 8) {  // two experts per pass: their loads share the trip to memory
    const bool two = j0 + 4 < p.n_experts;
    const u32x4* e0 = reinterpret_cast<const u32x4*>(p.centroids + (long long)j0 * p.d);
    const u32x4* e1 = reinterpret_cast<const u32x4*>(p.centroids + (long long)(two ? j0 + 4 : j0) * p.d);
    float acc0 = 0.f, acc1 = 0.f;
#pragma unroll 4
    for (int c = lane; c < p.d / 8; c += 64) {
      const u32x4 a = src[c], b0 = e0[c], b1 = e1[c];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc0 += bf16_lo(a[i]) * bf16_lo(b0[i]) + bf16_hi(a[i]) * bf16_hi(b0[i]);
        acc1 += bf16_lo(a[i]) * bf16_lo(b1[i]) + bf16_hi(a[i]) * bf16_hi(b1[i]);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      acc0 += __shfl_xor(acc0, o);
      acc1 += __shfl_xor(acc1, o);
    }
    if (lane == 0) {
      score[j0] = acc0;
      if (two) score[j0 + 4] = acc1;
    }
  }
  __syncthreads();
  if (tid == 0) {
    float m = -INFINITY;
    for (int j = 0; j < p.n_experts; ++j) m = fmaxf(m, score[j]);
    float z = 0.f;
    for (int j = 0; j < p.n_experts; ++j) z += expf(score[j] - m);
    int i1 = 0;
    for (int j = 1; j < p.n_experts; ++j)
      if (score[j] > score[i1]) i1 = j;
    int i2 = i1 == 0 ? 1 : 0;
    for (int j = 0; j < p.n_experts; ++j)
      if (j != i1 && score[j] > score[i2]) i2 = j;
    p.s_top[2 * row] = expf(score[i1] - m) / z;
    p.s_top[2 * row + 1] = expf(score[i2] - m) / z;
    p.idx[2 * row] = i1;
    p.idx[2 * row + 1] = i2;
  }
}

struct ActParams {
  const float *g, *up;  // [ksplit][n_experts][rows][f] fp32: partial gate and up projections
  uint16_t* h;          // [n_experts][rows padded to 32][f] bf16
  const int* sel;  // [2 rows]: the experts the rows selected
  int rows, rows_pad, f, ksplit;
  long long split_stride;
};

// h = silu(gate) * up, rounded to bf16 once; padding rows are zero-filled
__global__ __launch_bounds__(256) void gated_act_kernel(ActParams p) {
  const int e = blockIdx.y, row = blockIdx.x;
  {
    int mine = 0;
    for (int i = threadIdx.x & 63; i < 2 * p.rows; i += 64) mine |= (int)(p.sel[i] == e);
    if (!__any(mine)) return;  // nobody selected this expert (every wave finds the same)
  }
  uint16_t* h = p.h + ((long long)e * p.rows_pad + row) * p.f;
  if (row >= p.rows) {
    for (int c = threadIdx.x; c < p.f / 8; c += 256) reinterpret_cast<u32x4*>(h)[c] = u32x4{0u, 0u, 0u, 0u};
    return;
  }
  const float* g = p.g + ((long long)e * p.rows + row) * p.f;
  const float* up = p.up + ((long long)e * p.rows + row) * p.f;
  for (int c = threadIdx.x; c < p.f / 4; c += 256) {
    floatx4 a = reinterpret_cast<const floatx4*>(g)[c], b = reinterpret_cast<const floatx4*>(up)[c];
    for (int z = 1; z < p.ksplit; ++z) {
      a += reinterpret_cast<const floatx4*>(g + z * p.split_stride)[c];
      b += reinterpret_cast<const floatx4*>(up + z * p.split_stride)[c];
    }
    float o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = a[i] / (1.f + expf(-a[i])) * b[i];
    uint2 w;
    w.x = bf16_bits_rne(o[0]) | (bf16_bits_rne(o[1]) << 16);
    w.y = bf16_bits_rne(o[2]) | (bf16_bits_rne(o[3]) << 16);
    reinterpret_cast<uint2*>(h)[c] = w;
  }
}

struct SelectParams {
  int ksplit;
  long long split_stride;
  const float* y;     // [ksplit][n_experts][rows][d] fp32: the experts' (partial) outputs
  const uint16_t* u;  // [rows][d] bf16
  const float* s_top;
  const int* idx;
  uint16_t* f_top;    // [rows][2][d] bf16
  uint16_t* f_mix;    // [rows][d] bf16 or null
  int rows, d;
};

// f_top[r][k] = Expert_{idx[r][k]}(u_r) + u_r; f_mix[r] = sum_k s_k Expert_k(u_r) + u_r (Eq. 3)
__global__ __launch_bounds__(256) void select_kernel(SelectParams p) {
  const int row = blockIdx.x;
  const int i1 = p.idx[2 * row], i2 = p.idx[2 * row + 1];
  const float s1 = p.s_top[2 * row], s2 = p.s_top[2 * row + 1];
  const float* y1 = p.y + ((long long)i1 * p.rows + row) * p.d;
  const float* y2 = p.y + ((long long)i2 * p.rows + row) * p.d;
  const uint16_t* u = p.u + (long long)row * p.d;
  for (int c = blockIdx.y * 256 + threadIdx.x; c < p.d / 2; c += 256 * gridDim.y) {
    const unsigned uu = reinterpret_cast<const unsigned*>(u)[c];
    const float u0 = bf16_lo(uu), u1 = bf16_hi(uu);
    float2 a = reinterpret_cast<const float2*>(y1)[c], b = reinterpret_cast<const float2*>(y2)[c];
    for (int z = 1; z < p.ksplit; ++z) {
      const float2 az = reinterpret_cast<const float2*>(y1 + z * p.split_stride)[c];
      const float2 bz = reinterpret_cast<const float2*>(y2 + z * p.split_stride)[c];
      a.x += az.x; a.y += az.y;
      b.x += bz.x; b.y += bz.y;
    }
    reinterpret_cast<unsigned*>(p.f_top + ((long long)row * 2 + 0) * p.d)[c] =
        bf16_bits_rne(a.x + u0) | (bf16_bits_rne(a.y + u1) << 16);
    reinterpret_cast<unsigned*>(p.f_top + ((long long)row * 2 + 1) * p.d)[c] =
        bf16_bits_rne(b.x + u0) | (bf16_bits_rne(b.y + u1) << 16);
    if (p.f_mix)
      reinterpret_cast<unsigned*>(p.f_mix + (long long)row * p.d)[c] =
          bf16_bits_rne(s1 * a.x + s2 * b.x + u0) | (bf16_bits_rne(s1 * a.y + s2 * b.y + u1) << 16);
  }
}

struct MoePlan {
  int rows_pad, split1, split2;
  size_t x_off, g_off, up_off, h_off, y_off, total;
};
// k parts so that a projection with few output columns still fills the chip: a workgroup can
// pull only a fixed share of the memory bandwidth, so the weight stream needs about one
// workgroup per CU.  A part keeps at least 512 of k and a multiple of 128.
int pick_ksplit(int n_out, int k, int mb, int batch, int cus) {
  const int strip = mb <= 6 ? 512 : 256;
  const long long wgs = (long long)((n_out + strip - 1) / strip) * batch;
  int best = 1;
  for (int s = 2; s <= 8; ++s) {
    if (k % (128 * s) != 0 || k / s < 512) continue;
    if (wgs * s <= (long long)cus + cus / 8) best = s;
  }
  return best;
}
MoePlan moe_plan(int rows, int d, int f, int n) {
  MoePlan m;
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  m.rows_pad = (rows + 31) / 32 * 32;
  const int cus = device_cu_count();
  m.split1 = pick_ksplit(f, d, m.rows_pad / 32, 2 * n, cus);  // gate and up in one launch
  m.split2 = pick_ksplit(d, f, m.rows_pad / 32, n, cus);
  m.x_off = 0;
  m.g_off = up((size_t)m.rows_pad * d * 2);
  m.up_off = m.g_off + up((size_t)m.split1 * n * rows * f * 4);
  m.h_off = m.up_off + up((size_t)m.split1 * n * rows * f * 4);
  m.y_off = m.h_off + up((size_t)n * m.rows_pad * f * 2);
  m.total = m.y_off + up((size_t)m.split2 * n * rows * d * 4);
  return m;
}


// ------------------------------------------------------------------ plain linear layer
struct LinFinishParams {
  const float* part;        // [ksplit][m*n]
  const uint16_t* residual; // [m*n] bf16 or null
  float* out_f32;           // or null
  uint16_t* out_bf16;       // or null
  long long n_out;
  int ksplit;
};
__global__ __launch_bounds__(256) void linear_finish_kernel(LinFinishParams p) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < p.n_out; i += (long long)gridDim.x * 256) {
    float v = p.part[i];
    for (int z = 1; z < p.ksplit; ++z) v += p.part[i + z * p.n_out];
    if (p.residual) v += __uint_as_float((unsigned)p.residual[i] << 16);
    if (p.out_f32) p.out_f32[i] = v;
    if (p.out_bf16) p.out_bf16[i] = (uint16_t)bf16_bits_rne(v);
  }
}

int linear_ksplit(int m, int n, int k) {
  int s = pick_ksplit(n, k, (m + 31) / 32, 1, device_cu_count());
  while (s > 1 && (size_t)s * m * n * 4 > ((size_t)64 << 20)) --s;
  while (s > 1 && (k % (128 * s) != 0 || k / s < 512)) --s;
  return s;
}

struct RowPlan {
  int parts, part_len, ksplit;
  size_t x_bytes, ms_off, cv_off, ci_off, part_off, total;
};

// logits = sum of the k parts' partial products (fixed order)
__global__ __launch_bounds__(256) void sum_parts_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                        long long n, int ksplit) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
    float v = part[i];
    for (int z = 1; z < ksplit; ++z) v += part[i + z * n];
    out[i] = v;
  }
}
RowPlan row_plan(int rows, int d_model, int vocab) {
  RowPlan r;
  const size_t m = 2 * (size_t)rows, m_pad = (m + 31) / 32 * 32;
  r.parts = (vocab + kPartMax - 1) / kPartMax;
  r.part_len = ((vocab + r.parts - 1) / r.parts + 3) / 4 * 4;
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  r.x_bytes = up(m_pad * (size_t)d_model * 2);
  r.ms_off = r.x_bytes;
  r.cv_off = r.ms_off + up(m * r.parts * 2 * 4);
  r.ci_off = r.cv_off + up(m * r.parts * kMaxTopK * 4);
  r.part_off = r.ci_off + up(m * r.parts * kMaxTopK * 4);
  // a small vocabulary gives few 512-row strips: split k until the chip is full (partials of at most 64 MB)
  r.ksplit = pick_ksplit(vocab, d_model, (int)(m_pad / 32), 1, device_cu_count());
  while (r.ksplit > 1 && (size_t)r.ksplit * m * vocab * 4 > ((size_t)64 << 20)) --r.ksplit;
  while (r.ksplit > 1 && (d_model % (128 * r.ksplit) != 0 || d_model / r.ksplit < 512)) --r.ksplit;
  r.total = r.part_off + (r.ksplit > 1 ? up((size_t)r.ksplit * m * vocab * 4) : 0);
  return r;
}

}  // namespace

size_t draft_heads_workspace_bytes(int rows, int d_model, int vocab) { return row_plan(rows, d_model, vocab).total; }

hipError_t launch_draft_heads(const DraftHeadsArgs& a, hipStream_t stream) {
  const int m = 2 * a.rows, m_pad = (m + 31) / 32 * 32;
  const RowPlan rp = row_plan(a.rows, a.d_model, a.vocab);
  char* ws = static_cast<char*>(a.workspace);
  MixParams mp;
  mp.f_top = static_cast<const unsigned short*>(a.f_top);
  mp.s_top = a.s_top;
  mp.x = reinterpret_cast<unsigned short*>(ws);
  mp.rows = a.rows; mp.d = a.d_model; mp.mode = a.mode; mp.alpha = a.alpha; mp.beta = a.beta;
  hipLaunchKernelGGL(head_inputs_kernel, dim3(m_pad), dim3(256), 0, stream, mp);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  GemmParams gp;
  gp.x = reinterpret_cast<const uint16_t*>(ws);
  gp.w = static_cast<const uint16_t*>(a.w_head);
  gp.y = a.logits;
  gp.m = m; gp.n = a.vocab; gp.k = a.d_model;
  gp.ldw = a.d_model; gp.ldy = a.vocab;
  gp.batch = 1; gp.x_batch = gp.w_batch = gp.y_batch = 0; gp.sel = nullptr; gp.n_sel = 0; gp.w2 = nullptr; gp.y2 = nullptr;
  gp.ksplit = rp.ksplit; gp.y_split = (long long)m * a.vocab;
  if (rp.ksplit > 1) gp.y = reinterpret_cast<float*>(ws + rp.part_off);
  e = launch_gemm(gp, stream);
  if (e != hipSuccess) return e;
  if (rp.ksplit > 1) {
    const long long n_out = (long long)m * a.vocab;
    const unsigned grid = (unsigned)((n_out + 1023) / 1024 < 2048 ? (n_out + 1023) / 1024 : 2048);
    hipLaunchKernelGGL(sum_parts_kernel, dim3(grid), dim3(256), 0, stream, gp.y, a.logits, n_out, rp.ksplit);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }

  SoftParams sp;
  sp.logits = a.logits; sp.probs = a.draft_probs; sp.tk_ids = a.topk_tokens; sp.tk_probs = a.topk_probs;
  sp.part_ms = reinterpret_cast<float*>(ws + rp.ms_off);
  sp.part_cv = reinterpret_cast<float*>(ws + rp.cv_off);
  sp.part_ci = reinterpret_cast<int*>(ws + rp.ci_off);
  sp.n_rows = m; sp.vocab = a.vocab; sp.k = a.top_k; sp.parts = rp.parts; sp.part_len = rp.part_len;
  sp.inv_temp = 1.0f / a.temperature;
  hipLaunchKernelGGL(row_parts_kernel, dim3(m * rp.parts), dim3(kPartThreads), 0, stream, sp);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(row_finish_kernel, dim3(a.draft_probs ? m * rp.parts : m), dim3(kPartThreads), 0, stream, sp);
  return hipGetLastError();
}

size_t moe_experts_workspace_bytes(int rows, int d_model, int d_ff, int n_experts) {
  return moe_plan(rows, d_model, d_ff, n_experts).total;
}

hipError_t launch_moe_experts(const MoeArgs& a, hipStream_t stream) {
  const MoePlan mp = moe_plan(a.rows, a.d_model, a.d_ff, a.n_experts);
  char* ws = static_cast<char*>(a.workspace);
  hipError_t e;
  RouterParams rp;
  rp.u = static_cast<const uint16_t*>(a.u); rp.centroids = static_cast<const uint16_t*>(a.centroids);
  rp.x = reinterpret_cast<uint16_t*>(ws + mp.x_off);
  rp.s_top = a.s_top; rp.idx = a.expert_idx;
  rp.rows = a.rows; rp.d = a.d_model; rp.n_experts = a.n_experts;
  hipLaunchKernelGGL(router_kernel, dim3(mp.rows_pad), dim3(256), 0, stream, rp);
  if ((e = hipGetLastError()) != hipSuccess) return e;

  GemmParams gp;
  gp.x = rp.x; gp.m = a.rows; gp.n = a.d_ff; gp.k = a.d_model; gp.ldw = a.d_model; gp.ldy = a.d_ff;
  gp.batch = a.n_experts; gp.x_batch = 0; gp.w_batch = (long long)a.d_ff * a.d_model;
  gp.y_batch = (long long)a.rows * a.d_ff; gp.sel = a.expert_idx; gp.n_sel = 2 * a.rows;
  gp.ksplit = mp.split1; gp.y_split = (long long)a.n_experts * a.rows * a.d_ff;
  gp.w = static_cast<const uint16_t*>(a.w_gate); gp.y = reinterpret_cast<float*>(ws + mp.g_off);
  gp.w2 = static_cast<const uint16_t*>(a.w_up); gp.y2 = reinterpret_cast<float*>(ws + mp.up_off);
  if ((e = launch_gemm(gp, stream)) != hipSuccess) return e;  // gate and up projections of all experts
  gp.w2 = nullptr; gp.y2 = nullptr;

  ActParams ap;
  ap.g = reinterpret_cast<const float*>(ws + mp.g_off); ap.up = reinterpret_cast<const float*>(ws + mp.up_off);
  ap.h = reinterpret_cast<uint16_t*>(ws + mp.h_off); ap.sel = a.expert_idx;
  ap.rows = a.rows; ap.rows_pad = mp.rows_pad; ap.f = a.d_ff;
  ap.ksplit = mp.split1; ap.split_stride = gp.y_split;
  hipLaunchKernelGGL(gated_act_kernel, dim3(mp.rows_pad, a.n_experts), dim3(256), 0, stream, ap);
  if ((e = hipGetLastError()) != hipSuccess) return e;

  gp.x = ap.h; gp.m = a.rows; gp.n = a.d_model; gp.k = a.d_ff; gp.ldw = a.d_ff; gp.ldy = a.d_model;
  gp.x_batch = (long long)mp.rows_pad * a.d_ff; gp.w_batch = (long long)a.d_model * a.d_ff;
  gp.y_batch = (long long)a.rows * a.d_model;
  gp.ksplit = mp.split2; gp.y_split = (long long)a.n_experts * a.rows * a.d_model;
  gp.w = static_cast<const uint16_t*>(a.w_down); gp.y = reinterpret_cast<float*>(ws + mp.y_off);
  if ((e = launch_gemm(gp, stream)) != hipSuccess) return e;

  SelectParams sp;
  sp.y = reinterpret_cast<const float*>(ws + mp.y_off); sp.u = rp.u; sp.s_top = a.s_top; sp.idx = a.expert_idx;
  sp.f_top = static_cast<uint16_t*>(a.f_top); sp.f_mix = static_cast<uint16_t*>(a.f_mix);
  sp.rows = a.rows; sp.d = a.d_model;
  sp.ksplit = mp.split2; sp.split_stride = gp.y_split;
  const unsigned chunks = (unsigned)(a.d_model / 512 < 8 ? (a.d_model / 512 > 0 ? a.d_model / 512 : 1) : 8);
  hipLaunchKernelGGL(select_kernel, dim3(a.rows, chunks), dim3(256), 0, stream, sp);
  return hipGetLastError();
}

size_t linear_workspace_bytes(int m, int n, int k) {
  return ((size_t)linear_ksplit(m, n, k) * m * n * 4 + 255) / 256 * 256;
}

hipError_t launch_linear(const LinearArgs& a, hipStream_t stream) {
  const int ks = linear_ksplit(a.m, a.n, a.k);
  const bool direct = ks == 1 && !a.residual && !a.out_bf16 && a.out_f32;
  GemmParams gp;
  gp.x = static_cast<const uint16_t*>(a.x); gp.w = static_cast<const uint16_t*>(a.w);
  gp.y = direct ? a.out_f32 : static_cast<float*>(a.workspace);
  gp.m = a.m; gp.n = a.n; gp.k = a.k; gp.ldw = a.k; gp.ldy = a.n;
  gp.batch = 1; gp.x_batch = gp.w_batch = gp.y_batch = 0; gp.sel = nullptr; gp.n_sel = 0; gp.w2 = nullptr; gp.y2 = nullptr;
  gp.ksplit = ks; gp.y_split = (long long)a.m * a.n;
  hipError_t e = launch_gemm(gp, stream);
  if (e != hipSuccess || direct) return e;
  LinFinishParams fp;
  fp.part = gp.y; fp.residual = static_cast<const uint16_t*>(a.residual); fp.out_f32 = a.out_f32;
  fp.out_bf16 = static_cast<uint16_t*>(a.out_bf16); fp.n_out = (long long)a.m * a.n; fp.ksplit = ks;
  const unsigned grid = (unsigned)((fp.n_out + 1023) / 1024 < 2048 ? (fp.n_out + 1023) / 1024 : 2048);
  hipLaunchKernelGGL(linear_finish_kernel, dim3(grid), dim3(256), 0, stream, fp);
  return hipGetLastError();
}

}  // namespace jk
