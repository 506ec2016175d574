// Token acceptance over the verified draft tree (gfx950).
//
// Section 2.1 of the paper: candidates are judged in order with acceptance
// probability min(1, p/q); at a rejection the distribution becomes
// norm(max(0, p - q)) (steps 2-3).  Section 3.2: greedy decoding is strict
// top-1 verification.  On a tree the rule is applied sibling by sibling, left
// to right (Section 3.1.2 puts the higher-scoring expert's candidates on the
// left), each node carrying its own draft distribution.
//
// Kernels
//   row_reduce_kernel   one pass over the [rows, vocab] logits: per (row,
//                       chunk) either (max, argmax) or (max, sum exp) partials
//   walk_greedy_kernel  one workgroup per tree: merges the partials per row,
//                       marks every node whose token equals its parent row's
//                       argmax, then descends from the prefix
//   walk_sample_kernel  one workgroup per tree: descends from the prefix; a
//                       rejection costs one pass over the vocabulary that
//                       writes the unnormalised residual to the workspace and
//                       reduces its sum; the bonus token is found by a blocked
//                       prefix sum over the final distribution.  All sampling
//                       arithmetic is fp64: the inverse-CDF draw resolves steps
//                       of ~1/vocab, which fp32 terms cannot do reproducibly
#include <cstdlib>
#include <mutex>

#include "jk_internal.h"

namespace jk {
namespace {

constexpr int kChunk = 4096;        // vocabulary entries per row_reduce workgroup
constexpr int kWalkThreads = 1024;  // threads of a sampling walk

__host__ __device__ inline int n_chunks(int vocab) { return (vocab + kChunk - 1) / kChunk; }

// ------------------------------------------------------------------ row reductions
template <bool SAMPLE>
__global__ __launch_bounds__(256) void row_reduce_kernel(const float* __restrict__ logits, int vocab,
                                                         double temp, float* __restrict__ pmax,
                                                         int* __restrict__ pidx, double* __restrict__ psum) {
  __shared__ float s_max[4];
  __shared__ int s_idx[4];
  __shared__ double s_sum[4];
  const int chunk = blockIdx.x;
  const long long row = blockIdx.y;
  const float* src = logits + row * vocab;
  const int v0 = chunk * kChunk;
  const int v1 = min(vocab, v0 + kChunk);
  const int tid = threadIdx.x;

  float vals[16];
  float best = -INFINITY;
  int bidx = 0x7fffffff;
  const bool vec = ((vocab & 3) == 0);  // rows stay 16-byte aligned
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int v = v0 + (j * 256 + tid) * 4;
    if (vec && v + 3 < v1) {
      const float4 x = *reinterpret_cast<const float4*>(src + v);
      vals[4 * j] = x.x; vals[4 * j + 1] = x.y; vals[4 * j + 2] = x.z; vals[4 * j + 3] = x.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) vals[4 * j + e] = (v + e < v1) ? src[v + e] : -INFINITY;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float x = vals[4 * j + e];
      if (x > best) { best = x; bidx = v + e; }  // ascending v inside a thread keeps the lowest id
    }
  }
  // block (max, lowest index of the max)
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o);
    const int oi = __shfl_xor(bidx, o);
    if (ob > best || (ob == best && oi < bidx)) { best = ob; bidx = oi; }
  }
  if ((tid & 63) == 0) { s_max[tid >> 6] = best; s_idx[tid >> 6] = bidx; }
  __syncthreads();
  best = s_max[0]; bidx = s_idx[0];
#pragma unroll
  for (int w = 1; w < 4; ++w)
    if (s_max[w] > best || (s_max[w] == best && s_idx[w] < bidx)) { best = s_max[w]; bidx = s_idx[w]; }

  const long long slot = row * gridDim.x + chunk;
  if (!SAMPLE) {
    if (tid == 0) { pmax[slot] = best; pidx[slot] = bidx; }
    return;
  }
  // sum of exp(x/T - max/T) over the chunk, all in fp64 (same operations as the definition,
  // so a decision of the walk differs from exact arithmetic only at ~1e-15 relative)
  const double mref = (best == -INFINITY) ? 0.0 : (double)best / temp;
  double acc = 0.0;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc += exp((double)vals[i] / temp - mref);
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  if ((tid & 63) == 0) s_sum[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) { pmax[slot] = best; psum[slot] = s_sum[0] + s_sum[1] + s_sum[2] + s_sum[3]; }
}

// A parent entry that breaks -1 <= parent[k] < k counts as -1, and a token id outside the vocabulary is
// clamped into it; either is recorded in the workspace's sticky error word (err may be null).
__device__ __forceinline__ void report(unsigned* err, unsigned bit) {
  if (err) __hip_atomic_fetch_or(err, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int sanitize_parent(int pa, int k, unsigned* err) {
  if (pa >= -1 && pa < k) return pa;
  report(err, kDevErrBadTree);
  return -1;
}

// ------------------------------------------------------------------ greedy walk
__global__ __launch_bounds__(128) void walk_greedy_kernel(int n_tree, int nch, int vocab, int max_depth,
                                                          const int* __restrict__ tokens,
                                                          const int* __restrict__ parent,
                                                          const float* __restrict__ pmax,
                                                          const int* __restrict__ pidx, int* __restrict__ out_path,
                                                          int* __restrict__ out_len, int* __restrict__ out_bonus,
                                                          unsigned* err) {
  __shared__ int amax[JK_MAX_TREE + 1];
  __shared__ int par_s[JK_MAX_TREE];
  __shared__ int ok[JK_MAX_TREE];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int rows = n_tree + 1;
  for (int r = tid; r < rows; r += blockDim.x) {
    const long long base = ((long long)b * rows + r) * nch;
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int c0 = 0; c0 < nch; c0 += 8) {  // eight partials in flight at a time
      float v[8];
      int id[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool in = c0 + u < nch;
        v[u] = in ? pmax[base + c0 + u] : -INFINITY;
        id[u] = in ? pidx[base + c0 + u] : 0x7fffffff;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)  // chunks ascend in token id: strict > keeps the lowest id
        if (v[u] > best) { best = v[u]; bi = id[u]; }
    }
    amax[r] = (bi == 0x7fffffff) ? 0 : bi;  // a row of -inf only: id 0, the first maximum
  }
  if (tid < n_tree) par_s[tid] = sanitize_parent(parent[(long long)b * n_tree + tid], tid, err);
  __syncthreads();
  if (tid < n_tree) {
    const int tk = tokens[(long long)b * n_tree + tid];
    const int tc = min(max(tk, 0), vocab - 1);  // as in the sampling walks: an id outside the vocabulary is clamped, and reported
    if (tc != tk) report(err, kDevErrBadToken);
    ok[tid] = (tc == amax[par_s[tid] + 1]);
  }
  __syncthreads();
  if (tid < 64) {  // wave 0 descends: the first accepted child of c, found with two ballots per level
    const int lane = tid;
    const bool in0 = lane < n_tree, in1 = lane + 64 < n_tree;
    const int p0 = in0 ? par_s[lane] : -2, p1 = in1 ? par_s[lane + 64] : -2;
    const bool ok0 = in0 && ok[lane], ok1 = in1 && ok[lane + 64];
    int c = -1, len = 0;
    // (nodes are numbered topologically: a child has a larger index than its parent; the walk
    // stops at max_depth accepted nodes, and the extra token then comes from the last one's row)
    while (len < max_depth) {
      const unsigned long long m0 = __ballot(ok0 && p0 == c), m1 = __ballot(ok1 && p1 == c);
      const int k = m0 ? __ffsll((long long)m0) - 1 : (m1 ? 63 + __ffsll((long long)m1) : -1);
      if (k < 0) break;
      if (lane == 0) out_path[(long long)b * max_depth + len] = k;
      ++len;
      c = k;
    }
    if (lane != 0) return;
    for (int i = len; i < max_depth; ++i) out_path[(long long)b * max_depth + i] = -1;
    out_len[b] = len;
    out_bonus[b] = amax[c + 1];
  }
}

// ------------------------------------------------------------------ sampling walk
__device__ double block_sum_f64(double v, double* red) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int w = threadIdx.x >> 6;
  __syncthreads();  // protects red[] against the previous use
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  double r = 0.0;
  for (int i = 0; i < kWalkThreads / 64; ++i) r += red[i];
  return r;
}

struct WalkParams {
  int n_tree, vocab, nch, max_depth;
  double temp;
  const int *tokens, *parent;
  const float *logits, *draft, *uniforms;
  const int* draft_row;  // or null: row b*n_tree + k
  long long n_draft_rows;
  const float* pmax;
  const double* psum;
  double* resid;  // [batch][2][vocab] unnormalised residuals (ping-pong)
  int *out_path, *out_len, *out_bonus;
  unsigned* err;  // the workspace's sticky device error word
};

__global__ __launch_bounds__(kWalkThreads) void walk_sample_kernel(WalkParams p) {
  __shared__ int par_s[JK_MAX_TREE];
  __shared__ double red[kWalkThreads / 64];
  __shared__ double seg_incl[kWalkThreads];
  __shared__ int s_found;

  const int b = blockIdx.x, tid = threadIdx.x;
  const int N = p.n_tree, V = p.vocab;
  const int rows = N + 1;
  if (tid < N) {
    par_s[tid] = sanitize_parent(p.parent[(long long)b * N + tid], tid, p.err);
    const int t = p.tokens[(long long)b * N + tid];
    if (t < 0 || t >= V) report(p.err, kDevErrBadToken);
  }
  __syncthreads();

  const int* tok = p.tokens + (long long)b * N;
  const float* uni = p.uniforms + (long long)b * rows;
  double* res0 = p.resid + (long long)b * 2 * V;

  int c = -1, len = 0;
  // current distribution at c: either softmax of row c+1 (fresh) or resid[cur] / res_s
  bool fresh = true;
  int cur = 0;
  double res_s = 1.0;
  double row_max = 0.0;  // max of row / T
  double row_z = 1.0;
  const float* row = nullptr;

  auto load_row_stats = [&](int r) {
    row = p.logits + ((long long)b * rows + r) * V;
    const long long base = ((long long)b * rows + r) * p.nch;
    float mx = -INFINITY;
    for (int i = 0; i < p.nch; ++i) mx = fmaxf(mx, p.pmax[base + i]);
    const double mref = (mx == -INFINITY) ? 0.0 : (double)mx / p.temp;
    double z = 0.0;
    for (int i = 0; i < p.nch; ++i) {
      const float mc = p.pmax[base + i];
      if (mc != -INFINITY) z += p.psum[base + i] * exp((double)mc / p.temp - mref);
    }
    row_max = mref;
    row_z = z;
  };
  // probability of token v under the current distribution (every thread may call it)
  auto prob = [&](int v) -> double {
    if (fresh) return exp((double)row[v] / p.temp - row_max) / row_z;
    return res0[(long long)cur * V + v] / res_s;
  };

  load_row_stats(0);
  int k = 0;  // children of c are searched from k upwards (topological numbering)
  while (len < p.max_depth) {  // (at the cap the token after c comes from c's own row, untouched)
    // next child of c, left to right
    int child = -1;
    for (int j = k; j < N; ++j)
      if (par_s[j] == c) { child = j; break; }
    if (child < 0) break;
    const int x = min(max(tok[child], 0), V - 1);  // a token id outside the vocabulary must not fault
    long long qr = (long long)b * N + child;
    if (p.draft_row) {
      qr = p.draft_row[qr];
      qr = qr < 0 ? 0 : (qr >= p.n_draft_rows ? p.n_draft_rows - 1 : qr);
    }
    const float* qk = p.draft + qr * V;
    const double lhs = (double)uni[child] * (double)qk[x];
    const double rhs = prob(x);
    if (lhs < rhs) {
      if (tid == 0) p.out_path[(long long)b * p.max_depth + len] = child;
      ++len;
      c = child;
      k = child + 1;
      fresh = true;
      load_row_stats(c + 1);
      continue;
    }
    // rejected: r = max(0, p - q_k), written unnormalised to the other buffer
    double* dst = res0 + (long long)(fresh ? 0 : (cur ^ 1)) * V;
    double part = 0.0;
    for (int v = tid; v < V; v += kWalkThreads) {
      const double r = fmax(0.0, prob(v) - (double)qk[v]);
      dst[v] = r;
      part += r;
    }
    const double s = block_sum_f64(part, red);  // its barriers also order dst[] for later readers
    if (s > 0.0) {
      cur = fresh ? 0 : (cur ^ 1);
      fresh = false;
      res_s = s;
    }
    k = child + 1;
  }

  // ---- bonus token: smallest v whose cumulative probability exceeds u * total
  const int seg = (V + kWalkThreads - 1) / kWalkThreads;
  const int s0 = min(V, tid * seg), s1 = min(V, s0 + seg);
  double part = 0.0;
  for (int v = s0; v < s1; ++v) part += prob(v);
  seg_incl[tid] = part;
  if (tid == 0) s_found = -1;
  __syncthreads();
  // inclusive scan over the 1024 segment sums (Hillis-Steele in LDS)
  for (int o = 1; o < kWalkThreads; o <<= 1) {
    const double add = (tid >= o) ? seg_incl[tid - o] : 0.0;
    __syncthreads();
    seg_incl[tid] += add;
    __syncthreads();
  }
  const double total = seg_incl[kWalkThreads - 1];
  const double target = (double)uni[N] * total;
  const double excl = (tid == 0) ? 0.0 : seg_incl[tid - 1];
  if (s1 > s0 && excl <= target && seg_incl[tid] > target) {
    double run = excl;
    int found = -1;
    for (int v = s0; v < s1; ++v) {
      run += prob(v);
      if (run > target) { found = v; break; }
    }
    // rounding between the scanned and the re-added sums can leave the segment without a hit
    if (found < 0) found = s1 - 1;
    atomicMax(&s_found, found);
  }
  __syncthreads();
  const int hit = s_found;  // every thread reads the same value before anyone may change it
  __syncthreads();
  if (hit < 0) {
    // u * total not below the last cumulative value: largest v with positive probability
    int last = -1;
    for (int v = s0; v < s1; ++v)
      if (prob(v) > 0.0) last = v;
    if (last >= 0) atomicMax(&s_found, last);
  }
  __syncthreads();
  if (tid == 0) {
    for (int i = len; i < p.max_depth; ++i) p.out_path[(long long)b * p.max_depth + i] = -1;
    p.out_len[b] = len;
    p.out_bonus[b] = s_found < 0 ? 0 : s_found;
  }
}

// ------------------------------------------------------------------ library-owned scratch
// For the entry point that takes no workspace (callers that cannot allocate device memory):
// the (max, argmax) partials of the greedy walk live in this array instead.  Every GPU the
// library runs on holds its own copy at its own address until the process ends; in host code
// the array's name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[JK_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, looked up once

hipError_t scratch_address(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));  // the current device's copy
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

// Where do consecutive workgroups run?  Every workgroup of a small grid records the id of the XCD
// it is on (the attention kernel merges its key splits inside one XCD's L2 and relies on the
// hardware dealing workgroup n to XCD n mod 8).
__global__ void xcd_probe_kernel(unsigned* out) {
  unsigned id;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(id));
  if (threadIdx.x == 0) out[blockIdx.x] = id & 0xfu;
}

struct WsLayout {
  size_t coop, pmax, pidx, psum, resid, total;  // (the error word's header sits in front of them)
};
WsLayout ws_layout(int batch, int n_tree, int vocab, int mode, bool caller_workspace = true) {
  WsLayout w{};
  const size_t rows = (size_t)batch * (n_tree + 1);
  const size_t slots = rows * n_chunks(vocab);
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  size_t off = kWsErrBytes;
  // the per-tree blocks of the cooperative walk come first, in every caller's workspace and for
  // every mode: their words keep their place and are never overlaid by another call's partials,
  // so a workspace needs zeroing only once whatever calls take turns on it (the library's own
  // scratch array serves greedy calls only and has no such blocks)
  w.coop = off; off += caller_workspace ? up(accept_coop_bytes()) : 0;
  w.pmax = off; off += up(slots * sizeof(float));
  w.pidx = off; off += up(slots * sizeof(int));
  w.psum = off; off += (mode == JK_SAMPLE) ? up(slots * sizeof(double)) : 0;
  w.resid = off; off += (mode == JK_SAMPLE) ? up((size_t)batch * 2 * vocab * sizeof(double)) : 0;
  w.total = off;
  return w;
}

}  // namespace

size_t accept_workspace_bytes(int batch, int n_tree, int vocab, int mode) {
  return ws_layout(batch, n_tree, vocab, mode).total;
}

// Synchronous, for jk_init: resolves the scratch array of the current device and runs the probe
// in it.  *round_robin: workgroups whose numbers agree modulo 8 were all on one XCD.
hipError_t probe_xcd_placement(hipStream_t stream, bool* round_robin) {
  constexpr int kProbeWgs = 256;
  void* base = nullptr;
  hipError_t e = scratch_address(&base);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(xcd_probe_kernel, dim3(kProbeWgs), dim3(64), 0, stream, static_cast<unsigned*>(base));
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  unsigned ids[kProbeWgs];
  e = hipMemcpyAsync(ids, base, sizeof(ids), hipMemcpyDeviceToHost, stream);
  if (e != hipSuccess) return e;
  e = hipStreamSynchronize(stream);
  if (e != hipSuccess) return e;
  bool ok = true;
  for (int n = 8; n < kProbeWgs; ++n) ok = ok && ids[n] == ids[n & 7];
  *round_robin = ok;
  return hipSuccess;
}

size_t accept_greedy_static_bytes(int batch, int n_tree, int vocab) {
  return ws_layout(batch, n_tree, vocab, JK_GREEDY, false).total;
}

// Greedy acceptance with the partials in the library's own scratch array: the same two
// kernels as launch_accept, no workspace argument, nothing allocated.  Nothing in the array
// needs clearing: every partial the walk reads is written by the reduction of the same call.
hipError_t launch_accept_greedy_static(const AcceptArgs& a, hipStream_t stream) {
  void* base = nullptr;
  hipError_t e = scratch_address(&base);
  if (e != hipSuccess) return e;
  const WsLayout w = ws_layout(a.batch, a.n_tree, a.vocab, JK_GREEDY, false);
  if (w.total > (size_t)JK_STATIC_SCRATCH_BYTES) return hipErrorInvalidValue;  // (checked by the caller too)
  char* ws = static_cast<char*>(base);
  float* pmax = reinterpret_cast<float*>(ws + w.pmax);
  int* pidx = reinterpret_cast<int*>(ws + w.pidx);
  const int nch = n_chunks(a.vocab);
  hipLaunchKernelGGL(row_reduce_kernel<false>, dim3(nch, a.batch * (a.n_tree + 1)), dim3(256), 0, stream, a.logits,
                     a.vocab, 1.0, pmax, pidx, static_cast<double*>(nullptr));
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(walk_greedy_kernel, dim3(a.batch), dim3(128), 0, stream, a.n_tree, nch, a.vocab, a.max_depth, a.tokens,
                     a.parent, pmax, pidx, a.out_path, a.out_len, a.out_bonus, static_cast<unsigned*>(nullptr));
  return hipGetLastError();
}

hipError_t launch_accept(const AcceptArgs& a, hipStream_t stream) {
  const WsLayout w = ws_layout(a.batch, a.n_tree, a.vocab, a.mode);
  char* ws = static_cast<char*>(a.workspace);
  float* pmax = reinterpret_cast<float*>(ws + w.pmax);
  int* pidx = reinterpret_cast<int*>(ws + w.pidx);
  double* psum = reinterpret_cast<double*>(ws + w.psum);
  double* resid = reinterpret_cast<double*>(ws + w.resid);
  const int nch = n_chunks(a.vocab);
  const dim3 grid(nch, a.batch * (a.n_tree + 1));
  if (a.mode == JK_GREEDY) {
    hipLaunchKernelGGL(row_reduce_kernel<false>, grid, dim3(256), 0, stream, a.logits, a.vocab, 1.0, pmax, pidx,
                       psum);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(walk_greedy_kernel, dim3(a.batch), dim3(128), 0, stream, a.n_tree, nch, a.vocab, a.max_depth,
                       a.tokens, a.parent, pmax, pidx, a.out_path, a.out_len, a.out_bonus,
                       reinterpret_cast<unsigned*>(ws));
    return hipGetLastError();
  }
  {
    int W = 0, slice = 0;
    // (tuning/testing: accept_single forces the one-workgroup walk)
    if (!tuning().accept_single && accept_coop_plan(a.batch, a.vocab, device_cu_count(), &W, &slice))
      return launch_accept_coop(a, ws + w.coop, W, slice, stream);
  }
  const double temp = (double)a.temperature;
  hipLaunchKernelGGL(row_reduce_kernel<true>, grid, dim3(256), 0, stream, a.logits, a.vocab, temp, pmax, pidx,
                     psum);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  WalkParams wp;
  wp.n_tree = a.n_tree; wp.vocab = a.vocab; wp.nch = nch; wp.max_depth = a.max_depth;
  wp.temp = temp;
  wp.tokens = a.tokens; wp.parent = a.parent;
  wp.logits = a.logits; wp.draft = a.draft_probs; wp.uniforms = a.uniforms;
  wp.draft_row = a.draft_row; wp.n_draft_rows = a.n_draft_rows;
  wp.pmax = pmax; wp.psum = psum; wp.resid = resid;
  wp.out_path = a.out_path; wp.out_len = a.out_len; wp.out_bonus = a.out_bonus;
  wp.err = reinterpret_cast<unsigned*>(ws);
  hipLaunchKernelGGL(walk_sample_kernel, dim3(a.batch), dim3(kWalkThreads), 0, stream, wp);
  return hipGetLastError();
}

}  // namespace jk
