// Growing the draft token tree on the device (gfx950), one depth at a time, from the candidate
// lists that jk_draft_heads returns (Section 3.1.2 of the paper: both activated experts propose
// their own top-k candidates for every expanded node, the expert with the larger router score
// on the left; top-k construction as in a dynamically built tree).
//
//   grow      per sequence: a new node for every (frontier node, expert, rank) in that order,
//             score = parent's score * candidate probability; the `width` best new nodes (ties
//             to the lower index) become the next frontier, listed in increasing index.
//   finalize  per sequence: the n_keep best nodes (ties to the lower index; a node never scores
//             above its parent, so ancestors come along), renumbered in increasing old index.
//   gather    the kept nodes' draft distributions as the dense [batch][n_tree][vocab] array that
//             jk_accept_path takes.
// All choices are made by counting how many entries beat a given one (no sorting network, no
// reduction rounds): at most a few hundred entries per sequence.
#include <climits>

#include "jk_internal.h"

namespace jk {
namespace {

constexpr int kTreeThreads = 256;
constexpr int kMaxGrowNodes = 1024;  // node capacity per sequence the kernels are laid out for

// larger score first, equal scores by increasing index (both operands always evaluated)
__device__ __forceinline__ int beats(float av, int ai, float bv, int bi) {
  return (int)(av > bv) | ((int)(av == bv) & (int)(ai < bi));
}

// How many threads with a smaller index raised `flag`, and how many did in all: ballots within
// the waves, the four wave totals through LDS (s_cnt: kTreeThreads / 64 ints; the caller's
// later use of it must follow a barrier).
__device__ __forceinline__ int count_before(bool flag, int t, int* s_cnt, int& total) {
  const unsigned long long m = __ballot(flag);
  const int lane = t & 63, wave = t >> 6;
  const int in_wave = __popcll(m & ((1ull << lane) - 1ull));
  if (lane == 0) s_cnt[wave] = __popcll(m);
  __syncthreads();
  int before = in_wave;
  total = 0;
#pragma unroll
  for (int w = 0; w < kTreeThreads / 64; ++w) {
    const int c = s_cnt[w];
    before += w < wave ? c : 0;
    total += c;
  }
  return before;
}

__global__ __launch_bounds__(kTreeThreads) void grow_kernel(TreeGrowArgs a) {
  __shared__ float s_sc[kTreeThreads];
  __shared__ int s_cnt[kTreeThreads / 64];
  __shared__ int s_first;
  const int b = blockIdx.x, t = threadIdx.x;
  const int C = a.n_front * 2 * a.top_k;  // <= kTreeThreads (checked by the host)
  const int n0 = min(max(a.n_nodes[b], 0), a.max_nodes);  // (a count the caller forgot to clear must not fault)
  const int id = n0 + t;
  const bool valid = t < C && id < a.max_nodes;
  float sc = -INFINITY;
  if (valid) {
    const int f = t / (2 * a.top_k), e = (t / a.top_k) & 1;
    const long long row = (long long)b * a.n_front + f;
    const int pid = a.frontier_in ? a.frontier_in[row] : -1;
    const bool has_parent = pid >= 0 && pid < n0;
    const float ps = has_parent ? a.score[(long long)b * a.max_nodes + pid] : 1.0f;
    sc = ps * a.cand_p[row * 2 * a.top_k + (t - f * 2 * a.top_k)];
    const long long at = (long long)b * a.max_nodes + id;
    a.tokens[at] = a.cand_tok[row * 2 * a.top_k + (t - f * 2 * a.top_k)];
    a.parent[at] = has_parent ? pid : -1;
    a.score[at] = sc;
    a.q_row[at] = a.q_row_base + (int)(2 * row) + e;
  }
  s_sc[t] = sc;
  if (t == 0) s_first = INT_MAX;
  __syncthreads();
  int rank = 0;  // (entries from C on hold -inf and a larger index: they beat nobody)
#pragma unroll 8
  for (int i = 0; i < C; ++i) rank += beats(s_sc[i], i, sc, t);
  const bool sel = valid && rank < a.width;
  int total;
  const int slot = count_before(sel, t, s_cnt, total);
  if (sel) {
    a.frontier_out[(long long)b * a.width + slot] = id;
    if (slot == 0) s_first = id;
  }
  __syncthreads();
  // fewer new nodes than frontier slots: the rest repeats the first entry (-1 if there is none)
  if (t >= total && t < a.width) a.frontier_out[(long long)b * a.width + t] = s_first == INT_MAX ? -1 : s_first;
  if (t == 0) a.n_nodes[b] = min(n0 + C, a.max_nodes);
}

// The last draft pass with a mixture head and a contrastive head (Section 3.2): children from
// head 0's list, then the `width` best children get head 1's list of their parent as children.
__global__ __launch_bounds__(kTreeThreads) void grow_tail_kernel(TreeGrowArgs a, int k1, int k2) {
  __shared__ float s_sc[kTreeThreads];
  __shared__ int s_cnt[kTreeThreads / 64];
  __shared__ int s_child[kTreeThreads];  // chosen children by slot: node id, frontier slot
  __shared__ int s_slot_f[kTreeThreads];
  const int b = blockIdx.x, t = threadIdx.x;
  const int C = a.n_front * k1;
  const int n0 = min(max(a.n_nodes[b], 0), a.max_nodes);
  const int id = n0 + t;
  const bool valid = t < C && id < a.max_nodes;
  const long long base = (long long)b * a.max_nodes;
  float sc = -INFINITY;
  const int f = t / k1, j = t - f * k1;
  if (valid) {
    const long long row = (long long)b * a.n_front + f;
    const int pid = a.frontier_in ? a.frontier_in[row] : -1;
    const bool has_parent = pid >= 0 && pid < n0;
    const float ps = has_parent ? a.score[base + pid] : 1.0f;
    sc = ps * a.cand_p[row * 2 * a.top_k + j];
    a.tokens[base + id] = a.cand_tok[row * 2 * a.top_k + j];
    a.parent[base + id] = has_parent ? pid : -1;
    a.score[base + id] = sc;
    a.q_row[base + id] = a.q_row_base + (int)(2 * row);
  }
  s_sc[t] = sc;
  __syncthreads();
  int rank = 0;
#pragma unroll 8
  for (int i = 0; i < C; ++i) rank += beats(s_sc[i], i, sc, t);
  const bool sel = valid && rank < a.width;
  int total;
  const int slot = count_before(sel, t, s_cnt, total);
  if (sel) {
    s_child[slot] = id;
    s_slot_f[slot] = f;
  }
  __syncthreads();
  const int n1 = min(n0 + C, a.max_nodes);
  const int G = total * k2;
  const int gid = n1 + t;
  if (t < G && gid < a.max_nodes) {
    const int s = t / k2, j2 = t - s * k2;
    const int c = s_child[s];
    const long long row = (long long)b * a.n_front + s_slot_f[s];
    a.tokens[base + gid] = a.cand_tok[(row * 2 + 1) * a.top_k + j2];
    a.parent[base + gid] = c;
    a.score[base + gid] = s_sc[c - n0] * a.cand_p[(row * 2 + 1) * a.top_k + j2];
    a.q_row[base + gid] = a.q_row_base + (int)(2 * row) + 1;
  }
  if (t == 0) a.n_nodes[b] = min(n1 + G, a.max_nodes);
}

// One depth of a predefined tree shape: new node j hangs under frontier slot shape_slot[j] and
// takes candidate shape_rank[j] of that slot's list of expert shape_expert[j].
__global__ __launch_bounds__(kTreeThreads) void fill_static_kernel(TreeGrowArgs a, const int* __restrict__ shape_slot,
                                                                   const int* __restrict__ shape_expert,
                                                                   const int* __restrict__ shape_rank, int n_new,
                                                                   const int* __restrict__ next_index, int n_next,
                                                                   int* __restrict__ new_ids) {
  const int b = blockIdx.x, t = threadIdx.x;
  const int n0 = min(max(a.n_nodes[b], 0), a.max_nodes);
  const long long base = (long long)b * a.max_nodes;
  for (int j = t; j < n_new; j += kTreeThreads) {
    const int id = n0 + j;
    const bool valid = id < a.max_nodes;
    if (valid) {
      const int f = min(max(shape_slot[j], 0), a.n_front - 1);
      const int e = shape_expert[j] != 0 ? 1 : 0;
      const int r = min(max(shape_rank[j], 0), a.top_k - 1);
      const long long row = (long long)b * a.n_front + f;
      const int pid = a.frontier_in ? a.frontier_in[row] : -1;
      const bool has_parent = pid >= 0 && pid < n0;
      const float ps = has_parent ? a.score[base + pid] : 1.0f;
      a.tokens[base + id] = a.cand_tok[(row * 2 + e) * a.top_k + r];
      a.parent[base + id] = has_parent ? pid : -1;
      a.score[base + id] = ps * a.cand_p[(row * 2 + e) * a.top_k + r];
      a.q_row[base + id] = a.q_row_base + (int)(2 * row) + e;
    }
    if (new_ids) new_ids[(long long)b * n_new + j] = valid ? id : -1;
  }
  if (a.frontier_out)
    for (int i = t; i < n_next; i += kTreeThreads) {
      const int j = min(max(next_index[i], 0), n_new - 1);
      a.frontier_out[(long long)b * n_next + i] = n0 + j < a.max_nodes ? n0 + j : -1;
    }
  __syncthreads();  // everybody has read n_nodes
  if (t == 0) a.n_nodes[b] = min(n0 + n_new, a.max_nodes);
}

__global__ __launch_bounds__(kTreeThreads) void finalize_kernel(TreeFinalArgs a) {
  __shared__ float s_sc[kMaxGrowNodes];
  __shared__ short s_keep[kMaxGrowNodes];
  __shared__ short s_new[kMaxGrowNodes];
  __shared__ int s_cnt[kTreeThreads / 64];
  const int b = blockIdx.x, t = threadIdx.x;
  const int n = min(max(a.n_nodes[b], 0), a.max_nodes);
  const long long base = (long long)b * a.max_nodes;
  for (int i = t; i < kMaxGrowNodes; i += kTreeThreads) s_sc[i] = i < n ? a.score[base + i] : -INFINITY;
  __syncthreads();
  for (int i = t; i < kMaxGrowNodes; i += kTreeThreads) {
    int rank = 0;
    const float sc = s_sc[i];
    if (i < n) {
#pragma unroll 8
      for (int j = 0; j < n; ++j) rank += beats(s_sc[j], j, sc, i);
    }
    s_keep[i] = (i < n && rank < a.n_keep) ? 1 : 0;
  }
  __syncthreads();
  int carried = 0;  // kept nodes in the chunks before this one (the same in every thread)
  for (int i0 = 0; i0 < n; i0 += kTreeThreads) {
    const int i = i0 + t;
    int total;
    const int before = count_before(i < n && s_keep[i], t, s_cnt, total);
    if (i < n) s_new[i] = (short)(carried + before);
    carried += total;
    __syncthreads();  // s_cnt is written again by the next chunk
  }
  for (int i = t; i < n; i += kTreeThreads) {
    if (!s_keep[i]) continue;
    const long long o = (long long)b * a.n_keep + s_new[i];
    const int pid = a.parent[base + i];
    a.out_tokens[o] = a.tokens[base + i];
    a.out_parent[o] = (pid >= 0 && pid < i) ? (int)s_new[pid] : -1;  // (a kept node's parent is kept)
    a.out_q_row[o] = a.q_row[base + i];
    if (a.out_old) a.out_old[o] = i;
  }
  const int n_valid = min(n, a.n_keep);
  for (int i = n_valid + t; i < a.n_keep; i += kTreeThreads) {  // a tree with fewer nodes than asked for
    const long long o = (long long)b * a.n_keep + i;
    a.out_tokens[o] = -1;
    a.out_parent[o] = -1;
    a.out_q_row[o] = 0;
    if (a.out_old) a.out_old[o] = -1;
  }
  if (t == 0) a.n_valid[b] = n_valid;
}

typedef float floatx4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void gather_rows_kernel(const float* __restrict__ q_all, const int* __restrict__ q_row,
                                                          float* __restrict__ out, int vocab, long long n_q_rows) {
  const long long node = blockIdx.x;
  long long r = q_row[node];
  r = r < 0 ? 0 : (r >= n_q_rows ? n_q_rows - 1 : r);  // must not fault on a bad row number
  const float* src = q_all + r * vocab;
  float* dst = out + node * vocab;
  const bool vec = (vocab & 3) == 0 && ((reinterpret_cast<size_t>(q_all) | reinterpret_cast<size_t>(out)) & 15) == 0;
  if (vec) {
    for (int c = blockIdx.y * 256 + threadIdx.x; c < vocab / 4; c += 256 * gridDim.y)
      reinterpret_cast<floatx4*>(dst)[c] = reinterpret_cast<const floatx4*>(src)[c];
  } else {
    for (int c = blockIdx.y * 256 + threadIdx.x; c < vocab; c += 256 * gridDim.y) dst[c] = src[c];
  }
}

}  // namespace

int tree_max_nodes() { return kMaxGrowNodes; }

hipError_t launch_tree_grow(const TreeGrowArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(grow_kernel, dim3(a.batch), dim3(kTreeThreads), 0, stream, a);
  return hipGetLastError();
}
hipError_t launch_tree_grow_tail(const TreeGrowArgs& a, int k1, int k2, hipStream_t stream) {
  hipLaunchKernelGGL(grow_tail_kernel, dim3(a.batch), dim3(kTreeThreads), 0, stream, a, k1, k2);
  return hipGetLastError();
}
hipError_t launch_tree_fill_static(const TreeGrowArgs& a, const int* slot, const int* expert, const int* rank, int n_new,
                                   const int* next_index, int n_next, int* new_ids, hipStream_t stream) {
  hipLaunchKernelGGL(fill_static_kernel, dim3(a.batch), dim3(kTreeThreads), 0, stream, a, slot, expert, rank, n_new,
                     next_index, n_next, new_ids);
  return hipGetLastError();
}
hipError_t launch_tree_finalize(const TreeFinalArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(finalize_kernel, dim3(a.batch), dim3(kTreeThreads), 0, stream, a);
  return hipGetLastError();
}
hipError_t launch_gather_rows(const float* q_all, const int* q_row, float* out, long long n_nodes, int vocab,
                              long long n_q_rows, hipStream_t stream) {
  const unsigned chunks = (unsigned)(vocab / 4096 < 1 ? 1 : (vocab / 4096 > 16 ? 16 : vocab / 4096));
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)n_nodes, chunks), dim3(256), 0, stream, q_all, q_row, out,
                     vocab, n_q_rows);
  return hipGetLastError();
}

}  // namespace jk
