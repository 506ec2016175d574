// Speculative-sampling acceptance walk, cooperative version (gfx950).
//
// Same rule as the single-workgroup walk (Section 2.1 steps 2-3 of the paper:
// accept with probability min(1, p/q), continue with norm(max(0, p - q)) after
// a rejection; siblings tried left to right, Section 3.1.2), spread over W
// workgroups per tree.  Workgroup w owns the vocabulary slice
// [w*SL, (w+1)*SL) and keeps the current distribution of that slice in LDS as
// fp64, so that a rejection only streams the rejected node's draft
// distribution from HBM.  Logits rows are read lazily: only the rows of nodes
// the walk actually reaches (at most depth+1 of the N+1 rows).
//
// Every workgroup follows the same control flow.  Scalars that depend on the
// whole vocabulary (row maximum and normaliser, residual mass, cumulative sums
// for the final draw) are exchanged through a small table in the workspace:
// each workgroup publishes its partial under a tag that is unique to the call
// and the exchange number, then reads the W partials once all tags have
// appeared.  All workgroups reduce the same values in the same order, so they
// take identical decisions.  Waiting is bounded: if a partner never shows up
// (the W workgroups of a tree are not all resident) the walk gives up and
// reports accept_len = -1 instead of hanging; the last workgroup of a tree to
// finish publishes the results and moves the call number on (see TreeWords), so
// a call that gave up leaves nothing behind that a later call could mistake.
#include "jk_internal.h"

namespace jk {
namespace {

constexpr int kCoopThreads = 256;  // (512 measured 8 % faster for one tree and 60 % slower for eight: two workgroups per CU then)
constexpr int kCoopWaves = kCoopThreads / 64;
constexpr unsigned kDefaultSpinLimit = 1u << 12;  // polls before giving up: a few milliseconds

// One workgroup's contribution to an exchange: two doubles, cut into four 32-bit halves,
// each stored in a 64-bit word together with the exchange's 32-bit tag.  A word is written
// and read with one 64-bit access, so a reader that sees the tag also sees the half that
// belongs to it: no fences and no ordering between the words are needed.
struct Slot {  // 32 bytes
  unsigned long long word[4];
};

// Per-tree words in the workspace header.  `epoch` numbers the calls: every exchange of a call is
// tagged with epoch + 1, and only the LAST workgroup of the tree to finish moves it on (it counts
// the finished ones in `finish` and returns that to zero), so that workgroups that start late -
// even after the others have given up and left - still read the call's own epoch and can never
// publish a tag that a later call would take for its own.  The results travel the same way: the
// workgroup that owns the final draw leaves (tag, token) in `bonus`, workgroup 0 (tag, length) in
// `len`, a workgroup that gave up its tag in `fail`; the last to finish reads the three and is
// the only writer of accept_len and bonus_token.
struct TreeWords {  // 64 bytes
  unsigned long long epoch;
  unsigned long long bonus, len, fail;
  unsigned finish;
  unsigned pad[7];
};

// What a tree owns in the workspace: its words and two exchange tables of up to 64 slots.  Tree b's
// block sits at b * sizeof(TreeBlock) whatever the batch size, mode or vocabulary of a call is, and
// the blocks of all kCoopMaxTrees trees are set aside in every acceptance workspace (see
// accept_coop_bytes), so calls of different shapes and modes can share one workspace.
struct TreeBlock {  // 4160 bytes
  TreeWords words;
  Slot slots[2 * 64];
};

struct CoopParams {
  int n_tree, vocab, max_depth, W, slice;
  double inv_temp;  // 1 / temperature
  const int *tokens, *parent;
  const float *logits, *draft, *uniforms;
  const int* draft_row;  // or null: row b*n_tree + k of draft
  long long n_draft_rows;
  TreeBlock* trees;  // [batch] words and exchange tables of each tree (zero before the first use of the workspace)
  unsigned spin_limit;
  int *out_path, *out_len, *out_bonus;
  unsigned* err;  // the workspace's sticky device error word
};

__device__ __forceinline__ double block_sum(double v, double* red) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  double s = 0.0;  // (waves in order: the same sum in every workgroup)
#pragma unroll
  for (int i = 0; i < kCoopWaves; i += 2) s += red[i] + red[i + 1];
  return s;
}
__device__ __forceinline__ double block_max(double v, double* red) {
  for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  double m = red[0];
#pragma unroll
  for (int i = 1; i < kCoopWaves; ++i) m = fmax(m, red[i]);
  return m;
}

__global__ __launch_bounds__(kCoopThreads) void walk_sample_coop_kernel(CoopParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  double* cur = reinterpret_cast<double*>(smem);   // [slice] current distribution of my slice
  __shared__ double red[kCoopWaves];
  __shared__ double xa[64], xb[64];                // the W partials of an exchange
  __shared__ unsigned xh[256];                     // their 32-bit halves as they arrive
  __shared__ int par_s[JK_MAX_TREE];
  __shared__ int tok_s[JK_MAX_TREE];
  __shared__ int s_fail, s_found;
  __shared__ double xw[64];                        // weights of the W partial softmax sums
  __shared__ double rej_inv[JK_MAX_TREE];          // 1 / residual mass of the rejected siblings at this node
  __shared__ int rej_k[JK_MAX_TREE];
  __shared__ float pf_q[JK_MAX_TREE + 2];          // prefetched scalars of the next candidate (see below)
  __shared__ float uni_s[JK_MAX_TREE + 1];

  const int tid = threadIdx.x;
  const int W = p.W;
  const int b = blockIdx.x / W, w = blockIdx.x % W;
  const int N = p.n_tree, V = p.vocab, rows = N + 1;
  const int v_lo = min(V, w * p.slice), v_hi = min(V, v_lo + p.slice);
  const int n_mine = v_hi - v_lo;
  constexpr int kPer = 4096 / kCoopThreads;        // slice elements per thread at most

  // the tree's small arrays: loads go out now, the values are parked in LDS after the first
  // logits row has been processed (nothing needs them before), so their latency is hidden
  int pa_reg = -1, tok_reg = 0;
  float uni_reg = 0.f;
  if (tid < N) {
    pa_reg = p.parent[(long long)b * N + tid];
    tok_reg = p.tokens[(long long)b * N + tid];
  }
  if (tid <= N) uni_reg = p.uniforms[(long long)b * rows + tid];
  if (tid == 0) s_fail = 0;
  TreeWords* tw = &p.trees[b].words;
  const unsigned long long epoch = __hip_atomic_load(&tw->epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();

  // the draft distribution of node k (a row of p.draft)
  auto q_of = [&](int k) -> const float* {
    long long r = (long long)b * N + k;
    if (p.draft_row) {
      r = p.draft_row[r];
      r = r < 0 ? 0 : (r >= p.n_draft_rows ? p.n_draft_rows - 1 : r);  // a bad row number must not fault
    }
    return p.draft + r * V;
  };

  // smallest j >= from with parent c, or -1: every wave looks at all (at most 128) nodes, two
  // per lane, so no barrier is needed and all waves get the same answer
  auto find_child = [&](int c, int from) -> int {
    const int lane = tid & 63;
    const bool h0 = lane < N && lane >= from && par_s[lane] == c;
    const bool h1 = lane + 64 < N && lane + 64 >= from && par_s[lane + 64] == c;
    const unsigned long long m0 = __ballot(h0), m1 = __ballot(h1);
    return m0 ? __ffsll((long long)m0) - 1 : (m1 ? 63 + __ffsll((long long)m1) : -1);
  };

  const int n_per = (p.slice + kCoopThreads - 1) / kCoopThreads;  // slice elements per thread (uniform)
  Slot* slots = p.trees[b].slots;
  unsigned n_exch = 0;

  // all-gather of one (a, b) pair per workgroup; results in xa[0..W), xb[0..W).
  // Tags: 22 bits of call epoch, 10 bits of exchange number (at most N + depth + 2 < 1024 per
  // call).  Both tables are rewritten by every call (a call has at least two exchanges), so
  // a stale word is at most one epoch old and can never carry the current tag.
  auto exchange = [&](double a, double bb, double pad_a) {
    ++n_exch;
    const unsigned tag = (unsigned)(((epoch + 1) & 0x3FFFFFull) << 10) | (n_exch & 0x3FFu);
    Slot* tab = slots + (n_exch & 1) * W;
    if (tid < 4) {
      const unsigned long long bits = (unsigned long long)__double_as_longlong(tid < 2 ? a : bb);
      const unsigned half = (unsigned)(bits >> (32 * (tid & 1)));
      __hip_atomic_store(&tab[w].word[tid], ((unsigned long long)tag << 32) | half, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tid < 4 * W) {
      unsigned long long* src = &tab[tid >> 2].word[tid & 3];
      unsigned long long v;
      unsigned spins = 0;
      while ((unsigned)((v = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) >> 32) != tag) {
        if (++spins > p.spin_limit || s_fail) { s_fail = 1; v = 0; break; }
        __builtin_amdgcn_s_sleep(1);
      }
      xh[tid] = (unsigned)v;
    }
    __syncthreads();
    if (tid < W) {
      xa[tid] = __longlong_as_double((long long)(((unsigned long long)xh[4 * tid + 1] << 32) | xh[4 * tid]));
      xb[tid] = __longlong_as_double((long long)(((unsigned long long)xh[4 * tid + 3] << 32) | xh[4 * tid + 2]));
    } else if (tid < 64) {
      xa[tid] = pad_a;  // the reductions below always run over 64 entries
      xb[tid] = 0.0;
    }
    __syncthreads();
  };
  // sum of 64 LDS doubles in a fixed order (four interleaved chains): identical in every workgroup
  auto sum64 = [&](const double* v) {
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
#pragma unroll
    for (int i = 0; i < 64; i += 4) {
      a0 += v[i];
      a1 += v[i + 1];
      a2 += v[i + 2];
      a3 += v[i + 3];
    }
    return (a0 + a1) + (a2 + a3);
  };

  double row_m = 0.0, row_inv_z = 1.0;  // max of row/T, and 1 / sum of exp(row/T - max), of the current row
  const float* row = nullptr;

  // softmax of logits row r over my slice into cur[]; (row_m, row_inv_z) for everybody
  auto load_row = [&](int r) {
    row = p.logits + ((long long)b * rows + r) * V;
    double z[kPer];
    double lm = -INFINITY;
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      if (u >= n_per) break;
      const int i = tid + u * kCoopThreads;
      z[u] = i < n_mine ? (double)row[v_lo + i] * p.inv_temp : -INFINITY;
      lm = fmax(lm, z[u]);
    }
    const double m_w = block_max(lm, red);
    const double m_use = (m_w == -INFINITY) ? 0.0 : m_w;
    double ls = 0.0;
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      if (u >= n_per) break;
      z[u] = exp(z[u] - m_use);
      ls += z[u];
    }
    const double z_w = block_sum(ls, red);
    exchange(m_w, z_w, -INFINITY);
    double M0 = -INFINITY, M1 = -INFINITY;
#pragma unroll
    for (int i = 0; i < 64; i += 2) {
      M0 = fmax(M0, xa[i]);
      M1 = fmax(M1, xa[i + 1]);
    }
    const double M = fmax(M0, M1);
    const double M_use = (M == -INFINITY) ? 0.0 : M;
    if (tid < 64) xw[tid] = xb[tid] * exp(xa[tid] - M_use);  // 0 for an empty slice (-inf) and for the padding
    __syncthreads();
    const double Z = sum64(xw);  // same numbers, same order in every workgroup
    row_m = M_use;
    row_inv_z = 1.0 / Z;
    const double sc = exp(m_use - M_use) * row_inv_z;
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      if (u >= n_per) break;
      const int i = tid + u * kCoopThreads;
      if (i < n_mine) cur[i] = z[u] * sc;
    }
    __syncthreads();
  };

  // Scalars a candidate's test needs, gathered by one thread each and parked in LDS:
  // pf_q[i] = q_{rej_k[i]}[x] for the n_rej siblings rejected so far, then q_child[x], then
  // logits_row[x], with x the candidate's token.  `extra` >= 0 adds one more (pending)
  // rejected sibling to the list: the gather for the next sibling is issued before the
  // current one's fate is known, so that its latency hides behind the exchange.
  auto gather_issue = [&](int child, int n_rej, int extra) -> float {
    const int x = tok_s[child];
    const int n_list = n_rej + (extra >= 0 ? 1 : 0);
    float v = 0.f;
    if (tid < n_list) {
      const int kq = tid < n_rej ? rej_k[tid] : extra;
      v = q_of(kq)[x];
    } else if (tid == n_list) {
      v = q_of(child)[x];
    } else if (tid == n_list + 1) {
      v = row[x];
    }
    return v;
  };
  auto gather_park = [&](float v, int n_list) {
    if (tid < n_list + 2) pf_q[tid] = v;
  };

  int c = -1, len = 0, n_rej = 0;
  load_row(0);
  if (tid < N) {
    par_s[tid] = (pa_reg >= -1 && pa_reg < tid) ? pa_reg : -1;
    tok_s[tid] = min(max(tok_reg, 0), V - 1);  // a token id outside the vocabulary must not fault
    if (w == 0) {  // both repairs are recorded in the workspace's error word
      if (par_s[tid] != pa_reg) __hip_atomic_fetch_or(p.err, kDevErrBadTree, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (tok_s[tid] != tok_reg) __hip_atomic_fetch_or(p.err, kDevErrBadToken, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (tid <= N) uni_s[tid] = uni_reg;
  __syncthreads();
  int child = find_child(-1, 0);
  bool have_pf = false;     // pf_q[] and qreg[] already hold `child`'s data
  float qreg[kPer];         // q_child over my slice
  while (!s_fail && child >= 0) {
    const float* qk = q_of(child);
    if (!have_pf) {
      const float v = gather_issue(child, n_rej, -1);
#pragma unroll
      for (int u = 0; u < kPer; ++u) {
        const int i = tid + u * kCoopThreads;
        qreg[u] = i < n_mine ? qk[v_lo + i] : 0.f;
      }
      gather_park(v, n_rej);
      __syncthreads();
    }
    // probability of token x under the current distribution: the same chain of operations in
    // every workgroup (global data only), so that all take the same decision
    double px = exp((double)pf_q[n_rej + 1] * p.inv_temp - row_m) * row_inv_z;
    for (int i = 0; i < n_rej; ++i) px = fmax(0.0, px - (double)pf_q[i]) * rej_inv[i];
    const double lhs = (double)uni_s[child] * (double)pf_q[n_rej];
    if (lhs < px) {
      if (tid == 0 && w == 0) p.out_path[(long long)b * p.max_depth + len] = child;
      ++len;
      c = child;
      n_rej = 0;
      have_pf = false;
      __syncthreads();  // pf_q is rewritten for the first child
      load_row(c + 1);
      // at max_depth accepted nodes the walk stops: the token after c is drawn from c's own row
      child = len < p.max_depth ? find_child(c, c + 1) : -1;
      continue;
    }
    // rejected: candidate residual of my slice and its mass
    double part = 0.0;
    double res[kPer];
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      if (u >= n_per) break;
      const int i = tid + u * kCoopThreads;
      res[u] = i < n_mine ? fmax(0.0, cur[i] - (double)qreg[u]) : 0.0;
      part += res[u];
    }
    // the next sibling's data go out now; they arrive while the exchange is under way
    const int nxt_child = find_child(c, child + 1);
    float pv = 0.f;
    float qnext[kPer];
    if (nxt_child >= 0) {
      pv = gather_issue(nxt_child, n_rej, child);
      const float* qn = q_of(nxt_child);
#pragma unroll
      for (int u = 0; u < kPer; ++u) {
        const int i = tid + u * kCoopThreads;
        qnext[u] = i < n_mine ? qn[v_lo + i] : 0.f;
      }
    }
    const double s_w = block_sum(part, red);
    exchange(s_w, 0.0, 0.0);
    const double s = sum64(xa);
    have_pf = false;
    if (s > 0.0) {
      const double inv_s = 1.0 / s;
#pragma unroll
      for (int u = 0; u < kPer; ++u) {
        const int i = tid + u * kCoopThreads;
        if (i < n_mine) cur[i] = res[u] * inv_s;
      }
      if (tid == 0) { rej_k[n_rej] = child; rej_inv[n_rej] = inv_s; }
      if (nxt_child >= 0) {  // the prefetched list assumed exactly this rejection
        gather_park(pv, n_rej + 1);
#pragma unroll
        for (int u = 0; u < kPer; ++u) qreg[u] = qnext[u];  // (registers: nothing to skip)
        have_pf = true;
      }
      ++n_rej;
    }
    __syncthreads();
    child = nxt_child;
  }
  // ---- final draw: smallest v whose cumulative probability exceeds u * total
  if (!s_fail) {
    double part = 0.0;
    int last_pos = -1;
    // contiguous segments per thread so that the in-slice order is the vocabulary order
    const int seg = (n_mine + kCoopThreads - 1) / kCoopThreads;
    const int i0 = min(n_mine, tid * seg), i1 = min(n_mine, i0 + seg);
    for (int i = i0; i < i1; ++i) {
      part += cur[i];
      if (cur[i] > 0.0) last_pos = v_lo + i;
    }
    // scan of the 256 segment sums: wave scan, then wave offsets.  A thread's interval is
    // [off + excl, off + incl) with excl taken from its left neighbour's incl, so that the
    // intervals of threads, waves and workgroups tile [0, total) exactly, rounding included.
    double incl = part;
    for (int o = 1; o < 64; o <<= 1) {
      const double t = __shfl_up(incl, o);
      if ((tid & 63) >= o) incl += t;
    }
    double excl = __shfl_up(incl, 1);
    if ((tid & 63) == 0) excl = 0.0;
    __syncthreads();
    if ((tid & 63) == 63) red[tid >> 6] = incl;
    int lp = last_pos;
    for (int o = 32; o > 0; o >>= 1) lp = max(lp, __shfl_xor(lp, o));
    __shared__ int s_lp[kCoopWaves];
    if ((tid & 63) == 0) s_lp[tid >> 6] = lp;
    __syncthreads();
    double woff = 0.0;
    for (int i = 0; i < (tid >> 6); ++i) woff += red[i];
    double t_w = 0.0;  // (in wave order, like the offsets: the last wave's interval ends exactly at the total)
    int lp_w = -1;
#pragma unroll
    for (int i = 0; i < kCoopWaves; ++i) {
      t_w += red[i];
      lp_w = max(lp_w, s_lp[i]);
    }
    exchange(t_w, (double)lp_w, 0.0);
    if (!s_fail) {
      double before = 0.0, total = 0.0;
      int last_any = -1;
      for (int i = 0; i < W; ++i) {
        if (i < w) before += xa[i];
        total += xa[i];
        last_any = max(last_any, (int)xb[i]);
      }
      const double target = (double)uni_s[N] * total;
      if (tid == 0) s_found = -1;
      __syncthreads();
      // is the crossing inside my segment?
      const double lo = before + (woff + excl), hi = before + (woff + incl);
      if (i1 > i0 && lo <= target && hi > target) {
        double run = lo;
        int found = -1;
        for (int i = i0; i < i1; ++i) {
          run += cur[i];
          if (run > target) { found = v_lo + i; break; }
        }
        if (found < 0) found = v_lo + i1 - 1;  // rounding between the scanned and the re-added sums
        atomicMax(&s_found, found);
      }
      __syncthreads();
      const bool mine = s_found >= 0;
      // nobody crosses (u * total not below the last cumulative value): largest v with p > 0.
      // Decided identically everywhere: workgroup w' owns the crossing iff
      // before(w') <= target < before(w') + t(w'); sums of the same numbers in the same order.
      bool any = false;
      {
        double acc = 0.0;
        for (int i = 0; i < W; ++i) {
          if (acc <= target && acc + xa[i] > target) any = true;
          acc += xa[i];
        }
      }
      if (tid == 0) {
        const unsigned long long tag = (epoch + 1) << 32;
        if (mine || (!any && w == 0)) {
          const int token = mine ? s_found : (last_any < 0 ? 0 : last_any);
          __hip_atomic_store(&tw->bonus, tag | (unsigned)token, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (w == 0) {
          for (int i = len; i < p.max_depth; ++i) p.out_path[(long long)b * p.max_depth + i] = -1;
          __hip_atomic_store(&tw->len, tag | (unsigned)len, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
  }
  // ---- the end of this workgroup: say so; the last one of the tree publishes the results
  if (tid == 0) {
    const unsigned long long tag = (epoch + 1) << 32;
    if (s_fail) __hip_atomic_store(&tw->fail, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // (the words above went through to memory; wait for that before the count can tell anybody)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    const unsigned done = __hip_atomic_fetch_add(&tw->finish, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (done == (unsigned)W - 1) {
      __hip_atomic_store(&tw->finish, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned long long f = __hip_atomic_load(&tw->fail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned long long l = __hip_atomic_load(&tw->len, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned long long t = __hip_atomic_load(&tw->bonus, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const bool ok = f != tag && (l >> 32) == (tag >> 32) && (t >> 32) == (tag >> 32);
      p.out_len[b] = ok ? (int)(unsigned)l : -1;
      p.out_bonus[b] = ok ? (int)(unsigned)t : -1;
      if (!ok) __hip_atomic_fetch_or(p.err, kDevErrWalkWait, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&tw->epoch, epoch + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

}  // namespace

// The blocks of kCoopMaxTrees trees are part of every acceptance workspace, whatever a call's mode and
// batch size: nothing else is ever laid over them, so greedy and sampling calls of any shapes can
// take turns on one workspace without disturbing the words the cooperative walk keeps between calls.
constexpr int kCoopMaxTrees = 512;
size_t accept_coop_bytes() { return (size_t)kCoopMaxTrees * sizeof(TreeBlock); }

bool accept_coop_plan(int batch, int vocab, int cus, int* W, int* slice) {
  if (batch > kCoopMaxTrees) return false;
  int w = (2 * cus) / batch;
  if (w > 64) w = 64;
  if (w < 1) return false;
  const int sl = (vocab + w - 1) / w;
  if (sl > 4096) return false;  // 4096 doubles of LDS and 16 slice elements per thread
  *W = w;
  *slice = sl;
  return true;
}

hipError_t launch_accept_coop(const AcceptArgs& a, void* coop_ws, int W, int slice, hipStream_t stream) {
  CoopParams cp;
  cp.err = static_cast<unsigned*>(a.workspace);
  cp.n_tree = a.n_tree; cp.vocab = a.vocab; cp.max_depth = a.max_depth; cp.W = W; cp.slice = slice;
  cp.inv_temp = 1.0 / (double)a.temperature;
  cp.tokens = a.tokens; cp.parent = a.parent;
  cp.logits = a.logits; cp.draft = a.draft_probs; cp.uniforms = a.uniforms;
  cp.draft_row = a.draft_row; cp.n_draft_rows = a.n_draft_rows;
  cp.trees = static_cast<TreeBlock*>(coop_ws);
  cp.spin_limit = tuning().spin_limit >= 0 ? (unsigned)tuning().spin_limit : kDefaultSpinLimit;
  cp.out_path = a.out_path; cp.out_len = a.out_len; cp.out_bonus = a.out_bonus;
  const size_t lds = (size_t)slice * sizeof(double);
  static LdsLimitRaised raised;
  if (hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(walk_sample_coop_kernel), 4096 * 8, raised); e != hipSuccess)
    return e;
  hipLaunchKernelGGL(walk_sample_coop_kernel, dim3(a.batch * W), dim3(kCoopThreads), lds, stream, cp);
  return hipGetLastError();
}

// Calibration: a pure 128-bit streaming read of `bytes` bytes (nothing is computed or written
// unless the data happen to hash to a magic value), the ceiling any HBM-bound kernel of the same
// size can be compared with.
typedef unsigned int probe_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_read_kernel(const probe_u32x4* __restrict__ src, size_t n_chunks,
                                                          unsigned* sink) {
  probe_u32x4 acc = {0u, 0u, 0u, 0u};
  const size_t stride = (size_t)gridDim.x * 256;
#pragma unroll 4
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_chunks; i += stride) acc += src[i];
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) sink[0] = acc.x;
}
hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t stream) {
  const size_t n = bytes / 16;
  if (n == 0) return hipSuccess;
  const unsigned grid = (unsigned)((n + 1023) / 1024 < 16384 ? (n + 1023) / 1024 : 16384);  // ~4 chunks per thread
  hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(256), 0, stream, static_cast<const probe_u32x4*>(src), n,
                     static_cast<unsigned*>(sink));
  return hipGetLastError();
}

// zero fill as a kernel (safe inside HIP-graph capture, unlike a memset node)
__global__ void zero_fill_kernel(unsigned long long* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0ull;
}
hipError_t launch_zero_fill(void* p, size_t bytes, hipStream_t stream) {
  const size_t n = bytes / 8;
  if (n == 0) return hipSuccess;
  const unsigned grid = (unsigned)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
  hipLaunchKernelGGL(zero_fill_kernel, dim3(grid), dim3(256), 0, stream, static_cast<unsigned long long*>(p), n);
  return hipGetLastError();
}

}  // namespace jk
