// C-ABI entry points of libjakiro_verify: argument checks, launch planning,
// kernel launches.  No device memory is allocated here and nothing synchronises.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <initializer_list>

#include "jk_internal.h"

namespace jk {

int device_cu_count() {
  static int cus = 0;  // same value whoever writes it first
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      cus = 256;
  }
  return cus;
}

namespace {
int env_int(const char* name, int fallback) {
  const char* e = std::getenv(name);
  return e && *e ? std::atoi(e) : fallback;
}
Tuning tuning_from_env() {
  Tuning t;
  t.attn_wm = env_int("JK_ATTN_WM", 0);
  t.attn_wn = env_int("JK_ATTN_WN", 0);
  t.attn_splits = env_int("JK_ATTN_SPLITS", 0);
  t.attn_fused = env_int("JK_ATTN_FUSED", -1);
  t.attn_deep = env_int("JK_ATTN_DEEP", -1);
  t.accept_single = env_int("JK_ACCEPT_SINGLE", 0);
  t.spin_limit = env_int("JK_SPIN_LIMIT", -1);
  t.verbose = env_int("JK_ATTN_VERBOSE", 0);
  return t;
}
}  // namespace

Tuning& tuning() {
  static Tuning t = tuning_from_env();  // the environment is read once, here
  return t;
}

namespace {
constexpr int kMaxDevices = 64;
int g_xcd_state[kMaxDevices];  // per device: 0 not checked (jk_init not called), 1 round-robin verified, 2 not round-robin
}  // namespace

bool xcd_placement_verified() {
  int dev = -1;
  return hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices && g_xcd_state[dev] == 1;
}

namespace {
bool desc_ok(const jk_attn_desc& d) {
  if (d.batch < 1 || d.n_tree < 1 || d.n_tree > JK_MAX_TREE) return false;
  if (d.n_q_heads < 1 || d.n_kv_heads < 1 || d.n_q_heads % d.n_kv_heads) return false;
  if (d.dtype != JK_BF16 && d.dtype != JK_F32) return false;
  if (!(d.scale >= 0.f) || !std::isfinite(d.scale)) return false;
  return true;
}
bool shape_supported(const jk_attn_desc& d) {
  if (d.dtype == JK_BF16) return d.head_dim == 64 || d.head_dim == 128;
  return d.head_dim >= 4 && d.head_dim <= 256 && d.head_dim % 4 == 0;
}
}  // namespace

// Constants of the attention plan's time estimate, each measured on an MI355X at head_dim 128 with
// bench.py (forced plans through jk_set_tuning; the kernel's own time stamps in a -DJK_TIMING build):
struct PlanModel {
  double round_4x1 = 1.31;      // us per round (a pair of 32-key tiles) of a 4x1 workgroup alone on its CU: c3, 4 pairs in 5.26 us
  double round_2x2 = 0.95;      // us per round (one tile per key column) of a 2x2 workgroup: c2 sweep of split counts
  double share2_4x1 = 1.58;     // two 4x1 workgroups on one CU take this many times one's time: c5, 1 against 2 per CU
  double share_2x2_slope = 0.75;  // 2x2 workgroups sharing a CU: time x (0.75 per workgroup + 0.25): c7 and c4 sweeps
  double cu_pull = 22.0e3;      // bytes per us one CU draws from HBM with one round in flight (32 KB / 1.3 us round trip)
  double stream = 4.0e6;        // bytes per us all CUs together: c4, 178 MB per call
  double startup = 2.7;         // us before a workgroup's first K/V data are there (c3 time stamps: 2.6 - 2.8); with two
                                // workgroups on a CU one's start hides under the other's loop (c7: 4 splits beat 2)
  double merge_fused_fixed = 2.0, merge_fused_per_mb = 0.1;   // merge inside the kernel: c3 time stamps, xchg probe
  double merge_kernel_fixed = 3.0, merge_kernel_per_mb = 0.28, merge_kernel_per_mb_busy = 0.4;  // second launch: c3/c2/c5 traces
};

bool make_attn_plan(const jk_attn_desc& d, int max_prefix_len, bool fused_allowed, AttnPlan* pl) {
  static const PlanModel km;
  if (!desc_ok(d) || !shape_supported(d) || max_prefix_len < 0 || max_prefix_len > (1 << 24)) return false;
  const int G = d.n_q_heads / d.n_kv_heads;
  pl->m_rows = d.n_tree * G;
  const long long units = (long long)d.batch * d.n_kv_heads;
  if (d.dtype == JK_BF16) {
    // Candidates: 4x1 or 2x2 waves (32-row blocks x key interleave) per workgroup.  Fewer
    // rows per workgroup means more workgroups per KV head without more KV splits: the K/V
    // stream is then re-read by the row tiles (from L2, they run side by side on one XCD)
    // instead of partial outputs being written and read back once per split.
    const int n_tiles = (max_prefix_len + kTileKeys - 1) / kTileKeys + (d.n_tree + kTileKeys - 1) / kTileKeys;
    const double kv_bytes = 2.0 * (max_prefix_len + d.n_tree) * d.head_dim * 2.0;
    const int slots = device_cu_count();  // one workgroup per CU measured best (partials cost more than idle slots)
    const Tuning& tn = tuning();
    const int forced_wm = tn.attn_wm, forced_wn = tn.attn_wn, forced_s = tn.attn_splits;  // tuning overrides
    const int fused_mode = !fused_allowed ? 0 : tn.attn_fused;  // 0 never, 1 whenever possible, -1 when it pays
    static const int kArr[][2] = {{2, 2}, {4, 1}};  // waves along rows x along keys
    bool forced_ok = false;
    for (const auto& a : kArr) forced_ok |= (a[0] == forced_wm && a[1] == forced_wn);
    double best_cost = 0.0;
    bool have = false;
    for (const auto& a : kArr) {
      const int wm = a[0], wn = a[1];
      if (forced_ok ? (wm != forced_wm || wn != forced_wn) : (wm > 2 && pl->m_rows <= 16 * wm)) continue;  // mostly padding rows
      const int q_rows = 32 * wm;
      const int n_qtiles = (pl->m_rows + q_rows - 1) / q_rows;
      const long long wgs = units * n_qtiles;
      const int kt = wn == 1 ? 2 : 1;  // a lone key column pairs its tiles (hand-pipelined two-tile path)
      const int max_by_tiles = n_tiles / (2 * wn * kt) > 0 ? n_tiles / (2 * wn * kt) : 1;  // >= 2 rounds per split
      // every split count that leaves a split at least two rounds is priced
      const long long s_top = forced_s >= 1 && forced_s <= kMaxSplits ? 1 : (max_by_tiles < kMaxSplits ? max_by_tiles : kMaxSplits);
      for (long long sc = 1; sc <= s_top; ++sc) {
        long long s = sc;
        if (forced_s >= 1 && forced_s <= kMaxSplits) s = forced_s;
        // a split's tiles stay within what a workgroup can keep page ids for (paged caches)
        const long long s_min = (n_tiles + kMaxTilesPerSplit - 1) / kMaxTilesPerSplit;
        if (s < s_min) s = s_min;
        if (s > kMaxSplits) continue;
        // Estimated time of a call, in microseconds, from what was measured on an MI355X at
        // head_dim 128: a workgroup runs a round (2 tiles per key column) in about 0.95 us as
        // 2x2 waves and 1.33 us as 4x1 waves (which cover twice the rows, hand-pipelined);
        // workgroups beyond one per CU share its throughput; the K/V stream (re-read from L2
        // by the row tiles at a quarter of the price) moves at about 4 TB/s while every CU
        // pulls, so CUs with one workgroup more than the average stretch it; partial outputs
        // (bf16, written, flushed at the kernel boundary and read back) cost about 0.28 us per MB.
        const double t_round = (wn == 1 ? km.round_4x1 : km.round_2x2) * d.head_dim / 128.0;
        // rounds of the longest split: the 4x1 arrangement deals tiles (an odd last tile costs about
        // half a round), the 2x2 arrangement whole rounds
        double rounds;
        if (wn == 1) {
          // (the kernel's own dealing: full prefix tiles evenly, a lone last tile a little over half a
          // pair; the tail - two full tiles a tile - with the last split)
          const long long F = max_prefix_len / kTileKeys, tail = n_tiles - F;
          auto pairs_of = [](long long tiles) { return 0.5 * (double)(tiles / 2 * 2) + ((tiles & 1) ? 0.55 : 0.0); };
          if (s == 1) {
            rounds = pairs_of(F) + 1.07 * (double)tail;
          } else {
            const long long per = (F + 2 * tail + s - 1) / s;
            long long f_last = per - 2 * tail;
            f_last = (f_last < 0 ? 0 : (f_last > F ? F : f_last)) & ~1LL;
            const long long rest = F - f_last, most = (rest + s - 2) / (s - 1);
            const double last = pairs_of(f_last) + 1.07 * (double)tail;
            rounds = pairs_of(most) > last ? pairs_of(most) : last;
          }
        } else {
          rounds = (double)(((n_tiles + wn * kt - 1) / (wn * kt) + s - 1) / s);
        }
        const double per_cu = (double)(wgs * s) / slots;
        // 4x1 workgroups that share a CU overlap each other's matrix and vector phases: two of
        // them take 1.58 times one's time (measured on c5), plus a part of a workgroup of tail
        const double share =
            per_cu > 1.0 ? (wn == 1 ? 0.5 * km.share2_4x1 * (per_cu + 0.3 > 2.0 ? per_cu + 0.3 : 2.0)
                                    : km.share_2x2_slope * per_cu + (1.0 - km.share_2x2_slope))
                         : 1.0;
        const double imbalance = per_cu > 1.0 ? std::ceil(per_cu) / per_cu : 1.0;
        const double loop_us = rounds * t_round * share;
        // (a CU pulls about 22 GB/s on its own: fewer workgroups than CUs stream slower than 4 TB/s)
        const double active = (double)(wgs * s < slots ? wgs * s : slots);
        const double rate = active * km.cu_pull < km.stream ? active * km.cu_pull : km.stream;  // bytes per microsecond
        const double stream_us = imbalance * (double)units * kv_bytes * (1.0 + 0.25 * (n_qtiles - 1)) / rate;
        // Merge inside the kernel: possible when every workgroup is resident at once (here: at most
        // one per CU, or two when forced) and the workgroup numbering puts all splits of a (unit, row
        // tile) group on one XCD: logical ids are dealt to the 8 XCDs in contiguous ranges of
        // total / 8, and a unit's ids are contiguous, so every unit's range must sit inside one.
        // (and one thread per (row of a slice, split padded to a power of two); partials below 2^31 bytes)
        int s_pow2 = 1;
        while (s_pow2 < s) s_pow2 *= 2;
        bool can_fuse = fused_mode != 0 && s > 1 && wgs <= kMaxFusedGroups &&
                        ((q_rows + s - 1) / s) * s_pow2 <= 64 * wm * wn &&
                        (double)units * s * n_qtiles * q_rows * d.head_dim * 2.0 < 2.0e9 &&
                        wgs * s <= (long long)slots * 2;  // (two of these workgroups fit a CU: all resident)
        if (can_fuse) {
          const long long per_unit = s * n_qtiles, per_xcd = (wgs * s + 7) / 8;
          for (long long u = 0; u < units && can_fuse; ++u)
            can_fuse = (u * per_unit) / per_xcd == ((u + 1) * per_unit - 1) / per_xcd;
        }
        // Partials (bf16): merged inside the kernel they are written once and read once through the XCD's L2
        // (about 2 us of exchange latency whatever their size plus 0.1 us per MB); with the stand-alone merge
        // kernel they cost a second launch (about 3 us) and 0.28 us per MB when the grid is one turn
        // of workgroups and they are stored through to memory, 0.4 when they take the ordinary route
        const double part_mb = 1.0e-6 * (double)units * s * pl->m_rows * d.head_dim * 2.0;
        const double partial_us =
            s <= 1 ? 0.0
            : can_fuse ? km.merge_fused_fixed + km.merge_fused_per_mb * part_mb
                       : km.merge_kernel_fixed + (per_cu > 1.0 && wn == 1 ? km.merge_kernel_per_mb_busy : km.merge_kernel_per_mb) * part_mb;
        // (near ties go to the count that gives every CU a workgroup: 2 % for an idle CU)
        // (measured for the 2x2 arrangement only; two 4x1 workgroups on a CU get in each other's way from the start: c3, 20 - 32 splits)
        const double start_us = km.startup * (wn == 2 && per_cu >= 1.5 ? 0.5 : 1.0);
        const double cost = ((loop_us > stream_us ? loop_us : stream_us) + partial_us + start_us) * (active < slots ? 1.02 : 1.0);
        if (!have || cost < best_cost) {
          have = true;
          best_cost = cost;
          pl->wm = wm; pl->wn = wn; pl->kt = kt; pl->q_rows = q_rows; pl->n_qtiles = n_qtiles; pl->splits = (int)s;
          pl->fused = can_fuse ? 1 : 0;
        }
      }
    }
    if (!have) return false;
    pl->m_pad = pl->n_qtiles * pl->q_rows;
    // The six-tile ring of the 2x2 arrangement: two rounds in flight for a workgroup that has its CU to itself
    // and a long way to stream (at least eight rounds: c6 59.3 -> 56.1 us); never where two workgroups may share
    // a CU, since only one with the deeper ring fits.
    {
      const long long all_wgs = units * pl->n_qtiles * pl->splits;
      const long long rounds_per_split = ((n_tiles + 1) / 2 + pl->splits - 1) / pl->splits;
      const bool fits = pl->wn == 2 && all_wgs <= slots;
      pl->deep = fits && (tn.attn_deep == 1 || (tn.attn_deep < 0 && rounds_per_split >= 8)) ? 1 : 0;
    }
  } else {
    pl->fused = 0;
    pl->deep = 0;
    pl->wm = pl->wn = pl->kt = 1;
    pl->q_rows = 1;
    pl->n_qtiles = pl->m_rows;
    pl->m_pad = pl->m_rows;
    const long long keys = (long long)max_prefix_len + d.n_tree;
    long long s = (keys + 1023) / 1024;  // each fp32 workgroup holds at most 1024 scores
    if (s > kMaxSplits) return false;  // fp32 path: at most 64 * 1024 keys
    pl->splits = (int)s;
  }
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  const size_t rows = (size_t)units * pl->splits * pl->m_pad;
  const bool need_parts = (d.dtype == JK_F32) || pl->splits > 1;
  pl->part_o_bytes = need_parts ? up(rows * d.head_dim * (d.dtype == JK_BF16 ? 2 : sizeof(float))) : 0;
  pl->part_ml_bytes = need_parts ? up(rows * sizeof(float2)) : 0;
  pl->total_bytes = kAttnHeaderBytes + pl->part_o_bytes + pl->part_ml_bytes;
  return true;
}

}  // namespace jk

using namespace jk;

extern "C" {

size_t jk_tree_verify_attention_workspace(const jk_attn_desc* desc, int32_t max_prefix_len) {
  // Whether the splits are merged inside the kernel depends on jk_init having verified the device,
  // and the two plans may cut the work differently: the size covers both, so that it is a function
  // of the descriptor and the bound alone.
  AttnPlan a, b;
  if (!desc || !make_attn_plan(*desc, max_prefix_len, false, &a) || !make_attn_plan(*desc, max_prefix_len, true, &b))
    return 0;
  return a.total_bytes > b.total_bytes ? a.total_bytes : b.total_bytes;
}

jk_status jk_tree_verify_attention_plan(const jk_attn_desc* desc, int32_t max_prefix_len, int32_t* plan_out) {
  if (!desc || !plan_out) return JK_ERR_INVALID_ARG;
  AttnPlan pl;
  if (!make_attn_plan(*desc, max_prefix_len, xcd_placement_verified(), &pl)) return JK_ERR_UNSUPPORTED;
  plan_out[0] = pl.wm; plan_out[1] = pl.wn; plan_out[2] = pl.kt; plan_out[3] = pl.n_qtiles;
  plan_out[4] = pl.splits; plan_out[5] = pl.fused;
  return JK_OK;
}

static jk_status attention_common(const jk_attn_desc* desc, const jk_paged_kv* pages, const void* q,
                                  const void* k_cache, const void* v_cache, const void* k_tree, const void* v_tree,
                                  const int32_t* parent, const int32_t* prefix_len, int32_t max_prefix_len, void* out,
                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!desc || !q || !k_tree || !v_tree || !parent || !prefix_len || !out) return JK_ERR_INVALID_ARG;
  if (max_prefix_len < 0) return JK_ERR_INVALID_ARG;
  if (max_prefix_len > 0 && (!k_cache || !v_cache)) return JK_ERR_INVALID_ARG;
  const jk_attn_desc& d = *desc;
  if (!desc_ok(d)) return JK_ERR_INVALID_ARG;
  if (!shape_supported(d)) return JK_ERR_UNSUPPORTED;
  const int64_t align = (d.dtype == JK_BF16) ? 8 : 4;
  const size_t es = (d.dtype == JK_BF16) ? 2 : 4;
  const int64_t strides[] = {d.q_stride_b, d.q_stride_t, d.q_stride_h, d.kc_stride_b, d.kc_stride_l,
                             d.kc_stride_h, d.kt_stride_b, d.kt_stride_t, d.kt_stride_h, d.o_stride_b,
                             d.o_stride_t, d.o_stride_h};
  for (int64_t s : strides)
    if (s < 0 || s % align) return JK_ERR_INVALID_ARG;
  if (d.q_stride_t < d.head_dim && d.n_tree > 1) return JK_ERR_INVALID_ARG;
  // the bf16 kernel addresses a tile's rows with 32-bit byte offsets from the tile's first row
  if (d.dtype == JK_BF16 && (d.kc_stride_l > (1 << 24) || d.kt_stride_t > (1 << 24))) return JK_ERR_UNSUPPORTED;
  const void* ptrs[] = {q, k_cache, v_cache, k_tree, v_tree, out};
  for (const void* p : ptrs)
    if (reinterpret_cast<uintptr_t>(p) % (align * es)) return JK_ERR_INVALID_ARG;
  if (pages) {
    if (d.dtype != JK_BF16) return JK_ERR_UNSUPPORTED;
    if (!pages->block_table || pages->page_size < 1 || pages->max_blocks < 1 || pages->n_pages < 1)
      return JK_ERR_INVALID_ARG;
    if (pages->page_size % kTileKeys) return JK_ERR_UNSUPPORTED;  // a page holds whole 32-key tiles
    if (pages->page_stride < 0 || pages->page_stride % align) return JK_ERR_INVALID_ARG;
    if ((long long)pages->max_blocks * pages->page_size < max_prefix_len) return JK_ERR_INVALID_ARG;
  }

  AttnPlan pl;
  if (!make_attn_plan(d, max_prefix_len, xcd_placement_verified(), &pl)) return JK_ERR_UNSUPPORTED;
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256) return JK_ERR_WORKSPACE;
  if (workspace_bytes < pl.total_bytes) return JK_ERR_WORKSPACE;
  if (tuning().verbose)
    std::fprintf(stderr, "jk attention plan: waves %dx%d, %d tile(s) per wave and round, %d row tile(s), %d split(s)%s%s\n",
                 pl.wm, pl.wn, pl.kt, pl.n_qtiles, pl.splits, pl.fused ? ", merged in the kernel" : "", pl.deep ? ", six-tile ring" : "");

  AttnArgs a;
  a.q = q; a.k_cache = k_cache; a.v_cache = v_cache; a.k_tree = k_tree; a.v_tree = v_tree;
  a.parent = parent; a.prefix_len = prefix_len; a.out = out;
  char* ws = static_cast<char*>(workspace);
  a.err = reinterpret_cast<unsigned*>(ws);
  a.sync = reinterpret_cast<unsigned*>(ws + kWsErrBytes);
  a.part_o = reinterpret_cast<float*>(ws + kAttnHeaderBytes);
  a.part_ml = reinterpret_cast<float2*>(ws + kAttnHeaderBytes + pl.part_o_bytes);
  a.d = d;
  a.max_prefix_len = max_prefix_len;
  a.block_table = pages ? pages->block_table : nullptr;
  a.max_blocks = pages ? pages->max_blocks : 0;
  a.page_size = pages ? pages->page_size : 0;
  a.n_pages = pages ? pages->n_pages : 0;
  a.page_stride = pages ? pages->page_stride : 0;
  const float scale = d.scale > 0.f ? d.scale : 1.0f / std::sqrt((float)d.head_dim);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (d.dtype == JK_BF16) {
    a.scale_log2 = scale * 1.44269504088896340736f;
    e = launch_tva_bf16(a, pl, stream);
    if (e == hipSuccess && pl.splits > 1 && !pl.fused) e = launch_tva_combine(a, pl, stream);
  } else {
    a.scale_log2 = scale;  // the fp32 path works in natural units
    e = launch_tva_f32(a, pl, stream);
    if (e == hipSuccess) e = launch_tva_combine(a, pl, stream);
  }
  return e == hipSuccess ? JK_OK : JK_ERR_HIP;
}

jk_status jk_tree_verify_attention(const jk_attn_desc* desc, const void* q, const void* k_cache,
                                   const void* v_cache, const void* k_tree, const void* v_tree,
                                   const int32_t* parent, const int32_t* prefix_len, int32_t max_prefix_len,
                                   void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return attention_common(desc, nullptr, q, k_cache, v_cache, k_tree, v_tree, parent, prefix_len, max_prefix_len, out,
                          workspace, workspace_bytes, hip_stream);
}

jk_status jk_tree_verify_attention_paged(const jk_attn_desc* desc, const jk_paged_kv* pages, const void* q,
                                         const void* k_pool, const void* v_pool, const void* k_tree,
                                         const void* v_tree, const int32_t* parent, const int32_t* prefix_len,
                                         int32_t max_prefix_len, void* out, void* workspace, size_t workspace_bytes,
                                         void* hip_stream) {
  if (!pages) return JK_ERR_INVALID_ARG;
  return attention_common(desc, pages, q, k_pool, v_pool, k_tree, v_tree, parent, prefix_len, max_prefix_len, out,
                          workspace, workspace_bytes, hip_stream);
}

size_t jk_accept_path_workspace(int32_t batch, int32_t n_tree, int32_t vocab, int32_t mode) {
  if (batch < 1 || n_tree < 1 || n_tree > JK_MAX_TREE || vocab < 1) return 0;
  if (mode != JK_GREEDY && mode != JK_SAMPLE) return 0;
  return accept_workspace_bytes(batch, n_tree, vocab, mode);
}

static jk_status accept_common(int32_t batch, int32_t n_tree, int32_t vocab, int32_t max_depth,
                               const int32_t* tree_tokens, const int32_t* parent, const float* target_logits,
                               int32_t mode, float temperature, const float* draft_probs, const int32_t* draft_row,
                               int64_t n_draft_rows, const float* uniforms, int32_t* out_path,
                               int32_t* out_accept_len, int32_t* out_bonus_token, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
  if (batch < 1 || vocab < 1 || max_depth < 1) return JK_ERR_INVALID_ARG;
  if (n_tree < 1) return JK_ERR_INVALID_ARG;
  if (n_tree > JK_MAX_TREE) return JK_ERR_UNSUPPORTED;
  if (mode != JK_GREEDY && mode != JK_SAMPLE) return JK_ERR_INVALID_ARG;
  if (!tree_tokens || !parent || !target_logits || !out_path || !out_accept_len || !out_bonus_token)
    return JK_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(target_logits) % 16) return JK_ERR_INVALID_ARG;
  if ((long long)batch * (n_tree + 1) > 65535) return JK_ERR_UNSUPPORTED;
  if (mode == JK_SAMPLE) {
    if (!draft_probs || !uniforms) return JK_ERR_INVALID_ARG;
    if (!(temperature > 0.f) || !std::isfinite(temperature)) return JK_ERR_INVALID_ARG;
    if (draft_row && n_draft_rows < 1) return JK_ERR_INVALID_ARG;
  }
  const size_t need = accept_workspace_bytes(batch, n_tree, vocab, mode);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256) return JK_ERR_WORKSPACE;
  if (workspace_bytes < need) return JK_ERR_WORKSPACE;
  AcceptArgs a;
  a.batch = batch; a.n_tree = n_tree; a.vocab = vocab; a.max_depth = max_depth; a.mode = mode;
  a.temperature = temperature;
  a.tokens = tree_tokens; a.parent = parent; a.logits = target_logits;
  a.draft_probs = draft_probs; a.uniforms = uniforms;
  a.draft_row = draft_row; a.n_draft_rows = n_draft_rows;
  a.out_path = out_path; a.out_len = out_accept_len; a.out_bonus = out_bonus_token;
  a.workspace = workspace;
  return launch_accept(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? JK_OK : JK_ERR_HIP;
}

jk_status jk_accept_path(int32_t batch, int32_t n_tree, int32_t vocab, int32_t max_depth,
                         const int32_t* tree_tokens, const int32_t* parent, const float* target_logits,
                         int32_t mode, float temperature, const float* draft_probs, const float* uniforms,
                         int32_t* out_path, int32_t* out_accept_len, int32_t* out_bonus_token, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  return accept_common(batch, n_tree, vocab, max_depth, tree_tokens, parent, target_logits, mode, temperature,
                       draft_probs, nullptr, 0, uniforms, out_path, out_accept_len, out_bonus_token, workspace,
                       workspace_bytes, hip_stream);
}

jk_status jk_accept_path_greedy_static(int32_t batch, int32_t n_tree, int32_t vocab, int32_t max_depth,
                                       const int32_t* tree_tokens, const int32_t* parent,
                                       const float* target_logits, int32_t* out_path, int32_t* out_accept_len,
                                       int32_t* out_bonus_token, void* hip_stream) {
  if (batch < 1 || vocab < 1 || max_depth < 1 || n_tree < 1) return JK_ERR_INVALID_ARG;
  if (n_tree > JK_MAX_TREE) return JK_ERR_UNSUPPORTED;
  if (!tree_tokens || !parent || !target_logits || !out_path || !out_accept_len || !out_bonus_token)
    return JK_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(target_logits) % 16) return JK_ERR_INVALID_ARG;
  if ((long long)batch * (n_tree + 1) > 65535) return JK_ERR_UNSUPPORTED;
  if (accept_greedy_static_bytes(batch, n_tree, vocab) > (size_t)JK_STATIC_SCRATCH_BYTES) return JK_ERR_SCRATCH_LIMIT;
  AcceptArgs a;
  a.batch = batch; a.n_tree = n_tree; a.vocab = vocab; a.max_depth = max_depth; a.mode = JK_GREEDY;
  a.temperature = 1.f;
  a.tokens = tree_tokens; a.parent = parent; a.logits = target_logits;
  a.draft_probs = nullptr; a.uniforms = nullptr; a.draft_row = nullptr; a.n_draft_rows = 0;
  a.out_path = out_path; a.out_len = out_accept_len; a.out_bonus = out_bonus_token;
  a.workspace = nullptr;
  return launch_accept_greedy_static(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? JK_OK : JK_ERR_HIP;
}

jk_status jk_accept_path_rows(int32_t batch, int32_t n_tree, int32_t vocab, int32_t max_depth,
                              const int32_t* tree_tokens, const int32_t* parent, const float* target_logits,
                              int32_t mode, float temperature, const float* draft_rows_all, int64_t n_draft_rows,
                              const int32_t* draft_row, const float* uniforms, int32_t* out_path,
                              int32_t* out_accept_len, int32_t* out_bonus_token, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  if (mode == JK_SAMPLE && !draft_row) return JK_ERR_INVALID_ARG;
  return accept_common(batch, n_tree, vocab, max_depth, tree_tokens, parent, target_logits, mode, temperature,
                       draft_rows_all, draft_row, n_draft_rows, uniforms, out_path, out_accept_len, out_bonus_token,
                       workspace, workspace_bytes, hip_stream);
}

static jk_status commit_common(const jk_attn_desc* desc, const jk_paged_kv* pages, int n_layers, const void* k_tree, const void* v_tree,
                               void* k_cache, void* v_cache, const int32_t* path, const int32_t* accept_len,
                               int32_t max_depth, int32_t cache_capacity, int32_t* prefix_len, int32_t advance,
                               void* hip_stream) {
  if (!desc || !k_tree || !v_tree || !k_cache || !v_cache || !path || !accept_len || !prefix_len)
    return JK_ERR_INVALID_ARG;
  const jk_attn_desc& d = *desc;
  if (d.batch < 1 || d.n_tree < 1 || d.n_tree > JK_MAX_TREE || d.n_kv_heads < 1 || d.head_dim < 1)
    return JK_ERR_INVALID_ARG;
  if (d.dtype != JK_BF16 && d.dtype != JK_F32) return JK_ERR_INVALID_ARG;
  if (max_depth < 1 || cache_capacity < 1) return JK_ERR_INVALID_ARG;
  if ((long long)d.batch * max_depth > 0x7fffffffLL || n_layers > 65535) return JK_ERR_UNSUPPORTED;
  const int64_t es = d.dtype == JK_BF16 ? 2 : 4;
  const int64_t align = 16 / es;  // elements per 16-byte chunk
  if (d.head_dim % align) return JK_ERR_UNSUPPORTED;
  const int64_t strides[] = {d.kc_stride_b, d.kc_stride_l, d.kc_stride_h, d.kt_stride_b, d.kt_stride_t, d.kt_stride_h};
  for (int64_t s : strides)
    if (s < 0 || s % align) return JK_ERR_INVALID_ARG;
  if (n_layers == 0) {  // (with several layers the tensor pointers live on the device and cannot be checked here)
    const void* ptrs[] = {k_tree, v_tree, k_cache, v_cache};
    for (const void* p : ptrs)
      if (reinterpret_cast<uintptr_t>(p) % 16) return JK_ERR_INVALID_ARG;
  }
  if (pages) {
    if (!pages->block_table || pages->page_size < 1 || pages->max_blocks < 1 || pages->n_pages < 1)
      return JK_ERR_INVALID_ARG;
    if (pages->page_stride < 0 || pages->page_stride % align) return JK_ERR_INVALID_ARG;
    if ((long long)pages->max_blocks * pages->page_size < cache_capacity) return JK_ERR_INVALID_ARG;
  }
  CommitArgs a;
  a.d = d;
  a.k_tree = k_tree; a.v_tree = v_tree; a.k_cache = k_cache; a.v_cache = v_cache;
  a.path = path; a.accept_len = accept_len; a.prefix_len = prefix_len;
  a.max_depth = max_depth; a.capacity = cache_capacity; a.advance = advance != 0;
  a.n_layers = n_layers;
  a.block_table = pages ? pages->block_table : nullptr;
  a.max_blocks = pages ? pages->max_blocks : 0;
  a.page_size = pages ? pages->page_size : 0;
  a.n_pages = pages ? pages->n_pages : 0;
  a.page_stride = pages ? pages->page_stride : 0;
  return launch_commit(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? JK_OK : JK_ERR_HIP;
}

jk_status jk_commit_path(const jk_attn_desc* desc, const void* k_tree, const void* v_tree, void* k_cache,
                         void* v_cache, const int32_t* path, const int32_t* accept_len, int32_t max_depth,
                         int32_t cache_capacity, int32_t* prefix_len, int32_t advance, void* hip_stream) {
  return commit_common(desc, nullptr, 0, k_tree, v_tree, k_cache, v_cache, path, accept_len, max_depth,
                       cache_capacity, prefix_len, advance, hip_stream);
}

jk_status jk_commit_path_layers(const jk_attn_desc* desc, int32_t n_layers, const void* const* k_tree,
                                const void* const* v_tree, void* const* k_cache, void* const* v_cache,
                                const int32_t* path, const int32_t* accept_len, int32_t max_depth,
                                int32_t cache_capacity, int32_t* prefix_len, int32_t advance, void* hip_stream) {
  if (n_layers < 1) return JK_ERR_INVALID_ARG;
  return commit_common(desc, nullptr, n_layers, k_tree, v_tree,
                       const_cast<void**>(reinterpret_cast<void* const*>(k_cache)),
                       const_cast<void**>(reinterpret_cast<void* const*>(v_cache)), path, accept_len, max_depth,
                       cache_capacity, prefix_len, advance, hip_stream);
}

jk_status jk_commit_path_layers_paged(const jk_attn_desc* desc, const jk_paged_kv* pages, int32_t n_layers,
                                      const void* const* k_tree, const void* const* v_tree, void* const* k_pool,
                                      void* const* v_pool, const int32_t* path, const int32_t* accept_len,
                                      int32_t max_depth, int32_t* prefix_len, int32_t advance, void* hip_stream) {
  if (n_layers < 1 || !pages) return JK_ERR_INVALID_ARG;
  const long long cap = (long long)pages->max_blocks * pages->page_size;
  return commit_common(desc, pages, n_layers, k_tree, v_tree,
                       const_cast<void**>(reinterpret_cast<void* const*>(k_pool)),
                       const_cast<void**>(reinterpret_cast<void* const*>(v_pool)), path, accept_len, max_depth,
                       (int32_t)(cap > 0x7fffffffLL ? 0x7fffffffLL : cap), prefix_len, advance, hip_stream);
}

size_t jk_draft_heads_workspace(int32_t rows, int32_t d_model, int32_t vocab) {
  if (rows < 1 || rows > 128 || d_model < 128 || d_model > 16384 || d_model % 128 || vocab < 1 ||
      vocab > (1 << 24))
    return 0;
  return draft_heads_workspace_bytes(rows, d_model, vocab);
}

jk_status jk_draft_heads(const jk_draft_heads_desc* desc, const void* f_top, const float* s_top,
                         const void* w_head, float* logits, float* draft_probs, int32_t* topk_tokens,
                         float* topk_probs, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!desc || !f_top || !s_top || !w_head || !logits || !topk_tokens || !topk_probs) return JK_ERR_INVALID_ARG;
  const jk_draft_heads_desc& d = *desc;
  if (d.rows < 1 || d.d_model < 1 || d.vocab < 1 || d.top_k < 1 || d.top_k > d.vocab) return JK_ERR_INVALID_ARG;
  if (d.mode != JK_HEADS_DECOUPLED && d.mode != JK_HEADS_CONTRASTIVE) return JK_ERR_INVALID_ARG;
  if (!(d.temperature > 0.f) || !std::isfinite(d.temperature)) return JK_ERR_INVALID_ARG;
  if (d.mode == JK_HEADS_CONTRASTIVE && (!std::isfinite(d.alpha) || !std::isfinite(d.beta))) return JK_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(f_top) % 16 || reinterpret_cast<uintptr_t>(w_head) % 16) return JK_ERR_INVALID_ARG;
  if (d.rows > 128 || d.d_model < 128 || d.d_model > 16384 || d.d_model % 128 || d.top_k > 16) return JK_ERR_UNSUPPORTED;
  if ((long long)2 * d.rows * d.vocab > 0x7fffffffLL * 4) return JK_ERR_UNSUPPORTED;
  if (d.vocab > (1 << 24)) return JK_ERR_UNSUPPORTED;
  const size_t need = draft_heads_workspace_bytes(d.rows, d.d_model, d.vocab);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < need) return JK_ERR_WORKSPACE;
  DraftHeadsArgs a;
  a.rows = d.rows; a.d_model = d.d_model; a.vocab = d.vocab; a.top_k = d.top_k; a.mode = d.mode;
  a.temperature = d.temperature; a.alpha = d.alpha; a.beta = d.beta;
  a.f_top = f_top; a.w_head = w_head; a.s_top = s_top;
  a.logits = logits; a.draft_probs = draft_probs; a.topk_probs = topk_probs; a.topk_tokens = topk_tokens;
  a.workspace = workspace;
  return launch_draft_heads(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? JK_OK : JK_ERR_HIP;
}

static bool moe_desc_ok(const jk_moe_desc& d) {
  return d.rows >= 1 && d.d_model >= 1 && d.d_ff >= 1 && d.n_experts >= 2;
}
static bool moe_desc_supported(const jk_moe_desc& d) {
  return d.rows <= 128 && d.d_model >= 128 && d.d_model <= 65536 && d.d_model % 128 == 0 && d.d_ff >= 128 &&
         d.d_ff <= 65536 && d.d_ff % 128 == 0 && d.n_experts <= 64;
}

size_t jk_moe_experts_workspace(const jk_moe_desc* desc) {
  if (!desc || !moe_desc_ok(*desc) || !moe_desc_supported(*desc)) return 0;
  return moe_experts_workspace_bytes(desc->rows, desc->d_model, desc->d_ff, desc->n_experts);
}

jk_status jk_moe_experts(const jk_moe_desc* desc, const void* u, const void* centroids, const void* w_gate,
                         const void* w_up, const void* w_down, void* f_top, float* s_top, int32_t* expert_idx,
                         void* f_mix, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!desc || !u || !centroids || !w_gate || !w_up || !w_down || !f_top || !s_top || !expert_idx)
    return JK_ERR_INVALID_ARG;
  if (!moe_desc_ok(*desc)) return JK_ERR_INVALID_ARG;
  for (const void* ptr : {u, centroids, w_gate, w_up, w_down, (const void*)f_top, (const void*)f_mix})
    if (reinterpret_cast<uintptr_t>(ptr) % 16) return JK_ERR_INVALID_ARG;
  if (!moe_desc_supported(*desc)) return JK_ERR_UNSUPPORTED;
  const size_t need = moe_experts_workspace_bytes(desc->rows, desc->d_model, desc->d_ff, desc->n_experts);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < need) return JK_ERR_WORKSPACE;
  MoeArgs a;
  a.rows = desc->rows; a.d_model = desc->d_model; a.d_ff = desc->d_ff; a.n_experts = desc->n_experts;
  a.u = u; a.centroids = centroids; a.w_gate = w_gate; a.w_up = w_up; a.w_down = w_down;
  a.f_top = f_top; a.f_mix = f_mix; a.s_top = s_top; a.expert_idx = expert_idx; a.workspace = workspace;
  return launch_moe_experts(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? JK_OK : JK_ERR_HIP;
}

static bool tree_state_ok(const jk_tree_state* s) {
  return s && s->tokens && s->parent && s->score && s->q_row && s->n_nodes && s->max_nodes >= 1;
}

jk_status jk_tree_grow(const jk_tree_state* state, int32_t batch, int32_t n_front, int32_t top_k, int32_t width,
                       int32_t q_row_base, const int32_t* frontier_in, const int32_t* cand_tokens,
                       const float* cand_probs, int32_t* frontier_out, void* hip_stream) {
  if (!tree_state_ok(state) || !cand_tokens || !cand_probs || !frontier_out) return JK_ERR_INVALID_ARG;
  if (batch < 1 || n_front < 1 || top_k < 1 || width < 1 || q_row_base < 0) return JK_ERR_INVALID_ARG;
  if (!frontier_in && n_front != 1) return JK_ERR_INVALID_ARG;
  if (state->max_nodes > tree_max_nodes() || (long long)n_front * 2 * top_k > 256 || width > 256 || batch > 65535)
    return JK_ERR_UNSUPPORTED;
  TreeGrowArgs a;
  a.batch = batch; a.n_front = n_front; a.top_k = top_k; a.width = width; a.max_nodes = state->max_nodes;
  a.q_row_base = q_row_base;
  a.tokens = state->tokens; a.parent = state->parent; a.q_row = state->q_row; a.n_nodes = state->n_nodes;
  a.score = state->score;
  a.frontier_in = frontier_in; a.cand_tok = cand_tokens; a.cand_p = cand_probs; a.frontier_out = frontier_out;
  return launch_tree_grow(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? JK_OK : JK_ERR_HIP;
}

jk_status jk_tree_grow_tail(const jk_tree_state* state, int32_t batch, int32_t n_front, int32_t top_k, int32_t k1,
                            int32_t k2, int32_t width, int32_t q_row_base, const int32_t* frontier_in,
                            const int32_t* cand_tokens, const float* cand_probs, void* hip_stream) {
  if (!tree_state_ok(state) || !cand_tokens || !cand_probs) return JK_ERR_INVALID_ARG;
  if (batch < 1 || n_front < 1 || top_k < 1 || k1 < 1 || k2 < 1 || k1 > top_k || k2 > top_k || width < 1 ||
      q_row_base < 0)
    return JK_ERR_INVALID_ARG;
  if (!frontier_in && n_front != 1) return JK_ERR_INVALID_ARG;
  if (state->max_nodes > tree_max_nodes() || (long long)n_front * k1 > 256 || (long long)width * k2 > 256 ||
      batch > 65535)
    return JK_ERR_UNSUPPORTED;
  TreeGrowArgs a;
  a.batch = batch; a.n_front = n_front; a.top_k = top_k; a.width = width; a.max_nodes = state->max_nodes;
  a.q_row_base = q_row_base;
  a.tokens = state->tokens; a.parent = state->parent; a.q_row = state->q_row; a.n_nodes = state->n_nodes;
  a.score = state->score;
  a.frontier_in = frontier_in; a.cand_tok = cand_tokens; a.cand_p = cand_probs; a.frontier_out = nullptr;
  return launch_tree_grow_tail(a, k1, k2, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? JK_OK : JK_ERR_HIP;
}

jk_status jk_tree_fill_static(const jk_tree_state* state, int32_t batch, int32_t n_front, int32_t top_k,
                              int32_t q_row_base, const int32_t* frontier_in, const int32_t* cand_tokens,
                              const float* cand_probs, const int32_t* shape_slot, const int32_t* shape_expert,
                              const int32_t* shape_rank, int32_t n_new, const int32_t* next_index, int32_t n_next,
                              int32_t* frontier_out, int32_t* new_ids, void* hip_stream) {
  if (!tree_state_ok(state) || !cand_tokens || !cand_probs || !shape_slot || !shape_expert || !shape_rank)
    return JK_ERR_INVALID_ARG;
  if (batch < 1 || n_front < 1 || top_k < 1 || n_new < 1 || n_next < 0 || q_row_base < 0) return JK_ERR_INVALID_ARG;
  if (!frontier_in && n_front != 1) return JK_ERR_INVALID_ARG;
  if (n_next > 0 && (!next_index || !frontier_out)) return JK_ERR_INVALID_ARG;
  if (state->max_nodes > tree_max_nodes() || n_new > 4096 || n_next > 4096 || batch > 65535) return JK_ERR_UNSUPPORTED;
  TreeGrowArgs a;
  a.batch = batch; a.n_front = n_front; a.top_k = top_k; a.width = n_next; a.max_nodes = state->max_nodes;
  a.q_row_base = q_row_base;
  a.tokens = state->tokens; a.parent = state->parent; a.q_row = state->q_row; a.n_nodes = state->n_nodes;
  a.score = state->score;
  a.frontier_in = frontier_in; a.cand_tok = cand_tokens; a.cand_p = cand_probs;
  a.frontier_out = n_next > 0 ? frontier_out : nullptr;
  return launch_tree_fill_static(a, shape_slot, shape_expert, shape_rank, n_new, next_index, n_next, new_ids,
                                 static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? JK_OK
             : JK_ERR_HIP;
}

jk_status jk_tree_finalize(const jk_tree_state* state, int32_t batch, int32_t n_keep, int32_t* tree_tokens,
                           int32_t* parent, int32_t* q_row, int32_t* old_index, int32_t* n_valid, void* hip_stream) {
  if (!tree_state_ok(state) || !tree_tokens || !parent || !q_row || !n_valid) return JK_ERR_INVALID_ARG;
  if (batch < 1 || n_keep < 1 || n_keep > state->max_nodes) return JK_ERR_INVALID_ARG;
  if (state->max_nodes > tree_max_nodes() || batch > 65535) return JK_ERR_UNSUPPORTED;
  TreeFinalArgs a;
  a.batch = batch; a.n_keep = n_keep; a.max_nodes = state->max_nodes;
  a.tokens = state->tokens; a.parent = state->parent; a.q_row = state->q_row; a.n_nodes = state->n_nodes;
  a.score = state->score;
  a.out_tokens = tree_tokens; a.out_parent = parent; a.out_q_row = q_row; a.out_old = old_index; a.n_valid = n_valid;
  return launch_tree_finalize(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? JK_OK : JK_ERR_HIP;
}

jk_status jk_gather_draft_probs(int32_t batch, int32_t n_tree, int32_t vocab, const float* q_all, int64_t n_q_rows,
                                const int32_t* q_row, float* draft_probs, void* hip_stream) {
  if (!q_all || !q_row || !draft_probs || batch < 1 || n_tree < 1 || vocab < 1 || n_q_rows < 1)
    return JK_ERR_INVALID_ARG;
  if ((long long)batch * n_tree > 0x7fffffffLL) return JK_ERR_UNSUPPORTED;
  return launch_gather_rows(q_all, q_row, draft_probs, (long long)batch * n_tree, vocab, n_q_rows,
                            static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? JK_OK
             : JK_ERR_HIP;
}

static bool linear_shape_ok(int32_t m, int32_t n, int32_t k) {
  return m >= 1 && m <= 256 && n >= 1 && k >= 128 && k % 128 == 0 && k <= (1 << 20) && n <= (1 << 24);
}

size_t jk_linear_workspace(int32_t m, int32_t n, int32_t k) {
  return linear_shape_ok(m, n, k) ? linear_workspace_bytes(m, n, k) : 0;
}

jk_status jk_linear(int32_t m, int32_t n, int32_t k, const void* x, const void* w, const void* residual,
                    void* out_bf16, float* out_f32, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!x || !w || (!out_bf16 && !out_f32) || m < 1 || n < 1 || k < 1) return JK_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(x) % 16 || reinterpret_cast<uintptr_t>(w) % 16) return JK_ERR_INVALID_ARG;
  if (!linear_shape_ok(m, n, k)) return JK_ERR_UNSUPPORTED;
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < linear_workspace_bytes(m, n, k))
    return JK_ERR_WORKSPACE;
  LinearArgs a;
  a.m = m; a.n = n; a.k = k; a.x = x; a.w = w; a.residual = residual; a.out_f32 = out_f32; a.out_bf16 = out_bf16;
  a.workspace = workspace;
  return launch_linear(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? JK_OK : JK_ERR_HIP;
}

jk_status jk_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256) return JK_ERR_WORKSPACE;
  return launch_zero_fill(workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? JK_OK
             : JK_ERR_HIP;
}

jk_status jk_stream_read_probe(const void* src, size_t bytes, void* sink, void* hip_stream) {
  if (!src || !sink || reinterpret_cast<uintptr_t>(src) % 16) return JK_ERR_INVALID_ARG;
  return launch_stream_read(src, bytes, sink, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? JK_OK
                                                                                                  : JK_ERR_HIP;
}

jk_status jk_init(void* hip_stream) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return JK_ERR_HIP;
  bool rr = false;
  if (probe_xcd_placement(static_cast<hipStream_t>(hip_stream), &rr) != hipSuccess) return JK_ERR_HIP;
  g_xcd_state[dev] = rr ? 1 : 2;
  return JK_OK;
}

jk_status jk_set_tuning(const char* name, int32_t value) {
  if (!name) return JK_ERR_INVALID_ARG;
  Tuning& t = tuning();
  const struct { const char* name; int* field; } table[] = {
      {"attn_wm", &t.attn_wm}, {"attn_wn", &t.attn_wn}, {"attn_splits", &t.attn_splits},
      {"attn_fused", &t.attn_fused}, {"attn_deep", &t.attn_deep}, {"accept_single", &t.accept_single}, {"spin_limit", &t.spin_limit},
      {"verbose", &t.verbose}};
  for (const auto& e : table)
    if (std::strcmp(name, e.name) == 0) {
      *e.field = value;
      return JK_OK;
    }
  return JK_ERR_INVALID_ARG;
}

int32_t jk_last_device_error(const void* workspace) {
  if (!workspace) return -1;
  unsigned word = 0;
  if (hipMemcpy(&word, workspace, sizeof(word), hipMemcpyDeviceToHost) != hipSuccess) return -1;
  return (int32_t)(word & 0x7fffffffu);
}

jk_status jk_validate_tree(const int32_t* parent_host, int32_t n_tree) {
  if (!parent_host || n_tree < 1 || n_tree > JK_MAX_TREE) return JK_ERR_INVALID_ARG;
  for (int32_t i = 0; i < n_tree; ++i)
    if (parent_host[i] < -1 || parent_host[i] >= i) return JK_ERR_BAD_TREE;
  return JK_OK;
}

const char* jk_status_string(int32_t status) {
  switch (status) {
    case JK_OK: return "ok";
    case JK_ERR_INVALID_ARG: return "invalid argument";
    case JK_ERR_BAD_TREE: return "parent[] violates -1 <= parent[i] < i";
    case JK_ERR_UNSUPPORTED: return "unsupported shape";
    case JK_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case JK_ERR_HIP: return "HIP runtime error";
    case JK_ERR_SCRATCH_LIMIT: return "input too large for the library's built-in scratch buffer";
    default: return "unknown status";
  }
}

const char* jk_version(void) { return "0.1"; }

}  // extern "C"
