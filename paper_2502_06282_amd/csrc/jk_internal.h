// Internal declarations shared by the library's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "jakiro_verify.h"

namespace jk {
// The dynamic-LDS limit of a kernel is an attribute it has per device: raised on a device's first launch of
// that kernel (idempotent, so a race between host threads is harmless).  `done` is the caller's static table.
struct LdsLimitRaised {
  bool on_device[64] = {};
};
inline hipError_t raise_lds_limit(const void* kernel, int bytes, LdsLimitRaised& done) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < 64;
  if (tracked && done.on_device[dev]) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && tracked) done.on_device[dev] = true;
  return e;
}
}  // namespace jk

namespace jk {

constexpr int kWaveSize = 64;
constexpr int kTileKeys = 32;      // keys per attention tile (one MFMA M-block)
constexpr int kMaxSplits = 64;     // upper bound on KV splits per (sequence, KV head)
constexpr int kMaxTilesPerSplit = 1024;  // so that a split's page ids (paged caches) fit a workgroup's LDS table

// How one attention call is cut into workgroups.  Derived on the host from the
// descriptor and the prefix bound only, so that the workspace query and the
// launch always agree.
struct AttnPlan {
  int wm;          // waves along the query-row axis (32 rows each)
  int wn;          // waves along the key axis (key columns of a round)
  int kt;          // consecutive 32-key tiles a wave takes per round (1 or 2)
  int q_rows;      // query rows per workgroup = 32 * wm
  int n_qtiles;    // workgroups along the query-row axis
  int m_rows;      // T * G query rows per KV head
  int m_pad;       // n_qtiles * q_rows
  int splits;      // KV splits
  int fused;       // bf16 path: the splits are merged inside the attention kernel (no second launch)
  int deep;        // bf16 path, 2x2 waves: the six-tile K/V ring (one workgroup per CU, two rounds in flight)
  size_t part_o_bytes, part_ml_bytes, total_bytes;  // total = header + partials
};

// Every attention and acceptance workspace starts with a header: 256 bytes whose first word is the
// sticky device error word (jk_last_device_error), then, in an attention workspace, one 64-byte line
// of synchronisation words per (unit, row tile) group for the merge inside the kernel.  The header
// must be zero before the first use of a workspace and is kept consistent by the calls themselves.
constexpr size_t kWsErrBytes = 256;
constexpr int kMaxFusedGroups = 508;
constexpr size_t kAttnHeaderBytes = kWsErrBytes + (size_t)kMaxFusedGroups * 64;  // 32 KiB
static_assert(kAttnHeaderBytes == JK_WORKSPACE_HEADER_BYTES, "public constant");

// Device error bits (public names in jakiro_verify.h)
constexpr unsigned kDevErrBadTree = 1u, kDevErrBadToken = 2u, kDevErrBadPage = 4u, kDevErrMergeWait = 8u,
                   kDevErrWalkWait = 16u;

// Overrides for experiments and tests (jk_set_tuning; seeded once from the JK_* environment
// variables when the library is loaded).  0 / -1 mean "let the library decide".
struct Tuning {
  int attn_wm = 0, attn_wn = 0, attn_splits = 0;
  int attn_fused = -1;     // -1 automatic, 0 never, 1 whenever the grid allows it
  int attn_deep = -1;      // six-tile K/V ring of the 2x2 arrangement: -1 automatic, 0 never, 1 whenever one workgroup per CU is planned
  int accept_single = 0;   // 1: one-workgroup sampling walk
  int spin_limit = -1;     // polls of the bounded waits (-1: default)
  int verbose = 0;
};
Tuning& tuning();

// whether this device places consecutive workgroups round-robin over its XCDs (checked by jk_init)
bool xcd_placement_verified();

bool make_attn_plan(const jk_attn_desc& d, int max_prefix_len, bool fused_allowed, AttnPlan* plan);

struct AttnArgs {
  const void *q, *k_cache, *v_cache, *k_tree, *v_tree;
  const int32_t* parent;
  const int32_t* prefix_len;
  void* out;
  float* part_o;    // [B*Hkv][splits][m_pad][D], fp32 (fp32 path) or bf16 (bf16 path)
  float2* part_ml;  // [B*Hkv][splits][m_pad]  (running max in log2 units, sum)
  unsigned* err;    // the workspace's device error word
  unsigned* sync;   // the workspace's group synchronisation words (merge inside the kernel)
  jk_attn_desc d;
  int max_prefix_len;
  float scale_log2;  // softmax scale * log2(e)
  // paged cache (bf16 path only): nullptr / 0 for a contiguous cache
  const int32_t* block_table;
  int max_blocks, page_size, n_pages;
  long long page_stride;
};

hipError_t launch_tva_bf16(const AttnArgs& a, const AttnPlan& p, hipStream_t stream);
hipError_t launch_tva_f32(const AttnArgs& a, const AttnPlan& p, hipStream_t stream);
hipError_t launch_tva_combine(const AttnArgs& a, const AttnPlan& p, hipStream_t stream);

struct AcceptArgs {
  int batch, n_tree, vocab, max_depth, mode;
  float temperature;
  const int32_t *tokens, *parent;
  const float *logits, *draft_probs, *uniforms;
  int32_t *out_path, *out_len, *out_bonus;
  void* workspace;
  // optional indirection: node k of sequence b uses row draft_row[b*n_tree + k] (clamped into
  // [0, n_draft_rows)) of draft_probs instead of row b*n_tree + k
  const int32_t* draft_row;
  long long n_draft_rows;
};
size_t accept_workspace_bytes(int batch, int n_tree, int vocab, int mode);
hipError_t launch_accept(const AcceptArgs& a, hipStream_t stream);
size_t accept_greedy_static_bytes(int batch, int n_tree, int vocab);
hipError_t launch_accept_greedy_static(const AcceptArgs& a, hipStream_t stream);
hipError_t probe_xcd_placement(hipStream_t stream, bool* round_robin);
int device_cu_count();

struct CommitArgs {
  jk_attn_desc d;
  const void *k_tree, *v_tree;
  void *k_cache, *v_cache;
  const int32_t *path, *accept_len;
  int32_t* prefix_len;
  int max_depth, capacity, advance;
  int n_layers;  // 0: the four pointers are the tensors; > 0: device arrays of that many tensor pointers
  // paged caches: nullptr / 0 for contiguous ones
  const int32_t* block_table;
  int max_blocks, page_size, n_pages;
  long long page_stride;
};
hipError_t launch_commit(const CommitArgs& a, hipStream_t stream);

// cooperative sampling walk (several workgroups per tree)
size_t accept_coop_bytes();
bool accept_coop_plan(int batch, int vocab, int cus, int* W, int* slice);
hipError_t launch_accept_coop(const AcceptArgs& a, void* coop_ws, int W, int slice, hipStream_t stream);
hipError_t launch_zero_fill(void* p, size_t bytes, hipStream_t stream);
hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t stream);

// draft head step (two heads over the shared output embedding)
struct DraftHeadsArgs {
  int rows, d_model, vocab, top_k, mode;
  float temperature, alpha, beta;
  const void *f_top, *w_head;
  const float* s_top;
  float *logits, *draft_probs, *topk_probs;
  int32_t* topk_tokens;
  void* workspace;
};
size_t draft_heads_workspace_bytes(int rows, int d_model, int vocab);
hipError_t launch_draft_heads(const DraftHeadsArgs& a, hipStream_t stream);

// router + expert MLPs of the draft layer
struct MoeArgs {
  int rows, d_model, d_ff, n_experts;
  const void *u, *centroids, *w_gate, *w_up, *w_down;
  void *f_top, *f_mix;
  float* s_top;
  int32_t* expert_idx;
  void* workspace;
};
size_t moe_experts_workspace_bytes(int rows, int d_model, int d_ff, int n_experts);
hipError_t launch_moe_experts(const MoeArgs& a, hipStream_t stream);

// draft tree growth
struct TreeGrowArgs {
  int batch, n_front, top_k, width, max_nodes, q_row_base;
  int32_t *tokens, *parent, *q_row, *n_nodes;  // state [batch][max_nodes], [batch]
  float* score;
  const int32_t* frontier_in;  // [batch][n_front] or null (the root)
  const int32_t* cand_tok;     // [batch*n_front][2][top_k]
  const float* cand_p;
  int32_t* frontier_out;       // [batch][width]
};
struct TreeFinalArgs {
  int batch, n_keep, max_nodes;
  const int32_t *tokens, *parent, *q_row, *n_nodes;
  const float* score;
  int32_t *out_tokens, *out_parent, *out_q_row, *out_old, *n_valid;
};
int tree_max_nodes();
hipError_t launch_tree_grow(const TreeGrowArgs& a, hipStream_t stream);
hipError_t launch_tree_grow_tail(const TreeGrowArgs& a, int k1, int k2, hipStream_t stream);
hipError_t launch_tree_fill_static(const TreeGrowArgs& a, const int* slot, const int* expert, const int* rank, int n_new,
                                   const int* next_index, int n_next, int* new_ids, hipStream_t stream);
hipError_t launch_tree_finalize(const TreeFinalArgs& a, hipStream_t stream);
hipError_t launch_gather_rows(const float* q_all, const int* q_row, float* out, long long n_nodes, int vocab,
                              long long n_q_rows, hipStream_t stream);

// plain linear layer on the skinny GEMM
struct LinearArgs {
  int m, n, k;
  const void *x, *w, *residual;
  float* out_f32;
  void* out_bf16;
  void* workspace;
};
size_t linear_workspace_bytes(int m, int n, int k);
hipError_t launch_linear(const LinearArgs& a, hipStream_t stream);

}  // namespace jk
