// Commit of the accepted path to the KV cache of one layer (gfx950).
//
// What it computes (Section 2.1 step 3 of the paper: accepted tokens are
// appended to the sequence, the rest of the draft is dropped): the key/value
// rows of the accepted tree nodes, in path order, become the next rows of the
// cache.  A plain gather-copy: one workgroup per (layer, sequence, path
// position) moves that node's K and V rows of all KV heads with 16-byte
// accesses; the layers of a model go in one launch (the copy is a few tens of
// KB per layer, so a launch per layer would cost more than the copies).  The
// prefix length is advanced by a second, tiny kernel, because every workgroup
// of the first still reads the old value.
#include "jk_internal.h"

namespace jk {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct CommitParams {
  const unsigned char *kt, *vt;    // one layer: the tensors; several layers: device arrays of n_layers pointers
  unsigned char *kc, *vc;
  const int32_t *path, *accept_len;
  int32_t* prefix_len;
  int T, Hkv, max_depth, capacity;
  int row_chunks;                  // 16-byte chunks per (node, KV head) row
  long long kc_sb, kc_sl, kc_sh, kt_sb, kt_st, kt_sh;  // strides in bytes
  // paged caches: kc / vc are page pools and position t of sequence b lives in page
  // block_table[b * max_blocks + t / page_size], slot t % page_size
  const int32_t* block_table;
  int max_blocks, page_size, n_pages;
  long long page_sb;  // page stride in bytes
};

// rows of sequence b that are committed: accept_len cut to [0, max_depth], ended in front of
// the first node id outside [0, T), and limited to the room left in the cache
__device__ __forceinline__ int committed_rows(const CommitParams& p, int b, int L) {
  int n = p.accept_len[b];
  n = n < 0 ? 0 : (n > p.max_depth ? p.max_depth : n);
  for (int i = 0; i < n; ++i) {
    const int node = p.path[(long long)b * p.max_depth + i];
    if (node < 0 || node >= p.T) { n = i; break; }
  }
  const int room = p.capacity - L;
  return n < room ? n : (room > 0 ? room : 0);
}

// grid: x = sequence * max_depth + path position, y = layer
template <bool LAYERS>
__global__ __launch_bounds__(256) void commit_rows_kernel(CommitParams p) {
  const int b = blockIdx.x / p.max_depth, i = blockIdx.x % p.max_depth;
  int L = p.prefix_len[b];
  L = L < 0 ? 0 : L;
  if (i >= committed_rows(p, b, L)) return;
  const int node = p.path[(long long)b * p.max_depth + i];
  const unsigned char *kt = p.kt, *vt = p.vt;
  unsigned char *kc = p.kc, *vc = p.vc;
  if (LAYERS) {
    kt = reinterpret_cast<const unsigned char* const*>(p.kt)[blockIdx.y];
    vt = reinterpret_cast<const unsigned char* const*>(p.vt)[blockIdx.y];
    kc = reinterpret_cast<unsigned char* const*>(p.kc)[blockIdx.y];
    vc = reinterpret_cast<unsigned char* const*>(p.vc)[blockIdx.y];
  }
  const unsigned char* ks = kt + b * p.kt_sb + node * p.kt_st;
  const unsigned char* vs = vt + b * p.kt_sb + node * p.kt_st;
  long long dst = b * p.kc_sb + (long long)(L + i) * p.kc_sl;
  if (p.block_table) {
    const int pos = L + i, pi = pos / p.page_size;  // pi < max_blocks: pos < capacity <= max_blocks * page_size
    int page = p.block_table[(long long)b * p.max_blocks + pi];
    page = page < 0 ? 0 : (page >= p.n_pages ? p.n_pages - 1 : page);
    dst = page * p.page_sb + (long long)(pos - pi * p.page_size) * p.kc_sl;
  }
  unsigned char* kd = kc + dst;
  unsigned char* vd = vc + dst;
  const int total = p.Hkv * p.row_chunks;
  for (int c = threadIdx.x; c < total; c += 256) {
    const int h = c / p.row_chunks, o = (c % p.row_chunks) * 16;
    const u32x4 kv = *reinterpret_cast<const u32x4*>(ks + h * p.kt_sh + o);
    const u32x4 vv = *reinterpret_cast<const u32x4*>(vs + h * p.kt_sh + o);
    *reinterpret_cast<u32x4*>(kd + h * p.kc_sh + o) = kv;
    *reinterpret_cast<u32x4*>(vd + h * p.kc_sh + o) = vv;
  }
}

__global__ void advance_len_kernel(CommitParams p, int batch) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= batch) return;
  int L = p.prefix_len[b];
  L = L < 0 ? 0 : L;
  p.prefix_len[b] = L + committed_rows(p, b, L);
}

}  // namespace

hipError_t launch_commit(const CommitArgs& a, hipStream_t stream) {
  const jk_attn_desc& d = a.d;
  const long long es = d.dtype == JK_BF16 ? 2 : 4;
  CommitParams p;
  p.kt = static_cast<const unsigned char*>(a.k_tree);
  p.vt = static_cast<const unsigned char*>(a.v_tree);
  p.kc = static_cast<unsigned char*>(a.k_cache);
  p.vc = static_cast<unsigned char*>(a.v_cache);
  p.path = a.path; p.accept_len = a.accept_len; p.prefix_len = a.prefix_len;
  p.T = d.n_tree; p.Hkv = d.n_kv_heads; p.max_depth = a.max_depth; p.capacity = a.capacity;
  p.row_chunks = (int)(d.head_dim * es / 16);
  p.kc_sb = d.kc_stride_b * es; p.kc_sl = d.kc_stride_l * es; p.kc_sh = d.kc_stride_h * es;
  p.kt_sb = d.kt_stride_b * es; p.kt_st = d.kt_stride_t * es; p.kt_sh = d.kt_stride_h * es;
  p.block_table = a.block_table; p.max_blocks = a.max_blocks; p.page_size = a.page_size; p.n_pages = a.n_pages;
  p.page_sb = a.page_stride * es;
  const dim3 grid((unsigned)(d.batch * a.max_depth), (unsigned)(a.n_layers > 0 ? a.n_layers : 1));
  if (a.n_layers > 0)
    hipLaunchKernelGGL(commit_rows_kernel<true>, grid, dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL(commit_rows_kernel<false>, grid, dim3(256), 0, stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !a.advance) return e;
  hipLaunchKernelGGL(advance_len_kernel, dim3((unsigned)((d.batch + 255) / 256)), dim3(256), 0, stream, p, d.batch);
  return hipGetLastError();
}

}  // namespace jk
