// dam_kv_evict_plan, dam_kv_compact, dam_kv_remap_lists: KV-cache eviction for decode under
// pattern masks.
//
// Paper (arXiv 2506.11104): Sec. 2 notes that local attention patterns allow the KV cache to be
// evicted beyond the attention span; with the mask of Sec. 4.3 a row i of the pattern region keeps
// key j iff i - j is a matched diagonal or j is a matched column. For the query heads h of one KV
// head g, a cached key j <= p is therefore still attended by some row i >= p iff j is a matched
// column of such an h, or j >= p - r_max(g), r_max the largest matched diagonal of the group.
// The compacted cache of (sequence, g) holds the live columns first (ascending), then a ring of
// W_g = r_max + 1 rows in which key j sits at position j mod W_g, so that no row ever moves while
// the position advances: a new key overwrites the one that has just left the window.
// The layout, the kernels and the entry points are this library's own.
#include <math.h>

#include <algorithm>

#include "dam_internal.h"

namespace {
using namespace dam;

struct EvictArgs {
  int B, Hq, Hkv, P, pos, row_chunks;  // row_chunks: 16-byte pieces per K or V row
  int cap, ccap;
  int64_t kv_sb, kv_sh, kv_ss, c_sb, c_sh, c_ss;  // strides in 16-byte pieces
};

// The flag arrays are walked in chunks of kChunk columns, one workgroup per (chunk, KV head).
constexpr int kChunk = 4096;

__global__ void k_evict_init(int Hkv, int *__restrict__ window) {
  for (int g = threadIdx.x; g < Hkv; g += blockDim.x) window[g] = 0;
}

// Per KV head: W = 1 + largest matched diagonal of its query heads (maximum over the chunks), and per
// chunk the number of matched columns <= pos of their union.
__global__ __launch_bounds__(256) void k_evict_count(EvictArgs a, const uint8_t *__restrict__ diag_flag,
                                                     const uint8_t *__restrict__ vert_flag, int *__restrict__ window,
                                                     int *__restrict__ chunk_cnt) {
  __shared__ int s_max[4], s_cnt[4];
  const int chunk = blockIdx.x, g = blockIdx.y, G = a.Hq / a.Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int rmax = -1, n = 0;
  const int last = min(a.P - 1, a.pos);
  const int x_end = min(a.P, (chunk + 1) * kChunk);
  for (int x = chunk * kChunk + threadIdx.x; x < x_end; x += 256) {
    bool any_d = false, any_c = false;
    for (int q = 0; q < G; ++q) {
      any_d |= diag_flag[(int64_t)(g * G + q) * a.P + x] != 0;
      any_c |= vert_flag[(int64_t)(g * G + q) * a.P + x] != 0;
    }
    if (any_d) rmax = x;  // x grows with the loop
    if (any_c && x <= last) ++n;
  }
  for (int off = 32; off; off >>= 1) {
    rmax = max(rmax, __shfl_xor(rmax, off));
    n += __shfl_xor(n, off);
  }
  if (lane == 0) {
    s_max[wave] = rmax;
    s_cnt[wave] = n;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int w = max(max(s_max[0], s_max[1]), max(s_max[2], s_max[3])) + 1;
    if (w > 0) atomicMax(&window[g], w);  // an integer maximum: the order of the chunks does not matter
    chunk_cnt[g * gridDim.x + chunk] = (s_cnt[0] + s_cnt[1]) + (s_cnt[2] + s_cnt[3]);
  }
}

// Offsets of every chunk's columns (chunk_cnt becomes an exclusive prefix), col_ptr, rows, total.
__global__ void k_evict_offsets(int Hkv, int n_chunks, int *__restrict__ chunk_cnt, const int *__restrict__ window,
                                int *__restrict__ col_ptr, int *__restrict__ rows, int64_t *__restrict__ col_total) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  int64_t at = 0;
  for (int g = 0; g < Hkv; ++g) {
    col_ptr[g] = (int)at;
    for (int c = 0; c < n_chunks; ++c) {
      const int n = chunk_cnt[g * n_chunks + c];
      chunk_cnt[g * n_chunks + c] = (int)at;
      at += n;
    }
    if (rows) rows[g] = (int)(at - col_ptr[g]) + window[g];
  }
  col_ptr[Hkv] = (int)at;
  *col_total = at;
}

// The live columns of one chunk of one KV head, ascending, from the chunk's offset on. Thread t owns a
// contiguous stretch of the chunk.
__global__ __launch_bounds__(256) void k_evict_fill(EvictArgs a, const uint8_t *__restrict__ vert_flag,
                                                    const int *__restrict__ chunk_base, int *__restrict__ cols,
                                                    int64_t capacity) {
  __shared__ int s_wave[4];
  const int chunk = blockIdx.x, g = blockIdx.y, G = a.Hq / a.Hkv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_cols = min(a.P, a.pos + 1);
  constexpr int per = kChunk / 256;
  const int x0 = chunk * kChunk + threadIdx.x * per, x1 = min(n_cols, x0 + per);
  auto live = [&](int x) {
    bool any = false;
    for (int q = 0; q < G; ++q) any |= vert_flag[(int64_t)(g * G + q) * a.P + x] != 0;
    return any;
  };
  unsigned mine_bits = 0;  // the stretch is 16 columns long
  for (int x = x0; x < x1; ++x) mine_bits |= (live(x) ? 1u : 0u) << (x - x0);
  const int mine = __popc(mine_bits);
  int incl = mine;
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  int before = 0;
  for (int w = 0; w < wave; ++w) before += s_wave[w];
  int64_t at = (int64_t)chunk_base[g * gridDim.x + chunk] + before + incl - mine;
  while (mine_bits) {
    const int b = __ffs(mine_bits) - 1;
    mine_bits &= mine_bits - 1;
    if (at < capacity) cols[at] = x0 + b;
    ++at;
  }
}

// Gather of the live rows of (sequence b, KV head g) into the compacted caches: row s of the
// compacted cache is column cols[s] for s < n_col, else the key j of the window [pos - W + 1, pos]
// with j mod W == s - n_col. A row is moved by row_chunks adjacent lanes, 16 bytes each, K and V.
__global__ __launch_bounds__(256) void k_kv_compact(EvictArgs a, const int *__restrict__ window,
                                                    const int *__restrict__ col_ptr, const int *__restrict__ cols,
                                                    const uint4 *__restrict__ kc, const uint4 *__restrict__ vc,
                                                    uint4 *__restrict__ kd, uint4 *__restrict__ vd) {
  const int pair = blockIdx.y, b = pair / a.Hkv, g = pair % a.Hkv;
  const int n_col = col_ptr[g + 1] - col_ptr[g], W = window[g];
  const int n_rows = min(n_col + W, a.ccap);
  const int rows_per_block = 256 / a.row_chunks;
  const int sub = threadIdx.x % a.row_chunks;
  const int64_t src0 = (int64_t)b * a.kv_sb + (int64_t)g * a.kv_sh + sub;
  const int64_t dst0 = (int64_t)b * a.c_sb + (int64_t)g * a.c_sh + sub;
  for (int s = blockIdx.x * rows_per_block + threadIdx.x / a.row_chunks; s < n_rows; s += gridDim.x * rows_per_block) {
    int j;
    if (s < n_col) {
      j = cols[col_ptr[g] + s];
    } else {
      const int r = s - n_col;               // ring position
      j = a.pos - (a.pos - r) % W;            // the key <= pos congruent to r; negative: the slot is still empty
      if (a.pos < r) j = -1;
    }
    if (j < 0 || j >= a.cap) continue;
    kd[dst0 + (int64_t)s * a.c_ss] = kc[src0 + (int64_t)j * a.kv_ss];
    vd[dst0 + (int64_t)s * a.c_ss] = vc[src0 + (int64_t)j * a.kv_ss];
  }
}

// kept_idx (cache positions) -> rows of the compacted cache, list by list (one workgroup per
// (sequence, query head) list): a live column by its rank among the group's columns (binary search),
// any other key by its ring position.
__global__ __launch_bounds__(256) void k_remap_lists(EvictArgs a, const int *__restrict__ window,
                                                     const int *__restrict__ col_ptr, const int *__restrict__ cols,
                                                     const int *__restrict__ kept_ptr, const int *__restrict__ kept_idx,
                                                     int *__restrict__ kept_slot) {
  const int item = blockIdx.x, hq = item % a.Hq, g = hq / (a.Hq / a.Hkv);
  const int c0 = col_ptr[g], n_col = col_ptr[g + 1] - c0, W = window[g];
  const int64_t lo = kept_ptr[item], hi = kept_ptr[item + 1];
  for (int64_t e = lo + threadIdx.x; e < hi; e += 256) {
    const int j = kept_idx[e];
    int left = 0, right = n_col;  // first column >= j
    while (left < right) {
      const int mid = (left + right) >> 1;
      if (cols[c0 + mid] < j) left = mid + 1;
      else right = mid;
    }
    int slot;
    if (left < n_col && cols[c0 + left] == j) slot = left;
    else slot = W > 0 ? n_col + j % W : -1;
    kept_slot[e] = slot;
  }
}

int validate(const dam_evict_params *p) {
  if (!p) return DAM_ERR_INVALID_ARG;
  if (p->batch < 1 || p->hq < 1 || p->hkv < 1 || p->hq % p->hkv || p->n_flags < 1 || p->pos < 0) return DAM_ERR_INVALID_ARG;
  return DAM_OK;
}

int validate_caches(const dam_evict_params *p) {
  if (p->dtype != DAM_F32 && p->dtype != DAM_BF16) return DAM_ERR_UNSUPPORTED;
  const int elt = p->dtype == DAM_BF16 ? 2 : 4, per16 = 16 / elt;
  if (p->head_dim < 1 || (p->head_dim * elt) % 16 || p->head_dim * elt / 16 > 256) return DAM_ERR_UNSUPPORTED;
  if (p->kv_capacity < 1 || p->compact_capacity < 1 || p->pos >= p->kv_capacity) return DAM_ERR_INVALID_ARG;
  for (int x = 0; x < 3; ++x)
    if (p->kv_stride[x] < 0 || p->kv_stride[x] % per16 || p->compact_stride[x] < 0 || p->compact_stride[x] % per16)
      return DAM_ERR_INVALID_ARG;
  return DAM_OK;
}

EvictArgs make_args(const dam_evict_params *p, bool caches) {
  EvictArgs a = {};
  a.B = p->batch; a.Hq = p->hq; a.Hkv = p->hkv; a.P = p->n_flags; a.pos = p->pos;
  if (caches) {
    const int elt = p->dtype == DAM_BF16 ? 2 : 4, per16 = 16 / elt;
    a.row_chunks = p->head_dim * elt / 16;
    a.cap = p->kv_capacity; a.ccap = p->compact_capacity;
    a.kv_sb = p->kv_stride[0] / per16; a.kv_sh = p->kv_stride[1] / per16; a.kv_ss = p->kv_stride[2] / per16;
    a.c_sb = p->compact_stride[0] / per16; a.c_sh = p->compact_stride[1] / per16; a.c_ss = p->compact_stride[2] / per16;
  }
  return a;
}

}  // namespace

extern "C" size_t dam_kv_evict_workspace(const dam_evict_params *p) {
  if (validate(p) != DAM_OK) return 0;
  const size_t n_chunks = ((size_t)p->n_flags + kChunk - 1) / kChunk;
  return align_up((size_t)p->hkv * n_chunks * sizeof(int), 256);
}

extern "C" int dam_kv_evict_plan(const dam_evict_params *p, const uint8_t *diag_flag, const uint8_t *vert_flag,
                                 int32_t *window, int32_t *col_ptr, int32_t *cols, int64_t col_capacity,
                                 int32_t *rows, int64_t *col_total, void *ws, size_t ws_bytes, void *stream_v) {
  const int bad = validate(p);
  if (bad != DAM_OK) return bad;
  if (!diag_flag || !vert_flag || !window || !col_ptr || !col_total || col_capacity < 0) return DAM_ERR_INVALID_ARG;
  if (col_capacity > 0 && !cols) return DAM_ERR_INVALID_ARG;
  if (!ws || ws_bytes < dam_kv_evict_workspace(p)) return DAM_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream_v);
  const EvictArgs a = make_args(p, false);
  int *chunk_cnt = static_cast<int *>(ws);
  const int n_chunks = (p->n_flags + kChunk - 1) / kChunk;
  k_evict_init<<<1, 64, 0, st>>>(p->hkv, window);
  k_evict_count<<<dim3(n_chunks, p->hkv), 256, 0, st>>>(a, diag_flag, vert_flag, window, chunk_cnt);
  k_evict_offsets<<<1, 64, 0, st>>>(p->hkv, n_chunks, chunk_cnt, window, col_ptr, rows, col_total);
  if (cols && col_capacity > 0)
    k_evict_fill<<<dim3(n_chunks, p->hkv), 256, 0, st>>>(a, vert_flag, chunk_cnt, cols, col_capacity);
  return launch_status();
}

extern "C" int dam_kv_compact(const dam_evict_params *p, const int32_t *window, const int32_t *col_ptr,
                              const int32_t *cols, const void *kcache, const void *vcache, void *kcompact,
                              void *vcompact, void *stream_v) {
  int bad = validate(p);
  if (bad == DAM_OK) bad = validate_caches(p);
  if (bad != DAM_OK) return bad;
  if (!window || !col_ptr || !cols || !kcache || !vcache || !kcompact || !vcompact) return DAM_ERR_INVALID_ARG;
  const EvictArgs a = make_args(p, true);
  const int rows_per_block = 256 / a.row_chunks;
  const int blocks_x = std::max(1, std::min((p->compact_capacity + rows_per_block - 1) / rows_per_block,
                                            std::max(1, 2048 / (p->batch * p->hkv))));
  k_kv_compact<<<dim3(blocks_x, p->batch * p->hkv), 256, 0, static_cast<hipStream_t>(stream_v)>>>(
      a, window, col_ptr, cols, static_cast<const uint4 *>(kcache), static_cast<const uint4 *>(vcache),
      static_cast<uint4 *>(kcompact), static_cast<uint4 *>(vcompact));
  return launch_status();
}

extern "C" int dam_kv_remap_lists(const dam_evict_params *p, const int32_t *window, const int32_t *col_ptr,
                                  const int32_t *cols, const int32_t *kept_ptr, const int32_t *kept_idx,
                                  int32_t *kept_slot, void *stream_v) {
  const int bad = validate(p);
  if (bad != DAM_OK) return bad;
  if (!window || !col_ptr || !cols || !kept_ptr || !kept_idx || !kept_slot) return DAM_ERR_INVALID_ARG;
  const EvictArgs a = make_args(p, false);
  k_remap_lists<<<p->batch * p->hq, 256, 0, static_cast<hipStream_t>(stream_v)>>>(a, window, col_ptr, cols, kept_ptr, kept_idx,
                                                                                  kept_slot);
  return launch_status();
}
