// dam_sparse_attn_decode: one query row per (sequence, query head) over an explicit kept-key list.
//
// Paper (arXiv 2506.11104): Sec. 3 (scaled dot-product attention) with the mask of Sec. 4.3 applied
// as -inf before the softmax; the kept list is row p of the head's mask.
//
// HBM-bound gather of 2 * head_dim * sizeof(T) bytes per kept key. A K or V row is read by LPR
// adjacent lanes with one 16-byte load each (a whole row per load instruction group, fully
// coalesced); every lane keeps 4 keys in flight. The kept list is split over several workgroups
// per head so that all 256 CUs stream; partial (max, sum, O) triples are merged by log-sum-exp.
// Workgroups are numbered so that all query heads sharing a KV head run on the same XCD and hit
// the same L2 for the rows their lists have in common. The grouped-query form (one merged list per
// KV head) takes the matrix-core kernel of dam_decode_mfma.hip for bf16 and head_dim 128, and the
// plain-ALU kernel here otherwise; both feed the same merge pass.
#include <hip/hip_bf16.h>
#include <math.h>

#include <algorithm>
#include <atomic>

#include "dam_internal.h"

namespace {
using namespace dam;

constexpr int kXcd = 8;
constexpr int kUnroll = 4;  // keys in flight per lane (K and V fragment each); 4 to 6 measured best at c5 (8: 4 % slower)

struct DecodeArgs {
  int B, Hq, Hkv, cap, splits, shared_lists;
  float scale;
  int64_t q_sb, q_sh, kv_sb, kv_sh, kv_ss, o_sb, o_sh;
};

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// 16 bytes that no other workgroup reads again (the grouped kernel reads every cached row once): a
// non-temporal load, so that the rows stream past the caches instead of displacing each other there
// (c5: 105 -> 98 us; the per-head kernel, whose heads share rows through L2, gains nothing from it).
__device__ __forceinline__ uint4 load_once(const void *p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// 16 bytes of a row, kept as loaded; dot() and axpy() interpret them.
template <typename T>
struct Frag;

template <>
struct Frag<float> {
  static constexpr int N = 4;  // elements per 16 bytes
  __device__ static float dot(const uint4 &a, const uint4 &b) {
    float d = __uint_as_float(a.x) * __uint_as_float(b.x);
    d = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), d);
    d = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), d);
    return fmaf(__uint_as_float(a.w), __uint_as_float(b.w), d);
  }
  __device__ static void axpy(float (&o)[4], float w, const uint4 &v) {
    o[0] = fmaf(w, __uint_as_float(v.x), o[0]);
    o[1] = fmaf(w, __uint_as_float(v.y), o[1]);
    o[2] = fmaf(w, __uint_as_float(v.z), o[2]);
    o[3] = fmaf(w, __uint_as_float(v.w), o[3]);
  }
};

template <>
struct Frag<__hip_bfloat16> {
  static constexpr int N = 8;
  // exact fp32 products of bf16 pairs, fp32 accumulation (v_dot2_f32_bf16)
  __device__ static float dot(const uint4 &a, const uint4 &b) {
    float d = 0.0f;
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.x), __builtin_bit_cast(bf16x2, b.x), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.y), __builtin_bit_cast(bf16x2, b.y), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.z), __builtin_bit_cast(bf16x2, b.z), d, false);
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.w), __builtin_bit_cast(bf16x2, b.w), d, false);
  }
  __device__ static void axpy(float (&o)[8], float w, const uint4 &v) {
    const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      o[2 * k] = fmaf(w, __uint_as_float(u[k] << 16), o[2 * k]);
      o[2 * k + 1] = fmaf(w, __uint_as_float(u[k] & 0xFFFF0000u), o[2 * k + 1]);
    }
  }
};

// Sum over the LPR adjacent lanes that share a row (LPR = 8, 16 or 32), on the DPP network.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}

template <int LPR>
__device__ __forceinline__ float row_sum(float d) {
  d += dpp_move<0xB1>(d);   // quad_perm [1,0,3,2]
  d += dpp_move<0x4E>(d);   // quad_perm [2,3,0,1]
  d += dpp_move<0x141>(d);  // row_half_mirror: the other quad of the 8
  if (LPR >= 16) d += dpp_move<0x140>(d);  // row_mirror: the other half of the 16
  if (LPR >= 32) d += __shfl_xor(d, 16);
  return d;
}

// A listed key outside the cache is pulled to its nearest row: the result is then wrong, but no
// address leaves the head's rows. Applied where the row address is formed, not where the index is
// fetched: there it would make the pass wait for the index load (and, the counter being in order,
// for the rows in flight before it).
__device__ __forceinline__ int in_cache(int row, int cap) { return min(max(row, 0), cap - 1); }

__device__ __forceinline__ void store_out(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_out(__hip_bfloat16 *p, float v) { *p = __float2bfloat16(v); }

// Partial result of one split: running max m, sum l (relative to m) and un-normalised O.
template <typename T, int D>
__global__ __launch_bounds__(256) void k_decode_partial(DecodeArgs a, const T *__restrict__ q,
                                                        const T *__restrict__ kc,
                                                        const T *__restrict__ vc,
                                                        const int *__restrict__ kept_ptr,
                                                        const int *__restrict__ kept_idx,
                                                        float *__restrict__ part_o,
                                                        float *__restrict__ part_ml, T *__restrict__ out,
                                                        float *__restrict__ lse) {
  constexpr int N = Frag<T>::N;        // elements per lane
  constexpr int LPR = D / N;           // lanes per row
  constexpr int GROUPS = 256 / LPR;    // rows in flight per pass of the block
  __shared__ float s_o[GROUPS][D];
  __shared__ float s_m[GROUPS], s_l[GROUPS];

  // XCD-aware numbering: block n runs on XCD n % 8; all splits and query heads of one
  // (sequence, KV head) pair are given ids with the same n % 8.
  const int G = a.Hq / a.Hkv;
  const int per_pair = G * a.splits;
  const int n_pairs = a.B * a.Hkv;
  const int n = blockIdx.x;
  const int xcd = n % kXcd, slot = n / kXcd;
  const int pair = (slot / per_pair) * kXcd + xcd;
  if (pair >= n_pairs) return;
  const int within = slot % per_pair;
  const int hq_in = within / a.splits, split = within % a.splits;
  const int b = pair / a.Hkv, hkv = pair % a.Hkv;
  const int hq = hkv * G + hq_in;
  const int item = b * a.Hq + hq;

  const int group = threadIdx.x / LPR, sub = threadIdx.x % LPR;
  const int list = a.shared_lists ? hq : item;  // one list per head for the whole batch, or one per (sequence, head)
  const int64_t lo = kept_ptr[list], hi = kept_ptr[list + 1];
  const int64_t len = hi - lo;
  const int64_t chunk = (len + a.splits - 1) / a.splits;
  const int64_t beg = lo + (int64_t)split * chunk;
  const int64_t end = std::min<int64_t>(hi, beg + chunk);

  const uint4 qf = *reinterpret_cast<const uint4 *>(q + b * a.q_sb + hq * a.q_sh + sub * N);
  const T *kb = kc + b * a.kv_sb + hkv * a.kv_sh + sub * N;
  const T *vb = vc + b * a.kv_sb + hkv * a.kv_sh + sub * N;
  const float sl2 = a.scale * 1.4426950408889634f;  // logits in log2 units

  float m = -INFINITY, l = 0.0f, o[N];
#pragma unroll
  for (int e = 0; e < N; ++e) o[e] = 0.0f;

  // The key indices of the next pass are fetched while the rows of the current one are in flight,
  // so that a pass costs one memory round trip, not two.
  int rows[kUnroll];
  int64_t p0 = beg + group * kUnroll;
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) rows[u] = p0 < end ? kept_idx[p0 + u < end ? p0 + u : p0] : 0;
  for (; p0 < end; p0 += GROUPS * kUnroll) {
    uint4 kf[kUnroll], vf[kUnroll];
    float s[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t row = in_cache(rows[u], a.cap);
      kf[u] = *reinterpret_cast<const uint4 *>(kb + row * a.kv_ss);
      vf[u] = *reinterpret_cast<const uint4 *>(vb + row * a.kv_ss);
    }
    const int64_t pn = p0 + GROUPS * kUnroll;
    if (pn < end) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) rows[u] = kept_idx[pn + u < end ? pn + u : pn];
    }
    float mx = m;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const float d = row_sum<LPR>(Frag<T>::dot(qf, kf[u]));
      s[u] = p0 + u < end ? d * sl2 : -INFINITY;
      mx = fmaxf(mx, s[u]);
    }
    const float corr = __builtin_amdgcn_exp2f(m - mx);  // m = -inf, mx finite -> 0; p0 < end guarantees mx finite
    l *= corr;
#pragma unroll
    for (int e = 0; e < N; ++e) o[e] *= corr;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const float w = __builtin_amdgcn_exp2f(s[u] - mx);
      l += w;
      Frag<T>::axpy(o, w, vf[u]);
    }
    m = mx;
  }

  // merge the groups of this block
  if (sub == 0) {
    s_m[group] = m;
    s_l[group] = l;
  }
#pragma unroll
  for (int e = 0; e < N; ++e) s_o[group][sub * N + e] = o[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float M = -INFINITY;
    for (int g = 0; g < GROUPS; ++g) M = fmaxf(M, s_m[g]);
    float Lsum = 0.0f, acc = 0.0f;
    if (M > -INFINITY)
      for (int g = 0; g < GROUPS; ++g) {
        const float w = exp2f(s_m[g] - M);
        Lsum += w * s_l[g];
        acc += w * s_o[g][threadIdx.x];
      }
    if (a.splits == 1) {  // the whole list was handled here: normalise and store, no merge pass
      store_out(out + b * a.o_sb + hq * a.o_sh + threadIdx.x, Lsum > 0.0f ? acc / Lsum : 0.0f);
      if (lse && threadIdx.x == 0)
        lse[item] = Lsum > 0.0f ? (M + log2f(Lsum)) * 0.6931471805599453f : -INFINITY;
    } else {
      const int64_t slot_out = (int64_t)item * a.splits + split;
      part_o[slot_out * D + threadIdx.x] = acc;
      if (threadIdx.x == 0) {
        part_ml[slot_out * 2] = M;
        part_ml[slot_out * 2 + 1] = Lsum;
      }
    }
  }
}

// Grouped-query form: one workgroup per (sequence, KV head, split) walks the merged list of the KV
// head's query heads; every listed K / V row is read once and enters the softmax state of exactly
// the heads whose member bit is set. A wave's 32 consecutive entries mostly belong to one run of the
// list (kept by several heads, or by one head only), so a head with no member bit in the wave's
// entries of a pass is skipped for the whole pass (wave-uniform branch).
template <typename T, int D, int GM>
__global__ __launch_bounds__(256) void k_decode_group(DecodeArgs a, const T *__restrict__ q,
                                                      const T *__restrict__ kc, const T *__restrict__ vc,
                                                      const int *__restrict__ kept_ptr,
                                                      const int *__restrict__ kept_idx,
                                                      const uint8_t *__restrict__ kept_member,
                                                      float *__restrict__ part_o, float *__restrict__ part_ml,
                                                      T *__restrict__ out, float *__restrict__ lse) {
  constexpr int N = Frag<T>::N;
  constexpr int LPR = D / N;
  constexpr int GROUPS = 256 / LPR;
  __shared__ float s_o[GROUPS][D];
  __shared__ float s_m[GROUPS], s_l[GROUPS];

  const int G = a.Hq / a.Hkv;  // <= GM
  const int split = blockIdx.x % a.splits, pair = blockIdx.x / a.splits;
  const int b = pair / a.Hkv, hkv = pair % a.Hkv;
  const int group = threadIdx.x / LPR, sub = threadIdx.x % LPR;
  const int list = a.shared_lists ? hkv : pair;
  // the splits take the list's blocks of GROUPS * kUnroll entries in turn, so that each gets its share of
  // every run (the run kept by several heads costs several times the arithmetic of the others)
  const int64_t end = kept_ptr[list + 1];
  const int64_t stride = (int64_t)a.splits * GROUPS * kUnroll;

  uint4 qf[GM];
#pragma unroll
  for (int x = 0; x < GM; ++x)
    qf[x] = x < G ? *reinterpret_cast<const uint4 *>(q + b * a.q_sb + (hkv * G + x) * a.q_sh + sub * N)
                  : uint4{0u, 0u, 0u, 0u};
  const T *kb = kc + b * a.kv_sb + hkv * a.kv_sh + sub * N;
  const T *vb = vc + b * a.kv_sb + hkv * a.kv_sh + sub * N;
  const float sl2 = a.scale * 1.4426950408889634f;

  float m[GM], l[GM], o[GM][N];
#pragma unroll
  for (int x = 0; x < GM; ++x) {
    m[x] = -INFINITY;
    l[x] = 0.0f;
#pragma unroll
    for (int e = 0; e < N; ++e) o[x][e] = 0.0f;
  }

  int rows[kUnroll];
  unsigned who[kUnroll];  // member bits; 0 past the end of the stretch
  int64_t p0 = kept_ptr[list] + ((int64_t)split * GROUPS + group) * kUnroll;
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const bool ok = p0 + u < end;
    rows[u] = p0 < end ? kept_idx[ok ? p0 + u : p0] : 0;
    who[u] = ok ? kept_member[p0 + u] : 0u;
  }
  for (; p0 < end; p0 += stride) {
    uint4 kf[kUnroll], vf[kUnroll];
    unsigned cur[kUnroll], anyone = 0;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t row = in_cache(rows[u], a.cap);
      kf[u] = load_once(kb + row * a.kv_ss);
      vf[u] = load_once(vb + row * a.kv_ss);
      cur[u] = who[u];
      anyone |= who[u];
    }
    const int64_t pn = p0 + stride;
    if (pn < end) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const bool ok = pn + u < end;
        rows[u] = kept_idx[ok ? pn + u : pn];
        who[u] = ok ? kept_member[pn + u] : 0u;
      }
    }
#pragma unroll
    for (int x = 0; x < GM; ++x) {
      if (x < G && __ballot((anyone >> x) & 1)) {  // some entry of this wave's pass is kept by head x
        float s[kUnroll];
        float mx = m[x];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          const float d = row_sum<LPR>(Frag<T>::dot(qf[x], kf[u]));
          s[u] = (cur[u] >> x) & 1 ? d * sl2 : -INFINITY;
          mx = fmaxf(mx, s[u]);
        }
        // a lane whose entries all belong to other heads, before its first own one: mx = -inf, state stays 0
        const float ref = mx == -INFINITY ? 0.0f : mx;
        const float corr = __builtin_amdgcn_exp2f(m[x] - ref);  // m = -inf -> 0
        l[x] *= corr;
#pragma unroll
        for (int e = 0; e < N; ++e) o[x][e] *= corr;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          const float w = __builtin_amdgcn_exp2f(s[u] - ref);
          l[x] += w;
          Frag<T>::axpy(o[x], w, vf[u]);
        }
        m[x] = mx;
      }
    }
  }

  // merge the row groups of this block, one head after the other through the same staging area
#pragma unroll
  for (int x = 0; x < GM; ++x) {
    if (x < G) {
      __syncthreads();
      if (sub == 0) {
        s_m[group] = m[x];
        s_l[group] = l[x];
      }
#pragma unroll
      for (int e = 0; e < N; ++e) s_o[group][sub * N + e] = o[x][e];
      __syncthreads();
      if (threadIdx.x < D) {
        const int hq = hkv * G + x;
        const int item = b * a.Hq + hq;
        float M = -INFINITY;
        for (int gI = 0; gI < GROUPS; ++gI) M = fmaxf(M, s_m[gI]);
        float Lsum = 0.0f, acc = 0.0f;
        if (M > -INFINITY)
          for (int gI = 0; gI < GROUPS; ++gI) {
            const float w = exp2f(s_m[gI] - M);  // a group that saw no key of this head: m = -inf, w = 0
            Lsum += w * s_l[gI];
            acc += w * s_o[gI][threadIdx.x];
          }
        if (a.splits == 1) {
          store_out(out + b * a.o_sb + hq * a.o_sh + threadIdx.x, Lsum > 0.0f ? acc / Lsum : 0.0f);
          if (lse && threadIdx.x == 0)
            lse[item] = Lsum > 0.0f ? (M + log2f(Lsum)) * 0.6931471805599453f : -INFINITY;
        } else {
          const int64_t slot_out = (int64_t)item * a.splits + split;
          part_o[slot_out * D + threadIdx.x] = acc;
          if (threadIdx.x == 0) {
            part_ml[slot_out * 2] = M;
            part_ml[slot_out * 2 + 1] = Lsum;
          }
        }
      }
    }
  }
}

template <typename T, int D>
__global__ void k_decode_merge(DecodeArgs a, const float *__restrict__ part_o,
                               const float *__restrict__ part_ml, T *__restrict__ out,
                               float *__restrict__ lse) {
  const int item = blockIdx.x;
  const int b = item / a.Hq, hq = item % a.Hq;
  const int t = threadIdx.x;
  float M = -INFINITY;
  for (int s = 0; s < a.splits; ++s) M = fmaxf(M, part_ml[((int64_t)item * a.splits + s) * 2]);
  float L = 0.0f, acc = 0.0f;
  if (M > -INFINITY)
    for (int s = 0; s < a.splits; ++s) {
      const int64_t at = (int64_t)item * a.splits + s;
      const float w = exp2f(part_ml[at * 2] - M);
      L += w * part_ml[at * 2 + 1];
      acc += w * part_o[at * D + t];
    }
  const float res = L > 0.0f ? acc / L : 0.0f;
  store_out(out + b * a.o_sb + hq * a.o_sh + t, res);
  if (lse && t == 0)
    lse[item] = L > 0.0f ? (M + log2f(L)) * 0.6931471805599453f : -INFINITY;
}

int pick_splits(int64_t items, int64_t max_kept) {
  // Enough workgroups to put two on every CU (512), each with at least 256 keys; one split (and no
  // merge pass) when the batch alone provides them.
  int64_t s = (512 + items - 1) / items;
  s = std::min<int64_t>(s, std::max<int64_t>(1, max_kept / 256));
  return (int)std::min<int64_t>(std::max<int64_t>(s, 1), 64);
}

// Splits of the grouped form, and whether the call takes the matrix-core kernel (one wave per
// workgroup: four per CU, each with at least two blocks of 32 entries).
int group_splits(const dam_decode_params *p, int64_t max_kept, bool *mfma) {
  const int64_t items = (int64_t)p->batch * p->hkv;
  *mfma = decode_group_mfma_fits(p);
  if (!*mfma) return pick_splits(items, max_kept);
  int64_t s = (1024 + items - 1) / items;
  s = std::min<int64_t>(s, std::max<int64_t>(1, max_kept / 64));
  return (int)std::min<int64_t>(std::max<int64_t>(s, 1), 64);
}

int validate(const dam_decode_params *p, const void *q, const void *kc, const void *vc,
             const int32_t *kept_ptr, const int32_t *kept_idx, int64_t max_kept, const void *out) {
  if (!p || !q || !kc || !vc || !kept_ptr || !out) return DAM_ERR_INVALID_ARG;
  if (p->batch < 1 || p->hq < 1 || p->hkv < 1 || p->hq % p->hkv || p->kv_capacity < 1) return DAM_ERR_INVALID_ARG;
  if (max_kept < 0 || (max_kept > 0 && !kept_idx)) return DAM_ERR_INVALID_ARG;
  if (p->dtype != DAM_F32 && p->dtype != DAM_BF16) return DAM_ERR_UNSUPPORTED;
  if (p->head_dim != 64 && p->head_dim != 128) return DAM_ERR_UNSUPPORTED;
  const int align = p->dtype == DAM_BF16 ? 8 : 4;  // elements per 16 bytes
  const int64_t strides[] = {p->q_stride[0], p->q_stride[1], p->kv_stride[0], p->kv_stride[1], p->kv_stride[2]};
  for (int64_t s : strides)
    if (s < 0 || s % align) return DAM_ERR_INVALID_ARG;
  if (p->o_stride[0] < 0 || p->o_stride[1] < 0) return DAM_ERR_INVALID_ARG;
  if (!(p->scale >= 0.0f)) return DAM_ERR_INVALID_ARG;
  return DAM_OK;
}

template <typename T, int D>
void launch(const DecodeArgs &a, const void *q, const void *kc, const void *vc, const int32_t *kept_ptr,
            const int32_t *kept_idx, void *out, float *lse, float *part_o, float *part_ml, hipStream_t st) {
  const int G = a.Hq / a.Hkv;
  const int n_pairs = a.B * a.Hkv;
  const int rounds = (n_pairs + kXcd - 1) / kXcd;
  const int blocks = rounds * kXcd * G * a.splits;
  k_decode_partial<T, D><<<blocks, 256, 0, st>>>(a, static_cast<const T *>(q), static_cast<const T *>(kc),
                                                static_cast<const T *>(vc), kept_ptr, kept_idx, part_o, part_ml,
                                                static_cast<T *>(out), lse);
  if (a.splits > 1) k_decode_merge<T, D><<<a.B * a.Hq, D, 0, st>>>(a, part_o, part_ml, static_cast<T *>(out), lse);
}

}  // namespace

extern "C" size_t dam_sparse_attn_decode_workspace(const dam_decode_params *p, int64_t max_kept) {
  if (!p || p->batch < 1 || p->hq < 1 || p->head_dim < 1 || max_kept < 0) return 0;
  const int splits = pick_splits((int64_t)p->batch * p->hq, max_kept);
  Carver c(nullptr);
  c.take<float>((size_t)p->batch * p->hq * splits * p->head_dim);
  c.take<float>((size_t)p->batch * p->hq * splits * 2);
  return c.off;
}

extern "C" int dam_sparse_attn_decode(const dam_decode_params *p, const void *q, const void *kcache,
                                      const void *vcache, const int32_t *kept_ptr, const int32_t *kept_idx,
                                      int64_t max_kept, void *out, float *lse, void *ws, size_t ws_bytes,
                                      void *stream_v) {
  const int bad = validate(p, q, kcache, vcache, kept_ptr, kept_idx, max_kept, out);
  if (bad != DAM_OK) return bad;
  if (!ws || ws_bytes < dam_sparse_attn_decode_workspace(p, max_kept)) return DAM_ERR_WORKSPACE;
  DecodeArgs a;
  a.B = p->batch; a.Hq = p->hq; a.Hkv = p->hkv; a.cap = p->kv_capacity;
  a.splits = pick_splits((int64_t)p->batch * p->hq, max_kept);
  a.shared_lists = p->shared_lists != 0;
  a.scale = p->scale > 0.0f ? p->scale : 1.0f / sqrtf((float)p->head_dim);
  a.q_sb = p->q_stride[0]; a.q_sh = p->q_stride[1];
  a.kv_sb = p->kv_stride[0]; a.kv_sh = p->kv_stride[1]; a.kv_ss = p->kv_stride[2];
  a.o_sb = p->o_stride[0]; a.o_sh = p->o_stride[1];
  Carver c(ws);
  float *part_o = c.take<float>((size_t)a.B * a.Hq * a.splits * p->head_dim);
  float *part_ml = c.take<float>((size_t)a.B * a.Hq * a.splits * 2);
  hipStream_t st = static_cast<hipStream_t>(stream_v);
  if (p->dtype == DAM_BF16) {
    if (p->head_dim == 128) launch<__hip_bfloat16, 128>(a, q, kcache, vcache, kept_ptr, kept_idx, out, lse, part_o, part_ml, st);
    else launch<__hip_bfloat16, 64>(a, q, kcache, vcache, kept_ptr, kept_idx, out, lse, part_o, part_ml, st);
  } else {
    if (p->head_dim == 128) launch<float, 128>(a, q, kcache, vcache, kept_ptr, kept_idx, out, lse, part_o, part_ml, st);
    else launch<float, 64>(a, q, kcache, vcache, kept_ptr, kept_idx, out, lse, part_o, part_ml, st);
  }
  return launch_status();
}

namespace {

template <typename T, int D>
void launch_group(const DecodeArgs &a, const void *q, const void *kc, const void *vc, const int32_t *kept_ptr,
                  const int32_t *kept_idx, const uint8_t *kept_member, void *out, float *lse, float *part_o,
                  float *part_ml, hipStream_t st) {
  const int blocks = a.B * a.Hkv * a.splits;
  if (a.Hq / a.Hkv <= 4)
    k_decode_group<T, D, 4><<<blocks, 256, 0, st>>>(a, static_cast<const T *>(q), static_cast<const T *>(kc),
                                                    static_cast<const T *>(vc), kept_ptr, kept_idx, kept_member, part_o,
                                                    part_ml, static_cast<T *>(out), lse);
  else
    k_decode_group<T, D, 8><<<blocks, 256, 0, st>>>(a, static_cast<const T *>(q), static_cast<const T *>(kc),
                                                    static_cast<const T *>(vc), kept_ptr, kept_idx, kept_member, part_o,
                                                    part_ml, static_cast<T *>(out), lse);
  if (a.splits > 1) k_decode_merge<T, D><<<a.B * a.Hq, D, 0, st>>>(a, part_o, part_ml, static_cast<T *>(out), lse);
}

}  // namespace

extern "C" size_t dam_sparse_attn_decode_grouped_workspace(const dam_decode_params *p, int64_t max_kept) {
  if (!p || p->batch < 1 || p->hq < 1 || p->hkv < 1 || p->head_dim < 1 || max_kept < 0) return 0;
  if (p->hq % p->hkv) return 0;
  bool mfma;
  const int splits = group_splits(p, max_kept, &mfma);
  Carver c(nullptr);
  c.take<float>((size_t)p->batch * p->hq * splits * p->head_dim);
  c.take<float>((size_t)p->batch * p->hq * splits * 2);
  return c.off;
}

namespace {

// The grouped-query decode behind both of its entry points: arguments already validated, ws large enough.
int decode_grouped_run(const dam_decode_params *p, const void *q, const void *kcache, const void *vcache,
                       const int32_t *kept_ptr, const int32_t *kept_idx, const uint8_t *kept_member, int64_t max_kept,
                       void *out, float *lse, void *ws, hipStream_t st, const uint8_t *plan_table = nullptr,
                       int n_flags = 0, int pos = 0) {
  DecodeArgs a;
  a.B = p->batch; a.Hq = p->hq; a.Hkv = p->hkv; a.cap = p->kv_capacity;
  bool mfma;
  a.splits = group_splits(p, max_kept, &mfma);
  a.shared_lists = p->shared_lists != 0;
  a.scale = p->scale > 0.0f ? p->scale : 1.0f / sqrtf((float)p->head_dim);
  a.q_sb = p->q_stride[0]; a.q_sh = p->q_stride[1];
  a.kv_sb = p->kv_stride[0]; a.kv_sh = p->kv_stride[1]; a.kv_ss = p->kv_stride[2];
  a.o_sb = p->o_stride[0]; a.o_sh = p->o_stride[1];
  Carver c(ws);
  float *part_o = c.take<float>((size_t)a.B * a.Hq * a.splits * p->head_dim);
  float *part_ml = c.take<float>((size_t)a.B * a.Hq * a.splits * 2);
  if (mfma) {
    // matrix-core pass; with more than four splits its partial results go through the merge pass
    const int rc = launch_decode_group_mfma(p, a.splits, a.scale, q, kcache, vcache, kept_ptr, kept_idx, kept_member, part_o,
                                            part_ml, out, lse, st, plan_table, n_flags, pos);
    if (rc != DAM_OK) return rc;
    if (!decode_group_mfma_merges(a.splits))
      k_decode_merge<__hip_bfloat16, 128><<<a.B * a.Hq, 128, 0, st>>>(a, part_o, part_ml, static_cast<__hip_bfloat16 *>(out), lse);
  } else if (plan_table) {
    return DAM_ERR_UNSUPPORTED;  // plans are decoded by the matrix-core kernel only
  } else if (p->dtype == DAM_BF16) {
    if (p->head_dim == 128) launch_group<__hip_bfloat16, 128>(a, q, kcache, vcache, kept_ptr, kept_idx, kept_member, out, lse, part_o, part_ml, st);
    else launch_group<__hip_bfloat16, 64>(a, q, kcache, vcache, kept_ptr, kept_idx, kept_member, out, lse, part_o, part_ml, st);
  } else {
    if (p->head_dim == 128) launch_group<float, 128>(a, q, kcache, vcache, kept_ptr, kept_idx, kept_member, out, lse, part_o, part_ml, st);
    else launch_group<float, 64>(a, q, kcache, vcache, kept_ptr, kept_idx, kept_member, out, lse, part_o, part_ml, st);
  }
  return launch_status();
}

int validate_grouped(const dam_decode_params *p, const void *q, const void *kcache, const void *vcache,
                     const int32_t *kept_ptr, const int32_t *kept_idx, const uint8_t *kept_member, int64_t max_kept,
                     const void *out) {
  const int bad = validate(p, q, kcache, vcache, kept_ptr, kept_idx, max_kept, out);
  if (bad != DAM_OK) return bad;
  if (max_kept > 0 && !kept_member) return DAM_ERR_INVALID_ARG;
  if (p->hq / p->hkv > 8) return DAM_ERR_UNSUPPORTED;  // member bits are a byte
  return DAM_OK;
}

}  // namespace

extern "C" int dam_sparse_attn_decode_grouped(const dam_decode_params *p, const void *q, const void *kcache,
                                              const void *vcache, const int32_t *kept_ptr, const int32_t *kept_idx,
                                              const uint8_t *kept_member, int64_t max_kept, void *out, float *lse,
                                              void *ws, size_t ws_bytes, void *stream_v) {
  const int bad = validate_grouped(p, q, kcache, vcache, kept_ptr, kept_idx, kept_member, max_kept, out);
  if (bad != DAM_OK) return bad;
  if (!ws || ws_bytes < dam_sparse_attn_decode_grouped_workspace(p, max_kept)) return DAM_ERR_WORKSPACE;
  return decode_grouped_run(p, q, kcache, vcache, kept_ptr, kept_idx, kept_member, max_kept, out, lse, ws,
                            static_cast<hipStream_t>(stream_v));
}

// The grouped decode from a position-independent plan of a pattern mask: no list is built per step.
extern "C" int dam_sparse_attn_decode_patterns(const dam_decode_params *p, const void *q, const void *kcache,
                                               const void *vcache, const int32_t *plan_ptr, const int32_t *plan_val,
                                               const uint8_t *plan_member, const uint8_t *plan_table, int32_t n_flags,
                                               int32_t pos, int64_t max_entries, void *out, float *lse, void *ws,
                                               size_t ws_bytes, void *stream_v) {
  const int bad = validate_grouped(p, q, kcache, vcache, plan_ptr, plan_val, plan_member, max_entries, out);
  if (bad != DAM_OK) return bad;
  if (!plan_table || n_flags < 1 || pos < 0 || pos >= p->kv_capacity) return DAM_ERR_INVALID_ARG;
  if (!decode_group_mfma_fits(p)) return DAM_ERR_UNSUPPORTED;  // bf16, head_dim 128, rows of a head within 4 GiB
  dam_decode_params shared = *p;
  shared.shared_lists = 1;  // a plan belongs to the heads, not to a sequence
  if (!ws || ws_bytes < dam_sparse_attn_decode_grouped_workspace(&shared, max_entries)) return DAM_ERR_WORKSPACE;
  return decode_grouped_run(&shared, q, kcache, vcache, plan_ptr, plan_val, plan_member, max_entries, out, lse, ws,
                            static_cast<hipStream_t>(stream_v), plan_table, n_flags, pos);
}

// ------------------------------------------------------------------------------------------------
// dam_sparse_attn_decode_grouped for callers that cannot allocate: the partial results of the splits live in
// a fixed array in device memory that belongs to the library instead of a caller's workspace.
constexpr size_t kStaticScratchBytes = DAM_DECODE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
// the array's device address on each GPU (every GPU holds its own copy of the array at its own address);
// looked up once per device, at the first call made with that device current
std::atomic<void *> g_scratch_at[kMaxDevices];

int scratch_address(void **at) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DAM_ERR_DEVICE;
  void *ptr = g_scratch_at[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return DAM_ERR_DEVICE;
    g_scratch_at[dev].store(ptr, std::memory_order_release);  // (two threads racing here store the same address)
  }
  *at = ptr;
  return DAM_OK;
}
}  // namespace

extern "C" size_t dam_sparse_attn_decode_grouped_static_limit(void) { return kStaticScratchBytes; }

extern "C" int dam_sparse_attn_decode_grouped_static(const dam_decode_params *p, const void *q, const void *kcache,
                                                     const void *vcache, const int32_t *kept_ptr,
                                                     const int32_t *kept_idx, const uint8_t *kept_member,
                                                     int64_t max_kept, void *out, float *lse, void *stream_v) {
  const int bad = validate_grouped(p, q, kcache, vcache, kept_ptr, kept_idx, kept_member, max_kept, out);
  if (bad != DAM_OK) return bad;
  const size_t need = dam_sparse_attn_decode_grouped_workspace(p, max_kept);
  if (need == 0 || need > kStaticScratchBytes) return DAM_ERR_WORKSPACE;  // the call does not fit the fixed array
  void *ws = nullptr;
  const int st = scratch_address(&ws);
  if (st != DAM_OK) return st;
  // nothing to clear: every split writes its partial result before the merge pass reads it
  return decode_grouped_run(p, q, kcache, vcache, kept_ptr, kept_idx, kept_member, max_kept, out, lse, ws,
                            static_cast<hipStream_t>(stream_v));
}
