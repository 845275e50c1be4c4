// dam_sparse_attn_prefill: masked causal self-attention evaluated only inside the listed tiles.
//
// Paper (arXiv 2506.11104): Sec. 3 (S = Q K^T / sqrt(d_k), softmax, O = A V) with the per-head mask
// of Sec. 4.3 applied as -inf before the softmax. The tiling, the online softmax and the use of
// the block index are this library's own.
//
// bf16 kernel (head_dim 128, tiles 128 x 128), one workgroup of 4 waves per (head, query tile),
// each wave owning 32 query rows:
//   S^T = K Q^T on v_mfma_f32_32x32x16_bf16 (A = K rows from LDS, B = Q rows held in registers).
//     In the transposed product a lane's 64 accumulators all belong to ONE query, so the row max
//     and row sum of the online softmax are in-lane reductions plus a single exchange between the
//     two half-waves.
//   O^T += V^T P^T on the same instruction: the accumulator layout of S^T is, up to a fixed
//     permutation of each 16-key group, already the B-operand layout, so P never leaves
//     registers. V is transposed once per call into the workspace with that permutation baked in
//     (padded with zeros to whole tiles), which makes the V^T tile a plain row copy into LDS.
//   Tiles not in the block index are never touched; kind-1 (full) tiles skip the element mask.
// fp32 kernel (the 1e-4 variant): plain ALU code, one query row per group of head_dim/4 lanes,
// iterating only over the set bits of the row's tile words.
#include <hip/hip_bf16.h>
#include <math.h>

#include <algorithm>

#include "dam_internal.h"

namespace {
using namespace dam;

constexpr int kXcd = 8;

struct AttnArgs {
  int B, Hq, Hkv, S, nQt, tile_m, tile_n, wpr, s_pad;
  float scale;
  int64_t q_sb, q_sh, q_ss, k_sb, k_sh, k_ss, v_sb, v_sh, v_ss, o_sb, o_sh, o_ss;
};

// Work numbering shared by both kernels. Block n runs on XCD n % 8. All query heads of one
// (batch, KV head) pair get ids on one XCD so that they share that XCD's L2 copy of K / V;
// within a pair the query tiles go last-first (the longest rows of the causal triangle first).
struct WorkItem {
  int b, hq, hkv, qt;
  bool valid;
};

__device__ __forceinline__ WorkItem decode_work(const AttnArgs &a, int n) {
  const int G = a.Hq / a.Hkv;
  const int per_pair = G * a.nQt;
  const int xcd = n % kXcd, slot = n / kXcd;
  const int pair = (slot / per_pair) * kXcd + xcd;
  const int within = slot % per_pair;
  WorkItem w;
  w.valid = pair < a.B * a.Hkv;
  w.b = pair / a.Hkv;
  w.hkv = pair % a.Hkv;
  w.qt = a.nQt - 1 - within / G;
  w.hq = w.hkv * G + within % G;
  return w;
}

inline int work_blocks(const AttnArgs &a) {
  const int n_pairs = a.B * a.Hkv;
  return (n_pairs + kXcd - 1) / kXcd * kXcd * (a.Hq / a.Hkv) * a.nQt;
}

// ================================================================================================
// fp32 variant
template <int D>
__global__ __launch_bounds__(256) void k_prefill_f32(AttnArgs a, const float *__restrict__ q,
                                                     const float *__restrict__ k,
                                                     const float *__restrict__ v,
                                                     const int *__restrict__ row_ptr,
                                                     const int *__restrict__ blk_col,
                                                     const uint64_t *__restrict__ tile_bits,
                                                     float *__restrict__ out, float *__restrict__ lse) {
  constexpr int N = 4, LPR = D / N, GROUPS = 256 / LPR;
  const WorkItem w = decode_work(a, blockIdx.x);
  if (!w.valid) return;
  const int group = threadIdx.x / LPR, sub = threadIdx.x % LPR;
  const int t0 = row_ptr[(int64_t)w.hq * (a.nQt + 1) + w.qt];
  const int t1 = row_ptr[(int64_t)w.hq * (a.nQt + 1) + w.qt + 1];
  const float *kb = k + w.b * a.k_sb + w.hkv * a.k_sh + sub * N;
  const float *vb = v + w.b * a.v_sb + w.hkv * a.v_sh + sub * N;
  for (int rl = group; rl < a.tile_m; rl += GROUPS) {
    const int i = w.qt * a.tile_m + rl;
    if (i >= a.S) break;
    const float4 qv = *reinterpret_cast<const float4 *>(q + w.b * a.q_sb + w.hq * a.q_sh + i * a.q_ss + sub * N);
    float m = -INFINITY, l = 0.0f;
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int t = t0; t < t1; ++t) {
      const int j0 = blk_col[t] * a.tile_n;
      for (int wd = 0; wd < a.wpr; ++wd) {
        uint64_t bits = tile_bits[((int64_t)t * a.tile_m + rl) * a.wpr + wd];
        while (bits) {
          const int j = j0 + wd * 64 + __ffsll((unsigned long long)bits) - 1;
          bits &= bits - 1;
          const float4 kv = *reinterpret_cast<const float4 *>(kb + j * a.k_ss);
          const float4 vv = *reinterpret_cast<const float4 *>(vb + j * a.v_ss);
          float d = qv.x * kv.x + qv.y * kv.y + qv.z * kv.z + qv.w * kv.w;
#pragma unroll
          for (int off = LPR / 2; off; off >>= 1) d += __shfl_xor(d, off);
          const float s = d * a.scale;
          const float mn = fmaxf(m, s);
          const float corr = expf(m - mn), p = expf(s - mn);
          l = l * corr + p;
          o.x = o.x * corr + p * vv.x;
          o.y = o.y * corr + p * vv.y;
          o.z = o.z * corr + p * vv.z;
          o.w = o.w * corr + p * vv.w;
          m = mn;
        }
      }
    }
    const float inv = l > 0.0f ? 1.0f / l : 0.0f;
    *reinterpret_cast<float4 *>(out + w.b * a.o_sb + w.hq * a.o_sh + i * a.o_ss + sub * N) =
        make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
    if (lse && sub == 0)
      lse[((int64_t)w.b * a.Hq + w.hq) * a.S + i] = l > 0.0f ? m + logf(l) : -INFINITY;
  }
}

// ================================================================================================
// bf16 MFMA variant
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int kD = 128;            // head dim
constexpr int kBM = 128, kBN = 128;
constexpr int kRowBytes = 272;     // 256 B of bf16 + 16 B pad: 16-byte reads of 16 consecutive rows
                                   // fall into 16 different bank groups
constexpr int kTileLds = 128 * kRowBytes;

// Position of key offset o (0..15) inside its 16-key group of the transposed V: the two middle
// groups of four are swapped so that the S^T accumulators of one lane are, in register order, the
// eight consecutive k-slots the B operand of the P V product expects.
__host__ __device__ constexpr int vt_slot(int o) { return 8 * ((o % 8) / 4) + 4 * (o / 8) + o % 4; }

// V [b][hkv][s][d] -> VT [b*Hkv + hkv][d][s_pad] with keys permuted inside groups of 16 and zeros
// beyond S. 64 x 64 element patches through LDS.
__global__ __launch_bounds__(256) void k_transpose_v(AttnArgs a, const __hip_bfloat16 *__restrict__ v,
                                                     __hip_bfloat16 *__restrict__ vt) {
  __shared__ unsigned short patch[64][66];
  const int s0 = blockIdx.x * 64, d0 = blockIdx.y * 64;
  const int pair = blockIdx.z, b = pair / a.Hkv, hkv = pair % a.Hkv;
  const unsigned short *src = reinterpret_cast<const unsigned short *>(v) + b * a.v_sb + hkv * a.v_sh;
  for (int e = threadIdx.x; e < 64 * 64; e += 256) {
    const int r = e / 64, c = e % 64;  // r: key, c: dim
    patch[r][c] = (s0 + r < a.S) ? src[(int64_t)(s0 + r) * a.v_ss + d0 + c] : (unsigned short)0;
  }
  __syncthreads();
  unsigned short *dst = reinterpret_cast<unsigned short *>(vt) + (int64_t)pair * kD * a.s_pad;
  for (int e = threadIdx.x; e < 64 * 64; e += 256) {
    const int c = e / 64, pos = e % 64;  // c: dim, pos: position inside the 64-key patch
    const int grp = pos / 16, slot = pos % 16;
    // inverse of vt_slot: slot -> key offset
    const int o = 8 * ((slot % 8) / 4) + 4 * (slot / 8) + slot % 4;
    dst[(int64_t)(d0 + c) * a.s_pad + s0 + pos] = patch[grp * 16 + o][c];
  }
}

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  // round to nearest even on both halves
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  const bf16x2 r = __builtin_convertvector((f32x2){lo, hi}, bf16x2);
  return __builtin_bit_cast(unsigned, r);
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_prefill_bf16(AttnArgs a, const __hip_bfloat16 *__restrict__ q,
                                                      const __hip_bfloat16 *__restrict__ k,
                                                      const __hip_bfloat16 *__restrict__ vt,
                                                      const int *__restrict__ row_ptr,
                                                      const int *__restrict__ blk_col,
                                                      const uint8_t *__restrict__ blk_kind,
                                                      const uint64_t *__restrict__ tile_bits,
                                                      __hip_bfloat16 *__restrict__ out,
                                                      float *__restrict__ lse) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  unsigned char *ldsK = lds, *ldsV = lds + kTileLds;

  const WorkItem w = decode_work(a, blockIdx.x);
  if (!w.valid) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int t0 = row_ptr[(int64_t)w.hq * (a.nQt + 1) + w.qt];
  const int t1 = row_ptr[(int64_t)w.hq * (a.nQt + 1) + w.qt + 1];
  const int qrow_l = wave * 32 + n;              // this lane's query row inside the tile
  const int qrow = w.qt * kBM + qrow_l;
  const bool qlive = qrow < a.S;

  // Q fragments: B operand of S^T = K Q^T. Chunk c covers dims 16c .. 16c+15; this lane holds
  // dims 16c + 8 hf .. + 7 of its query row.
  bf16x8 qf[8];
  {
    const __hip_bfloat16 *qp = q + w.b * a.q_sb + w.hq * a.q_sh + (int64_t)qrow * a.q_ss + 8 * hf;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      u32x4 raw = {0u, 0u, 0u, 0u};
      if (qlive) raw = *reinterpret_cast<const u32x4 *>(qp + 16 * c);
      qf[c] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  f32x16 oacc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[db][e] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;   // running max (raw logit units) and this lane's part of the sum
  const float c2 = a.scale * 1.4426950408889634f;

  const unsigned char *kg = reinterpret_cast<const unsigned char *>(k + w.b * a.k_sb + w.hkv * a.k_sh);
  const unsigned char *vg =
      reinterpret_cast<const unsigned char *>(vt + (int64_t)(w.b * a.Hkv + w.hkv) * kD * a.s_pad);

  for (int t = t0; t < t1; ++t) {
    const int kt = blk_col[t];
    const bool full = blk_kind[t] != 0;
    __syncthreads();  // every wave is done with the previous tile
    // K tile: 128 rows x 256 B; V^T tile: 128 dims x 256 B. 16 lanes copy one row.
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int chunk = tid + 256 * it, r = chunk >> 4, c16 = chunk & 15;
      const int key = kt * kBN + r;
      u32x4 kv = {0u, 0u, 0u, 0u};
      if (key < a.S) kv = *reinterpret_cast<const u32x4 *>(kg + (int64_t)key * a.k_ss * 2 + c16 * 16);
      const u32x4 vv = *reinterpret_cast<const u32x4 *>(vg + ((int64_t)r * a.s_pad + kt * kBN) * 2 + c16 * 16);
      *reinterpret_cast<u32x4 *>(ldsK + r * kRowBytes + c16 * 16) = kv;
      *reinterpret_cast<u32x4 *>(ldsV + r * kRowBytes + c16 * 16) = vv;
    }
    // this lane's mask words: row qrow_l of the tile, 128 keys = 4 dwords
    u32x4 mw = {~0u, ~0u, ~0u, ~0u};
    if (!full) mw = *reinterpret_cast<const u32x4 *>(tile_bits + ((int64_t)t * kBM + qrow_l) * 2);
    __syncthreads();

    // S^T = K Q^T: block kb holds keys 32 kb .. 32 kb + 31 (rows) x 32 queries (columns)
    f32x16 sacc[4];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[kb][e] = 0.0f;
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(ldsK + (kb * 32 + n) * kRowBytes + c * 32 + hf * 16);
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], sacc[kb], 0, 0, 0);
      }
    }
    // element mask: accumulator e of block kb is key 32 kb + 8 (e / 4) + 4 hf + e % 4
    if (!full) {
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) {
        const unsigned bits = mw[kb] >> (4 * hf);
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (!((bits >> (8 * (e / 4) + e % 4)) & 1u)) sacc[kb][e] = -INFINITY;
      }
    }
    // online softmax, one query per lane pair (lane, lane ^ 32)
    float mx = sacc[0][0];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[kb][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float m_ref = m_new == -INFINITY ? 0.0f : m_new;
    const float corr = __builtin_amdgcn_exp2f((m_run - m_ref) * c2);
    const float off = m_ref * c2;
    m_run = m_new;
    float psum = 0.0f;
    unsigned pk[4][8];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(sacc[kb][e] * c2 - off);
        const float p1 = __builtin_amdgcn_exp2f(sacc[kb][e + 1] * c2 - off);
        psum += p0 + p1;
        pk[kb][e / 2] = pack_bf16(p0, p1);
      }
    l_run = l_run * corr + psum;
    if (__ballot(corr != 1.0f)) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[db][e] *= corr;
    }
    // O^T += V^T P^T: for key block kb and half a, the B operand is accumulators 8a .. 8a+7 of
    // block kb (as bf16); the A operand is 16 bytes of row (32 db + n) of the V^T tile.
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        const u32x4 praw = {pk[kb][4 * h2], pk[kb][4 * h2 + 1], pk[kb][4 * h2 + 2], pk[kb][4 * h2 + 3]};
        const bf16x8 pf = __builtin_bit_cast(bf16x8, praw);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(ldsV + (db * 32 + n) * kRowBytes +
                                                             (kb * 32 + h2 * 16) * 2 + hf * 16);
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[db], 0, 0, 0);
        }
      }
  }

  // finish: total sum over both half-waves, normalise, store. Accumulator e of block db is
  // dim 32 db + 8 (e / 4) + 4 hf + e % 4 of this lane's query.
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
  if (qlive) {
    __hip_bfloat16 *op = out + w.b * a.o_sb + w.hq * a.o_sh + (int64_t)qrow * a.o_ss;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 pr;
        pr.x = pack_bf16(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv);
        pr.y = pack_bf16(oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv);
        *reinterpret_cast<uint2 *>(op + 32 * db + 8 * g + 4 * hf) = pr;
      }
    if (lse && hf == 0)
      lse[((int64_t)w.b * a.Hq + w.hq) * a.S + qrow] =
          l_tot > 0.0f ? (m_run * c2 + log2f(l_tot)) * 0.6931471805599453f : -INFINITY;
  }
}

int validate(const dam_attn_params *p, const void *q, const void *k, const void *v, const dam_mask_view *mk,
             const void *out) {
  if (!p || !q || !k || !v || !mk || !out) return DAM_ERR_INVALID_ARG;
  if (!mk->blk_row_ptr || !mk->blk_col || !mk->blk_kind || !mk->tile_bits) return DAM_ERR_INVALID_ARG;
  if (p->batch < 1 || p->hq < 1 || p->hkv < 1 || p->hq % p->hkv || p->seq < 1) return DAM_ERR_INVALID_ARG;
  if (p->tile_m < 64 || p->tile_n < 64 || p->tile_m % 64 || p->tile_n % 64) return DAM_ERR_INVALID_ARG;
  if (!(p->scale >= 0.0f)) return DAM_ERR_INVALID_ARG;
  const int align = p->dtype == DAM_BF16 ? 8 : 4;
  const int64_t *sets[4] = {p->q_stride, p->k_stride, p->v_stride, p->o_stride};
  for (auto s : sets)
    for (int x = 0; x < 3; ++x)
      if (s[x] < 0 || s[x] % align) return DAM_ERR_INVALID_ARG;
  if (p->dtype == DAM_BF16) {
    if (p->head_dim != 128 || p->tile_m != 128 || p->tile_n != 128) return DAM_ERR_UNSUPPORTED;
  } else if (p->dtype == DAM_F32) {
    if (p->head_dim != 64 && p->head_dim != 128) return DAM_ERR_UNSUPPORTED;
    if (p->tile_m > 128 || p->tile_n > 128) return DAM_ERR_UNSUPPORTED;
  } else {
    return DAM_ERR_UNSUPPORTED;
  }
  return DAM_OK;
}

AttnArgs make_args(const dam_attn_params *p) {
  AttnArgs a;
  a.B = p->batch; a.Hq = p->hq; a.Hkv = p->hkv; a.S = p->seq;
  a.tile_m = p->tile_m; a.tile_n = p->tile_n;
  a.nQt = (p->seq + p->tile_m - 1) / p->tile_m;
  a.wpr = p->tile_n / 64;
  a.s_pad = (p->seq + kBN - 1) / kBN * kBN;
  a.scale = p->scale > 0.0f ? p->scale : 1.0f / sqrtf((float)p->head_dim);
  a.q_sb = p->q_stride[0]; a.q_sh = p->q_stride[1]; a.q_ss = p->q_stride[2];
  a.k_sb = p->k_stride[0]; a.k_sh = p->k_stride[1]; a.k_ss = p->k_stride[2];
  a.v_sb = p->v_stride[0]; a.v_sh = p->v_stride[1]; a.v_ss = p->v_stride[2];
  a.o_sb = p->o_stride[0]; a.o_sh = p->o_stride[1]; a.o_ss = p->o_stride[2];
  return a;
}

}  // namespace

extern "C" size_t dam_sparse_attn_prefill_workspace(const dam_attn_params *p) {
  if (!p || p->batch < 1 || p->hkv < 1 || p->seq < 1) return 0;
  if (p->dtype != DAM_BF16) return 0;
  const size_t s_pad = ((size_t)p->seq + kBN - 1) / kBN * kBN;
  return align_up((size_t)p->batch * p->hkv * kD * s_pad * 2, 256);  // transposed V
}

extern "C" int dam_sparse_attn_prefill(const dam_attn_params *p, const void *q, const void *k, const void *v,
                                       const dam_mask_view *mk, void *out, float *lse, void *ws, size_t ws_bytes,
                                       void *stream_v) {
  const int bad = validate(p, q, k, v, mk, out);
  if (bad != DAM_OK) return bad;
  const size_t need = dam_sparse_attn_prefill_workspace(p);
  if (need && (!ws || ws_bytes < need)) return DAM_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream_v);
  const AttnArgs a = make_args(p);
  const int blocks = work_blocks(a);
  if (p->dtype == DAM_F32) {
    if (p->head_dim == 64)
      k_prefill_f32<64><<<blocks, 256, 0, st>>>(a, (const float *)q, (const float *)k, (const float *)v, mk->blk_row_ptr,
                                               mk->blk_col, mk->tile_bits, (float *)out, lse);
    else
      k_prefill_f32<128><<<blocks, 256, 0, st>>>(a, (const float *)q, (const float *)k, (const float *)v, mk->blk_row_ptr,
                                                mk->blk_col, mk->tile_bits, (float *)out, lse);
    return launch_status();
  }
  __hip_bfloat16 *vt = static_cast<__hip_bfloat16 *>(ws);
  k_transpose_v<<<dim3(a.s_pad / 64, kD / 64, a.B * a.Hkv), 256, 0, st>>>(a, (const __hip_bfloat16 *)v, vt);
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(k_prefill_bf16), hipFuncAttributeMaxDynamicSharedMemorySize,
                            2 * kTileLds) != hipSuccess)
      return DAM_ERR_DEVICE;
    attr_set = true;
  }
  k_prefill_bf16<<<blocks, 256, 2 * kTileLds, st>>>(a, (const __hip_bfloat16 *)q, (const __hip_bfloat16 *)k, vt,
                                                   mk->blk_row_ptr, mk->blk_col, mk->blk_kind, mk->tile_bits,
                                                   (__hip_bfloat16 *)out, lse);
  return launch_status();
}

extern "C" int dam_version(void) { return 1; }
