// dam_capture_accumulate and the capture half of dam_mask_build_from_qk: full causal attention
// probabilities of a captured sequence, summed into the statistics A (and C) or thresholded on
// the fly into the true mask.
//
// Paper (arXiv 2506.11104): Sec. 4.2.1 (sequences truncated to the pattern capture length are run
// with full attention), Sec. 4.2.2 (the attention weights are summed over the captured batches and
// the valid position pairs are counted), Sec. 4.2.3 (threshold) for the fused form. The two-pass
// organisation and the kernels are this library's own.
//
// Both forms take two passes over the causal triangle of Q K^T: the first one reduces every row to
// its log-sum-exp (never materialising the logits), the second one recomputes the logits and turns
// them into probabilities p = exp2(s - lse). bf16 inputs with head_dim 128 run on the matrix
// cores: S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so that the 16 accumulators of a lane belong
// to one query row and the row reductions are in-lane plus one exchange between the half-waves.
// Everything else (fp32 inputs, other head dims) goes through a plain one-row-per-workgroup kernel.
#include <hip/hip_bf16.h>
#include <math.h>

#include <algorithm>

#include "dam_internal.h"

namespace {
using namespace dam;

constexpr float kLog2e = 1.4426950408889634f;

struct CapArgs {
  int Hq, Hkv, n, L, d, tbw;
  float c2;  // scale * log2(e): logits in log2 units
  int64_t q_sh, q_ss, k_sh, k_ss;
};

// Ordered key of an fp32 value (increasing with the value; NaN counts as -inf): the form in which
// the true-mask threshold is handed over.
__device__ __forceinline__ unsigned key_of(float x) {
  if (x != x) x = -INFINITY;
  const unsigned b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

enum { kEmitBits = 0, kEmitSum = 1 };

// ================================================================================================
// Plain kernel: one workgroup per (row i, head h). The row's logits live in LDS between the
// reduction and the emission, so this kernel needs one pass only.
template <typename T>
__device__ __forceinline__ float dot_row(const float *__restrict__ qs, const T *__restrict__ krow, int d);

template <>
__device__ __forceinline__ float dot_row<float>(const float *__restrict__ qs, const float *__restrict__ krow, int d) {
  float acc = 0.0f;
  for (int t = 0; t < d; t += 4) {
    const float4 kv = *reinterpret_cast<const float4 *>(krow + t);
    acc = fmaf(qs[t], kv.x, acc);
    acc = fmaf(qs[t + 1], kv.y, acc);
    acc = fmaf(qs[t + 2], kv.z, acc);
    acc = fmaf(qs[t + 3], kv.w, acc);
  }
  return acc;
}

template <>
__device__ __forceinline__ float dot_row<__hip_bfloat16>(const float *__restrict__ qs, const __hip_bfloat16 *__restrict__ krow,
                                                         int d) {
  float acc = 0.0f;
  for (int t = 0; t < d; t += 8) {
    const uint4 kv = *reinterpret_cast<const uint4 *>(krow + t);
    const unsigned u[4] = {kv.x, kv.y, kv.z, kv.w};
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      acc = fmaf(qs[t + 2 * x], __uint_as_float(u[x] << 16), acc);
      acc = fmaf(qs[t + 2 * x + 1], __uint_as_float(u[x] & 0xFFFF0000u), acc);
    }
  }
  return acc;
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(__hip_bfloat16 x) { return __bfloat162float(x); }

template <typename T, int MODE>
__global__ __launch_bounds__(256) void k_capture_rows(CapArgs a, const T *__restrict__ q, const T *__restrict__ k,
                                                      const unsigned *__restrict__ theta_key,
                                                      uint64_t *__restrict__ true_bits, float *__restrict__ attn_sum,
                                                      float *__restrict__ attn_cnt) {
  extern __shared__ float smem[];  // [d] query, then [i + 1] logits
  __shared__ float red[4];
  const int i = a.n - 1 - blockIdx.x, h = blockIdx.y;  // long rows first
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float *qs = smem, *sv = smem + a.d;
  const T *qrow = q + (int64_t)h * a.q_sh + (int64_t)i * a.q_ss;
  for (int t = threadIdx.x; t < a.d; t += 256) qs[t] = to_f32(qrow[t]);
  __syncthreads();
  const T *kh = k + (int64_t)(h / (a.Hq / a.Hkv)) * a.k_sh;
  float mx = -INFINITY;
  for (int j = threadIdx.x; j <= i; j += 256) {
    const float s = dot_row<T>(qs, kh + (int64_t)j * a.k_ss, a.d) * a.c2;
    sv[j] = s;
    mx = fmaxf(mx, s);
  }
  for (int off = 32; off; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.0f;
  for (int j = threadIdx.x; j <= i; j += 256) sum += __builtin_amdgcn_exp2f(sv[j] - mx);
  for (int off = 32; off; off >>= 1) sum += __shfl_xor(sum, off);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  sum = (red[0] + red[1]) + (red[2] + red[3]);
  const float lse2 = mx + __builtin_amdgcn_logf(sum);  // v_log_f32 is the base-2 logarithm
  if (MODE == kEmitBits) {
    const unsigned theta = *theta_key;
    uint64_t *out = true_bits + ((int64_t)h * a.L + i) * a.tbw;
    for (int w = wave; w < a.tbw; w += 4) {
      const int j = w * 64 + lane;
      const bool keep = j <= i && key_of(__builtin_amdgcn_exp2f(sv[j <= i ? j : 0] - lse2)) >= theta;
      const uint64_t word = __ballot(keep);
      if (lane == 0) out[w] = word;
    }
  } else {
    float *arow = attn_sum + ((int64_t)h * a.L + i) * a.L;
    float *crow = attn_cnt ? attn_cnt + ((int64_t)h * a.L + i) * a.L : nullptr;
    for (int j = threadIdx.x; j <= i; j += 256) {
      arow[j] += __builtin_amdgcn_exp2f(sv[j] - lse2);
      if (crow) crow[j] += 1.0f;
    }
  }
}

// ================================================================================================
// Matrix-core kernels (bf16, head_dim 128). One workgroup of 4 waves per (head, tile of 128 query
// rows), each wave owning 32 rows; K moves through LDS in blocks of 32 keys (8 KiB), double
// buffered. A K row is 16 chunks of 16 bytes; chunk c of row r is stored at position c ^ (r & 15),
// so that the 16-byte operand reads of 16 consecutive rows cover all banks once.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int kRows = 128, kBlk = 32, kBlkBytes = kBlk * 256;

struct KStage {
  uint4 r[2];
};

// This thread's two 16-byte pieces of the K block starting at key0 (rows past the sequence end are
// redirected to the last row: such keys are masked by causality anyway).
__device__ __forceinline__ KStage k_fetch(const __hip_bfloat16 *__restrict__ kh, int64_t k_ss, int key0, int n_keys) {
  KStage st;
  const int row = threadIdx.x >> 4, chunk = threadIdx.x & 15;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int key = min(key0 + row + 16 * it, n_keys - 1);
    st.r[it] = *reinterpret_cast<const uint4 *>(kh + (int64_t)key * k_ss + chunk * 8);
  }
  return st;
}

__device__ __forceinline__ void k_stash(unsigned char *buf, const KStage &st) {
  const int row = threadIdx.x >> 4, chunk = threadIdx.x & 15;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int r = row + 16 * it;
    *reinterpret_cast<uint4 *>(buf + r * 256 + ((chunk ^ (r & 15)) << 4)) = st.r[it];
  }
}

// S^T block: accumulator e of lane (n = lane & 31, hf = lane >> 5) is the logit of query row n of
// the wave with key 8 (e / 4) + 4 hf + e % 4 of the block.
__device__ __forceinline__ f32x16 s_block(const unsigned char *buf, const bf16x8 (&qf)[8], int kbase) {
  f32x16 s = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(buf + (kbase ^ (c << 5)));
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], s, 0, 0, 0);
  }
  return s;
}

// PASS 0: log-sum-exp (log2 units) of every row. PASS 1: emission (MODE).
template <int PASS, int MODE>
__global__ __launch_bounds__(256) void k_capture_mfma(CapArgs a, const __hip_bfloat16 *__restrict__ q,
                                                      const __hip_bfloat16 *__restrict__ k, float *__restrict__ lse2,
                                                      const unsigned *__restrict__ theta_key,
                                                      uint64_t *__restrict__ true_bits, float *__restrict__ attn_sum,
                                                      float *__restrict__ attn_cnt) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kBlkBytes];
  const int nQt = (a.n + kRows - 1) / kRows;
  const int qt = nQt - 1 - blockIdx.x, h = blockIdx.y;  // long rows first
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int i = qt * kRows + wave * 32 + n;  // this lane's query row
  const bool live = i < a.n;
  const int wave_last = qt * kRows + wave * 32 + 31;
  const int kbase = n * 256 + ((hf ^ (n & 15)) << 4);
  const __hip_bfloat16 *kh = k + (int64_t)(h / (a.Hq / a.Hkv)) * a.k_sh;

  bf16x8 qf[8];
  {
    const __hip_bfloat16 *qp = q + (int64_t)h * a.q_sh + (int64_t)i * a.q_ss + 8 * hf;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      u32x4 raw = {0u, 0u, 0u, 0u};
      if (live) raw = *reinterpret_cast<const u32x4 *>(qp + 16 * c);
      qf[c] = __builtin_bit_cast(bf16x8, raw);
    }
  }
  // key blocks that hold a key <= the tile's last live row
  const int last_row = min(qt * kRows + kRows - 1, a.n - 1);
  const int nkb = last_row / kBlk + 1;

  float m_run = -INFINITY, l_run = 0.0f;                      // PASS 0
  const float my_lse = (PASS == 1 && live) ? lse2[(int64_t)h * a.L + i] : 0.0f;
  const unsigned theta = (PASS == 1 && MODE == kEmitBits) ? *theta_key : 0u;
  unsigned words[4] = {0u, 0u, 0u, 0u};                        // bits of the current 128-key group
  unsigned *out32 = reinterpret_cast<unsigned *>(true_bits + ((int64_t)h * a.L + (live ? i : 0)) * a.tbw);
  const int nw32 = a.tbw * 2;

  k_stash(lds, k_fetch(kh, a.k_ss, 0, a.n));
  __syncthreads();
  for (int kb = 0; kb < nkb; ++kb) {
    const unsigned char *buf = lds + (kb & 1) * kBlkBytes;
    KStage next;
    const bool more = kb + 1 < nkb;
    if (more) next = k_fetch(kh, a.k_ss, (kb + 1) * kBlk, a.n);
    const int key0 = kb * kBlk;
    if (key0 <= wave_last) {  // wave-uniform: otherwise the whole block lies above this wave's rows
      const f32x16 s = s_block(buf, qf, kbase);
      if (PASS == 0) {
        float t[16], mx = m_run;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = key0 + 8 * (e / 4) + 4 * hf + (e % 4);
          t[e] = j <= i ? s[e] * a.c2 : -INFINITY;
          mx = fmaxf(mx, t[e]);
        }
        const float ref = mx == -INFINITY ? 0.0f : mx;
        float add = 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) add += __builtin_amdgcn_exp2f(t[e] - ref);
        l_run = l_run * __builtin_amdgcn_exp2f(m_run - ref) + add;
        m_run = mx;
      } else if (MODE == kEmitBits) {
        unsigned mine = 0u;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int j = key0 + 8 * (e / 4) + 4 * hf + (e % 4);
          const float p = __builtin_amdgcn_exp2f(s[e] * a.c2 - my_lse);
          if (j <= i && key_of(p) >= theta) mine |= 1u << (8 * (e / 4) + 4 * hf + (e % 4));
        }
        mine |= (unsigned)__shfl_xor((int)mine, 32);
        const int slot = kb & 3;
        words[0] = slot == 0 ? mine : words[0];
        words[1] = slot == 1 ? mine : words[1];
        words[2] = slot == 2 ? mine : words[2];
        words[3] = slot == 3 ? mine : words[3];
      } else {
        float *arow = attn_sum + ((int64_t)h * a.L + (live ? i : 0)) * a.L;
        float *crow = attn_cnt ? attn_cnt + ((int64_t)h * a.L + (live ? i : 0)) * a.L : nullptr;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int j0 = key0 + 8 * g + 4 * hf;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (live && j0 + r <= i) {
              arow[j0 + r] += __builtin_amdgcn_exp2f(s[4 * g + r] * a.c2 - my_lse);
              if (crow) crow[j0 + r] += 1.0f;
            }
          }
        }
      }
    }
    if (PASS == 1 && MODE == kEmitBits && ((kb & 3) == 3 || kb + 1 == nkb)) {
      // the 128-key group is complete (blocks above this wave's rows contribute zeros)
      if (live && hf == 0) {
        const int w0 = (kb >> 2) * 4;
#pragma unroll
        for (int x = 0; x < 4; ++x)
          if (w0 + x < nw32) out32[w0 + x] = words[x];
      }
      words[0] = words[1] = words[2] = words[3] = 0u;
    }
    if (more) k_stash(lds + ((kb + 1) & 1) * kBlkBytes, next);
    __syncthreads();
  }
  if (PASS == 0) {
    const float m_o = __shfl_xor(m_run, 32), l_o = __shfl_xor(l_run, 32);
    const float M = fmaxf(m_run, m_o);  // finite: every live row holds key 0
    const float tot = l_run * __builtin_amdgcn_exp2f(m_run - M) + l_o * __builtin_amdgcn_exp2f(m_o - M);
    if (live && hf == 0) lse2[(int64_t)h * a.L + i] = M + __builtin_amdgcn_logf(tot);
  } else if (MODE == kEmitBits) {
    // words of the row past the tile's last key block: all zero (keys above the diagonal)
    if (live) {
      const int w_done = ((nkb + 3) / 4) * 4;
      for (int w = w_done + hf; w < nw32; w += 2) out32[w] = 0u;
    }
  }
}

bool mfma_path(const dam_capture_params *p) { return p->dtype == DAM_BF16 && p->head_dim == 128; }

CapArgs make_args(const dam_capture_params *p) {
  CapArgs a;
  a.Hq = p->hq; a.Hkv = p->hkv; a.n = p->len; a.L = p->pcl; a.d = p->head_dim;
  a.tbw = (p->pcl + 63) / 64;
  a.c2 = (p->scale > 0.0f ? p->scale : 1.0f / sqrtf((float)p->head_dim)) * kLog2e;
  a.q_sh = p->q_stride[0]; a.q_ss = p->q_stride[1];
  a.k_sh = p->k_stride[0]; a.k_ss = p->k_stride[1];
  return a;
}

template <int MODE>
void launch(const dam_capture_params *p, const void *q, const void *k, float *lse2, const unsigned *theta_key,
            uint64_t *true_bits, float *attn_sum, float *attn_cnt, hipStream_t st) {
  const CapArgs a = make_args(p);
  if (mfma_path(p)) {
    const dim3 grid((a.n + kRows - 1) / kRows, a.Hq);
    const __hip_bfloat16 *qb = static_cast<const __hip_bfloat16 *>(q), *kb = static_cast<const __hip_bfloat16 *>(k);
    k_capture_mfma<0, MODE><<<grid, 256, 0, st>>>(a, qb, kb, lse2, theta_key, true_bits, attn_sum, attn_cnt);
    k_capture_mfma<1, MODE><<<grid, 256, 0, st>>>(a, qb, kb, lse2, theta_key, true_bits, attn_sum, attn_cnt);
    return;
  }
  const dim3 grid(a.n, a.Hq);
  const size_t lds = (size_t)(a.d + a.n) * sizeof(float);
  if (p->dtype == DAM_BF16)
    k_capture_rows<__hip_bfloat16, MODE><<<grid, 256, lds, st>>>(a, static_cast<const __hip_bfloat16 *>(q),
                                                                static_cast<const __hip_bfloat16 *>(k), theta_key, true_bits,
                                                                attn_sum, attn_cnt);
  else
    k_capture_rows<float, MODE><<<grid, 256, lds, st>>>(a, static_cast<const float *>(q), static_cast<const float *>(k),
                                                       theta_key, true_bits, attn_sum, attn_cnt);
}

}  // namespace

namespace dam {

int capture_validate(const dam_capture_params *p, const void *q, const void *k) {
  if (!p || !q || !k) return DAM_ERR_INVALID_ARG;
  if (p->hq < 1 || p->hkv < 1 || p->hq % p->hkv || p->len < 1 || p->pcl < p->len) return DAM_ERR_INVALID_ARG;
  if (p->dtype != DAM_F32 && p->dtype != DAM_BF16) return DAM_ERR_UNSUPPORTED;
  if (p->head_dim < 8 || p->head_dim > 256 || p->head_dim % 8) return DAM_ERR_UNSUPPORTED;
  if (p->pcl > 8192) return DAM_ERR_UNSUPPORTED;  // a row's logits stay in LDS in the plain kernel
  if (!(p->scale >= 0.0f)) return DAM_ERR_INVALID_ARG;
  const int align = p->dtype == DAM_BF16 ? 8 : 4;  // elements per 16 bytes
  const int64_t strides[] = {p->q_stride[0], p->q_stride[1], p->k_stride[0], p->k_stride[1]};
  for (int64_t s : strides)
    if (s < 0 || s % align) return DAM_ERR_INVALID_ARG;
  return DAM_OK;
}

size_t capture_lse_bytes(const dam_capture_params *p) {
  return align_up((size_t)p->hq * (size_t)p->pcl * sizeof(float), 256);
}

void launch_capture_true_bits(const dam_capture_params *p, const void *q, const void *k, float *lse2,
                              const unsigned *theta_key, uint64_t *true_bits, hipStream_t st) {
  launch<kEmitBits>(p, q, k, lse2, theta_key, true_bits, nullptr, nullptr, st);
}

}  // namespace dam

extern "C" size_t dam_capture_workspace(const dam_capture_params *p) {
  if (!p || p->hq < 1 || p->pcl < 1) return 0;
  return dam::capture_lse_bytes(p);
}

extern "C" int dam_capture_accumulate(const dam_capture_params *p, const void *q, const void *k, float *attn_sum,
                                      float *attn_cnt, void *ws, size_t ws_bytes, void *stream_v) {
  const int bad = dam::capture_validate(p, q, k);
  if (bad != DAM_OK) return bad;
  if (!attn_sum) return DAM_ERR_INVALID_ARG;
  if (!ws || ws_bytes < dam_capture_workspace(p)) return DAM_ERR_WORKSPACE;
  launch<kEmitSum>(p, q, k, static_cast<float *>(ws), nullptr, nullptr, attn_sum, attn_cnt,
                   static_cast<hipStream_t>(stream_v));
  return dam::launch_status();
}
