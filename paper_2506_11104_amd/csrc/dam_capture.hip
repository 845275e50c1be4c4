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
// rows), each wave owning 32 rows; K moves through LDS in stages of 64 keys (16 KiB), double
// buffered, one barrier per stage. A K row is 16 chunks of 16 bytes; chunk c of row r is stored at
// position c ^ (r & 15), so that the 16-byte operand reads of 16 consecutive rows cover all banks.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int kRows = 128, kBlk = 32, kBlkBytes = kBlk * 256;
constexpr int kXcd = 8;
constexpr int kStageKeys = 64, kStageBytes = kStageKeys * 256;
constexpr int kPadRow = 36;  // floats per row of a wave's 32 x 32 transposition tile (16-byte aligned, conflict-free)

struct KStage {
  uint4 r[4];
};

// This thread's four 16-byte pieces of the 64 keys starting at key0. `kp` points at this thread's
// piece of key `threadIdx.x >> 4`; rows past the sequence end are redirected to the last row (such
// keys are masked by causality anyway), which only a sequence's last stage has to look at.
__device__ __forceinline__ KStage k_fetch(const __hip_bfloat16 *__restrict__ kp, int64_t k_ss, int key0, int n_keys) {
  KStage st;
  const __hip_bfloat16 *base = kp + (int64_t)key0 * k_ss;
  if (key0 + kStageKeys <= n_keys) {  // workgroup-uniform
#pragma unroll
    for (int it = 0; it < 4; ++it) st.r[it] = *reinterpret_cast<const uint4 *>(base + (int64_t)(16 * it) * k_ss);
  } else {
    const int row = threadIdx.x >> 4;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int over = max(key0 + row + 16 * it - (n_keys - 1), 0);
      st.r[it] = *reinterpret_cast<const uint4 *>(base + (int64_t)(16 * it - over) * k_ss);
    }
  }
  return st;
}

__device__ __forceinline__ void k_stash(unsigned char *buf, const KStage &st) {
  const int row = threadIdx.x >> 4, chunk = threadIdx.x & 15;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int r = row + 16 * it;
    *reinterpret_cast<uint4 *>(buf + r * 256 + ((chunk ^ (r & 15)) << 4)) = st.r[it];
  }
}

// One wave's quarter of a stage as four load-to-LDS copies (lane L of the wave fetches 16 bytes from
// gbase + voff[it] and writes them to LDS byte lds_at + 4096 it + 16 L): rows wave * 4 + L / 16 + 16 it
// of the stage, whose chunk order the lane offsets already permute. Inline assembly, so that the
// compiler neither tracks nor counts the copies: the kernel waits for them itself (s_waitcnt vmcnt)
// before the barrier that publishes the stage. gbase and lds_at are wave-uniform.
__device__ __forceinline__ void k_copy_stage(unsigned lds_at, const void *gbase, const unsigned (&voff)[4]) {
#define DAM_CAP_COPY(IT)                                                               \
  asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"    \
               :                                                                         \
               : "s"(lds_at), "n"(4096 * (IT)), "v"(voff[IT]), "s"(gbase)                \
               : "memory", "scc", "m0")
  DAM_CAP_COPY(0);
  DAM_CAP_COPY(1);
  DAM_CAP_COPY(2);
  DAM_CAP_COPY(3);
#undef DAM_CAP_COPY
}

// S^T block of 32 keys: accumulator e of lane (n = lane & 31, hf = lane >> 5) is the raw logit
// (before the scale) of query row n of the wave with key 8 (e / 4) + 4 hf + e % 4 of the block,
// added to the start value `s`. kaddr[c] is this lane's operand c in the block at LDS offset 0; OFF
// (a constant: buffer and half) lands in the instruction's offset field. All eight operand reads
// are issued before the first product: the chain then waits for one LDS round trip, not for eight.
template <int OFF>
__device__ __forceinline__ f32x16 s_block(const unsigned char *const (&kaddr)[8], const bf16x8 (&qf)[8], f32x16 s) {
  bf16x8 kf[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) kf[c] = *reinterpret_cast<const bf16x8 *>(kaddr[c] + OFF);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int c = 0; c < 8; ++c) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[c], qf[c], s, 0, 0, 0);
  return s;
}

// Bits 0 .. 31 of a 32-key block starting at key0 that are causal for row i (key <= i).
__device__ __forceinline__ unsigned causal_bits(int i, int key0) {
  const int u = i - key0;
  return u >= 31 ? 0xFFFFFFFFu : (u < 0 ? 0u : ((2u << u) - 1u));
}

// Position, among the 32 keys of a block, of accumulator e of a lane of the lower half-wave.
__device__ __forceinline__ constexpr int key_of_acc(int e) { return 8 * (e / 4) + (e % 4); }

// Start value of a block's accumulators: 0 where the key is causal for this lane's row, -inf where
// it is not (the products add to it). `mine` = the causal bits already shifted by 4 hf.
__device__ __forceinline__ f32x16 causal_start(unsigned mine) {
  f32x16 s;
  const int inv = (int)~mine;
#pragma unroll
  for (int e = 0; e < 16; ++e)
    s[e] = __int_as_float(__builtin_amdgcn_sbfe(inv, key_of_acc(e), 1) & (int)0xFF800000u);
  return s;
}

template <int V>
struct IntC {
  static constexpr int value = V;
};

// Emission of the summed form: probabilities p = exp2(logit * c2 - lse) of every causal pair, added to
// A (and 1 to C). The kernel is bound by the read-modify-write of A and C, so K simply moves global
// -> registers -> LDS one stage ahead, and a block's probabilities are transposed through LDS so that
// a row's 32 keys are read and written as one 128-byte line.
__global__ __launch_bounds__(256) void k_capture_sum(CapArgs a, const __hip_bfloat16 *__restrict__ q,
                                                     const __hip_bfloat16 *__restrict__ k,
                                                     const float *__restrict__ lse2, float *__restrict__ attn_sum,
                                                     float *__restrict__ attn_cnt) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kStageBytes + 4 * 32 * kPadRow * 4];
  // Workgroup numbering: workgroup g runs on XCD g % 8; all query heads and query tiles of one KV head
  // get ids with the same g % 8, so that one XCD's L2 holds that head's K; within a KV head the long
  // rows come first.
  const int nQt = (a.n + kRows - 1) / kRows;
  const int G = a.Hq / a.Hkv, per_kv = G * nQt;
  const int xcd = blockIdx.x % kXcd, slot = blockIdx.x / kXcd;
  const int kv = (slot / per_kv) * kXcd + xcd, within = slot % per_kv;
  if (kv >= a.Hkv) return;
  const int qt = nQt - 1 - within / G, h = kv * G + within % G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int wave_first = qt * kRows + wave * 32;
  const int i = wave_first + n;  // this lane's query row
  const bool live = i < a.n;
  const int kbase = n * 256 + ((hf ^ (n & 15)) << 4);
  const unsigned char *kaddr[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) kaddr[c] = lds + (kbase ^ (c << 5));
  const __hip_bfloat16 *kp = k + (int64_t)kv * a.k_sh + (int64_t)(threadIdx.x >> 4) * a.k_ss + (threadIdx.x & 15) * 8;

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
  // stages that hold a key <= the tile's last live row
  const int last_row = min(qt * kRows + kRows - 1, a.n - 1);
  const int n_stage = last_row / kStageKeys + 1;
  const float my_lse = live ? lse2[(int64_t)h * a.L + i] : 0.0f;
  float *tile = reinterpret_cast<float *>(lds + 2 * kStageBytes) + wave * 32 * kPadRow;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // One block of 32 keys: buffer BUF (= st & 1), half HALF of its stage.
  auto block = [&](auto bufc, auto halfc, int st) {
    constexpr int BUF = decltype(bufc)::value, HALF = decltype(halfc)::value;
    constexpr int OFF = BUF * kStageBytes + HALF * kBlkBytes;
    const int key0 = st * kStageKeys + HALF * kBlk;
    if (key0 > wave_first + 31) return;  // wave-uniform: the block lies above all rows of this wave
    const f32x16 s = s_block<OFF>(kaddr, qf, zero);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float4 pv;
      pv.x = __builtin_amdgcn_exp2f(__builtin_fmaf(s[4 * g], a.c2, -my_lse));
      pv.y = __builtin_amdgcn_exp2f(__builtin_fmaf(s[4 * g + 1], a.c2, -my_lse));
      pv.z = __builtin_amdgcn_exp2f(__builtin_fmaf(s[4 * g + 2], a.c2, -my_lse));
      pv.w = __builtin_amdgcn_exp2f(__builtin_fmaf(s[4 * g + 3], a.c2, -my_lse));
      *reinterpret_cast<float4 *>(tile + n * kPadRow + 8 * g + 4 * hf) = pv;
    }
    // the tile is private to the wave, whose LDS operations complete in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int col = (lane & 7) * 4, j0 = key0 + col;
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
      const int r = (lane >> 3) + 8 * pass, row = wave_first + r;
      const float4 pv = *reinterpret_cast<const float4 *>(tile + r * kPadRow + col);
      if (row < a.n && j0 <= row) {
        float *ap = attn_sum + ((int64_t)h * a.L + row) * a.L + j0;
        float *cp = attn_cnt ? attn_cnt + ((int64_t)h * a.L + row) * a.L + j0 : nullptr;
        if (j0 + 3 <= row && (a.L & 3) == 0) {
          float4 av = *reinterpret_cast<float4 *>(ap);
          av.x += pv.x; av.y += pv.y; av.z += pv.z; av.w += pv.w;
          *reinterpret_cast<float4 *>(ap) = av;
          if (cp) {
            float4 cv = *reinterpret_cast<float4 *>(cp);
            cv.x += 1.0f; cv.y += 1.0f; cv.z += 1.0f; cv.w += 1.0f;
            *reinterpret_cast<float4 *>(cp) = cv;
          }
        } else {
          const float pe[4] = {pv.x, pv.y, pv.z, pv.w};
#pragma unroll
          for (int x = 0; x < 4; ++x)
            if (j0 + x <= row) {
              ap[x] += pe[x];
              if (cp) cp[x] += 1.0f;
            }
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };

  // One stage of 64 keys out of buffer BUF (= st & 1); the next stage's rows travel through registers
  // meanwhile and are written to the other buffer behind the blocks.
  auto stage = [&](auto bufc, int st) {
    constexpr int BUF = decltype(bufc)::value;
    KStage next;
    const bool more = st + 1 < n_stage;
    if (more) next = k_fetch(kp, a.k_ss, (st + 1) * kStageKeys, a.n);
    block(bufc, IntC<0>{}, st);
    block(bufc, IntC<1>{}, st);
    if (more) k_stash(lds + (BUF ^ 1) * kStageBytes, next);
    __syncthreads();
  };

  k_stash(lds, k_fetch(kp, a.k_ss, 0, a.n));
  __syncthreads();
  for (int st = 0; st < n_stage; st += 2) {
    stage(IntC<0>{}, st);
    if (st + 1 < n_stage) stage(IntC<1>{}, st + 1);  // workgroup-uniform
  }
}

// ------------------------------------------------------------------------------------------------
// Pipelined form of the two passes that emit no probabilities: PASS 0 reduces every row to its
// log-sum-exp, PASS 1 compares every logit with the row's threshold and packs the true-mask bits.
// A wave works on its blocks of 32 keys one after the other (block g: keys 32 g .. 32 g + 31, in
// half g & 1 of LDS buffer (g >> 1) & 1, i.e. at byte (g & 3) * 8 KiB); in step g it issues
//   the eight products of block g + 1 (one dependent chain into the other accumulator set),
//   the vector work on the finished logits of block g, cut into eight slices that sit between
//     the products (the wave issues in order: what stands between two products of a chain runs
//     in the shadow of the first),
//   the operand reads of block g + 2, each into the registers its product has just consumed.
// So the operands run two blocks ahead of the vector work, and a stage of 64 keys must be resident
// one stage before its first product: the rows of stage st + 2 are copied (load-to-LDS) during stage st
// into the buffer of stage st itself, which no wave reads then: the operand reads of a stage all fall
// into the stage before it. One barrier per stage.
template <int PASS>
__global__ __launch_bounds__(256) void k_capture_pipe(CapArgs a, const __hip_bfloat16 *__restrict__ q,
                                                      const __hip_bfloat16 *__restrict__ k, float *__restrict__ lse2,
                                                      const unsigned *__restrict__ theta_key,
                                                      uint64_t *__restrict__ true_bits) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kStageBytes];
  // workgroup numbering as in k_capture_sum
  const int nQt = (a.n + kRows - 1) / kRows;
  const int G = a.Hq / a.Hkv, per_kv = G * nQt;
  const int xcd = blockIdx.x % kXcd, slot = blockIdx.x / kXcd;
  const int kv = (slot / per_kv) * kXcd + xcd, within = slot % per_kv;
  if (kv >= a.Hkv) return;
  const int qt = nQt - 1 - within / G, h = kv * G + within % G;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, hf = lane >> 5;
  const int wave_first = qt * kRows + wave * 32;
  const int i = wave_first + n;  // this lane's query row
  const bool live = i < a.n;
  const int kbase = n * 256 + ((hf ^ (n & 15)) << 4);
  const unsigned char *kaddr[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) kaddr[c] = lds + (kbase ^ (c << 5));
  // K rows reach LDS by load-to-LDS copies: thread t brings piece (t & 15) ^ (row & 15) of row
  // t >> 4 (+ 16 per copy) of a stage to position t & 15 of that row. Rows past the sequence end are
  // redirected to the last row (such keys are masked by causality anyway).
  const char *kh = reinterpret_cast<const char *>(k + (int64_t)kv * a.k_sh);
  const int64_t row_bytes = a.k_ss * 2;
  const int srow = threadIdx.x >> 4;
  const unsigned piece = (((threadIdx.x & 15) ^ (srow & 15)) << 4);
  unsigned voff_full[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) voff_full[it] = (unsigned)((srow + 16 * it) * row_bytes) + piece;
  const unsigned lds_mine =
      __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds + wave * 1024);
  auto copy_stage = [&](int st, int buf) {
    const int key0 = st * kStageKeys;
    const char *gbase = kh + (int64_t)key0 * row_bytes;
    if (key0 + kStageKeys <= a.n) {  // workgroup-uniform
      k_copy_stage(lds_mine + buf * kStageBytes, gbase, voff_full);
    } else {
      unsigned voff[4];
#pragma unroll
      for (int it = 0; it < 4; ++it) voff[it] = (unsigned)(min(srow + 16 * it, a.n - 1 - key0) * row_bytes) + piece;
      k_copy_stage(lds_mine + buf * kStageBytes, gbase, voff);
    }
  };

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
  const int last_row = min(qt * kRows + kRows - 1, a.n - 1);
  const int n_stage = last_row / kStageKeys + 1;        // stages that hold a key <= the tile's last live row
  const int diag_g = qt * 4 + wave;                     // the wave's last block: the one the diagonal crosses
  const int n_blocks = min(diag_g + 1, 2 * n_stage);    // blocks 0 .. n_blocks - 1 hold a key <= a row of the wave

  // PASS 0 state: reference m_ref (log2 units; moves only when a maximum outgrows it by more than 8,
  // so that the sum rarely has to be rescaled) and the sum of exp2(t - m_ref) over this lane's keys
  float m_ref = -INFINITY, l_run = 0.0f;
  // PASS 1: p >= theta  <=>  raw logit >= (lse + log2 theta) / c2 up to rounding. The threshold arrives as an
  // ordered key: 0 keeps every causal entry, all ones keeps none; so do theta <= 0 and theta = +inf.
  float thr = 0.0f;
  if (PASS == 1) {
    const float my_lse = live ? lse2[(int64_t)h * a.L + i] : 0.0f;
    const unsigned tk = *theta_key;
    const float theta = __uint_as_float((tk & 0x80000000u) ? (tk & 0x7FFFFFFFu) : ~tk);
    if (tk == 0u || theta <= 0.0f) thr = -INFINITY;
    else if (tk == 0xFFFFFFFFu || !(theta < INFINITY)) thr = INFINITY;
    else thr = (my_lse + __builtin_amdgcn_logf(theta)) / a.c2;
  }
  unsigned words[4] = {0u, 0u, 0u, 0u};  // bits of the current 128-key group of this lane's row
  unsigned *out32 = reinterpret_cast<unsigned *>(true_bits + ((int64_t)h * a.L + (live ? i : 0)) * a.tbw);
  const int nw32 = a.tbw * 2;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 S0 = zero, S1 = zero;  // logits of the even / odd blocks
  bf16x8 kf[8];                 // operands of the next chain

  // ---- vector work of one block, in slices -------------------------------------------------------
  float blk_off = 0.0f, add0 = 0.0f, add1 = 0.0f;   // PASS 0, between the slices of a block
  unsigned neg = 0u;                                // PASS 1
  // PASS 0, first part: the block's maximum decides whether the reference moves
  auto ref_update = [&](const f32x16 &s) {
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; e += 2) mx = fmaxf(fmaxf(s[e], s[e + 1]), mx);
    mx *= a.c2;  // c2 > 0
    const bool move = mx - m_ref > 8.0f;  // false while both are -inf (NaN)
    if (__ballot(move)) {
      if (move) {
        l_run *= __builtin_amdgcn_exp2f(m_ref - mx);  // m_ref = -inf: 0
        m_ref = mx;
      }
    }
    blk_off = m_ref == -INFINITY ? 0.0f : m_ref;
    add0 = add1 = 0.0f;
  };
  // elements e0 .. e1 - 1 of a block
  auto slice = [&](const f32x16 &s, auto e0c, auto e1c) {
    constexpr int E0 = decltype(e0c)::value, E1 = decltype(e1c)::value;
    if (PASS == 0) {
#pragma unroll
      for (int e = E0; e < E1; ++e) {
        const float w = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], a.c2, -blk_off));
        if (e & 1) add1 += w;
        else add0 += w;
      }
    } else {
      // logit >= thr <=> the difference is not negative: the sign bits are shifted into a word one
      // by one, the last accumulator first, so that accumulator e ends at bit e
#pragma unroll
      for (int e = E0; e < E1; ++e)
        neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(s[15 - e] - thr), 31);
    }
  };
  auto finish = [&](auto g4c, int g) {
    constexpr int G4 = decltype(g4c)::value;
    if (PASS == 0) {
      l_run += add0 + add1;
    } else {
      // the four nibbles go to the key positions of a lower half-wave lane and are inverted
      unsigned v = neg & 0xFFFFu;
      v = (v | (v << 8)) & 0x00FF00FFu;
      v = (v | (v << 4)) & 0x0F0F0F0Fu;
      unsigned mine = (v ^ 0x0F0F0F0Fu) << (4 * hf);
      mine |= (unsigned)__shfl_xor((int)mine, 32);
      if (g == diag_g) mine &= causal_bits(i, g * kBlk);  // wave-uniform
      words[G4] = mine;
    }
  };

  // ---- one step -----------------------------------------------------------------------------------
  // G4 = g & 3. cur = logits of block g, nxt = accumulators of block g + 1.
  auto step = [&](auto g4c, int g) {
    constexpr int G4 = decltype(g4c)::value;
    constexpr int OFF2 = ((G4 + 2) & 3) * kBlkBytes;  // where block g + 2 lies
    f32x16 &cur = (G4 & 1) ? S1 : S0;
    f32x16 &nxt = (G4 & 1) ? S0 : S1;
    if (g >= 0 && g + 2 < n_blocks) {
      // steady state: neither block g nor block g + 1 touches the diagonal
#define DAM_CAP_SEG(C, VALU)                                                                       \
  nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[C], qf[C], (C) == 0 ? zero : nxt, 0, 0, 0);      \
  kf[C] = *reinterpret_cast<const bf16x8 *>(kaddr[C] + OFF2);                                       \
  VALU;                                                                                             \
  __builtin_amdgcn_sched_barrier(0);
      if (PASS == 0) {
        // the maximum first (it needs every logit); its instructions are short and stay in front
        ref_update(cur);
        __builtin_amdgcn_sched_barrier(0);
        DAM_CAP_SEG(0, slice(cur, IntC<0>{}, IntC<2>{}))
        DAM_CAP_SEG(1, slice(cur, IntC<2>{}, IntC<4>{}))
        DAM_CAP_SEG(2, slice(cur, IntC<4>{}, IntC<6>{}))
        DAM_CAP_SEG(3, slice(cur, IntC<6>{}, IntC<8>{}))
        DAM_CAP_SEG(4, slice(cur, IntC<8>{}, IntC<10>{}))
        DAM_CAP_SEG(5, slice(cur, IntC<10>{}, IntC<12>{}))
        DAM_CAP_SEG(6, slice(cur, IntC<12>{}, IntC<14>{}))
        DAM_CAP_SEG(7, slice(cur, IntC<14>{}, IntC<16>{}))
      } else {
        DAM_CAP_SEG(0, slice(cur, IntC<0>{}, IntC<2>{}))
        DAM_CAP_SEG(1, slice(cur, IntC<2>{}, IntC<4>{}))
        DAM_CAP_SEG(2, slice(cur, IntC<4>{}, IntC<6>{}))
        DAM_CAP_SEG(3, slice(cur, IntC<6>{}, IntC<8>{}))
        DAM_CAP_SEG(4, slice(cur, IntC<8>{}, IntC<10>{}))
        DAM_CAP_SEG(5, slice(cur, IntC<10>{}, IntC<12>{}))
        DAM_CAP_SEG(6, slice(cur, IntC<12>{}, IntC<14>{}))
        DAM_CAP_SEG(7, slice(cur, IntC<14>{}, IntC<16>{}))
      }
#undef DAM_CAP_SEG
      finish(g4c, g);
      return;
    }
    // the first step (g = -1: only the chain of block 0) and the last ones of the wave
    const bool do_chain = g + 1 < n_blocks, do_read = g + 2 < n_blocks, do_valu = g >= 0 && g < n_blocks;
    if (do_chain) {
      // entries above the diagonal start from -inf, so that the products leave them there
      f32x16 acc = zero;
      if (PASS == 0 && g + 1 == diag_g) acc = causal_start(causal_bits(i, (g + 1) * kBlk) >> (4 * hf));
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[c], qf[c], acc, 0, 0, 0);
        if (do_read) kf[c] = *reinterpret_cast<const bf16x8 *>(kaddr[c] + OFF2);
      }
      nxt = acc;
    }
    if (do_valu) {
      if (PASS == 0) ref_update(cur);
      slice(cur, IntC<0>{}, IntC<16>{});
      finish(g4c, g);
    }
  };

  // One stage of 64 keys (st & 1 = B): the steps of its two blocks; the rows of stage st + 2 travel
  // through registers meanwhile and replace this stage's, which nobody reads any more.
  auto stage = [&](auto bc, int st) {
    constexpr int B = decltype(bc)::value;
    const bool more2 = st + 2 < n_stage;
    if (more2) copy_stage(st + 2, B);
    step(IntC<2 * B>{}, 2 * st);
    step(IntC<2 * B + 1>{}, 2 * st + 1);
    // this wave's copies have landed (and the bit stores of the group before: a whole stage old)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (PASS == 1 && (B == 1 || st + 1 >= n_stage)) {
      // the 128-key group is complete (blocks above this wave's rows contributed zeros)
      if (live && hf == 0) {
        const int w0 = (st >> 1) * 4;
        if (w0 + 3 < nw32 && (a.tbw & 1) == 0) {
          *reinterpret_cast<uint4 *>(out32 + w0) = make_uint4(words[0], words[1], words[2], words[3]);
        } else {
#pragma unroll
          for (int x = 0; x < 4; ++x)
            if (w0 + x < nw32) out32[w0 + x] = words[x];
        }
      }
      words[0] = words[1] = words[2] = words[3] = 0u;
    }
    __syncthreads();
  };

  copy_stage(0, 0);
  if (n_stage > 1) copy_stage(1, 1);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
#pragma unroll
  for (int c = 0; c < 8; ++c) kf[c] = *reinterpret_cast<const bf16x8 *>(kaddr[c]);
  step(IntC<3>{}, -1);
  __syncthreads();  // buffer 0 is rewritten at the end of stage 0: every wave has read block 0 and 1 by now
  for (int st = 0; st < n_stage; st += 2) {
    stage(IntC<0>{}, st);
    if (st + 1 < n_stage) stage(IntC<1>{}, st + 1);  // workgroup-uniform
  }
  if (PASS == 0) {
    const float m_o = __shfl_xor(m_ref, 32), l_o = __shfl_xor(l_run, 32);
    const float M = fmaxf(m_ref, m_o);  // finite: every live row holds key 0
    const float tot = l_run * __builtin_amdgcn_exp2f(m_ref - M) + l_o * __builtin_amdgcn_exp2f(m_o - M);
    if (live && hf == 0) lse2[(int64_t)h * a.L + i] = M + __builtin_amdgcn_logf(tot);
  } else {
    // words of the tile's rows past its last 128-key group: all zero (keys above the diagonal);
    // written by the whole workgroup, 16 bytes per thread along a row
    const int w_done = ((n_stage + 1) / 2) * 4, rest = nw32 - w_done;
    if (rest > 0) {
      const int rows = min(kRows, a.n - qt * kRows), per_row = (rest + 3) / 4;
      unsigned *tile_out = reinterpret_cast<unsigned *>(true_bits + ((int64_t)h * a.L + qt * kRows) * a.tbw);
      for (int x = threadIdx.x; x < rows * per_row; x += 256) {
        const int r = x / per_row, w = w_done + 4 * (x % per_row);
        unsigned *dst = tile_out + (int64_t)r * nw32 + w;
        if (w + 3 < nw32 && (a.tbw & 1) == 0) {
          *reinterpret_cast<uint4 *>(dst) = make_uint4(0u, 0u, 0u, 0u);
        } else {
          for (int y = 0; y < 4 && w + y < nw32; ++y) dst[y] = 0u;
        }
      }
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
    const int nQt = (a.n + kRows - 1) / kRows;
    const dim3 grid((a.Hkv + kXcd - 1) / kXcd * kXcd * (a.Hq / a.Hkv) * nQt);
    const __hip_bfloat16 *qb = static_cast<const __hip_bfloat16 *>(q), *kb = static_cast<const __hip_bfloat16 *>(k);
    k_capture_pipe<0><<<grid, 256, 0, st>>>(a, qb, kb, lse2, theta_key, true_bits);
    if (MODE == kEmitBits) k_capture_pipe<1><<<grid, 256, 0, st>>>(a, qb, kb, lse2, theta_key, true_bits);
    else k_capture_sum<<<grid, 256, 0, st>>>(a, qb, kb, lse2, attn_sum, attn_cnt);
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
  if (p->k_stride[1] >= (1 << 24)) return DAM_ERR_UNSUPPORTED;  // byte offsets inside a stage of 64 rows are 32-bit
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
