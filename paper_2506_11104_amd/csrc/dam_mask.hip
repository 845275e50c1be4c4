// dam_mask_build: attention statistics at the pattern capture length -> per-head sparse mask.
//
// Paper (arXiv 2506.11104): Sec. 4.2.2 (mean, clamp, Box-Cox, global-min shift), Sec. 4.2.3 (true
// mask by threshold tau), Sec. 4.2.4 (diagonal / vertical pattern pool, match score gamma against
// mu), Sec. 4.3 (mask of a length-S problem: true mask inside the L x L block, matched patterns
// continued elsewhere). The tile pooling, block index and kept lists are this library's own data
// structures for the sparse attention kernels.
//
// Everything here is streaming bit work bounded by HBM bandwidth: A is read once (lower triangle
// only for a single causal capture), one wave turns 64 keys into one mask word with a ballot, and
// the S x S mask is never materialised: any 64-key word of any row is recomputed on the fly from
// the true bits, the column bitset and a bit-reversed diagonal bitset (one funnel shift).
#include <math.h>

#include <algorithm>
#include <type_traits>

#include "dam_internal.h"

#pragma clang fp contract(off)

namespace {
using namespace dam;

// Workgroups of a launch whose items are short: enough to fill the chip twice (256 CUs x 8 workgroups of
// 256 threads); each takes several items in turn.
constexpr int kGridTarget = 4096;
constexpr int kHeadSub = 16;  // partial sums per head of the listed-tile counts

struct Geom {
  int H, L, S, P;            // P: length of the pattern flag arrays (L from a map, S when given)
  int tile_m, tile_n, nQt, nKt, wpr;
  int tbw;                   // words per true_bits row, ceil(L / 64)
  int pw;                    // words per pattern bitset, ceil(P / 64)
  int occw;                  // occupancy words per query tile, ceil(nKt / 64)
};

// ------------------------------------------------------------------------------------------------
// Sec. 4.2.2 in the fixed fp32 sequence (each op rounded to nearest, nothing contracted: this file
// is compiled with contraction off and with correctly rounded fp32 divide and square root; the
// __fsqrt_rn / __fdiv_rn intrinsics are NOT used because they map to the approximate forms).
__host__ __device__ __forceinline__ float clamp_mean(float a, float c, float eps) {
  const float denom = c + eps;
  const float abar = a / denom;
  return fmaxf(abar, eps);
}

template <int LAMBDA2>  // 2 * lambda: 1 -> lambda 0.5, 2 -> lambda 1
__host__ __device__ __forceinline__ float box_cox(float x) {
  if (LAMBDA2 == 1) {
    const float root = sqrtf(x);
    const float num = root - 1.0f;
    return num / 0.5f;
  }
  return x - 1.0f;
}

__global__ void k_copy_f32(float *dst, const float *src) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *dst = *src;
}

// General case: min over every stored entry. min B = B(min X) because every step after X is
// non-decreasing; X > 0, so its bit pattern orders like an unsigned integer.
__global__ void k_min_x(const float *__restrict__ A, const float *__restrict__ C, int64_t n, int L,
                        float eps, unsigned *xmin_bits) {
  float m = INFINITY;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
       e += (int64_t)gridDim.x * blockDim.x) {
    float a, c;
    if (C) {
      a = A[e];
      c = C[e];
    } else {  // only reached for L == 1 (a single valid pair per map)
      a = A[e];
      c = 1.0f;
    }
    m = fminf(m, clamp_mean(a, c, eps));
  }
  for (int off = 32; off; off >>= 1) m = fminf(m, __shfl_xor(m, off));
  if ((threadIdx.x & 63) == 0) atomicMin(xmin_bits, __float_as_uint(m));
}

template <int LAMBDA2>
__global__ void k_bmin_from_x(const unsigned *xmin_bits, float *bmin) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *bmin = box_cox<LAMBDA2>(__uint_as_float(*xmin_bits));
}

__global__ void k_fill_u32(unsigned *p, int64_t n, unsigned v) {
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n;
       e += (int64_t)gridDim.x * blockDim.x)
    p[e] = v;
}

// ------------------------------------------------------------------------------------------------
// Sec. 4.2.3: m[i][j] = (B - bmin >= tau) and j <= i. One wave = 4 rows x 4 words (256 keys); each
// lane owns one key per word so every load is a fully coalesced 256-byte row segment, and the
// 16 loads of a lane are independent. Entries above the diagonal are never kept, so never read.
constexpr int kTmRows = 64;  // rows per block (4 passes of 4 rows per wave)

// Every operation of the fixed fp32 sequence (divide by a positive constant, max, square root,
// subtract, compare) is rounded to nearest and therefore non-decreasing in its input, so the keep
// decision (Sec. 4.2.3) is a step function of the mean attention abar (of A itself when no count
// matrix is given: then abar = A / (1 + eps)): keep <=> value >= theta for one fp32 number theta.
// k_threshold finds theta by bisection over the ordered bit patterns of fp32, evaluating the exact
// sequence at each probe; k_true_mask then needs one comparison per element and stays bit-exact.
// Ordered key: increasing with the value over [-inf, +inf]; a NaN is treated as -inf, which is what
// the sequence does with it (fmaxf(NaN, eps) = eps, the smallest clamped value).
__host__ __device__ __forceinline__ unsigned key_of(float x) {
  const unsigned b = __builtin_bit_cast(unsigned, x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__host__ __device__ __forceinline__ float value_of(unsigned k) {
  return __builtin_bit_cast(float, (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}
constexpr unsigned kKeyNegInf = 0x007FFFFFu, kKeyPosInf = 0xFF800000u;
constexpr unsigned kKeepAll = 0u, kKeepNone = 0xFFFFFFFFu;

template <int LAMBDA2, bool FROM_A>
__host__ __device__ __forceinline__ bool keep_at(float v, float eps, float tau, float bmin) {
  const float x = FROM_A ? clamp_mean(v, 1.0f, eps) : fmaxf(v, eps);
  const float bstar = box_cox<LAMBDA2>(x) - bmin;
  return bstar >= tau;
}

// (host and device: the sequence is correctly rounded IEEE arithmetic on both, so when the minimum is known
// without looking at the data -- an override, or the closed form of a single causal capture -- the bisection runs
// on the host and the first kernel of the chain takes the key by value)
template <int LAMBDA2, bool FROM_A>
__host__ __device__ unsigned threshold_key(float eps, float tau, float bmin) {
  unsigned lo = kKeyNegInf, hi = kKeyPosInf;
  if (!keep_at<LAMBDA2, FROM_A>(value_of(hi), eps, tau, bmin)) return kKeepNone;
  if (keep_at<LAMBDA2, FROM_A>(value_of(lo), eps, tau, bmin)) return kKeepAll;
  while (hi - lo > 1u) {  // keep(lo) false, keep(hi) true
    const unsigned mid = lo + (hi - lo) / 2u;
    if (keep_at<LAMBDA2, FROM_A>(value_of(mid), eps, tau, bmin)) hi = mid;
    else lo = mid;
  }
  return hi;
}

template <int LAMBDA2, bool FROM_A>
__global__ void k_threshold(float eps, float tau, const float *__restrict__ bmin_p, unsigned *__restrict__ theta_key) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  *theta_key = threshold_key<LAMBDA2, FROM_A>(eps, tau, *bmin_p);
}

// minimum and key found on the host: into the workspace (and the caller's bmin) for the kernels that read them there
__global__ void k_set_threshold(float bmin, unsigned key, float *__restrict__ ws_bmin, unsigned *__restrict__ ws_key,
                                float *__restrict__ out_bmin) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  *ws_bmin = bmin;
  *ws_key = key;
  if (out_bmin) *out_bmin = bmin;
}

// ------------------------------------------------------------------------------------------------
// App. B: the alternative transforms between the mean map and the threshold (dam_transform other
// than Box-Cox). Every one of them is non-decreasing in the mean (raw sum: in the sum), so the same
// scheme applies: the statistics the transform needs are reduced over every stored entry, the
// minimum of the transformed map is the transform of the smallest input, and one thread bisects for
// the smallest input value that is kept. raw sum, average, min-max and square root are exact fp32
// sequences; log, Yeo-Johnson, arcsinh use the device's library functions and z-score sums in fp64
// with atomics, so their decisions can differ from another implementation's within rounding of the
// threshold.
struct TransformStats {
  unsigned xmin_bits, xmax_bits;  // X > 0: its bit pattern orders like an unsigned integer
  unsigned amin_key, abarmin_key; // ordered keys (see key_of) of the smallest sum and the smallest mean
  double sum, sumsq;              // of X
};

struct TransformCtx {
  int kind;
  float lambda, eps, tau, tmin, p0, p1;  // p0, p1: (mu, sigma) for z-score, (min X, max X) for min-max
};

__global__ void k_stats_init(TransformStats *st) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    st->xmin_bits = 0x7F800000u;
    st->xmax_bits = 0u;
    st->amin_key = kKeyPosInf;
    st->abarmin_key = kKeyPosInf;
    st->sum = 0.0;
    st->sumsq = 0.0;
  }
}

__global__ __launch_bounds__(256) void k_stats(const float *__restrict__ A, const float *__restrict__ C, int64_t n, int L,
                                               float eps, TransformStats *st) {
  float xmin = INFINITY, xmax = 0.0f;
  unsigned amin = kKeyPosInf, abarmin = kKeyPosInf;
  double sum = 0.0, sumsq = 0.0;
  const int64_t LL = (int64_t)L * L;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
    float a, c;
    if (C) {
      a = A[e];
      c = C[e];
    } else {
      const int64_t r = e % LL;
      const bool causal = r % L <= r / L;
      a = causal ? A[e] : 0.0f;
      c = causal ? 1.0f : 0.0f;
    }
    const float denom = c + eps;
    const float abar = a / denom;
    const float x = fmaxf(abar, eps);
    xmin = fminf(xmin, x);
    xmax = fmaxf(xmax, x);
    amin = min(amin, key_of(a != a ? -INFINITY : a));
    abarmin = min(abarmin, key_of(abar != abar ? -INFINITY : abar));
    sum += (double)x;
    sumsq += (double)x * (double)x;
  }
  for (int off = 32; off; off >>= 1) {
    xmin = fminf(xmin, __shfl_xor(xmin, off));
    xmax = fmaxf(xmax, __shfl_xor(xmax, off));
    amin = min(amin, (unsigned)__shfl_xor((int)amin, off));
    abarmin = min(abarmin, (unsigned)__shfl_xor((int)abarmin, off));
    sum += __shfl_xor(sum, off);
    sumsq += __shfl_xor(sumsq, off);
  }
  if ((threadIdx.x & 63) == 0) {
    atomicMin(&st->xmin_bits, __float_as_uint(xmin));
    atomicMax(&st->xmax_bits, __float_as_uint(xmax));
    atomicMin(&st->amin_key, amin);
    atomicMin(&st->abarmin_key, abarmin);
    atomicAdd(&st->sum, sum);
    atomicAdd(&st->sumsq, sumsq);
  }
}

// The transform of a mean value abar (raw sum: of a sum) in the fixed fp32 sequence.
__device__ float transform_of(const TransformCtx &c, float v) {
  if (c.kind == DAM_T_RAW_SUM || c.kind == DAM_T_AVERAGE) return v;
  const float x = fmaxf(v, c.eps);
  switch (c.kind) {
    case DAM_T_LOG:
      return logf(x);
    case DAM_T_YEO_JOHNSON: {
      const float x1 = x + 1.0f;
      if (c.lambda == 0.0f) return logf(x1);
      const float p = powf(x1, c.lambda);
      const float num = p - 1.0f;
      return num / c.lambda;
    }
    case DAM_T_ZSCORE: {
      const float num = x - c.p0;
      const float den = c.p1 + c.eps;
      return num / den;
    }
    case DAM_T_MINMAX: {
      const float num = x - c.p0;
      const float range = c.p1 - c.p0;
      const float den = range + c.eps;
      return num / den;
    }
    case DAM_T_SQRT:
      return sqrtf(x);
    default:  // DAM_T_ARCSINH
      return asinhf(x);
  }
}

// Context of the transform and the threshold key. from_a: the compared value is the sum of a single
// capture (the mean is sum / (1 + eps)); otherwise it is the mean itself (raw sum: always the sum).
__global__ void k_transform_threshold(int kind, float lambda, float eps, float tau, float tmin_override,
                                      const TransformStats *__restrict__ st, bool from_a, float n_entries,
                                      double n_exact, float *__restrict__ bmin, unsigned *__restrict__ theta_key) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  TransformCtx c;
  c.kind = kind; c.lambda = lambda; c.eps = eps; c.tau = tau; c.p0 = 0.0f; c.p1 = 0.0f;
  const float xmin = __uint_as_float(st->xmin_bits), xmax = __uint_as_float(st->xmax_bits);
  if (kind == DAM_T_ZSCORE) {
    const double mean = st->sum / n_exact;
    double var = st->sumsq / n_exact - mean * mean;
    if (var < 0.0) var = 0.0;
    c.p0 = (float)mean;
    c.p1 = (float)sqrt(var);
  } else if (kind == DAM_T_MINMAX) {
    c.p0 = xmin;
    c.p1 = xmax;
  }
  // every transform is non-decreasing: the minimum of the map is the transform of the smallest input
  float tmin;
  if (kind == DAM_T_RAW_SUM) tmin = value_of(st->amin_key);
  else if (kind == DAM_T_AVERAGE) tmin = value_of(st->abarmin_key);
  else tmin = transform_of(c, xmin);
  if (tmin_override == tmin_override) tmin = tmin_override;
  c.tmin = tmin;
  *bmin = tmin;
  auto keep = [&](float v) {
    if (kind != DAM_T_RAW_SUM && from_a) {
      const float denom = 1.0f + eps;
      v = v / denom;
    }
    const float t = transform_of(c, v);
    return t - c.tmin >= tau;
  };
  unsigned lo = kKeyNegInf, hi = kKeyPosInf;
  if (!keep(value_of(hi))) {
    *theta_key = kKeepNone;
    return;
  }
  if (keep(value_of(lo))) {
    *theta_key = kKeepAll;
    return;
  }
  while (hi - lo > 1u) {
    const unsigned mid = lo + (hi - lo) / 2u;
    if (keep(value_of(mid))) hi = mid;
    else lo = mid;
  }
  *theta_key = hi;
}

// The threshold key comes from the workspace (theta_key) or, when the host found it, by value (theta_key == nullptr:
// theta_val, and bmin_val goes to the caller's bmin from here, this being the first kernel of the chain).
struct Threshold {
  const unsigned *theta_key;
  unsigned theta_val;
  float bmin_val;
  float *bmin_out;
};

__device__ __forceinline__ unsigned take_threshold(const Threshold &t) {
  if (t.theta_key) return *t.theta_key;
  if (t.bmin_out && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0) *t.bmin_out = t.bmin_val;
  return t.theta_val;
}

template <bool FROM_A, bool RAW = false>
__global__ __launch_bounds__(256) void k_true_mask(const float *__restrict__ A, const float *__restrict__ C, int L,
                                                   int tbw, float eps, Threshold thr,
                                                   uint64_t *__restrict__ true_bits) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = blockIdx.z;
  const int w0 = blockIdx.x * 4;
  const unsigned theta = take_threshold(thr);
  const float *Ah = A + (int64_t)h * L * L;
  const float *Ch = FROM_A ? nullptr : C + (int64_t)h * L * L;
  constexpr int kIter = kTmRows / 16;  // passes of 4 rows per wave
#pragma unroll 2
  for (int it = 0; it < kIter; ++it) {
    const int r0 = blockIdx.y * kTmRows + (it * 4 + wave) * 4;
    float a[4][4], c[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int i = r0 + r, j = (w0 + k) * 64 + lane;
        const bool live = i < L && j <= i;
        a[r][k] = live ? Ah[(int64_t)i * L + j] : 0.0f;
        if (!FROM_A) c[r][k] = live ? Ch[(int64_t)i * L + j] : 0.0f;
      }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int i = r0 + r, j = (w0 + k) * 64 + lane;
        const bool live = i < L && j <= i;
        float v = a[r][k];
        if (!FROM_A && !RAW) v = v / (c[r][k] + eps);
        if (v != v) v = -INFINITY;
        const uint64_t word = __ballot(live && key_of(v) >= theta);
        if (lane == 0 && i < L && w0 + k < tbw) true_bits[((int64_t)h * L + i) * tbw + w0 + k] = word;
      }
  }
}

// The same for the common case (no count matrix, L a multiple of 4) at streaming speed: one wave per
// row, 16-byte loads, the live 256-key segments of a 2048-key span in flight at once, and the row's
// words gathered into lanes so that they leave as one coalesced store (single 8-byte stores from one
// lane made the store path the bottleneck).
__device__ __forceinline__ float4 load_once(const float4 *p) {
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
  return make_float4(t.x, t.y, t.z, t.w);
}

// FAST: theta is the key of a normal positive number (or keeps nothing, a NaN once decoded), and then
// key_of(v) >= theta is the plain comparison v >= value_of(theta): zeros, denormals and negative values
// lie below theta in either order, a NaN fails both. Segments that end before the diagonal then cost one
// comparison per element (0.490 -> 0.475 ms for 64 maps of 4096 x 4096).
template <bool FAST>
__device__ __forceinline__ void true_mask_row(const float *__restrict__ A, int L, int tbw, int h, int i_any, unsigned theta,
                                              uint64_t *__restrict__ true_bits, int lane) {
  const int i = __builtin_amdgcn_readfirstlane(i_any);
  const float4 *row = reinterpret_cast<const float4 *>(A + ((int64_t)h * L + i) * L);
  uint64_t *out = true_bits + ((int64_t)h * L + i) * tbw;
  const int nseg = i / 256 + 1;  // segments with a key <= i
  const int c = lane & 3;
  const float theta_f = value_of(theta);
  constexpr int kSeg = 8;  // 256-key segments in flight per pass
  for (int s0 = 0; s0 * 4 < tbw; s0 += kSeg) {
    float4 v[kSeg];
#pragma unroll
    for (int u = 0; u < kSeg; ++u) {
      const int j0 = (s0 + u) * 256 + lane * 4;
      v[u] = (s0 + u < nseg && j0 < L) ? load_once(row + (s0 + u) * 64 + lane) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    uint64_t mine = 0;  // word s0 * 4 + lane of the row
#pragma unroll
    for (int u = 0; u < kSeg; ++u) {
      if (s0 + u < nseg) {  // wave-uniform
        const int j0 = (s0 + u) * 256 + lane * 4;
        float x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
        uint64_t b[4];
        if (FAST && s0 + u < nseg - 1) {  // every key of the segment is <= i
#pragma unroll
          for (int e = 0; e < 4; ++e) b[e] = __ballot(x[e] >= theta_f);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float val = x[e] != x[e] ? -INFINITY : x[e];
            b[e] = __ballot(j0 + e <= i && key_of(val) >= theta);  // bit l: key 4 l + e of the segment
          }
        }
        // lane l of word w is key 64 w + l = component l % 4 of lane 16 w + l / 4
        const uint64_t sel = c == 0 ? b[0] : c == 1 ? b[1] : c == 2 ? b[2] : b[3];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint64_t word = __ballot((sel >> (16 * w + (lane >> 2))) & 1);
          if (lane == u * 4 + w) mine = word;
        }
      }
    }
    if (lane < 4 * kSeg && s0 * 4 + lane < tbw) out[s0 * 4 + lane] = mine;
  }
}

// Rows are taken in quads (one row per wave); quad 2 p holds rows 4 p .. 4 p + 3, quad 2 p + 1 the rows
// that complement them, L - 1 - (4 p .. 4 p + 3), so that a pair of quads is the same work whatever p.
// A workgroup takes several pairs in turn (a little faster than a workgroup per quad: 0.60 -> 0.59 ms for
// 64 maps of 4096 x 4096).
template <bool FAST>
__device__ __forceinline__ void true_mask_pairs(const float *__restrict__ A, int L, int tbw, int n_pairs, unsigned theta,
                                                uint64_t *__restrict__ true_bits) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = blockIdx.y;
  const int half = (L + 1) / 2;
  for (int pair = blockIdx.x; pair < n_pairs; pair += gridDim.x) {
    const int lo = pair * 4 + wave, hi = L - 1 - lo;
    if (lo >= half) continue;
    true_mask_row<FAST>(A, L, tbw, h, lo, theta, true_bits, lane);
    if (hi >= half) true_mask_row<FAST>(A, L, tbw, h, hi, theta, true_bits, lane);
  }
}

__global__ __launch_bounds__(256) void k_true_mask_rows(const float *__restrict__ A, int L, int tbw, int n_pairs,
                                                        Threshold thr, uint64_t *__restrict__ true_bits) {
  const unsigned theta = take_threshold(thr);
  if (theta >= 0x80800000u) true_mask_pairs<true>(A, L, tbw, n_pairs, theta, true_bits);  // key of FLT_MIN
  else true_mask_pairs<false>(A, L, tbw, n_pairs, theta, true_bits);
}

// Sec. 4.2.4 numerators: kept entries per column and per diagonal of the true mask, counted with
// carry-save adders on whole 64-bit words. A wave takes a chunk of 64 rows; lane l owns word l of
// every row (64 columns) and adds the 64 row words into a bit-sliced counter (slice k holds bit k of
// the 64 column counts), two logic operations per full adder. For the diagonals the row word is first
// re-aligned: word l of row i then holds m[i][i - r] for r = 64 l .. 64 l + 63 (a funnel shift of two
// adjacent words and a bit reversal), after which diagonals are columns. The slices of every chunk
// go to the workspace; k_pattern_finish sums them per pattern and applies the ratio test. No atomics.
constexpr int kSlices = 7;      // counts 0 .. 64
constexpr int kChunkRows = 64;

__device__ __forceinline__ void csa(uint64_t &carry, uint64_t &sum, uint64_t a, uint64_t b, uint64_t c) {
  const uint64_t u = a ^ b;
  carry = (a & b) | (u & c);
  sum = u ^ c;
}

// Form for rows of more than 128 words (capture lengths above 8192): a wave per 64 rows and 64 words,
// every word fetched from global memory by the lane that owns it (one launch for both pattern kinds: the
// upper half of the grid's x range counts diagonals).
__global__ __launch_bounds__(256) void k_pattern_slices_wide(const uint64_t *__restrict__ true_bits, int L, int tbw,
                                                        int n_chunks, uint64_t *__restrict__ vslices,
                                                        uint64_t *__restrict__ dslices) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = blockIdx.z;
  const int chunk = blockIdx.y * 4 + wave;
  const int xw = gridDim.x / 2;
  const bool DIAG = (int)blockIdx.x >= xw;  // block-uniform
  uint64_t *slices = DIAG ? dslices : vslices;
  const int wl = ((int)blockIdx.x - (DIAG ? xw : 0)) * 64 + lane;  // word of columns (or of diagonal offsets) owned by this lane
  if (chunk >= n_chunks || wl >= tbw) return;
  const int i0 = chunk * kChunkRows;
  const uint64_t *tb = true_bits + (int64_t)h * L * tbw;
  uint64_t s[kSlices];
#pragma unroll
  for (int k = 0; k < kSlices; ++k) s[k] = 0;
  // a column (offset) block that starts beyond the chunk's last row holds no kept entry
  if (64 * wl <= i0 + kChunkRows - 1) {
    for (int g = 0; g < kChunkRows; g += 8) {
      uint64_t w[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 + g + u;
        uint64_t x = 0;
        if (i < L) {
          if (!DIAG) {
            x = tb[(int64_t)i * tbw + wl];
          } else {
            const int jhi = i - 64 * wl;  // the column of offset r = 64 wl in this row
            if (jhi >= 0) {
              const int wj = jhi >> 6, sh = (jhi & 63) + 1;  // window = bits jhi-63 .. jhi of the row
              const uint64_t hi = tb[(int64_t)i * tbw + wj];
              const uint64_t lo = wj > 0 ? tb[(int64_t)i * tbw + wj - 1] : 0;
              const uint64_t win = sh == 64 ? hi : ((hi << (64 - sh)) | (lo >> sh));
              x = __brevll(win);                             // offset r = 64 wl + t at bit t
            }
          }
        }
        w[u] = x;
      }
      uint64_t t0, t1, f0, f1, e;
      csa(t0, s[0], s[0], w[0], w[1]);
      csa(t1, s[0], s[0], w[2], w[3]);
      csa(f0, s[1], s[1], t0, t1);
      csa(t0, s[0], s[0], w[4], w[5]);
      csa(t1, s[0], s[0], w[6], w[7]);
      csa(f1, s[1], s[1], t0, t1);
      csa(e, s[2], s[2], f0, f1);
      // add the eights into slices 3 .. 6 (ripple)
#pragma unroll
      for (int k = 3; k < kSlices; ++k) {
        const uint64_t c = s[k] & e;
        s[k] ^= e;
        e = c;
      }
    }
  }
  uint64_t *out = slices + (((int64_t)h * n_chunks + chunk) * kSlices) * tbw + wl;
#pragma unroll
  for (int k = 0; k < kSlices; ++k) out[(int64_t)k * tbw] = s[k];
}

// Form for rows of up to 128 words: one workgroup per (head, chunk of 64 rows) counts both pattern
// kinds from one copy of the chunk in LDS, so that the true mask is read once (its lower triangle
// only: a word past the chunk's diagonal holds nothing). W = the number of words up to that diagonal
// rounded up to a power of two (16 .. 128); thread t owns word t % W of the rows t / W, t / W + 256 / W, ...:
// for the columns that is the row's word itself, for the diagonals the window of the row that ends
// at column i - 64 w, reversed (two neighbouring words of the LDS copy, a funnel shift and a bit
// reversal). The 256 / W partial counters of a word are added through LDS (bit-sliced, 7 + 7 bits).
__global__ __launch_bounds__(256) void k_pattern_slices(const uint64_t *__restrict__ true_bits, int L, int tbw,
                                                        int n_chunks, int Wmax, uint64_t *__restrict__ vslices,
                                                        uint64_t *__restrict__ dslices) {
  extern __shared__ uint64_t sm[];  // [64][W] row words, afterwards [2][256 / W][kSlices][W] partial counters
  const int chunk = blockIdx.x, h = blockIdx.y, i0 = chunk * kChunkRows;
  const int rows = min(kChunkRows, L - i0);
  const int wmax = min(tbw, chunk + 1);  // words that can hold a kept entry of these rows
  int W = 16;                            // ... rounded up to a power of two: the threads share those words only
  while (W < wmax) W *= 2;
  W = min(W, Wmax);
  const int wl = threadIdx.x & (W - 1), sub = threadIdx.x / W, nsub = 256 / W;
  const uint64_t *tb = true_bits + ((int64_t)h * L + i0) * tbw;
  for (int r0 = sub; r0 < kChunkRows; r0 += 8 * nsub) {  // eight loads in flight per thread
    uint64_t v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int r = r0 + u * nsub;
      v[u] = (r < rows && wl < wmax) ? __builtin_nontemporal_load(tb + (int64_t)r * tbw + wl) : 0;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int r = r0 + u * nsub;
      if (r < kChunkRows) sm[r * W + wl] = v[u];
    }
  }
  __syncthreads();
  uint64_t sc[kSlices], sd[kSlices];
#pragma unroll
  for (int k = 0; k < kSlices; ++k) sc[k] = sd[k] = 0;
  const int wj = chunk - wl;  // word of column i - 64 wl, the same for every row of the chunk
  const int per_thread = kChunkRows / nsub;
  for (int g = 0; g < per_thread; g += 8) {
    uint64_t c[8], d[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int r = sub + nsub * (g + u);  // rows past the chunk's end are zero in LDS
      uint64_t xc = 0, xd = 0;
      if (g + u < per_thread) {
        xc = sm[r * W + wl];
        if (wj >= 0) {
          const int sh = r + 1;  // window = bits jhi - 63 .. jhi of the row, jhi = 64 wj + r
          const uint64_t hi = sm[r * W + wj];
          const uint64_t lo = wj > 0 ? sm[r * W + wj - 1] : 0;
          const uint64_t win = sh == 64 ? hi : ((hi << (64 - sh)) | (lo >> sh));
          xd = __brevll(win);  // offset r = 64 wl + t at bit t
        }
      }
      c[u] = xc;
      d[u] = xd;
    }
    uint64_t t0, t1, f0, f1, e;
    csa(t0, sc[0], sc[0], c[0], c[1]);
    csa(t1, sc[0], sc[0], c[2], c[3]);
    csa(f0, sc[1], sc[1], t0, t1);
    csa(t0, sc[0], sc[0], c[4], c[5]);
    csa(t1, sc[0], sc[0], c[6], c[7]);
    csa(f1, sc[1], sc[1], t0, t1);
    csa(e, sc[2], sc[2], f0, f1);
#pragma unroll
    for (int k = 3; k < kSlices; ++k) {
      const uint64_t cy = sc[k] & e;
      sc[k] ^= e;
      e = cy;
    }
    csa(t0, sd[0], sd[0], d[0], d[1]);
    csa(t1, sd[0], sd[0], d[2], d[3]);
    csa(f0, sd[1], sd[1], t0, t1);
    csa(t0, sd[0], sd[0], d[4], d[5]);
    csa(t1, sd[0], sd[0], d[6], d[7]);
    csa(f1, sd[1], sd[1], t0, t1);
    csa(e, sd[2], sd[2], f0, f1);
#pragma unroll
    for (int k = 3; k < kSlices; ++k) {
      const uint64_t cy = sd[k] & e;
      sd[k] ^= e;
      e = cy;
    }
  }
  __syncthreads();  // the row words are no longer needed: their place takes the partial counters
#pragma unroll
  for (int k = 0; k < kSlices; ++k) {
    sm[((0 * nsub + sub) * kSlices + k) * W + wl] = sc[k];
    sm[((1 * nsub + sub) * kSlices + k) * W + wl] = sd[k];
  }
  __syncthreads();
  if ((int)threadIdx.x < 2 * W) {
    const int kind = threadIdx.x / W;  // 0 columns, 1 diagonals
    uint64_t acc[kSlices];
#pragma unroll
    for (int k = 0; k < kSlices; ++k) acc[k] = 0;
    for (int x = 0; x < nsub; ++x) {
      uint64_t carry = 0;
#pragma unroll
      for (int k = 0; k < kSlices; ++k) {
        const uint64_t in = sm[((kind * nsub + x) * kSlices + k) * W + wl];
        const uint64_t u = acc[k] ^ in;
        const uint64_t cy = (acc[k] & in) | (u & carry);
        acc[k] = u ^ carry;
        carry = cy;
      }
    }
    if (wl < tbw) {
      uint64_t *out = (kind ? dslices : vslices) + (((int64_t)h * n_chunks + chunk) * kSlices) * tbw + wl;
#pragma unroll
      for (int k = 0; k < kSlices; ++k) out[(int64_t)k * tbw] = acc[k];
    }
  }
  // words past the chunk's diagonal: nothing counted
  const int rest = tbw - W;
  for (int x = threadIdx.x; x < 2 * kSlices * rest; x += 256) {
    const int kind = x / (kSlices * rest), k = (x / rest) % kSlices, w = W + x % rest;
    ((kind ? dslices : vslices) + (((int64_t)h * n_chunks + chunk) * kSlices) * tbw)[(int64_t)k * tbw + w] = 0;
  }
}

// gamma = count / size >= mu for pattern p of head h (Sec. 4.2.4), counts summed over the row chunks.
// The chunk counts stay bit-sliced while they are added: a thread owns one word of 64 patterns and a
// sixteenth of the chunks, ripple-adds their 7-slice counts into a wider bit-sliced sum (a full adder is
// five logic operations on 64 patterns at once), the sixteen sums of a word are added pairwise, and only
// then every thread extracts the integer counts of its patterns.
// blockIdx.z: 0 vertical, 1 diagonal patterns; blockIdx.x: group of 16 words.
constexpr int kAccSlices = 17;  // counts below 2^17: pcl is limited accordingly

template <int NIN>
__device__ __forceinline__ void sliced_add(uint64_t (&acc)[kAccSlices], const uint64_t (&in)[NIN], int nb) {
  uint64_t carry = 0;
#pragma unroll
  for (int k = 0; k < kAccSlices; ++k) {
    if (k < nb) {  // wave-uniform
      const uint64_t x = k < NIN ? in[k < NIN ? k : 0] : 0;
      const uint64_t u = acc[k] ^ x;
      const uint64_t c = (acc[k] & x) | (u & carry);
      acc[k] = u ^ carry;
      carry = c;
    }
  }
}

constexpr int kFinWords = 16;  // words (of 64 patterns) per workgroup of k_pattern_finish

__global__ __launch_bounds__(256) void k_pattern_finish(const uint64_t *__restrict__ vslices,
                                                        const uint64_t *__restrict__ dslices, int L, int tbw,
                                                        int n_chunks, int nb, float mu, int *__restrict__ vert_cnt,
                                                        int *__restrict__ diag_cnt, uint8_t *__restrict__ vert_flag,
                                                        uint8_t *__restrict__ diag_flag) {
  // thread t: word t % 16 of the group, chunks t / 16, t / 16 + 16, ...; the 16 partial sums of a word are
  // then added pairwise through LDS
  __shared__ uint64_t part[16][kAccSlices][kFinWords];
  const int wi = threadIdx.x & (kFinWords - 1), sub = threadIdx.x / kFinWords;
  const int h = blockIdx.y, word0 = blockIdx.x * kFinWords;
  const bool diag = blockIdx.z == 1;
  const uint64_t *slices = diag ? dslices : vslices;
  int *cnt_out = diag ? diag_cnt : vert_cnt;
  uint8_t *flag_out = diag ? diag_flag : vert_flag;
  const int wl = word0 + wi;
  uint64_t acc[kAccSlices];
#pragma unroll
  for (int k = 0; k < kAccSlices; ++k) acc[k] = 0;
  // rows above pattern p hold nothing of it: start at the chunk of the group's first pattern
  for (int chunk = word0 * 64 / kChunkRows + sub; chunk < n_chunks; chunk += 16) {
    uint64_t in[kSlices];
    const int64_t at = (((int64_t)h * n_chunks + chunk) * kSlices) * tbw + wl;
#pragma unroll
    for (int k = 0; k < kSlices; ++k) in[k] = wl < tbw ? slices[at + (int64_t)k * tbw] : 0;
    sliced_add(acc, in, nb);
  }
  for (int half = 8; half >= 1; half >>= 1) {
    if (sub >= half && sub < 2 * half) {
#pragma unroll
      for (int k = 0; k < kAccSlices; ++k) part[sub][k][wi] = acc[k];
    }
    __syncthreads();
    if (sub < half) {
      uint64_t in[kAccSlices];
#pragma unroll
      for (int k = 0; k < kAccSlices; ++k) in[k] = part[sub + half][k][wi];
      sliced_add(acc, in, nb);
    }
  }
  if (sub == 0) {
#pragma unroll
    for (int k = 0; k < kAccSlices; ++k) part[0][k][wi] = acc[k];
  }
  __syncthreads();
  const int p_end = min(L, (word0 + kFinWords) * 64);
  for (int p = word0 * 64 + threadIdx.x; p < p_end; p += 256) {
    const int wd = (p >> 6) - word0, t = p & 63;
    int cnt = 0;
#pragma unroll
    for (int k = 0; k < kAccSlices; ++k)
      if (k < nb) cnt |= (int)((part[0][k][wd] >> t) & 1) << k;
    const int64_t e = (int64_t)h * L + p;
    if (cnt_out) cnt_out[e] = cnt;
    const float size = (float)(L - p);
    flag_out[e] = (uint8_t)((float)cnt / size >= mu);
  }
}

// Flags -> bitsets. cbits bit c = column c matched. rrev bit q = diagonal (pw*64 - 1 - q) matched,
// i.e. the diagonal set reversed, so that the 64 offsets i-j, i-j-1, ... of one mask word are 64
// consecutive ascending bits. Four lanes build one word: each turns 16 flag bytes (one 16-byte
// load when the row is aligned) into 16 bits.
__device__ __forceinline__ unsigned flags16(const uint8_t *__restrict__ row, int first, int P, bool aligned) {
  unsigned bits = 0;
  if (aligned && first + 16 <= P) {
    const uint4 v = *reinterpret_cast<const uint4 *>(row + first);
    const unsigned x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      // per byte: non-zero -> 1, then gather the four 0/1 bytes into four adjacent bits
      const unsigned nz = ((((x[k] & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x[k]) & 0x80808080u) >> 7;
      bits |= (((nz * 0x00204081u) >> 21) & 0xFu) << (4 * k);
    }
  } else {
    for (int k = 0; k < 16; ++k)
      if (first + k < P && row[first + k] != 0) bits |= 1u << k;
  }
  return bits;
}

// (every thread of the workgroup calls this; 256 words per pass)
__device__ __forceinline__ void pattern_bitsets_of_head(const uint8_t *__restrict__ diag_flag,
                                                        const uint8_t *__restrict__ vert_flag, int P, int pw, int h,
                                                        uint64_t *__restrict__ cbits, uint64_t *__restrict__ rrev,
                                                        uint64_t *lds_copy) {  // both sets again, [2 pw], or nullptr
  const int part = threadIdx.x & 3;
  const uint8_t *drow = diag_flag + (int64_t)h * P, *vrow = vert_flag + (int64_t)h * P;
  const bool d_al = (reinterpret_cast<uintptr_t>(drow) & 15) == 0, v_al = (reinterpret_cast<uintptr_t>(vrow) & 15) == 0;
  for (int w0 = 0; w0 < pw; w0 += blockDim.x / 4) {
    const int w = w0 + (threadIdx.x >> 2);
    const bool live = w < pw;
    uint64_t cw = 0, rw = 0;
    if (live) {
      cw = (uint64_t)flags16(vrow, w * 64 + part * 16, P, v_al) << (16 * part);
      rw = (uint64_t)flags16(drow, (pw - 1 - w) * 64 + part * 16, P, d_al) << (16 * part);  // ascending offsets
    }
    cw |= __shfl_xor(cw, 1);
    cw |= __shfl_xor(cw, 2);
    rw |= __shfl_xor(rw, 1);
    rw |= __shfl_xor(rw, 2);
    if (live && part == 0) {
      const uint64_t rev = __brevll(rw);  // bit q of the word <- offset (pw*64 - 1) - (64 w + q)
      cbits[(int64_t)h * pw + w] = cw;
      rrev[(int64_t)h * pw + w] = rev;
      if (lds_copy) {
        lds_copy[w] = cw;
        lds_copy[pw + w] = rev;
      }
    }
  }
}

// Word w of a bitset of pw words, 0 outside it. The index is clamped before the address is formed: the
// set may live in LDS, and an address formed below the start of the LDS window is not an LDS address
// any more, even if an instruction offset would bring it back inside.
__device__ __forceinline__ uint64_t set_word(const uint64_t *__restrict__ bs, int w, int pw) {
  const bool ok = (unsigned)w < (unsigned)pw;
  const uint64_t v = bs[ok ? w : 0];
  return ok ? v : 0;
}

// ------------------------------------------------------------------------------------------------
// Sec. 4.3: the 64 mask bits of row i, keys [64 wj, 64 wj + 64) of one head.
__device__ __forceinline__ uint64_t diag_window(const uint64_t *__restrict__ rrev, int pw, int64_t u) {
  // bit t <- diagonal offset u - t; in the reversed set that is position s0 + t.
  const int64_t Q = (int64_t)pw * 64 - 1;
  const int64_t s0 = Q - u;
  if (s0 > Q || s0 + 63 < 0) return 0;
  const int64_t w0 = s0 >> 6;
  const int sh = (int)(s0 & 63);
  const uint64_t lo = set_word(rrev, (int)w0, pw);
  if (sh == 0) return lo;
  const uint64_t hi = set_word(rrev, (int)w0 + 1, pw);
  return (lo >> sh) | (hi << (64 - sh));
}

__device__ __forceinline__ uint64_t mask_word(const Geom &g, const uint64_t *__restrict__ tb_h,
                                              const uint64_t *__restrict__ cb_h,
                                              const uint64_t *__restrict__ rr_h, int i, int wj) {
  if (i >= g.S) return 0;
  const int64_t u = (int64_t)i - (int64_t)wj * 64;
  if (u < 0) return 0;
  const uint64_t causal = u >= 63 ? ~0ull : ((2ull << u) - 1);
  if (i < g.L) {  // top-left block (and the whole mask when S <= L): the true mask
    const int64_t left = (int64_t)g.L - (int64_t)wj * 64;  // > 0 because j <= i < L
    const uint64_t inside = left >= 64 ? ~0ull : ((1ull << left) - 1);
    return tb_h[(int64_t)i * g.tbw + wj] & causal & inside;
  }
  uint64_t pat = cb_h ? set_word(cb_h, wj, g.pw) : 0;  // cb_h == nullptr: the diagonal part alone
  pat |= diag_window(rr_h, g.pw, u);
  return pat & causal;
}

// Any set bit among positions [lo, hi] of a bitset of nw words (positions outside it read as 0).
__device__ __forceinline__ bool range_any(const uint64_t *__restrict__ bs, int nw, int64_t lo, int64_t hi) {
  lo = max(lo, (int64_t)0);
  hi = min(hi, (int64_t)nw * 64 - 1);
  if (lo > hi) return false;
  for (int64_t w = lo >> 6; w <= (hi >> 6); ++w) {
    uint64_t m = bs[w];
    if (w == (lo >> 6)) m &= ~0ull << (lo & 63);
    if (w == (hi >> 6)) m &= ~0ull >> (63 - (hi & 63));
    if (m) return true;
  }
  return false;
}

// Every bit set among positions [lo, hi] (all inside the bitset).
__device__ __forceinline__ bool range_all(const uint64_t *__restrict__ bs, int64_t lo, int64_t hi) {
  for (int64_t w = lo >> 6; w <= (hi >> 6); ++w) {
    uint64_t need = ~0ull;
    if (w == (lo >> 6)) need &= ~0ull << (lo & 63);
    if (w == (hi >> 6)) need &= ~0ull >> (63 - (hi & 63));
    if ((bs[w] & need) != need) return false;
  }
  return true;
}

// A tile strictly below the diagonal and outside the true-mask block holds only pattern entries:
// (i, j) is kept iff column j is matched or offset i - j is. Rows [i0, i1], columns [j0, j1].
//   any:  some column of the tile is matched, or some offset in [i0 - j1, i1 - j0] is;
//   full: every offset of that range is matched, or every column is, or every unmatched offset u
//         ("hole") only meets matched columns: columns [max(j0, i0 - u), min(j1, i1 - u)].
// Both are decided by one lane from a handful of bitset words. Returns bit0 any, bit1 full.
__device__ int pattern_tile_flags(const uint64_t *__restrict__ cb, const uint64_t *__restrict__ rr, int pw,
                                  int i0, int i1, int j0, int j1) {
  const int64_t Q = (int64_t)pw * 64 - 1;  // offset u sits at position Q - u of the reversed set
  const int a = i0 - j1, b = i1 - j0;      // offsets met by the tile, 0 <= a <= b
  const bool cols_in = cb && j0 <= Q;      // columns past the bitset are never matched; cb == nullptr: no columns
  const int jc1 = (int)min((int64_t)j1, Q);
  const bool any_c = cols_in && range_any(cb, pw, j0, jc1);
  const bool any_r = range_any(rr, pw, Q - b, Q - a);
  if (!any_c && !any_r) return 0;
  if (cols_in && j1 <= Q && range_all(cb, j0, j1)) return 3;
  // holes: offsets of [a, b] that are not matched (those past the bitset are all holes)
  bool full = true;
  if (b > Q) {  // offsets Q+1 .. b: their entries lie in columns [max(j0, i0 - b), min(j1, i1 - (Q + 1))]
    const int64_t lo = max((int64_t)j0, (int64_t)i0 - b), hi = min((int64_t)j1, (int64_t)i1 - (Q + 1));
    if (lo <= hi) full = cb && hi <= Q && range_all(cb, lo, hi);
  }
  const int64_t p_lo = max(Q - b, (int64_t)0), p_hi = Q - a;
  for (int64_t w = p_lo >> 6; full && w <= (p_hi >> 6); ++w) {
    uint64_t holes = ~rr[w];
    if (w == (p_lo >> 6)) holes &= ~0ull << (p_lo & 63);
    if (w == (p_hi >> 6)) holes &= ~0ull >> (63 - (p_hi & 63));
    while (holes && full) {
      const int64_t u = Q - (w * 64 + (__ffsll((unsigned long long)holes) - 1));
      holes &= holes - 1;
      const int64_t lo = max((int64_t)j0, (int64_t)i0 - u), hi = min((int64_t)j1, (int64_t)i1 - u);
      if (lo <= hi) full = cb && hi <= Q && range_all(cb, lo, hi);
    }
  }
  return full ? 3 : 1;
}

// Classes of whole tiles for square tiles of width T, per head (pattern region, tile strictly below
// the diagonal): the entries of tile (qt, kt) have the columns of key tile kt and exactly the offsets
// T d - (T - 1) .. T d + (T - 1), d = qt - kt. So "some column matched" / "all columns matched" is a
// property of kt alone and "some offset matched" / "all offsets matched" of d alone. The d classes
// are stored reversed (d at position 64 dw - 1 - d), like the diagonal set, so that the 64 key tiles
// of an occupancy word are 64 consecutive bits.
__device__ __forceinline__ void tile_classes_of_head(const Geom &g, const uint64_t *__restrict__ cb,  // the head's sets
                                                     const uint64_t *__restrict__ rr, int h, uint64_t *__restrict__ col_any,
                                                     uint64_t *__restrict__ col_all, uint64_t *__restrict__ off_any,
                                                     uint64_t *__restrict__ off_all) {
  const int lane = threadIdx.x & 63;
  const int T = g.tile_n;
  const int64_t Q = (int64_t)g.pw * 64 - 1;
  for (int w = threadIdx.x >> 6; w < g.occw; w += blockDim.x >> 6) {  // a wave per occupancy word
    {
      const int kt = w * 64 + lane;
      const int64_t j0 = (int64_t)kt * T, j1 = j0 + T - 1;
      const bool any = kt < g.nKt && range_any(cb, g.pw, j0, j1);
      const bool all = kt < g.nKt && j1 <= Q && range_all(cb, j0, j1);
      const uint64_t wa = __ballot(any), wf = __ballot(all);
      if (lane == 0) {
        col_any[(int64_t)h * g.occw + w] = wa;
        col_all[(int64_t)h * g.occw + w] = wf;
      }
    }
    {
      const int64_t d = (int64_t)g.occw * 64 - 1 - ((int64_t)w * 64 + lane);
      const int64_t a = d * T - (T - 1), b = d * T + (T - 1);  // offsets of the tile, a >= 1 when d >= 1
      const bool live = d >= 1 && d < g.nQt;
      const bool any = live && range_any(rr, g.pw, Q - b, Q - a);
      const bool all = live && b <= Q && range_all(rr, Q - b, Q - a);
      const uint64_t wa = __ballot(any), wf = __ballot(all);
      if (lane == 0) {
        off_any[(int64_t)h * g.occw + w] = wa;
        off_all[(int64_t)h * g.occw + w] = wf;
      }
    }
  }
}

// The column bitset and the reversed diagonal bitset of one head, copied into LDS by the whole
// workgroup when they fit (lds_words = 2 pw, else 0): every mask word then costs LDS reads instead
// of dependent global loads. Contains a barrier. The callers then run their body on the
// LDS array itself, in a call of its own: only then does the compiler know the address space of the sets and read
// them with LDS instructions (a pointer that may be either is read through the flat path, with waits on both counters).
constexpr size_t kMaxStagedBytes = 48 * 1024;
constexpr int kGuardFront = 4, kGuardBack = 2;

inline size_t staged_bytes(const Geom &g) {
  const size_t b = ((size_t)g.pw * 2 + kGuardFront + kGuardBack) * sizeof(uint64_t);
  return b <= kMaxStagedBytes ? b : 0;
}

// Layout: the column set (pw words), kGuardFront zero words, the reversed diagonal set (pw words), kGuardBack zero
// words: words -kGuardFront .. -1 and pw, pw + 1 of the staged diagonal set read as empty without a test.
__device__ __forceinline__ void stage_sets(uint64_t *lds_sets, int pw, const uint64_t *cb, const uint64_t *rr) {
  for (int x = threadIdx.x; x < pw; x += blockDim.x) {
    lds_sets[x] = cb[x];
    lds_sets[pw + kGuardFront + x] = rr[x];
  }
  if (threadIdx.x < kGuardFront + kGuardBack)
    lds_sets[threadIdx.x < kGuardFront ? pw + threadIdx.x : 2 * pw + threadIdx.x] = 0;
  __syncthreads();
}

// ------------------------------------------------------------------------------------------------
// Gathered column tiles (flag DAM_MASK_GATHER_COLUMNS). The mask is unchanged; its entries in query
// tiles of the pattern region are split into a diagonal part, listed in ordinary tiles, and a column
// part, listed in tiles whose 128 (tile_n) "keys" are matched columns taken in ascending order:
// gathered tile v of head h holds columns gidx[h][v tile_n ..], and row i keeps slot s iff
// c = gidx[s] <= i and i - c is not a matched diagonal (those entries belong to the diagonal part).
// A vertical stripe then costs its share of one dense tile per query tile instead of a whole tile.

// The matched columns below S of one head, ascending, padded with -1 up to the stride. One workgroup per
// head, a word of the column bitset per thread and pass.
__device__ __forceinline__ void gather_columns_of_head(const Geom &g, const uint64_t *__restrict__ cb,  // the head's column set
                                                       int stride, int h, int *__restrict__ gidx, int *__restrict__ gcnt) {
  __shared__ int s_wave[16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int *out = gidx + (int64_t)h * stride;
  const int n_cols = min(g.P, g.S);
  int base = 0;  // the same value in every thread
  for (int w0 = 0; w0 * 64 < n_cols; w0 += 1024) {  // a word of the column set per thread
    const int w = w0 + threadIdx.x;
    uint64_t m = (w < g.pw && w * 64 < n_cols) ? cb[w] : 0;
    if (w * 64 + 64 > n_cols && w * 64 < n_cols) m &= ~0ull >> (64 - (n_cols - w * 64));
    const int v = __popcll(m);
    int incl = v;
    for (int off = 1; off < 64; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    int before = base, all = 0;
    for (int x = 0; x < 16; ++x) {
      const int t = s_wave[x];
      if (x < wave) before += t;
      all += t;
    }
    int at = before + incl - v;
    while (m) {
      out[at++] = w * 64 + __ffsll((unsigned long long)m) - 1;
      m &= m - 1;
    }
    base += all;
    __syncthreads();  // s_wave is rewritten in the next pass
  }
  if (threadIdx.x == 0) gcnt[h] = base;
  // the empty slots: 16 bytes per store where the row allows it (rows are `stride` ints apart, a multiple of 64)
  const int first4 = (base + 3) & ~3;
  if ((reinterpret_cast<uintptr_t>(out) & 15) == 0) {
    if (base + (int)threadIdx.x < min(first4, stride)) out[base + threadIdx.x] = -1;
    for (int x = first4 + 4 * (int)threadIdx.x; x + 4 <= stride; x += 4 * blockDim.x)
      *reinterpret_cast<int4 *>(out + x) = make_int4(-1, -1, -1, -1);
    if ((int)threadIdx.x < (stride & 3)) out[(stride & ~3) + threadIdx.x] = -1;
  } else {
    for (int x = base + threadIdx.x; x < stride; x += blockDim.x) out[x] = -1;
  }
}

// Everything the block index needs from the pattern flags of one head, in one launch (one workgroup of 1024
// per head: the three steps are short chains of dependent work, and as separate kernels each paid a launch):
// the two bitsets, the tile classes, the gathered column list.
__global__ __launch_bounds__(1024) void k_pattern_prep(Geom g, const uint8_t *__restrict__ diag_flag,
                                                       const uint8_t *__restrict__ vert_flag, uint64_t *__restrict__ cbits,
                                                       uint64_t *__restrict__ rrev, bool classes,
                                                       uint64_t *__restrict__ col_any, uint64_t *__restrict__ col_all,
                                                       uint64_t *__restrict__ off_any, uint64_t *__restrict__ off_all,
                                                       int gstride, int *__restrict__ gidx, int *__restrict__ gcnt,
                                                       int *__restrict__ head_cnt, bool in_lds) {
  extern __shared__ uint64_t prep_sets[];  // in_lds: the head's two sets, [2 pw]
  const int h = blockIdx.x;
  if (threadIdx.x < kHeadSub) head_cnt[h * kHeadSub + threadIdx.x] = 0;  // the head's number of listed tiles: summed by k_tile_scan
  pattern_bitsets_of_head(diag_flag, vert_flag, g.P, g.pw, h, cbits, rrev, in_lds && classes ? prep_sets : nullptr);
  if (!classes) return;  // uniform over the grid
  __syncthreads();       // the sets are read back by other threads of this workgroup
  // (from the LDS copy when they fit: the steps below are chains of dependent reads. One call per address space,
  // so that the compiler knows which kind of read to use.)
  if (in_lds) {
    tile_classes_of_head(g, prep_sets, prep_sets + g.pw, h, col_any, col_all, off_any, off_all);
    if (gidx) gather_columns_of_head(g, prep_sets, gstride, h, gidx, gcnt);
  } else {
    tile_classes_of_head(g, cbits + (int64_t)h * g.pw, rrev + (int64_t)h * g.pw, h, col_any, col_all, off_any, off_all);
    if (gidx) gather_columns_of_head(g, cbits + (int64_t)h * g.pw, gstride, h, gidx, gcnt);
  }
}

// Transpose of the 64 x 64 bit matrix whose row l is the word x of lane l: lane r returns the word whose
// bit l is bit r of lane l's x. Six exchange steps on blocks of 32, 16, ... 1 bits.
__device__ __forceinline__ uint64_t transpose64(uint64_t x, int lane) {
  uint64_t m = 0x00000000FFFFFFFFull;
#pragma unroll
  for (int j = 32; j > 0; j >>= 1) {
    const uint64_t other = __shfl_xor(x, j);
    x = (lane & j) ? (((other >> j) & m) | (x & ~m)) : ((x & m) | ((other & m) << j));
    m ^= m << (j >> 1);
  }
  return x;
}

// Row bitmap of one gathered slot for the rows of query tile qt: bit r of word k is row 64 k + r of the
// tile. c < 0: an empty slot.
__device__ __forceinline__ void slot_rows(const Geom &g, const uint64_t *__restrict__ rr, int i0, int c,
                                          uint64_t (&keep)[4]) {
  const int row_words = g.tile_m / 64;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    keep[k] = 0;
    if (k < row_words && c >= 0) {
      const int r0 = 64 * k;                       // first row of the word
      const int first = c - i0 - r0;               // rows of the word from `first` on are causal
      uint64_t m = first <= 0 ? ~0ull : (first >= 64 ? 0ull : ~0ull << first);
      const int live = g.S - i0 - r0;              // rows of the word below `live` exist
      m &= live >= 64 ? ~0ull : (live <= 0 ? 0ull : ~0ull >> (64 - live));
      // offsets i - c of the word's rows, highest first, are 64 consecutive bits of the reversed set
      const uint64_t diag = __brevll(diag_window(rr, g.pw, (int64_t)i0 + r0 + 63 - c));
      keep[k] = m & ~diag;
    }
  }
}

// Pass 1 of the block index: which key tiles of query tile (h, qt) hold a kept entry / are full.
// One wave per query tile, 64 key tiles (one occupancy word) at a time, one lane per key tile. Tiles
// strictly below the diagonal and outside the true-mask block are decided by their lane alone (from
// the class bitsets, or by pattern_tile_flags); only the tiles on the diagonal or inside the
// true-mask block are then evaluated word by word by the whole wave. No LDS, no barrier.
__device__ __forceinline__ int tile_scan_row(const Geom &g, const uint64_t *__restrict__ tb, const uint64_t *__restrict__ cb,
                                              const uint64_t *__restrict__ rr, const uint64_t *__restrict__ col_any,
                                              const uint64_t *__restrict__ col_all, const uint64_t *__restrict__ off_any,
                                              const uint64_t *__restrict__ off_all, uint64_t *__restrict__ occ,
                                              uint64_t *__restrict__ full, int *__restrict__ cnt, const int *__restrict__ gidx,
                                              const int *__restrict__ gcnt, int gstride, uint64_t *__restrict__ vocc,
                                              uint64_t *__restrict__ vfull, int h, int qt, int lane) {
  const int i0 = qt * g.tile_m;
  const int i_last = min(g.S - 1, i0 + g.tile_m - 1);
  const int kmax = i_last / g.tile_n;
  // Square tiles, a whole row of tiles in the pattern region: 64 tiles at a time from the per-head
  // class bitsets. Only a tile that has matched and unmatched columns AND matched and unmatched
  // offsets needs the exact one-lane test for "full".
  const bool by_class = g.tile_m == g.tile_n && i0 >= g.L && i0 + g.tile_m <= g.S;
  // gathered columns: in a query tile of the pattern region the ordinary tiles hold the diagonal part only
  const bool split = gidx != nullptr && i0 >= g.L;
  const uint64_t *cbw = split ? nullptr : cb;
  const uint64_t *ca = col_any + (int64_t)h * g.occw, *cf = col_all + (int64_t)h * g.occw;
  const uint64_t *da = off_any + (int64_t)h * g.occw, *df = off_all + (int64_t)h * g.occw;
  const int words = g.tile_m * g.wpr;
  int total = 0;
  for (int w = 0; w <= (kmax >> 6); ++w) {  // (the words past the diagonal tile's are neither written nor read)
    const int kt = w * 64 + lane;
    int f = 0;
    if (kt <= kmax) {
      const int j0 = kt * g.tile_n, j1 = min(j0 + g.tile_n - 1, g.S - 1);
      f = 4;  // evaluate word by word
      if (i0 >= g.L && j1 <= i0) {
        bool exact = true;
        if (by_class) {
          const int d = qt - kt;  // >= 1 here
          const int64_t pos = (int64_t)g.occw * 64 - 1 - d;
          const bool c_any = !split && ((ca[w] >> lane) & 1), c_all = !split && ((cf[w] >> lane) & 1);
          const bool d_any = (da[pos >> 6] >> (pos & 63)) & 1, d_all = (df[pos >> 6] >> (pos & 63)) & 1;
          if (!(c_any && !c_all && d_any && !d_all)) {
            exact = false;
            f = ((c_any || d_any) ? 1 : 0) | ((c_all || d_all) ? 3 : 0);
          }
        }
        if (exact) {
          f = pattern_tile_flags(cbw, rr, g.pw, i0, i_last, j0, j1);
          // a tile cut by the end of the sequence is never full (its bits past S are zero)
          if (j0 + g.tile_n > g.S || i0 + g.tile_m > g.S) f &= 1;
        }
      }
    }
    uint64_t ow = __ballot(f & 1), fw = __ballot(f & 2);
    uint64_t need = __ballot(f & 4);
    while (need) {  // wave-uniform
      const int b = __ffsll((unsigned long long)need) - 1;
      need &= need - 1;
      bool any = false, all = true;
      for (int x = lane; x < words; x += 64) {
        const uint64_t m = mask_word(g, tb, cbw, rr, i0 + x / g.wpr, (w * 64 + b) * g.wpr + x % g.wpr);
        any |= m != 0;
        all &= m == ~0ull;
      }
      if (__ballot(any) != 0) ow |= 1ull << b;
      if (__ballot(!all) == 0) fw |= 1ull << b;
    }
    if (lane == 0) {
      occ[((int64_t)h * g.nQt + qt) * g.occw + w] = ow;
      full[((int64_t)h * g.nQt + qt) * g.occw + w] = fw;
    }
    total += __popcll(ow);
  }
  if (gidx) {
    // the gathered tiles of this query tile: one lane per slot, the rows of the tile as a bitmap
    const int n_gt = split ? (gcnt[h] + g.tile_n - 1) / g.tile_n : 0;
    const int *gi = gidx + (int64_t)h * gstride;
    const int row_words = g.tile_m / 64;
    // No matched diagonal lies beyond r_bound: the largest tile distance with a matched offset (the first set bit
    // of the reversed class words) covers offsets up to T d + T - 1. (Square tiles only: the classes are theirs.)
    int64_t r_bound = INT64_MAX;
    if (n_gt >= 4 && g.tile_m == g.tile_n) {  // (with a handful of gathered tiles the look-up costs more than it saves)
      int64_t first = -1;
      for (int w0 = 0; w0 < g.occw && first < 0; w0 += 64) {
        const uint64_t word = w0 + lane < g.occw ? da[w0 + lane] : 0;
        const uint64_t nz = __ballot(word != 0);
        if (nz) {
          const int wl = __ffsll((unsigned long long)nz) - 1;
          const uint64_t hit = __shfl(word, wl);
          first = (int64_t)(w0 + wl) * 64 + __ffsll((unsigned long long)hit) - 1;
        }
      }
      const int64_t dmax = first < 0 ? 0 : (int64_t)g.occw * 64 - 1 - first;
      r_bound = dmax * g.tile_n + g.tile_n - 1;
    }
    const int n_cols = split ? gcnt[h] : 0;
    for (int w = 0; w * 64 < n_gt; ++w) {  // (only the words that hold a gathered tile are written, and read)
      // A complete gathered tile whose columns all lie further above this query tile than any matched diagonal
      // reaches is full without looking: every row is causal for every slot and no offset i - c is a matched
      // one. A tile whose first column lies below the query tile's last row holds nothing (its columns ascend).
      // One lane per tile; the other tiles are evaluated slot by slot.
      bool certain = false, nothing = false;
      {
        const int v = w * 64 + lane;
        if (v < n_gt) {
          nothing = gi[v * g.tile_n] > i_last;
          if (r_bound != INT64_MAX && (v + 1) * g.tile_n <= n_cols && i0 + g.tile_m <= g.S) {
            const int cmax = gi[v * g.tile_n + g.tile_n - 1];  // the columns of a tile ascend
            certain = cmax >= 0 && (int64_t)i0 - cmax > r_bound;
          }
        }
      }
      const uint64_t sure = __ballot(certain), skip = sure | __ballot(nothing);
      uint64_t ow = sure, fw = sure;
      for (int v = w * 64; v < min(n_gt, w * 64 + 64); ++v) {
        if ((skip >> (v & 63)) & 1) continue;  // wave-uniform
        bool any = false, all = true;
        for (int wg = 0; wg < g.wpr; ++wg) {
          const int c = gi[v * g.tile_n + wg * 64 + lane];
          uint64_t keep[4];
          slot_rows(g, rr, i0, c, keep);
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if (k < row_words) {
              any |= keep[k] != 0;
              all &= keep[k] == ~0ull;
            }
        }
        if (__ballot(any) != 0) ow |= 1ull << (v & 63);
        if (__ballot(!all) == 0) fw |= 1ull << (v & 63);
      }
      if (lane == 0) {
        vocc[((int64_t)h * g.nQt + qt) * g.occw + w] = ow;
        vfull[((int64_t)h * g.nQt + qt) * g.occw + w] = fw;
      }
      total += __popcll(ow);
    }
  }
  if (lane == 0) cnt[(int64_t)h * g.nQt + qt] = total;
  return total;
}

// Exclusive scan of n counts by one block. group > 0: the result is laid out as [n / group]
// rows of group + 1 offsets (row r ends where row r + 1 begins); group == 0: plain [n + 1].
// Offsets are written as min(offset, clamp): with clamp = the capacity of the buffers the offsets point
// into, an index that does not fit is truncated to its first `capacity` entries and stays consistent
// with what the fill kernels wrote; *total is the unclamped sum.
// Every thread takes kScanItems consecutive counts per pass, so that the block-wide part (a wave
// scan, one exchange of the wave totals) is paid once per 8192 counts.
constexpr int kScanItems = 8;

// The scan itself, run by every thread of one workgroup of THREADS threads (a multiple of 64, at most 1024).
template <int THREADS>
__device__ __forceinline__ void block_exclusive_scan(const int *__restrict__ cnt, int64_t n, int group, int *__restrict__ ptr,
                                                     int64_t *__restrict__ total, int64_t clamp) {
  __shared__ int64_t wave_sum[2][16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t carry = 0;  // the same value in every thread
  int pass = 0;
  for (int64_t base = 0; base < n; base += THREADS * kScanItems, ++pass) {
    const int64_t e0 = base + (int64_t)threadIdx.x * kScanItems;
    int v[kScanItems];
#pragma unroll
    for (int x = 0; x < kScanItems; ++x) v[x] = e0 + x < n ? cnt[e0 + x] : 0;
    int64_t mine = 0;
#pragma unroll
    for (int x = 0; x < kScanItems; ++x) mine += v[x];
    int64_t incl = mine;
    for (int off = 1; off < 64; off <<= 1) {
      const int64_t up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    if (lane == 63) wave_sum[pass & 1][wave] = incl;
    __syncthreads();  // one barrier per pass: the totals of consecutive passes live in alternating buffers
    int64_t before = carry, all = 0;
    for (int w = 0; w < THREADS / 64; ++w) {
      const int64_t ws = wave_sum[pass & 1][w];
      if (w < wave) before += ws;
      all += ws;
    }
    int64_t excl = before + incl - mine;
    int64_t r = 0;
    int q = 0;
#pragma unroll
    for (int x = 0; x < kScanItems; ++x) {
      const int64_t e = e0 + x;
      if (e < n) {
        if (group > 0) {
          // row and position of count e: divided once per thread and pass (x == 0), stepped after that
          if (x == 0) {
            r = e / group;
            q = (int)(e - r * group);
          }
          ptr[r * (group + 1) + q] = (int)min(excl, clamp);
          if (q == 0 && r > 0) ptr[(r - 1) * (group + 1) + group] = (int)min(excl, clamp);
          if (++q == group) {
            q = 0;
            ++r;
          }
        } else {
          ptr[e] = (int)min(excl, clamp);
        }
      }
      excl += v[x];
    }
    carry += all;
  }
  if (threadIdx.x == 0) {
    if (group > 0) {
      if (n > 0) ptr[(n / group - 1) * (group + 1) + group] = (int)min(carry, clamp);
    } else {
      ptr[n] = (int)min(carry, clamp);
    }
    if (total) *total = carry;
  }
}

__global__ __launch_bounds__(1024) void k_exclusive_scan(const int *__restrict__ cnt, int64_t n,
                                                         int group, int *__restrict__ ptr,
                                                         int64_t *__restrict__ total, int64_t clamp) {
  block_exclusive_scan<1024>(cnt, n, group, ptr, total, clamp);
}

// Pass 1 as a kernel: a wave per query tile; the workgroup adds its four counts to the head's total. The CSR offsets
// need no launch of their own: every wave of the fill kernel adds up the totals of the heads before its own and the
// counts of the query tiles before its own. (Folding a scan into the last workgroup to finish was measured and
// dropped: it needs a device-wide release fence in every workgroup, which on this chip writes back the L2 of its
// XCD each time: 20 -> 190 us at S = 32768.)
__global__ __launch_bounds__(256) void k_tile_scan(Geom g, const uint64_t *__restrict__ true_bits,
                                                   const uint64_t *__restrict__ cbits,
                                                   const uint64_t *__restrict__ rrev,
                                                   const uint64_t *__restrict__ col_any,
                                                   const uint64_t *__restrict__ col_all,
                                                   const uint64_t *__restrict__ off_any,
                                                   const uint64_t *__restrict__ off_all,
                                                   uint64_t *__restrict__ occ,
                                                   uint64_t *__restrict__ full, int *__restrict__ cnt, bool staged,
                                                   const int *__restrict__ gidx, const int *__restrict__ gcnt,
                                                   int gstride, uint64_t *__restrict__ vocc,
                                                   uint64_t *__restrict__ vfull, int *__restrict__ head_cnt) {
  extern __shared__ uint64_t lds_sets[];
  __shared__ int wave_cnt[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = blockIdx.y, qt = blockIdx.x * 4 + wave;
  const uint64_t *tb = true_bits ? true_bits + (int64_t)h * g.L * g.tbw : nullptr;
  const uint64_t *cb = cbits + (int64_t)h * g.pw;
  const uint64_t *rr = rrev + (int64_t)h * g.pw;
  int mine = 0;
  if (staged) {  // uniform over the grid
    stage_sets(lds_sets, g.pw, cb, rr);
    if (qt < g.nQt)
      mine = tile_scan_row(g, tb, lds_sets, lds_sets + g.pw + kGuardFront, col_any, col_all, off_any, off_all, occ, full, cnt, gidx, gcnt,
                           gstride, vocc, vfull, h, qt, lane);
  } else if (qt < g.nQt) {
    mine = tile_scan_row(g, tb, cb, rr, col_any, col_all, off_any, off_all, occ, full, cnt, gidx, gcnt, gstride, vocc, vfull, h,
                         qt, lane);
  }
  // the head's total, for the offsets that the fill kernel derives itself (plain atomics, read by the next kernel
  // only; spread over kHeadSub words per head, because atomics on one address are served one after the other)
  if (lane == 0) wave_cnt[wave] = mine;
  __syncthreads();
  if (threadIdx.x == 0)
    atomicAdd(head_cnt + h * kHeadSub + (blockIdx.x & (kHeadSub - 1)), wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3]);
}

// Pass 2: write column, kind and the tile's element bits for every listed tile (below capacity). A wave per
// query tile (the four of a workgroup belong to one head and share its staged sets): the wave walks its own row
// of the index and writes every listed tile itself, a lane per tile row. With few query tiles in all (share = 4) the
// four waves of a workgroup share one query tile instead, each walking the whole row and taking every fourth
// tile: more waves, but the walk is then three quarters of the instructions.
template <bool STAGED>  // the head's pattern sets are staged in LDS (they fit), or read from global memory
__global__ __launch_bounds__(256) void k_tile_fill(Geom g, const uint64_t *__restrict__ true_bits,
                                                   const uint64_t *__restrict__ cbits,
                                                   const uint64_t *__restrict__ rrev,
                                                   const uint64_t *__restrict__ occ,
                                                   const uint64_t *__restrict__ full,
                                                   const int *__restrict__ tile_cnt, const int *__restrict__ head_cnt,
                                                   int *__restrict__ row_ptr, int64_t *__restrict__ blk_total,
                                                   int *__restrict__ blk_col,
                                                   uint8_t *__restrict__ blk_kind,
                                                   uint64_t *__restrict__ tile_bits, int64_t capacity,
                                                   bool skip_full_bits,
                                                   const int *__restrict__ gidx, const int *__restrict__ gcnt,
                                                   int gstride, const uint64_t *__restrict__ vocc,
                                                   const uint64_t *__restrict__ vfull, int share) {
  extern __shared__ uint64_t lds_sets[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = blockIdx.y;
  const int my_qt = share == 4 ? (int)blockIdx.x : (int)blockIdx.x * 4 + wave, my_turn = share == 4 ? wave : 0;
  const bool live = my_qt < g.nQt;
  const int qt = live ? my_qt : g.nQt - 1;  // (a spare wave reads a valid row and writes nothing)
  const uint64_t *tb = true_bits ? true_bits + (int64_t)h * g.L * g.tbw : nullptr;
  const uint64_t *cb = cbits + (int64_t)h * g.pw;
  const uint64_t *rr = rrev + (int64_t)h * g.pw;
  const uint64_t *oc = occ + ((int64_t)h * g.nQt + qt) * g.occw;
  const uint64_t *fl = full + ((int64_t)h * g.nQt + qt) * g.occw;
  // the walk below is a chain of dependent steps: its index words are fetched one word of 64 tiles ahead,
  // the first ones before the sets are staged, so that no step of the chain waits for memory alone
  // where this query tile's entries start: the listed tiles of the heads before h and of the query tiles before
  // qt (no scan kernel between the two passes: the counts are few enough for every wave to add up its own prefix)
  int64_t part = 0;
  for (int x = lane; x < h * kHeadSub; x += 64) part += head_cnt[x];
  const int *cnt_h = tile_cnt + (int64_t)h * g.nQt;
  for (int x = lane; x < qt; x += 64) part += cnt_h[x];
  const int my_cnt = cnt_h[qt];
  uint64_t ow_next = oc[0], fw_next = fl[0];
  if (STAGED) stage_sets(lds_sets, g.pw, cb, rr);
  if (!live) return;
  for (int off = 32; off; off >>= 1) part += __shfl_xor(part, off);
  const int64_t first = part;
  if (lane == 0 && my_turn == 0) {  // the CSR offsets, cut to the capacity like everything they point into
    int *rp = row_ptr + (int64_t)h * (g.nQt + 1);
    rp[qt] = (int)min(first, capacity);
    if (qt == g.nQt - 1) {
      rp[g.nQt] = (int)min(first + my_cnt, capacity);
      if (h == (int)gridDim.y - 1 && blk_total) *blk_total = first + my_cnt;
    }
  }
  const int i_last = min(g.S - 1, qt * g.tile_m + g.tile_m - 1);
  const int kmax = i_last / g.tile_n;
  const int words = g.tile_m * g.wpr;
  const int qw = g.tile_n / 4;  // quarter width in keys, a multiple of 16
  // gathered columns: the ordinary tiles of a query tile of the pattern region hold the diagonal part only
  const bool split = gidx != nullptr && qt * g.tile_m >= g.L;
  // the walk, once for sets in LDS and once for sets in global memory (see stage_sets)
  auto walk = [&](const uint64_t *cb, const uint64_t *rr, auto in_lds) __attribute__((always_inline)) {
  constexpr bool IN_LDS = decltype(in_lds)::value;
  if (split) cb = nullptr;
  // walk the listed tiles of this query tile in ascending order
  int rank = 0;
  for (int ow_i = 0; ow_i <= (kmax >> 6); ++ow_i) {
    uint64_t ow = ow_next;
    const uint64_t fw = fw_next;
    if (ow_i + 1 <= (kmax >> 6)) {
      ow_next = oc[ow_i + 1];
      fw_next = fl[ow_i + 1];
    }
    const uint64_t listed = ow;
    if (skip_full_bits) {
      // full tiles get a column and a kind only: all of the word's at once, lane j takes tile 64 ow_i + j
      const uint64_t below = (1ull << lane) - 1;
      const int r = rank + __popcll(listed & below);
      if (((listed & fw) >> lane) & 1) {
        const int64_t t = first + r;
        if (r % share == my_turn && t < capacity) {
          if (blk_col) blk_col[t] = ow_i * 64 + lane;
          if (blk_kind) blk_kind[t] = (uint8_t)31;
        }
      }
      ow &= ~fw;
    }
    const int rank0 = rank;
    rank += __popcll(listed);
    while (ow) {
      const int bit = __ffsll((unsigned long long)ow) - 1;
      const int kt = ow_i * 64 + bit;
      ow &= ow - 1;
      const int rk = rank0 + __popcll(listed & ((1ull << bit) - 1));
      const int64_t t = first + rk;
      const bool mine = rk % share == my_turn;
      if (!mine || t >= capacity) continue;
      // element words, and which key quarters of the tile hold a kept entry
      const bool is_full = (fw >> (kt & 63)) & 1;
      int quarters = 0, kind_q = 0;  // occupied key quarters: per lane (summed up by ballots below), or for the wave
      const bool quarters_used = !(words == 256 && g.wpr == 2 && qt * 128 >= g.L && qt * 128 + 128 <= g.S);
      if (words == 256 && g.wpr == 2 && qt * 128 >= g.L && qt * 128 + 128 <= g.S) {
        // 128 x 128 tile with every row in the pattern region: a lane takes rows lane and lane + 64 whole
        // (128 keys = two words). The offsets i - j of a row's 128 keys are 128 consecutive positions of the
        // reversed diagonal set, starting at Q - (i - 128 kt); row lane + 64 starts 64 positions below row lane,
        // so both rows come out of four consecutive words of the set: 256 bits, of which row lane + 64 takes
        // bits [sh, sh + 128) and row lane bits [64 + sh, 64 + sh + 128), as 32-bit funnel shifts.
        const int Q = g.pw * 64 - 1;
        const uint64_t c0 = cb ? set_word(cb, 2 * kt, g.pw) : 0, c1 = cb ? set_word(cb, 2 * kt + 1, g.pw) : 0;
        const int u_lane = (qt - kt) * 128 + lane;  // offset of the tile's first key in row lane, >= 0
        const int s0 = Q - u_lane;                  // (negative where the row's offsets lie beyond the pattern length)
        const int w0 = max(s0 >> 6, -3);            // from word -3 down all four words are outside the set
        // (staged sets carry four zero words in front and two behind: words -4 .. -1, pw and pw + 1 read as nothing)
        // (written out value by value: arrays indexed in unrolled loops end up in scratch memory here, because the
        // choice between neighbours below is turned into an index first)
        auto word = [&](int w) { return IN_LDS ? rr[w] : set_word(rr, w, g.pw); };
        const uint64_t wd0 = word(w0 - 1), wd1 = word(w0), wd2 = word(w0 + 1), wd3 = word(w0 + 2);
        const uint32_t e0 = (uint32_t)wd0, e1 = (uint32_t)(wd0 >> 32), e2 = (uint32_t)wd1, e3 = (uint32_t)(wd1 >> 32);
        const uint32_t e4 = (uint32_t)wd2, e5 = (uint32_t)(wd2 >> 32), e6 = (uint32_t)wd3, e7 = (uint32_t)(wd3 >> 32);
        const bool odd = (s0 & 32) != 0;
        const int r = s0 & 31;
        const uint32_t f0 = odd ? e1 : e0, f1 = odd ? e2 : e1, f2 = odd ? e3 : e2, f3 = odd ? e4 : e3;
        const uint32_t f4 = odd ? e5 : e4, f5 = odd ? e6 : e5, f6 = odd ? e7 : e6;
        uint32_t row[2][4];  // [u][dword]: row lane + 64 u
        row[1][0] = __builtin_amdgcn_alignbit(f1, f0, r);
        row[1][1] = __builtin_amdgcn_alignbit(f2, f1, r);
        row[1][2] = __builtin_amdgcn_alignbit(f3, f2, r);
        row[1][3] = __builtin_amdgcn_alignbit(f4, f3, r);
        row[0][0] = row[1][2];
        row[0][1] = row[1][3];
        row[0][2] = __builtin_amdgcn_alignbit(f5, f4, r);
        row[0][3] = __builtin_amdgcn_alignbit(f6, f5, r);
        const uint32_t cd[4] = {(uint32_t)c0, (uint32_t)(c0 >> 32), (uint32_t)c1, (uint32_t)(c1 >> 32)};
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int k = 0; k < 4; ++k) row[u][k] = is_full ? ~0u : (row[u][k] | cd[k]);
        if (kt == qt) {  // the diagonal tile (wave-uniform): keys up to the row's own only
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const int u0 = u_lane + 64 * u;  // = the row's index inside the tile
            const uint64_t lo = u0 >= 63 ? ~0ull : ((2ull << u0) - 1);
            const uint64_t hi = u0 >= 127 ? ~0ull : (u0 < 64 ? 0ull : ((2ull << (u0 - 64)) - 1));
            row[u][0] &= (uint32_t)lo; row[u][1] &= (uint32_t)(lo >> 32);
            row[u][2] &= (uint32_t)hi; row[u][3] &= (uint32_t)(hi >> 32);
          }
        }
        if (tile_bits) {
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            uint4 st;
            st.x = row[u][0]; st.y = row[u][1]; st.z = row[u][2]; st.w = row[u][3];
            *reinterpret_cast<uint4 *>(tile_bits + t * 256 + 2 * (lane + 64 * u)) = st;
          }
        }
        // a key quarter is 32 keys: one of the four 32-bit words of a row
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (__ballot((row[0][k] | row[1][k]) != 0)) kind_q |= 2 << k;
      } else if (words == 256 && g.wpr == 2) {
        // 128 x 128 tiles: four words per lane, evaluated together so that their loads overlap
        uint64_t m[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int w = lane + 64 * u;
          m[u] = is_full ? ~0ull : mask_word(g, tb, cb, rr, qt * 128 + (w >> 1), kt * 2 + (w & 1));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (tile_bits) tile_bits[t * 256 + lane + 64 * u] = m[u];
          if ((uint32_t)m[u]) quarters |= 1 << (2 * (lane & 1));
          if (m[u] >> 32) quarters |= 2 << (2 * (lane & 1));
        }
      } else
      for (int w = lane; w < words; w += 64) {
        const int wi = w % g.wpr;
        const uint64_t m = is_full ? ~0ull : mask_word(g, tb, cb, rr, qt * g.tile_m + w / g.wpr, kt * g.wpr + wi);
        if (tile_bits) tile_bits[t * words + w] = m;
        if (qw == 32) {  // 128-key tiles: a quarter is half a word
          if ((uint32_t)m) quarters |= 1 << (2 * wi);
          if (m >> 32) quarters |= 2 << (2 * wi);
        } else {
          for (int q = 0; q < 4; ++q) {
            // bits of this word that fall into quarter q: keys [q qw, (q + 1) qw) minus the word base
            const int lo = max(q * qw - wi * 64, 0), hi = min((q + 1) * qw - wi * 64, 64);
            if (hi > lo) {
              const uint64_t span = (hi - lo == 64 ? ~0ull : ((1ull << (hi - lo)) - 1)) << lo;
              if (m & span) quarters |= 1 << q;
            }
          }
        }
      }
      int kind = (is_full ? 1 : 0) | kind_q;
      if (quarters_used)
        for (int q = 0; q < 4; ++q)
          if (__ballot(quarters & (1 << q))) kind |= 2 << q;
      if (lane == 0) {
        if (blk_col) blk_col[t] = kt;
        if (blk_kind) blk_kind[t] = (uint8_t)kind;
      }
    }
  }
  if (!split) return;
  // the gathered tiles, after the ordinary ones: tile index nKt + v
  const uint64_t *voc = vocc + ((int64_t)h * g.nQt + qt) * g.occw;
  const uint64_t *vfl = vfull + ((int64_t)h * g.nQt + qt) * g.occw;
  const int n_gt = (gcnt[h] + g.tile_n - 1) / g.tile_n;
  const int *gi = gidx + (int64_t)h * gstride;
  const int i0 = qt * g.tile_m;
  // (a tile's columns are fetched while the tile before it is written: a load issued behind stores waits for them)
  int v_pre = -1, c_pre[4] = {-1, -1, -1, -1};  // (tiles are at most 256 wide: four groups of 64 slots)
  for (int ow_i = 0; ow_i * 64 < n_gt; ++ow_i) {
    uint64_t ow = voc[ow_i];
    const uint64_t vfw = vfl[ow_i];
    if (skip_full_bits) {
      // full tiles get a column and a kind only: all of the word's at once, lane j takes gathered tile 64 ow_i + j
      const uint64_t listed = ow;
      const int r = rank + __popcll(listed & ((1ull << lane) - 1));
      if (((listed & vfw) >> lane) & 1) {
        const int64_t t = first + r;
        if (r % share == my_turn && t < capacity) {
          if (blk_col) blk_col[t] = g.nKt + ow_i * 64 + lane;
          if (blk_kind) blk_kind[t] = (uint8_t)31;
        }
      }
    }
    const uint64_t listed_v = ow;
    const int rank0_v = rank;
    rank += __popcll(listed_v);
    if (skip_full_bits) ow &= ~vfw;
    while (ow) {
      const int bit = __ffsll((unsigned long long)ow) - 1;
      const int v = ow_i * 64 + bit;
      ow &= ow - 1;
      const int rk = rank0_v + __popcll(listed_v & ((1ull << bit) - 1));
      const int64_t t = first + rk;
      const bool mine = rk % share == my_turn;
      if (!mine || t >= capacity) continue;
      const bool is_full = (vfw >> (v & 63)) & 1;
      int c_all[4];
#pragma unroll
      for (int wg = 0; wg < 4; ++wg)
        if (wg < g.wpr) c_all[wg] = v == v_pre ? c_pre[wg] : gi[v * g.tile_n + wg * 64 + lane];
      if (ow) {  // the next listed tile of this word (if it turns out not to be this wave's, the fetch is wasted)
        v_pre = ow_i * 64 + __ffsll((unsigned long long)ow) - 1;
#pragma unroll
        for (int wg = 0; wg < 4; ++wg)
          if (wg < g.wpr) c_pre[wg] = gi[v_pre * g.tile_n + wg * 64 + lane];
      }
      int kind = 0;
#pragma unroll
      for (int wg = 0; wg < 4; ++wg) {  // the tile's slots, 64 at a time: lane = slot
        if (wg >= g.wpr) break;
        const int c = c_all[wg];
        uint64_t keep[4];
        slot_rows(g, rr, i0, c, keep);
        const bool any = (keep[0] | keep[1] | keep[2] | keep[3]) != 0;
        const uint64_t lanes_any = __ballot(any);
        for (int q = 0; q < 4; ++q) {  // quarter q: slots [q qw, (q + 1) qw)
          const int lo = q * qw - wg * 64, hi = lo + qw;
          if (hi > 0 && lo < 64) {
            const int a = max(lo, 0), b = min(hi, 64);
            const uint64_t span = (b - a == 64 ? ~0ull : ((1ull << (b - a)) - 1)) << a;
            if (lanes_any & span) kind |= 2 << q;
          }
        }
        if (tile_bits) {
          const uint64_t filled = __ballot(c >= 0);
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if (k < g.tile_m / 64) {
              // rows 64 k .. 64 k + 63 of the group: lane r gets the word (row 64 k + r, group wg), whose bit l is
              // slot l. Where every filled slot keeps all 64 rows (no row above a column, no matched offset met:
              // the usual case away from the diagonal) every row's word is the set of filled slots; otherwise the
              // 64 x 64 bits are transposed.
              const bool plain = __ballot(keep[k] != (c >= 0 ? ~0ull : 0ull)) == 0;  // wave-uniform
              tile_bits[t * words + (int64_t)(64 * k + lane) * g.wpr + wg] = plain ? filled : transpose64(keep[k], lane);
            }
        }
      }
      if (lane == 0) {
        if (blk_col) blk_col[t] = g.nKt + v;
        if (blk_kind) blk_kind[t] = (uint8_t)((is_full ? 1 : 0) | kind);
      }
    }
  }
  };
  if constexpr (STAGED)
    walk(lds_sets, lds_sets + g.pw + kGuardFront, std::true_type{});
  else
    walk(cb, rr, std::false_type{});
}

__global__ void k_dense_bits(Geom g, const uint64_t *__restrict__ true_bits,
                             const uint64_t *__restrict__ cbits, const uint64_t *__restrict__ rrev,
                             int sw, uint64_t *__restrict__ dense) {
  const int h = blockIdx.z, i = blockIdx.y;
  const int w = blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= sw) return;
  const uint64_t *tb = true_bits ? true_bits + (int64_t)h * g.L * g.tbw : nullptr;
  dense[((int64_t)h * g.S + i) * sw + w] =
      mask_word(g, tb, cbits + (int64_t)h * g.pw, rrev + (int64_t)h * g.pw, i, w);
}

// Kept-key lists of rows [row_begin, row_end): count, scan, fill (ascending).
__global__ __launch_bounds__(256) void k_row_count(Geom g, const uint64_t *__restrict__ true_bits,
                                                   const uint64_t *__restrict__ cbits,
                                                   const uint64_t *__restrict__ rrev, int row_begin,
                                                   int nrows, int *__restrict__ cnt) {
  __shared__ int total;
  const int h = blockIdx.y, i = row_begin + blockIdx.x;
  const uint64_t *tb = true_bits ? true_bits + (int64_t)h * g.L * g.tbw : nullptr;
  if (threadIdx.x == 0) total = 0;
  __syncthreads();
  int mine = 0;
  for (int w = threadIdx.x; w <= (i >> 6); w += blockDim.x)
    mine += __popcll(mask_word(g, tb, cbits + (int64_t)h * g.pw, rrev + (int64_t)h * g.pw, i, w));
  for (int off = 32; off; off >>= 1) mine += __shfl_xor(mine, off);
  if ((threadIdx.x & 63) == 0 && mine) atomicAdd(&total, mine);
  __syncthreads();
  if (threadIdx.x == 0) cnt[(int64_t)h * nrows + blockIdx.x] = total;
}

__global__ __launch_bounds__(256) void k_row_fill(Geom g, const uint64_t *__restrict__ true_bits,
                                                  const uint64_t *__restrict__ cbits,
                                                  const uint64_t *__restrict__ rrev, int row_begin,
                                                  int nrows, const int *__restrict__ kept_ptr,
                                                  int *__restrict__ kept_idx, int64_t capacity) {
  __shared__ int wave_sum[4];
  __shared__ int carry;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = blockIdx.y, i = row_begin + blockIdx.x;
  const uint64_t *tb = true_bits ? true_bits + (int64_t)h * g.L * g.tbw : nullptr;
  const int64_t first = kept_ptr[(int64_t)h * nrows + blockIdx.x];
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  const int nw = (i >> 6) + 1;
  for (int base = 0; base < nw; base += 256) {
    const int w = base + threadIdx.x;
    uint64_t m = w < nw ? mask_word(g, tb, cbits + (int64_t)h * g.pw, rrev + (int64_t)h * g.pw, i, w) : 0;
    const int v = __popcll(m);
    int incl = v;
    for (int off = 1; off < 64; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int before = carry;
    for (int x = 0; x < wave; ++x) before += wave_sum[x];
    int64_t at = first + before + incl - v;
    while (m) {
      const int b = __ffsll((unsigned long long)m) - 1;
      if (at < capacity) kept_idx[at] = w * 64 + b;
      ++at;
      m &= m - 1;
    }
    __syncthreads();
    if (threadIdx.x == 255) carry = before + incl;
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------------
// Kept lists of one row for grouped-query decoding (DAM_MASK_GROUP_LISTS): one list per group of G
// consecutive maps, holding each key some map of the group keeps once, in G + 1 runs (kept by two or
// more maps; by map 0 alone; by map 1 alone; ...), each ascending, with a byte of member bits per
// entry. A lane owns kPieceBits consecutive keys, a wave a chunk of 64 such pieces; the work is spread
// thin on purpose: the lists are short, so the time is the latency of the longest chain of dependent
// steps in one wave (its fullest piece), not throughput. Count per (group, run, chunk), exclusive
// scan in that order (which is the order of the output), fill.
constexpr int kMaxGroup = 8;
constexpr int kPieceBits = 8;
constexpr int kPiecesPerWord = 64 / kPieceBits;
constexpr int kChunkWords = 64 / kPiecesPerWord;  // mask words per wave

// This lane's piece of row i for the maps of group kv (m[x], zero for x >= G and beyond the row), and
// the bits set in at least two of them. Lane l: piece l % kPiecesPerWord of word chunk * kChunkWords +
// l / kPiecesPerWord.
__device__ __forceinline__ void group_pieces(const Geom &g, const uint64_t *__restrict__ true_bits,
                                             const uint64_t *__restrict__ cbits, const uint64_t *__restrict__ rrev,
                                             int kv, int G, int i, int chunk, int lane, unsigned (&m)[kMaxGroup],
                                             unsigned &shared) {
  const int w = chunk * kChunkWords + lane / kPiecesPerWord;
  const int shift = (lane % kPiecesPerWord) * kPieceBits;
  unsigned any = 0;
  shared = 0;
#pragma unroll
  for (int x = 0; x < kMaxGroup; ++x) {
    m[x] = 0;
    if (x < G && w <= (i >> 6)) {
      const int h = kv * G + x;
      const uint64_t word = mask_word(g, true_bits ? true_bits + (int64_t)h * g.L * g.tbw : nullptr,
                                      cbits + (int64_t)h * g.pw, rrev + (int64_t)h * g.pw, i, w);
      m[x] = (unsigned)(word >> shift) & ((1u << kPieceBits) - 1);
    }
    shared |= any & m[x];
    any |= m[x];
  }
}

__device__ __forceinline__ int wave_total(int v) {
  for (int off = 32; off; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// cnt[(kv * (G + 1) + run) * nchunks + chunk]
__global__ __launch_bounds__(256) void k_group_count(Geom g, const uint64_t *__restrict__ true_bits,
                                                     const uint64_t *__restrict__ cbits,
                                                     const uint64_t *__restrict__ rrev, int row, int G,
                                                     int nchunks, int *__restrict__ cnt) {
  const int lane = threadIdx.x & 63, chunk = blockIdx.x * 4 + (threadIdx.x >> 6), kv = blockIdx.y;
  if (chunk >= nchunks) return;  // whole waves
  unsigned m[kMaxGroup], shared;
  group_pieces(g, true_bits, cbits, rrev, kv, G, row, chunk, lane, m, shared);
  int *out = cnt + (int64_t)kv * (G + 1) * nchunks + chunk;
  const int c0 = wave_total(__popc(shared));
  if (lane == 0) out[0] = c0;
#pragma unroll
  for (int x = 0; x < kMaxGroup; ++x) {
    if (x < G) {
      const int c = wave_total(__popc(m[x] & ~shared));
      if (lane == 0) out[(int64_t)(1 + x) * nchunks] = c;
    }
  }
}

// first[e]: exclusive scan of cnt (n_groups * (G + 1) * nchunks + 1 entries)
__global__ __launch_bounds__(256) void k_group_fill(Geom g, const uint64_t *__restrict__ true_bits,
                                                    const uint64_t *__restrict__ cbits,
                                                    const uint64_t *__restrict__ rrev, int row, int G,
                                                    int nchunks, int n_groups, const int *__restrict__ first,
                                                    int *__restrict__ kept_ptr, int *__restrict__ kept_idx,
                                                    uint8_t *__restrict__ kept_member, int64_t capacity) {
  const int lane = threadIdx.x & 63, chunk = blockIdx.x * 4 + (threadIdx.x >> 6), kv = blockIdx.y;
  if (chunk >= nchunks) return;  // whole waves
  const int *mine_first = first + (int64_t)kv * (G + 1) * nchunks + chunk;
  if (chunk == 0 && lane == 0) {  // (offsets past the capacity of the list buffers are cut to it, like the block index')
    const int64_t clamp = kept_idx ? capacity : INT64_MAX;
    kept_ptr[kv] = (int)min((int64_t)mine_first[0], clamp);
    if (kv == n_groups - 1) kept_ptr[n_groups] = (int)min((int64_t)first[(int64_t)n_groups * (G + 1) * nchunks], clamp);
  }
  if (!kept_idx) return;
  unsigned m[kMaxGroup], shared;
  group_pieces(g, true_bits, cbits, rrev, kv, G, row, chunk, lane, m, shared);
  const int key0 = (chunk * kChunkWords + lane / kPiecesPerWord) * 64 + (lane % kPiecesPerWord) * kPieceBits;
#pragma unroll
  for (int r = 0; r <= kMaxGroup; ++r) {
    if (r <= G) {
      unsigned left = r == 0 ? shared : m[r - 1] & ~shared;  // lane's piece of run r
      const int v = __popc(left);
      int incl = v;
      for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
      }
      int64_t at = (int64_t)mine_first[(int64_t)r * nchunks] + incl - v;
      while (left) {
        const int bit = __ffs(left) - 1;
        left &= left - 1;
        unsigned who = r == 0 ? 0u : 1u << (r - 1);
        if (r == 0) {
#pragma unroll
          for (int y = 0; y < kMaxGroup; ++y) who |= ((m[y] >> bit) & 1u) << y;  // m[y] = 0 for y >= G
        }
        if (at < capacity) {
          kept_idx[at] = key0 + bit;
          if (kept_member) kept_member[at] = (uint8_t)who;
        }
        ++at;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Position-independent lists for grouped-query decoding in the pattern region (DAM_MASK_PATTERN_PLAN): per
// group of G maps first every diagonal offset matched by some map of the group, then every such column, each
// part in G + 1 runs (patterns of two or more maps; of map 0 alone; ...), each run ascending in the key it
// stands for. A diagonal r is stored as -1 - r (key p - r at position p), a column c as c. The diagonal part
// is the kept list of the last row of a P x P mask that has the group's diagonals and no columns (key j of
// that row is offset P - 1 - j), so the chunked count / scan / fill of the merged lists serves unchanged; the
// column part reads the column bitset itself. cnt / first: [((kv * 2 + part) * (G + 1) + run) * nchunks + chunk].
__device__ __forceinline__ void plan_pieces(const Geom &gp, const uint64_t *__restrict__ cbits,
                                            const uint64_t *__restrict__ rrev, int kv, int G, int part, int n_cols, int chunk,
                                            int lane, unsigned (&m)[kMaxGroup], unsigned &shared) {
  const int w = chunk * kChunkWords + lane / kPiecesPerWord;
  const int shift = (lane % kPiecesPerWord) * kPieceBits;
  unsigned any = 0;
  shared = 0;
#pragma unroll
  for (int x = 0; x < kMaxGroup; ++x) {
    m[x] = 0;
    if (x < G && w < gp.pw) {
      const int h = kv * G + x;
      uint64_t word;
      if (part == 0) {
        word = mask_word(gp, nullptr, nullptr, rrev + (int64_t)h * gp.pw, gp.S - 1, w);  // gp.S == P, gp.L == 0
      } else {
        word = cbits[(int64_t)h * gp.pw + w];
        const int left = n_cols - w * 64;  // columns of this word that exist
        word &= left >= 64 ? ~0ull : (left <= 0 ? 0ull : ~0ull >> (64 - left));
      }
      m[x] = (unsigned)(word >> shift) & ((1u << kPieceBits) - 1);
    }
    shared |= any & m[x];
    any |= m[x];
  }
}

__global__ __launch_bounds__(256) void k_plan_count(Geom gp, const uint64_t *__restrict__ cbits,
                                                    const uint64_t *__restrict__ rrev, int G, int n_cols, int nchunks,
                                                    int *__restrict__ cnt) {
  const int lane = threadIdx.x & 63, chunk = blockIdx.x * 4 + (threadIdx.x >> 6), kv = blockIdx.y, part = blockIdx.z;
  if (chunk >= nchunks) return;  // whole waves
  unsigned m[kMaxGroup], shared;
  plan_pieces(gp, cbits, rrev, kv, G, part, n_cols, chunk, lane, m, shared);
  int *out = cnt + (int64_t)(kv * 2 + part) * (G + 1) * nchunks + chunk;
  const int c0 = wave_total(__popc(shared));
  if (lane == 0) out[0] = c0;
#pragma unroll
  for (int x = 0; x < kMaxGroup; ++x) {
    if (x < G) {
      const int c = wave_total(__popc(m[x] & ~shared));
      if (lane == 0) out[(int64_t)(1 + x) * nchunks] = c;
    }
  }
}

__global__ __launch_bounds__(256) void k_plan_fill(Geom gp, const uint64_t *__restrict__ cbits,
                                                   const uint64_t *__restrict__ rrev, int G, int n_cols, int nchunks,
                                                   int n_groups, const int *__restrict__ first, int *__restrict__ kept_ptr,
                                                   int *__restrict__ kept_idx, uint8_t *__restrict__ kept_member,
                                                   int64_t capacity) {
  const int lane = threadIdx.x & 63, chunk = blockIdx.x * 4 + (threadIdx.x >> 6), kv = blockIdx.y, part = blockIdx.z;
  if (chunk >= nchunks) return;  // whole waves
  const int *mine_first = first + (int64_t)(kv * 2 + part) * (G + 1) * nchunks + chunk;
  if (chunk == 0 && lane == 0 && part == 0) {
    const int64_t clamp = kept_idx ? capacity : INT64_MAX;
    kept_ptr[kv] = (int)min((int64_t)mine_first[0], clamp);
    if (kv == n_groups - 1) kept_ptr[n_groups] = (int)min((int64_t)first[(int64_t)n_groups * 2 * (G + 1) * nchunks], clamp);
  }
  if (!kept_idx) return;
  unsigned m[kMaxGroup], shared;
  plan_pieces(gp, cbits, rrev, kv, G, part, n_cols, chunk, lane, m, shared);
  const int key0 = (chunk * kChunkWords + lane / kPiecesPerWord) * 64 + (lane % kPiecesPerWord) * kPieceBits;
  const int base = part == 0 ? key0 - gp.S : key0;  // diagonal part: key j of the virtual row P - 1 is -1 - (P - 1 - j) = j - P
#pragma unroll
  for (int r = 0; r <= kMaxGroup; ++r) {
    if (r <= G) {
      unsigned left = r == 0 ? shared : m[r - 1] & ~shared;
      const int v = __popc(left);
      int incl = v;
      for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
      }
      int64_t at = (int64_t)mine_first[(int64_t)r * nchunks] + incl - v;
      while (left) {
        const int bit = __ffs(left) - 1;
        left &= left - 1;
        unsigned who = r == 0 ? 0u : 1u << (r - 1);
        if (r == 0) {
#pragma unroll
          for (int y = 0; y < kMaxGroup; ++y) who |= ((m[y] >> bit) & 1u) << y;
        }
        if (at < capacity) {
          kept_idx[at] = base + bit;
          if (kept_member) kept_member[at] = (uint8_t)who;
        }
        ++at;
      }
    }
  }
}

// table[kv][r] = which maps of group kv have diagonal r matched (bit x: map kv * G + x)
__global__ void k_plan_table(const uint8_t *__restrict__ diag_flag, int P, int G, uint8_t *__restrict__ table) {
  const int kv = blockIdx.y;
  for (int r = blockIdx.x * blockDim.x + threadIdx.x; r < P; r += gridDim.x * blockDim.x) {
    unsigned who = 0;
    for (int x = 0; x < G; ++x) who |= (diag_flag[(int64_t)(kv * G + x) * P + r] ? 1u : 0u) << x;
    table[(int64_t)kv * P + r] = (uint8_t)who;
  }
}

int validate(const dam_mask_params *p, const float *attn_sum, const uint8_t *diag_in,
             const uint8_t *vert_in, const dam_mask_out *o) {
  if (!p || !o) return DAM_ERR_INVALID_ARG;
  if (p->mode != DAM_FROM_ATTN_MAP && p->mode != DAM_FROM_PATTERNS) return DAM_ERR_INVALID_ARG;
  if (p->n_maps < 1 || p->seq < 1) return DAM_ERR_INVALID_ARG;
  if (p->flags & ~(DAM_MASK_SKIP_FULL_TILE_BITS | DAM_MASK_GATHER_COLUMNS | DAM_MASK_GROUP_LISTS | DAM_MASK_PATTERN_PLAN))
    return DAM_ERR_INVALID_ARG;
  const bool plan = (p->flags & DAM_MASK_PATTERN_PLAN) != 0;
  if (plan && (!(p->flags & DAM_MASK_GROUP_LISTS) || !o->kept_ptr || !o->plan_table)) return DAM_ERR_INVALID_ARG;
  if ((p->flags & DAM_MASK_GROUP_LISTS) && o->kept_ptr) {
    if (p->group < 1 || p->group > kMaxGroup || p->n_maps % p->group) return DAM_ERR_INVALID_ARG;
    if (!plan && p->row_end != p->row_begin + 1) return DAM_ERR_UNSUPPORTED;
    if (o->kept_idx && !o->kept_member) return DAM_ERR_INVALID_ARG;
  }
  if ((p->flags & DAM_MASK_GATHER_COLUMNS) && (!o->gather_idx || !o->gather_cnt)) return DAM_ERR_INVALID_ARG;
  if (p->tile_m < 64 || p->tile_n < 64 || p->tile_m % 64 || p->tile_n % 64) return DAM_ERR_INVALID_ARG;
  if (p->tile_m > 256 || p->tile_n > 256) return DAM_ERR_UNSUPPORTED;
  if ((int64_t)(p->seq + p->tile_n - 1) / p->tile_n > 32768) return DAM_ERR_UNSUPPORTED;
  if (p->mode == DAM_FROM_ATTN_MAP) {
    if (p->pcl < 1 || !attn_sum || !o->true_bits) return DAM_ERR_INVALID_ARG;
    if (p->pcl >= (1 << kAccSlices)) return DAM_ERR_UNSUPPORTED;  // the match counts are summed in kAccSlices bits
    if (!(p->eps > 0.0f)) return DAM_ERR_INVALID_ARG;
    if (p->transform < DAM_T_BOXCOX || p->transform > DAM_T_ARCSINH) return DAM_ERR_INVALID_ARG;
    if (p->transform == DAM_T_BOXCOX && p->lambda != 0.5f && p->lambda != 1.0f) return DAM_ERR_UNSUPPORTED;
    if (isnan(p->lambda)) return DAM_ERR_INVALID_ARG;
    if (isnan(p->tau) || isnan(p->mu)) return DAM_ERR_INVALID_ARG;
  } else {
    if (p->pcl < 0 || !diag_in || !vert_in) return DAM_ERR_INVALID_ARG;
    if (p->pcl > 0 && !o->true_bits) return DAM_ERR_INVALID_ARG;
  }
  const bool blocks = o->blk_col || o->blk_kind || o->tile_bits || o->blk_total || o->blk_row_ptr;
  if (blocks && (!o->blk_row_ptr || !o->blk_total || o->blk_capacity < 0)) return DAM_ERR_INVALID_ARG;
  if ((o->blk_col || o->blk_kind || o->tile_bits) && o->blk_capacity < 1) return DAM_ERR_INVALID_ARG;
  if (o->dense_bits && p->seq > 65535) return DAM_ERR_UNSUPPORTED;
  if (o->kept_ptr || o->kept_idx || o->kept_total) {
    if (!o->kept_ptr || !o->kept_total || o->kept_capacity < 0) return DAM_ERR_INVALID_ARG;
    if (!plan && (p->row_begin < 0 || p->row_begin > p->row_end || p->row_end > p->seq)) return DAM_ERR_INVALID_ARG;
    if ((int64_t)p->n_maps * (p->row_end - p->row_begin) > (int64_t)1 << 30) return DAM_ERR_UNSUPPORTED;
  }
  return DAM_OK;
}

struct Workspace {
  float *bmin;
  unsigned *xmin_bits, *theta_key;
  TransformStats *stats;
  uint64_t *vslices, *dslices;
  uint8_t *diag_flag, *vert_flag;
  uint64_t *cbits, *rrev, *occ, *full, *col_any, *col_all, *off_any, *off_all, *vocc, *vfull;
  int *tile_cnt, *head_cnt, *row_cnt, *group_first;
  size_t bytes;
};

// Maps per list when a single row is listed: the group size with DAM_MASK_GROUP_LISTS, else 1 (a list per map is
// the same thing with groups of one: no key is shared, the only run is "map 0 alone", ascending).
int list_group(const dam_mask_params *p) {
  return (p->flags & DAM_MASK_GROUP_LISTS) && p->group >= 1 && p->group <= kMaxGroup ? p->group : 1;
}

// Chunks of kChunkWords mask words covering keys 0..row (one wave each in the group-list kernels).
int group_chunks(int row) { return ((row >> 6) + 1 + kChunkWords - 1) / kChunkWords; }

Geom geometry(const dam_mask_params *p) {
  Geom g;
  g.H = p->n_maps;
  g.L = p->pcl;
  g.S = p->seq;
  g.P = p->mode == DAM_FROM_ATTN_MAP ? p->pcl : p->seq;
  g.tile_m = p->tile_m;
  g.tile_n = p->tile_n;
  g.nQt = (g.S + g.tile_m - 1) / g.tile_m;
  g.nKt = (g.S + g.tile_n - 1) / g.tile_n;
  g.wpr = g.tile_n / 64;
  g.tbw = (g.L + 63) / 64;
  g.pw = (g.P + 63) / 64;
  g.occw = (g.nKt + 63) / 64;
  return g;
}

Workspace carve(const dam_mask_params *p, void *ws) {
  const Geom g = geometry(p);
  Carver c(ws);
  Workspace w;
  const size_t HL = (size_t)g.H * (size_t)(g.L > 0 ? g.L : 1);
  w.bmin = c.take<float>(1);
  w.xmin_bits = c.take<unsigned>(1);
  w.theta_key = c.take<unsigned>(1);
  w.stats = c.take<TransformStats>(1);
  const size_t n_slices = p->mode == DAM_FROM_ATTN_MAP
                              ? (size_t)g.H * (size_t)((g.L + kChunkRows - 1) / kChunkRows) * kSlices * (size_t)g.tbw
                              : 1;
  w.vslices = c.take<uint64_t>(n_slices);
  w.dslices = c.take<uint64_t>(n_slices);
  w.diag_flag = c.take<uint8_t>(HL);
  w.vert_flag = c.take<uint8_t>(HL);
  w.cbits = c.take<uint64_t>((size_t)g.H * g.pw);
  w.rrev = c.take<uint64_t>((size_t)g.H * g.pw);
  w.col_any = c.take<uint64_t>((size_t)g.H * g.occw);
  w.col_all = c.take<uint64_t>((size_t)g.H * g.occw);
  w.off_any = c.take<uint64_t>((size_t)g.H * g.occw);
  w.off_all = c.take<uint64_t>((size_t)g.H * g.occw);
  w.occ = c.take<uint64_t>((size_t)g.H * g.nQt * g.occw);
  w.full = c.take<uint64_t>((size_t)g.H * g.nQt * g.occw);
  const bool gather = (p->flags & DAM_MASK_GATHER_COLUMNS) != 0;
  w.vocc = c.take<uint64_t>(gather ? (size_t)g.H * g.nQt * g.occw : 1);
  w.vfull = c.take<uint64_t>(gather ? (size_t)g.H * g.nQt * g.occw : 1);
  w.tile_cnt = c.take<int>((size_t)g.H * g.nQt);
  w.head_cnt = c.take<int>((size_t)g.H * kHeadSub);
  const int nrows = p->row_end > p->row_begin ? p->row_end - p->row_begin : 0;
  size_t n_cnt = (size_t)g.H * (size_t)(nrows > 0 ? nrows : 1);
  size_t n_first = 1;
  if (nrows == 1 && p->row_begin >= 0) {  // a single row goes through the group-list kernels: run sizes per chunk, and their scan
    const int group = list_group(p);
    n_first = (size_t)(g.H / group) * (size_t)group_chunks(p->row_begin) * (size_t)(group + 1) + 1;
    n_cnt = std::max(n_cnt, n_first);
  }
  if (p->flags & DAM_MASK_PATTERN_PLAN) {  // two parts (diagonals, columns) over the P pattern positions
    const int group = list_group(p);
    n_first = std::max(n_first, (size_t)(g.H / group) * 2 * (size_t)group_chunks(g.P - 1) * (size_t)(group + 1) + 1);
    n_cnt = std::max(n_cnt, n_first);
  }
  w.row_cnt = c.take<int>(n_cnt);
  w.group_first = c.take<int>(n_first);
  w.bytes = c.off;
  return w;
}

// a1 and the threshold of a2. attn_sum / attn_cnt are only read in the general minimum. Returns how the
// true-mask kernel gets the key: by value when the host could find it (then that kernel also writes out_bmin),
// else from the workspace (in_workspace forces that form: the capture kernels read the key there).
Threshold stage_threshold(const dam_mask_params *p, const Geom &g, const Workspace &w, const float *attn_sum,
                          const float *attn_cnt, hipStream_t stream, float *out_bmin, bool in_workspace, bool *bmin_written) {
  const Threshold from_ws{w.theta_key, 0u, 0.0f, nullptr};
  *bmin_written = false;
  if (p->transform != DAM_T_BOXCOX) {
    // App. B alternatives: one reduction pass for the statistics, then minimum and threshold together
    const int64_t n = (int64_t)g.H * g.L * g.L;
    k_stats_init<<<1, 64, 0, stream>>>(w.stats);
    const int blocks = (int)std::min<int64_t>((n + 1023) / 1024, 256 * 16);
    k_stats<<<blocks, 256, 0, stream>>>(attn_sum, attn_cnt, n, g.L, p->eps, w.stats);
    k_transform_threshold<<<1, 64, 0, stream>>>(p->transform, p->lambda, p->eps, p->tau, p->bmin_override, w.stats,
                                                attn_cnt == nullptr, (float)n, (double)n, w.bmin, w.theta_key);
    return from_ws;
  }
  const bool half = p->lambda == 0.5f;
  // a1: the global minimum of the Box-Cox map. Known without the data when the caller overrides it, and for a single
  // causal capture with L >= 2 (some pair was never computed: its X is the clamp eps, and no X is smaller)
  if (!isnan(p->bmin_override) || (!attn_cnt && g.L >= 2)) {
    const float x_min = clamp_mean(0.0f, 0.0f, p->eps);
    const float bmin = !isnan(p->bmin_override) ? p->bmin_override : (half ? box_cox<1>(x_min) : box_cox<2>(x_min));
    unsigned key;
    if (half) key = attn_cnt ? threshold_key<1, false>(p->eps, p->tau, bmin) : threshold_key<1, true>(p->eps, p->tau, bmin);
    else key = attn_cnt ? threshold_key<2, false>(p->eps, p->tau, bmin) : threshold_key<2, true>(p->eps, p->tau, bmin);
    *bmin_written = true;
    if (in_workspace) {
      k_set_threshold<<<1, 64, 0, stream>>>(bmin, key, w.bmin, w.theta_key, out_bmin);
      return from_ws;
    }
    return Threshold{nullptr, key, bmin, out_bmin};
  }
  const int64_t n = (int64_t)g.H * g.L * g.L;
  k_fill_u32<<<1, 64, 0, stream>>>(w.xmin_bits, 1, 0x7F800000u);
  const int blocks = (int)std::min<int64_t>((n + 1023) / 1024, 256 * 16);
  k_min_x<<<blocks, 256, 0, stream>>>(attn_sum, attn_cnt, n, g.L, p->eps, w.xmin_bits);
  if (half) k_bmin_from_x<1><<<1, 64, 0, stream>>>(w.xmin_bits, w.bmin);
  else k_bmin_from_x<2><<<1, 64, 0, stream>>>(w.xmin_bits, w.bmin);
  // a2: the threshold, found once
  if (half) {
    if (attn_cnt) k_threshold<1, false><<<1, 64, 0, stream>>>(p->eps, p->tau, w.bmin, w.theta_key);
    else k_threshold<1, true><<<1, 64, 0, stream>>>(p->eps, p->tau, w.bmin, w.theta_key);
  } else {
    if (attn_cnt) k_threshold<2, false><<<1, 64, 0, stream>>>(p->eps, p->tau, w.bmin, w.theta_key);
    else k_threshold<2, true><<<1, 64, 0, stream>>>(p->eps, p->tau, w.bmin, w.theta_key);
  }
  return from_ws;
}

// a3: match scores of the true mask in o->true_bits; returns where the flags were written.
void stage_patterns(const dam_mask_params *p, const Geom &g, const Workspace &w, const dam_mask_out *o,
                    hipStream_t stream, const uint8_t **dflag, const uint8_t **vflag, bool bmin_written) {
  uint8_t *df = o->diag_flag ? o->diag_flag : w.diag_flag;
  uint8_t *vf = o->vert_flag ? o->vert_flag : w.vert_flag;
  const int n_chunks = (g.L + kChunkRows - 1) / kChunkRows;
  if (g.tbw <= 128) {
    int W = 16;
    while (W < g.tbw) W *= 2;
    const size_t lds = std::max<size_t>((size_t)kChunkRows * W, (size_t)2 * 256 * kSlices) * sizeof(uint64_t);
    k_pattern_slices<<<dim3(n_chunks, g.H), 256, lds, stream>>>(o->true_bits, g.L, g.tbw, n_chunks, W, w.vslices, w.dslices);
  } else {
    const dim3 sgrid(2 * ((g.tbw + 63) / 64), (n_chunks + 3) / 4, g.H);
    k_pattern_slices_wide<<<sgrid, 256, 0, stream>>>(o->true_bits, g.L, g.tbw, n_chunks, w.vslices, w.dslices);
  }
  int nb = 1;  // bits of the largest possible count, L
  while ((g.L >> nb) != 0) ++nb;
  k_pattern_finish<<<dim3((g.tbw + kFinWords - 1) / kFinWords, g.H, 2), 256, 0, stream>>>(w.vslices, w.dslices, g.L, g.tbw, n_chunks, nb, p->mu,
                                                                       o->vert_cnt, o->diag_cnt, vf, df);
  *dflag = df;
  *vflag = vf;
  if (o->bmin && !bmin_written) k_copy_f32<<<1, 64, 0, stream>>>(o->bmin, w.bmin);
}

// a4 + a5 and the kept lists: everything downstream of the stored artefact.
void stage_extension(const dam_mask_params *p, const Geom &g, const Workspace &w, const dam_mask_out *o,
                     const uint64_t *true_bits, const uint8_t *dflag, const uint8_t *vflag, hipStream_t stream) {
  const bool want_blocks = o->blk_row_ptr != nullptr;
  const bool want_lists = o->kept_ptr != nullptr;
  const bool gather = want_blocks && (p->flags & DAM_MASK_GATHER_COLUMNS) != 0;
  const int gstride = dam_gather_stride(p);
  const int *gidx = gather ? o->gather_idx : nullptr, *gcnt = gather ? o->gather_cnt : nullptr;
  if (want_blocks || want_lists || o->dense_bits) {
    const size_t prep_lds = want_blocks && (size_t)g.pw * 16 <= kMaxStagedBytes ? (size_t)g.pw * 16 : 0;
    k_pattern_prep<<<g.H, 1024, prep_lds, stream>>>(g, dflag, vflag, w.cbits, w.rrev, want_blocks, w.col_any, w.col_all, w.off_any,
                                                   w.off_all, gstride, gather ? o->gather_idx : nullptr,
                                                   gather ? o->gather_cnt : nullptr, w.head_cnt, prep_lds > 0);
  }
  // a4 + a5: tile occupancy, CSR offsets, tile bits
  if (want_blocks) {
    const size_t lds_sets = staged_bytes(g);
    const bool fill = o->blk_col || o->blk_kind || o->tile_bits;
    k_tile_scan<<<dim3((g.nQt + 3) / 4, g.H), 256, lds_sets, stream>>>(g, true_bits, w.cbits, w.rrev, w.col_any, w.col_all, w.off_any,
                                                                     w.off_all, w.occ, w.full, w.tile_cnt, lds_sets > 0, gidx,
                                                                     gcnt, gstride, w.vocc, w.vfull, w.head_cnt);
    if (fill) {
      // (the CSR offsets come out of the fill kernel: no scan launch between the two passes)
      const int share = (int64_t)g.H * g.nQt >= 2048 ? 1 : 4;  // enough query tiles to give every wave its own
      const dim3 fill_grid(share == 4 ? g.nQt : (g.nQt + 3) / 4, g.H);
      const bool skip_full = (p->flags & DAM_MASK_SKIP_FULL_TILE_BITS) != 0;
      if (lds_sets > 0)
        k_tile_fill<true><<<fill_grid, 256, lds_sets, stream>>>(
            g, true_bits, w.cbits, w.rrev, w.occ, w.full, w.tile_cnt, w.head_cnt, o->blk_row_ptr, o->blk_total, o->blk_col,
            o->blk_kind, o->tile_bits, o->blk_capacity, skip_full, gidx, gcnt, gstride, w.vocc, w.vfull, share);
      else
        k_tile_fill<false><<<fill_grid, 256, 0, stream>>>(
            g, true_bits, w.cbits, w.rrev, w.occ, w.full, w.tile_cnt, w.head_cnt, o->blk_row_ptr, o->blk_total, o->blk_col,
            o->blk_kind, o->tile_bits, o->blk_capacity, skip_full, gidx, gcnt, gstride, w.vocc, w.vfull, share);
    } else {  // the sizing call: offsets and total only
      k_exclusive_scan<<<1, 1024, 0, stream>>>(w.tile_cnt, (int64_t)g.H * g.nQt, g.nQt, o->blk_row_ptr, o->blk_total, INT64_MAX);
    }
  }
  if (o->dense_bits) {
    const int sw = (g.S + 63) / 64;
    k_dense_bits<<<dim3((sw + 255) / 256, g.S, g.H), 256, 0, stream>>>(g, true_bits, w.cbits, w.rrev, sw, o->dense_bits);
  }
  if (want_lists && (p->flags & DAM_MASK_PATTERN_PLAN)) {
    Geom gp = g;  // the P x P pattern-only mask whose last row lists the diagonals
    gp.L = 0;
    gp.S = g.P;
    const int G = list_group(p), n_groups = g.H / G, nchunks = group_chunks(g.P - 1), n_cols = std::min(g.P, g.S);
    const dim3 grid((nchunks + 3) / 4, n_groups, 2);
    k_plan_count<<<grid, 256, 0, stream>>>(gp, w.cbits, w.rrev, G, n_cols, nchunks, w.row_cnt);
    k_exclusive_scan<<<1, 1024, 0, stream>>>(w.row_cnt, (int64_t)n_groups * 2 * (G + 1) * nchunks, 0, w.group_first, o->kept_total,
                                             INT64_MAX);
    k_plan_fill<<<grid, 256, 0, stream>>>(gp, w.cbits, w.rrev, G, n_cols, nchunks, n_groups, w.group_first, o->kept_ptr,
                                          o->kept_capacity > 0 ? o->kept_idx : nullptr, o->kept_member, o->kept_capacity);
    k_plan_table<<<dim3((g.P + 255) / 256, n_groups), 256, 0, stream>>>(dflag, g.P, G, o->plan_table);
  } else if (want_lists) {
    const int nrows = p->row_end - p->row_begin;
    if (nrows == 1) {
      // one row (a decode step): the chunked kernels below, whose longest dependent chain is eight steps; lists per
      // map are groups of one
      const int G = list_group(p), n_groups = g.H / G, nchunks = group_chunks(p->row_begin);
      const dim3 grid((nchunks + 3) / 4, n_groups);
      k_group_count<<<grid, 256, 0, stream>>>(g, true_bits, w.cbits, w.rrev, p->row_begin, G, nchunks, w.row_cnt);
      k_exclusive_scan<<<1, 1024, 0, stream>>>(w.row_cnt, (int64_t)n_groups * (G + 1) * nchunks, 0, w.group_first, o->kept_total,
                                               INT64_MAX);
      k_group_fill<<<grid, 256, 0, stream>>>(g, true_bits, w.cbits, w.rrev, p->row_begin, G, nchunks, n_groups, w.group_first,
                                             o->kept_ptr, o->kept_capacity > 0 ? o->kept_idx : nullptr, o->kept_member,
                                             o->kept_capacity);
    } else if (nrows > 0) {
      k_row_count<<<dim3(nrows, g.H), 256, 0, stream>>>(g, true_bits, w.cbits, w.rrev, p->row_begin, nrows, w.row_cnt);
      const bool fill_lists = o->kept_idx && o->kept_capacity > 0;
      k_exclusive_scan<<<1, 1024, 0, stream>>>(w.row_cnt, (int64_t)g.H * nrows, 0, o->kept_ptr, o->kept_total,
                                               fill_lists ? o->kept_capacity : INT64_MAX);
      if (fill_lists)
        k_row_fill<<<dim3(nrows, g.H), 256, 0, stream>>>(g, true_bits, w.cbits, w.rrev, p->row_begin, nrows, o->kept_ptr,
                                                         o->kept_idx, o->kept_capacity);
    } else {
      k_exclusive_scan<<<1, 1024, 0, stream>>>(w.row_cnt, 0, 0, o->kept_ptr, o->kept_total, INT64_MAX);
    }
  }
}

}  // namespace

extern "C" int32_t dam_gather_stride(const dam_mask_params *p) {
  if (!p || p->seq < 1 || p->tile_n < 64 || p->pcl < 0) return 0;
  const int64_t P = p->mode == DAM_FROM_ATTN_MAP ? p->pcl : p->seq;
  const int64_t n = std::min<int64_t>(P, p->seq);
  return (int32_t)((n + p->tile_n - 1) / p->tile_n * p->tile_n);
}

extern "C" size_t dam_mask_build_workspace(const dam_mask_params *p) {
  if (!p || p->n_maps < 1 || p->seq < 1 || p->pcl < 0 || p->tile_m < 64 || p->tile_n < 64 ||
      p->tile_m % 64 || p->tile_n % 64)
    return 0;
  return carve(p, nullptr).bytes;
}

extern "C" int dam_mask_build(const dam_mask_params *p, const float *attn_sum, const float *attn_cnt,
                              const uint8_t *diag_in, const uint8_t *vert_in, const dam_mask_out *o,
                              void *ws, size_t ws_bytes, void *stream_v) {
  const int bad = validate(p, attn_sum, diag_in, vert_in, o);
  if (bad != DAM_OK) return bad;
  if (!ws || ws_bytes < dam_mask_build_workspace(p)) return DAM_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  const Geom g = geometry(p);
  const Workspace w = carve(p, ws);
  const uint8_t *dflag = diag_in, *vflag = vert_in;
  const uint64_t *true_bits = g.L > 0 ? o->true_bits : nullptr;

  if (p->mode == DAM_FROM_ATTN_MAP) {
    bool bmin_written;
    const Threshold thr = stage_threshold(p, g, w, attn_sum, attn_cnt, stream, o->bmin, false, &bmin_written);
    // a2: true mask, one comparison per element
    dim3 grid((g.tbw + 3) / 4, (g.L + kTmRows - 1) / kTmRows, g.H);
    if (attn_cnt && p->transform == DAM_T_RAW_SUM)
      k_true_mask<false, true><<<grid, 256, 0, stream>>>(attn_sum, attn_cnt, g.L, g.tbw, p->eps, thr, o->true_bits);
    else if (attn_cnt)
      k_true_mask<false><<<grid, 256, 0, stream>>>(attn_sum, attn_cnt, g.L, g.tbw, p->eps, thr, o->true_bits);
    else if (g.L % 4 == 0 && (reinterpret_cast<uintptr_t>(attn_sum) & 15) == 0) {
      const int n_pairs = (((g.L + 1) / 2) + 3) / 4;
      const int per_map = std::max(1, std::min(n_pairs, kGridTarget / g.H));
      k_true_mask_rows<<<dim3(per_map, g.H), 256, 0, stream>>>(attn_sum, g.L, g.tbw, n_pairs, thr, o->true_bits);
    } else
      k_true_mask<true><<<grid, 256, 0, stream>>>(attn_sum, attn_cnt, g.L, g.tbw, p->eps, thr, o->true_bits);
    stage_patterns(p, g, w, o, stream, &dflag, &vflag, bmin_written);
  }
  stage_extension(p, g, w, o, true_bits, dflag, vflag, stream);
  return launch_status();
}

// Sec. 4.2.1 - 4.3 for one captured sequence, from its Q and K: the probabilities are thresholded
// as the capture kernels produce them (dam_capture.hip); the rest is the path above.
extern "C" size_t dam_mask_build_from_qk_workspace(const dam_mask_params *p, const dam_capture_params *cp) {
  const size_t base = dam_mask_build_workspace(p);
  if (!base || !cp || cp->hq < 1 || cp->pcl < 1) return 0;
  return base + capture_lse_bytes(cp);
}

extern "C" int dam_mask_build_from_qk(const dam_mask_params *p, const dam_capture_params *cp, const void *q,
                                      const void *k, const dam_mask_out *o, void *ws, size_t ws_bytes,
                                      void *stream_v) {
  if (!p || !o || !cp) return DAM_ERR_INVALID_ARG;
  if (p->mode != DAM_FROM_ATTN_MAP) return DAM_ERR_INVALID_ARG;
  const float dummy_map = 0.0f;  // validate() only checks that a map pointer is present
  int bad = validate(p, &dummy_map, nullptr, nullptr, o);
  if (bad != DAM_OK) return bad;
  bad = capture_validate(cp, q, k);
  if (bad != DAM_OK) return bad;
  if (p->n_maps != cp->hq || p->pcl != cp->pcl || cp->len != cp->pcl || p->pcl < 2) return DAM_ERR_INVALID_ARG;
  if (p->transform != DAM_T_BOXCOX) return DAM_ERR_UNSUPPORTED;  // the other transforms need statistics of the whole map
  if (!ws || ws_bytes < dam_mask_build_from_qk_workspace(p, cp)) return DAM_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(stream_v);
  const Geom g = geometry(p);
  const Workspace w = carve(p, ws);
  float *lse2 = reinterpret_cast<float *>(static_cast<char *>(ws) + w.bytes);
  const uint8_t *dflag = nullptr, *vflag = nullptr;
  bool bmin_written;
  stage_threshold(p, g, w, nullptr, nullptr, stream, o->bmin, true, &bmin_written);
  launch_capture_true_bits(cp, q, k, lse2, w.theta_key, o->true_bits, stream);
  stage_patterns(p, g, w, o, stream, &dflag, &vflag, bmin_written);
  stage_extension(p, g, w, o, o->true_bits, dflag, vflag, stream);
  return launch_status();
}
