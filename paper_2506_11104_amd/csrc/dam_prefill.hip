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
//     registers; V stays row-major in LDS and its transposed A operand comes from the
//     transposing LDS read (ds_read_b64_tr_b16), addressed with the same permutation.
//   The unit of work is a block of 32 keys (an occupied key quarter of a listed tile). K / V blocks
//     move through two LDS rings of four slots filled by load-to-LDS instructions (no registers in
//     between), three blocks ahead of their use; one barrier per block. Within a wave the products
//     of three consecutive blocks are interleaved with the softmax arithmetic (see the kernel).
//     The blocks of a query tile are listed in LDS first (its tiles expanded 128 at a time by the whole
//     workgroup), so that an iteration reads one descriptor instead of walking tiles in scalar code.
//   Tiles not in the block index are never touched, key quarters of a tile without a kept entry are
//     never loaded, and full tiles skip the element mask.
// fp32 kernel (the 1e-4 variant): plain ALU code, one query row per group of head_dim/4 lanes,
// iterating only over the set bits of the row's tile words.
#include <hip/hip_bf16.h>
#include <math.h>

#include <algorithm>
#include <type_traits>
#include <utility>

#include "dam_internal.h"
#include "dam_mfma.h"

namespace {
using namespace dam;

constexpr int kXcd = 8;
// control words at the start of the bf16 kernel's workspace: the eight queue counters, then the redo list's
// length and its read cursor; the list itself (one int2 per work item at most) starts at byte kCtlBytes
constexpr int kRedoCount = 8, kRedoNext = 9, kCtlWords = 10, kCtlBytes = 256;

struct AttnArgs {
  int B, Hq, Hkv, S, nQt, nKt, tile_m, tile_n, wpr;
  int gather_rows, gather_stride;  // gathered column tiles (tile index >= nKt), 0 when the index has none
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
                                                     const uint8_t *__restrict__ blk_kind,
                                                     const uint64_t *__restrict__ tile_bits,
                                                     const int *__restrict__ gather_idx,
                                                     float *__restrict__ out, float *__restrict__ lse) {
  constexpr int N = 4, LPR = D / N, GROUPS = 256 / LPR;
  // a workgroup takes GROUPS rows of a query tile at a time; blockIdx.y spreads a tile's passes over workgroups
  // (a row's keys are folded in one after the other: the more rows in flight, the better)
  const WorkItem w = decode_work(a, blockIdx.x);
  if (!w.valid) return;
  const int group = threadIdx.x / LPR, sub = threadIdx.x % LPR;
  const int t0 = row_ptr[(int64_t)w.hq * (a.nQt + 1) + w.qt];
  const int t1 = row_ptr[(int64_t)w.hq * (a.nQt + 1) + w.qt + 1];
  const float *kb = k + w.b * a.k_sb + w.hkv * a.k_sh + sub * N;
  const float *vb = v + w.b * a.v_sb + w.hkv * a.v_sh + sub * N;
  for (int rl = blockIdx.y * GROUPS + group; rl < a.tile_m; rl += GROUPS * gridDim.y) {
    const int i = w.qt * a.tile_m + rl;
    if (i >= a.S) break;
    const float4 qv = *reinterpret_cast<const float4 *>(q + w.b * a.q_sb + w.hq * a.q_sh + i * a.q_ss + sub * N);
    float m = -INFINITY, l = 0.0f;
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int t = t0; t < t1; ++t) {
      // (a column or a key outside its range, from a list that was never filled, is pulled inside it)
      const int col = min(max(blk_col[t], 0), a.nKt + (gather_idx ? a.gather_stride / a.tile_n : 0) - 1);
      // a gathered tile (index >= nKt): slot s of the tile stands for the head's matched column gcols[s]
      const int *gcols = col >= a.nKt ? gather_idx + (int64_t)w.hq * a.gather_stride + (col - a.nKt) * a.tile_n : nullptr;
      const int j0 = col * a.tile_n;
      const bool full = blk_kind[t] & 1;  // every entry kept: the tile's words are not read (they may be unwritten)
      for (int wd = 0; wd < a.wpr; ++wd) {
        uint64_t bits = full ? ~0ull : tile_bits[((int64_t)t * a.tile_m + rl) * a.wpr + wd];
        while (bits) {
          // the rows of up to four kept keys are fetched together (their addresses depend on the bits, so nothing
          // else hides the latency), then folded into the running softmax one after the other, in key order
          constexpr int U = 4;
          float4 kv[U], vv[U];
          bool have[U];
#pragma unroll
          for (int u = 0; u < U; ++u) {
            have[u] = bits != 0;
            const int slot = wd * 64 + (have[u] ? __ffsll((unsigned long long)bits) - 1 : 0);
            const int j = min(max(gcols ? gcols[slot] : j0 + slot, 0), a.S - 1);
            bits &= bits - 1;  // (0 stays 0)
            kv[u] = *reinterpret_cast<const float4 *>(kb + j * a.k_ss);
            vv[u] = *reinterpret_cast<const float4 *>(vb + j * a.v_ss);
          }
#pragma unroll
          for (int u = 0; u < U; ++u) {
            if (!have[u]) break;  // uniform over the lanes of a row
            float d = qv.x * kv[u].x + qv.y * kv[u].y + qv.z * kv[u].z + qv.w * kv[u].w;
#pragma unroll
            for (int off = LPR / 2; off; off >>= 1) d += __shfl_xor(d, off);
            const float s = d * a.scale;
            const float mn = fmaxf(m, s);
            const float corr = expf(m - mn), p = expf(s - mn);
            l = l * corr + p;
            o.x = o.x * corr + p * vv[u].x;
            o.y = o.y * corr + p * vv[u].y;
            o.z = o.z * corr + p * vv[u].z;
            o.w = o.w * corr + p * vv[u].w;
            m = mn;
          }
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
constexpr int kBM = 128, kBN = 128;

// LDS layout. Rows are 256 B = 16 chunks of 16 B and are not padded, because the global -> LDS
// copies are done by the load-to-LDS instruction, which writes the 64 lanes of a wave to 1 KiB of
// consecutive LDS. Bank conflicts are avoided by permuting the chunks of a row instead:
//   K row r: chunk c lives at position c ^ (r & 15)        (16-byte reads of 16 consecutive rows
//            and one logical chunk then cover all 64 banks once)
//   V row r: chunk c lives at position c ^ ((r & 3) << 2)  (a transposing read touches 4 rows x 64 B
//            per half-wave; the four 64-byte groups land in different bank quarters)
// The permutation is applied on the global side of the copy (which chunk a lane fetches).

// Scheduling hints: instruction classes of __builtin_amdgcn_sched_group_barrier.
#define DAM_SCHED_MFMA 0x008
#define DAM_SCHED_DSREAD 0x100

// ================================================================================================
// Block-pipelined bf16 kernel. The unit of work is a block of 32 keys (one occupied key quarter of
// a listed tile). In iteration b a wave issues, interleaved in one instruction stream,
//     the 8 MFMAs of S_{b+1} = K_{b+1} Q^T   (one dependent chain),
//     the 8 MFMAs of O^T += V_{b-1}^T P_{b-1}^T (four independent accumulators),
//     the softmax arithmetic of block b (VALU) on S_b, which finished one iteration earlier,
// so that the matrix pipe and the vector ALU of a SIMD are busy at the same time from within one
// wave. K and V blocks live in two LDS rings of four 8 KiB slots each, filled by load-to-LDS
// copies issued three iterations ahead (K_{b+4} and V_{b+2} in iteration b); one barrier per
// iteration. The stream is padded with "dummy" blocks (mask bits all zero, so S = -inf and P = 0)
// at both ends, which keeps every iteration identical.
constexpr int kBlkKeys = 32;
constexpr int kBlkBytes = kBlkKeys * 256;
constexpr int kRing = 4;
constexpr int kVRing = kRing * kBlkBytes;  // byte offset of the V ring; K ring at 0
constexpr int kBitsRing = 2 * kRing * kBlkBytes;  // mask words: 4 slots x 4 waves x 64 lanes x 4 B
constexpr int kBlkList = kBitsRing + kRing * 1024;  // the block list of the current segment of tiles
constexpr int kSegTiles = 128;                      // listed tiles expanded into the list at a time
constexpr int kListEntries = kSegTiles * 4 + 1;     // up to four blocks per tile, and the dummy that ends the list
constexpr int kPipeLds = kBlkList + kListEntries * 8;

struct Blk {
  int key0;        // first key of the block (gathered tile: first row of the block in the gathered copy)
  int bits_off;    // byte offset of row 0's mask word for the block from the tile row's first mask word
  int flags;       // bit 0: tile is full (no mask), bit 1: dummy, bit 2: gathered tile (offsets into the gathered copies)
};

// FAST: the softmax without a running maximum. A weight is exp2(logit * scale * log2 e) itself: one multiply and
// one exponential per entry, no row maximum, no subtraction, no rescaling of O. (Folding the factor into the
// bf16 queries would save the multiply, but rounds every logit by up to 2^-9 of its size: 8 % in the weight of a
// logit of 70.) That is exact as long as the weights stay inside the range of fp32 and bf16 (both have 8
// exponent bits); the kernel checks the row sums at the end of a work item and sends the item to the variant
// with a running reference (FAST = false) when a sum left [2^-100, 2^100].
// seen / seen_full: does this lane's row have a kept entry at all (an empty row is not a failed one).
template <int PH, bool FAST>
__device__ __forceinline__ void pipe_iter(const unsigned char *__restrict__ lds, const bf16x8 (&qf)[8],
                                          f32x16 (&oacc)[4], const f32x16 &sA, f32x16 &sB,
                                          const unsigned (&pPrev)[8], unsigned (&pCur)[8], float &m_run,
                                          float &l_run, unsigned &seen, int &seen_full, int flags_next, int bits_addr,
                                          float c2, int kbase, int vbase, int hf) {
  // kbase ^ (c << 5) is this lane's address of chunk pair c of its K row, vbase ^ (db << 6) that of
  // dim block db in its V rows (the chunk permutations are XORs, see the layout note)
  int kaddr[8], vaddr[4];
#pragma unroll
  for (int c = 0; c < 8; ++c) kaddr[c] = kbase ^ (c << 5);
#pragma unroll
  for (int db = 0; db < 4; ++db) vaddr[db] = vbase ^ (db << 6);
  constexpr int KS = PH * kBlkBytes;                          // slot of K_{b+1}
  constexpr int VS = kVRing + ((PH + 2) & 3) * kBlkBytes;     // slot of V_{b-1}
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  // The first product of the S_{b+1} chain. Accumulator e is key 8 (e / 4) + 4 hf + e % 4 of the block
  // and starts at 0 (kept) or -inf (masked); a full tile needs no mask words and starts from a literal
  // zero (wave-uniform branch), and so does a block of a partial tile whose 32 x 32 entries of this wave
  // are all kept (a band edge crosses only some of the sixteen such squares of a tile).
  const bf16x8 kf0 = lds_read_b128(lds, KS + kaddr[0]);
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (flags_next & 1) {
    if (FAST) seen_full = 1;
    sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf0, qf[0], zero, 0, 0, 0);
  } else {
    unsigned bits_next = *reinterpret_cast<const unsigned *>(lds + kBitsRing + PH * 1024 + bits_addr);
    if (flags_next & 2) bits_next = 0u;  // dummy block: nothing kept
    if (FAST) seen |= bits_next;
    if (__builtin_amdgcn_ballot_w64(bits_next != 0xFFFFFFFFu) == 0) {
      sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf0, qf[0], zero, 0, 0, 0);
    } else {
      const int inv = (int)~(bits_next >> (4 * hf));
      // sign-extended one-bit field (0 or all ones), then the bits of -inf; the extract is written as an
      // instruction because the compiler turns the builtin into a three-operation compare and select
      mask_init(sB, inv, std::make_integer_sequence<int, 16>{});
      sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf0, qf[0], sB, 0, 0, 0);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- operand fetches, in the order the MFMAs consume them
  bf16x8 kf[8];
  s16x8 vf[2][4];
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    if (x > 0) kf[x] = lds_read_b128(lds, KS + kaddr[x]);
    const int a2 = x >> 2, db = x & 3;
    const s16x4 r0 = lds_read_tr(lds, VS + vaddr[db] + (a2 * 16) * 256);
    const s16x4 r1 = lds_read_tr(lds, VS + vaddr[db] + (a2 * 16 + 8) * 256);
    vf[a2][db] = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
  }
  // ---- matrix work: the rest of the S_{b+1} chain and P_{b-1} V_{b-1}, alternating
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    if (x > 0) sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[x], qf[x], sB, 0, 0, 0);
    const int a2 = x >> 2, db = x & 3;
    const u32x4 praw = {pPrev[4 * a2], pPrev[4 * a2 + 1], pPrev[4 * a2 + 2], pPrev[4 * a2 + 3]};
    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[a2][db]),
                                                       __builtin_bit_cast(bf16x8, praw), oacc[db], 0, 0, 0);
  }
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  if (FAST) {
    // ---- vector work: the weights of block b and their sum, nothing else
#pragma unroll
    for (int e = 0; e < 16; e += 2) {
      const float p0 = __builtin_amdgcn_exp2f(sA[e] * c2);
      const float p1 = __builtin_amdgcn_exp2f(sA[e + 1] * c2);
      pCur[e / 2] = pack_bf16(p0, p1);
      // the row sum is taken over the rounded weights the P V product uses
      l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pCur[e / 2]), ones, l_run, false);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) asm volatile("" ::"v"(pCur[e]));
    // ---- interleave: a few operand reads ahead, then per MFMA three VALU ops and the reads it needs
    __builtin_amdgcn_sched_group_barrier(DAM_SCHED_DSREAD, 12, 0);
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      if (x > 0) {
        __builtin_amdgcn_sched_group_barrier(DAM_SCHED_MFMA, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
      }
      __builtin_amdgcn_sched_group_barrier(DAM_SCHED_DSREAD, 2, 0);
      __builtin_amdgcn_sched_group_barrier(DAM_SCHED_MFMA, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
      __builtin_amdgcn_sched_group_barrier(DAM_SCHED_DSREAD, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    return;
  }
  // ---- vector work: online softmax of block b; one query per lane pair (lane, lane ^ 32)
  float mx = fmaxf(fmaxf(sA[0], sA[1]), sA[2]);
#pragma unroll
  for (int e = 3; e < 15; e += 2) mx = fmaxf(fmaxf(sA[e], sA[e + 1]), mx);
  mx = fmaxf(mx, sA[15]);
  {
    // the other half-wave's maximum of the same query row: one swap of the 32-lane halves (operands
    // both mx: the results are the lower half's values in all lanes, and the upper half's)
    typedef __attribute__((ext_vector_type(2))) unsigned u32x2_t;
    const u32x2_t sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
    mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
  }
  // m_run is the reference the weights are taken against, not necessarily the running maximum: it
  // only moves when the maximum has grown past it by more than 8 in log2 units (weights then stay
  // below 2^8, far inside the range of bf16 and of the fp32 sums), so that O rarely has to be rescaled.
  // The quotient O / l at the end does not depend on the reference. (-inf) - (-inf) is NaN: no move.
  const float m_top = fmaxf(m_run, mx);
  const bool move = (m_top - m_run) * c2 > 8.0f;
  const float m_new = move ? m_top : m_run;
  const float m_ref = m_new == -INFINITY ? 0.0f : m_new;
  const float off = m_ref * c2;
  const float m_old = m_run;
  m_run = m_new;
  float psum = 0.0f;
#pragma unroll
  for (int e = 0; e < 16; e += 2) {
    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sA[e], c2, -off));
    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sA[e + 1], c2, -off));
    pCur[e / 2] = pack_bf16(p0, p1);
    // the row sum is taken over the rounded weights the P V product uses
    psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pCur[e / 2]), ones, psum, false);
  }
  // keep the weights of block b inside this block of code (they are only consumed an iteration later
  // and would otherwise be sunk below the matrix work)
#pragma unroll
  for (int e = 0; e < 8; ++e) asm volatile("" ::"v"(pCur[e]));
  // ---- interleave: a few operand reads ahead, then per MFMA pair three reads and eight VALU ops
  __builtin_amdgcn_sched_group_barrier(DAM_SCHED_DSREAD, 12, 0);
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    if (x > 0) {
      __builtin_amdgcn_sched_group_barrier(DAM_SCHED_MFMA, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
    }
    __builtin_amdgcn_sched_group_barrier(DAM_SCHED_DSREAD, 2, 0);
    __builtin_amdgcn_sched_group_barrier(DAM_SCHED_MFMA, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
    __builtin_amdgcn_sched_group_barrier(DAM_SCHED_DSREAD, 1, 0);
  }
  __builtin_amdgcn_sched_barrier(0);
  // O and the row sum were accumulated against the old reference: when some row's reference moved,
  // rescale them, after P_{b-1} V_{b-1} is in (rare after the first blocks of a row)
  if (__ballot(move)) {
    const float corr = move ? __builtin_amdgcn_exp2f((m_old - m_ref) * c2) : 1.0f;  // old = -inf: 0
    l_run *= corr;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[db][e] *= corr;
  }
  l_run += psum;
}

// The FAST iteration laid out by hand in eight segments, one per pair of products (S chain step x, P V step x).
// The wave issues in order, so what stands between the last product of one iteration and the first of the next
// is time the matrix pipe of this wave idles: the bookkeeping of an iteration (decoding the next descriptor,
// issuing the five copies, fetching the descriptor after that) therefore sits inside the stream of products,
// one piece per segment (bk(x)), behind the operand reads (the copies are volatile statements that LDS reads do
// not move across), and only the flag test, the wait for the copies, the barrier and the first operand reads
// remain between two iterations.
// PART says which of the three streams the iteration holds: kAll in the steady state; the first iteration of a
// pass (block -1, kChainOnly) has no weights to compute and nothing to add to O, the second one (block 0,
// kNoPV) nothing to add to O yet (P_{-1} is zero). (The last iteration, whose block is the trailing dummy, stays
// whole: a second way out of the loop's iterations makes the compiler copy the 64 accumulators of O every time.)
enum { kAll = 0, kChainOnly = 1, kNoPV = 2 };
template <int PH, int PART, class Bk>
__device__ __forceinline__ void pipe_iter_seg(const unsigned char *__restrict__ lds, const bf16x8 (&qf)[8],
                                              f32x16 (&oacc)[4], const f32x16 &sA, f32x16 &sB,
                                              const unsigned (&pPrev)[8], unsigned (&pCur)[8], float &l_run,
                                              unsigned &seen, int &seen_full, int flags_next, int bits_addr, float c2,
                                              int kbase, int vbase, int hf, Bk &&bk) {
  int kaddr[8], vaddr[4];
#pragma unroll
  for (int c = 0; c < 8; ++c) kaddr[c] = kbase ^ (c << 5);
#pragma unroll
  for (int db = 0; db < 4; ++db) vaddr[db] = vbase ^ (db << 6);
  constexpr int KS = PH * kBlkBytes;                          // slot of K_{b+1}
  constexpr int VS = kVRing + ((PH + 2) & 3) * kBlkBytes;     // slot of V_{b-1}
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  bf16x8 kf[8];
  s16x8 vf[2][4];
  constexpr bool kChain = true, kWeights = PART != kChainOnly, kPV = PART == kAll;
  auto fetch = [&](int x) {
    if (kChain) kf[x] = lds_read_b128(lds, KS + kaddr[x]);
    if (kPV) {
      const int a2 = x >> 2, db = x & 3;
      const s16x4 r0 = lds_read_tr(lds, VS + vaddr[db] + (a2 * 16) * 256);
      const s16x4 r1 = lds_read_tr(lds, VS + vaddr[db] + (a2 * 16 + 8) * 256);
      vf[a2][db] = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
    }
  };
  // ---- the operands of the first four segments, and this row's mask word of the block
  const bool full_tile = (flags_next & 1) != 0;
  unsigned bits_next = 0xFFFFFFFFu;
  if (kChain && !full_tile) bits_next = *reinterpret_cast<const unsigned *>(lds + kBitsRing + PH * 1024 + bits_addr);
#pragma unroll
  for (int x = 0; x < 4; ++x) fetch(x);
  __builtin_amdgcn_sched_barrier(0);
  if (kChain) {
    if (full_tile) {
      seen_full = 1;
    } else {
      if (flags_next & 2) bits_next = 0u;  // dummy block: nothing kept
      seen |= bits_next;
    }
  }
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // no entry of this wave's 32 x 32 square is kept (wave-uniform): every logit is -inf without any product. (The
  // weights of such a square and its products with V stay: branches around them cost more than they save.)
  const bool skip_s = __builtin_amdgcn_ballot_w64(bits_next != 0u) == 0;
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    const int a2 = x >> 2, db = x & 3;
    // P_{b-1} V_{b-1}, step x (first: it needs no mask)
    if (kPV) {
      const u32x4 praw = {pPrev[4 * a2], pPrev[4 * a2 + 1], pPrev[4 * a2 + 2], pPrev[4 * a2 + 3]};
      oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[a2][db]),
                                                         __builtin_bit_cast(bf16x8, praw), oacc[db], 0, 0, 0);
    }
    // S_{b+1} chain, step x. Accumulator e is key 8 (e / 4) + 4 hf + e % 4 of the block and starts at 0 (kept)
    // or -inf (masked); a block whose 32 x 32 entries of this wave are all kept starts from a literal zero
    if (kChain) {
      if (x == 0) {
        if (__builtin_amdgcn_ballot_w64(bits_next != 0xFFFFFFFFu) == 0) {
          sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0], qf[0], zero, 0, 0, 0);
        } else if (skip_s) {
#pragma unroll
          for (int e = 0; e < 16; ++e) sB[e] = -INFINITY;
        } else {
          const int inv = (int)~(bits_next >> (4 * hf));
          mask_init(sB, inv, std::make_integer_sequence<int, 16>{});
          sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0], qf[0], sB, 0, 0, 0);
        }
      } else if (!skip_s) {
        sB = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[x], qf[x], sB, 0, 0, 0);
      }
    }
    if (x < 4) fetch(x + 4);
    // the weights of two entries of block b and their part of the row sum
    if (kWeights) {
      const float p0 = __builtin_amdgcn_exp2f(sA[2 * x] * c2);
      const float p1 = __builtin_amdgcn_exp2f(sA[2 * x + 1] * c2);
      pCur[x] = pack_bf16(p0, p1);
      l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pCur[x]), ones, l_run, false);
      asm volatile("" ::"v"(pCur[x]));
    }
    if (kChain) bk(std::integral_constant<int, 0>{} , x);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// RAGGED: the sequence length is not a multiple of the block size, so the last block of a row of tiles
// may reach past the end of K and V.
// GATHER: the block index may hold gathered column tiles (tile index >= nKt), whose K / V rows come from
// the per-head gathered copies.
// FAST: the softmax without a running maximum (see pipe_iter). Work items come from the eight queues; an item
// in which some row's sum of weights left the safe range is appended to the redo list (ctl[kRedoCount], then
// `redo`), and the FAST = false instantiation, launched behind this one, takes exactly those items and overwrites
// their rows. With well-scaled inputs the list stays empty.
template <bool RAGGED, bool GATHER, bool FAST>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_prefill_bf16_pipe(
    AttnArgs a, const __hip_bfloat16 *__restrict__ q, const __hip_bfloat16 *__restrict__ k,
    const __hip_bfloat16 *__restrict__ v, const int *__restrict__ row_ptr, const int *__restrict__ blk_col,
    const uint8_t *__restrict__ blk_kind, const uint64_t *__restrict__ tile_bits, __hip_bfloat16 *__restrict__ out,
    float *__restrict__ lse, int *__restrict__ ctl, int2 *__restrict__ redo, const __hip_bfloat16 *__restrict__ kgath,
    const __hip_bfloat16 *__restrict__ vgath) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  __shared__ int s_item[2];
  __shared__ int s_wsum[4];
  __shared__ int s_bad;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, hf = lane >> 5;
  const float c2 = a.scale * 1.4426950408889634f;
  if (!FAST && ctl[kRedoCount] == 0) return;  // nothing to redo (the usual case): leave before any set-up
  if (FAST && tid == 0) s_bad = 0;
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds;

  // LDS byte offsets of this lane's operand fragments inside a block (layout note above), chunk pair 0
  // and dim block 0; the others differ by an XOR
  const int kbase = n * 256 + ((hf ^ (n & 15)) << 4);
  const int vbase = (4 * hf + ((n & 15) >> 2)) * 256 + (((n & 15) >> 2) << 6) + 32 * (n >> 4) + 8 * (n & 3);
  // load-to-LDS copies of a block: instruction `it` (0, 1) of wave w fills rows 16 it + 4 w .. + 3; a
  // lane's byte offset from the block's first row is constant
  const int sub = lane >> 4, pos = lane & 15;
  const int row0 = wave * 4 + sub;
  const unsigned kss2 = (unsigned)a.k_ss * 2u, vss2 = (unsigned)a.v_ss * 2u;  // row strides in bytes
  const unsigned koff = (unsigned)row0 * kss2 + ((pos ^ (row0 & 15)) << 4);
  const unsigned voff = (unsigned)row0 * vss2 + ((pos ^ (sub << 2)) << 4);
  const unsigned boff = (unsigned)((wave * 32 + n) * 16);  // this lane's row in a tile's mask words
  const int bits_addr = wave * 256 + lane * 4;             // where its copy lands inside a bits slot
  const unsigned lds_kv = __builtin_amdgcn_readfirstlane(lds_base + wave * 1024);              // this wave's part of a K/V slot
  const unsigned lds_bits = __builtin_amdgcn_readfirstlane(lds_base + kBitsRing + wave * 256);  // ... of a bits slot

  // The first two iterations of an item multiply weights that are exactly zero (the leading dummy
  // blocks) with whatever the V ring holds: it has to be finite. Later items find the previous item's
  // V rows there; the first one would find what an earlier kernel left in LDS, so clear the ring once.
  for (int at = tid * 16; at < kRing * kBlkBytes; at += 256 * 16)
    *reinterpret_cast<uint4 *>(lds + kVRing + at) = make_uint4(0u, 0u, 0u, 0u);

  const int G = a.Hq / a.Hkv, n_pairs = a.B * a.Hkv, per_pair = G * a.nQt;
  const int my_xcd = __builtin_amdgcn_s_getreg((3 << 11) | 20) & (kXcd - 1);  // XCC_ID, 4 bits
  int hop = 0;
  int prev_item = -1, prev_queue = 0;  // (thread 0 only) the item just finished
  while (true) {
    __syncthreads();  // previous item: every wave is done with the LDS rings, with s_item and with s_bad
    if (tid == 0) {
      int item = -1, queue = 0;
      if (FAST) {
        if (s_bad) {  // some row of the previous item needs the running reference: hand the item over
          redo[atomicAdd(&ctl[kRedoCount], 1)] = make_int2(prev_item, prev_queue);
          s_bad = 0;
        }
        for (; hop < kXcd; ++hop) {
          queue = (my_xcd + hop) & (kXcd - 1);
          const int pairs_here = (n_pairs - queue + kXcd - 1) / kXcd;  // pairs p with p % 8 == queue
          const int got = atomicAdd(&ctl[queue], 1);
          if (got < pairs_here * per_pair) {
            item = got;
            break;
          }
        }
      } else {
        const int got = atomicAdd(&ctl[kRedoNext], 1);
        if (got < ctl[kRedoCount]) {  // (written by the kernel before this one)
          const int2 e = redo[got];
          item = e.x;
          queue = e.y;
        }
      }
      s_item[0] = item;
      s_item[1] = queue;
      prev_item = item;
      prev_queue = queue;
    }
    __syncthreads();
    const int item = __builtin_amdgcn_readfirstlane(s_item[0]), queue = __builtin_amdgcn_readfirstlane(s_item[1]);
    if (item < 0) break;
    const int pair = (item / per_pair) * kXcd + queue, within = item % per_pair;
    const int wb = pair / a.Hkv, whkv = pair % a.Hkv;
    const int wqt = a.nQt - 1 - within / G, whq = whkv * G + within % G;
    const int t0 = __builtin_amdgcn_readfirstlane(row_ptr[(int64_t)whq * (a.nQt + 1) + wqt]);
    const int t1 = __builtin_amdgcn_readfirstlane(row_ptr[(int64_t)whq * (a.nQt + 1) + wqt + 1]);
    const int qrow_l = wave * 32 + n;  // this lane's query row inside the tile
    const int qrow = wqt * kBM + qrow_l;
    const bool qlive = qrow < a.S;
    const unsigned char *kg = reinterpret_cast<const unsigned char *>(k + wb * a.k_sb + whkv * a.k_sh);
    const unsigned char *vg = reinterpret_cast<const unsigned char *>(v + wb * a.v_sb + whkv * a.v_sh);
    // the head's gathered column rows (tiles with index >= nKt): [gather_rows] rows at the row stride of K
    // (of V), so that a block of them is addressed exactly like a block of the cache
    const int64_t g_rows = ((int64_t)wb * a.Hq + whq) * a.gather_rows;
    const unsigned char *kgg = reinterpret_cast<const unsigned char *>(kgath) + g_rows * kss2;
    const unsigned char *vgg = reinterpret_cast<const unsigned char *>(vgath) + g_rows * vss2;

    // ---- the stream of occupied 32-key blocks of this query tile. The listed tiles are expanded, kSegTiles at
    // a time, into a list of block descriptors in LDS (two words: first key, and mask offset | flags << 28),
    // closed by a dummy entry that every read past the end returns. The pipeline then reads one descriptor per
    // iteration (fetched before the previous iteration's barrier, so that nothing waits for it) instead of
    // walking tiles and quarters in scalar code, which cost a sixth of the instructions of an iteration.
    uint2 *blk_list = reinterpret_cast<uint2 *>(lds + kBlkList);
    int n_blk = 0;      // entries of the current list before the dummy
    int cursor = 0;     // index of the descriptor held in pre_raw
    uint2 pre_raw = make_uint2(0u, 2u << 28);
    auto list_read = [&](int i) { return blk_list[min(i, n_blk)]; };  // the same address in every lane
    auto decode = [&](const uint2 &raw) {
      const int key0 = __builtin_amdgcn_readfirstlane((int)raw.x);
      const unsigned meta = (unsigned)__builtin_amdgcn_readfirstlane((int)raw.y);
      return Blk{key0, (int)(meta & 0x0FFFFFFFu), (int)(meta >> 28)};
    };
    // tiles [seg0, seg0 + n_seg) -> list; called by the whole workgroup, ends with a barrier
    auto expand = [&](int seg0, int n_seg) {
      int quarters = 0, col = 0, full = 0;
      if (tid < n_seg) {
        const int kind = blk_kind[seg0 + tid];
        // a column outside the index's range (a list that was never filled) is pulled inside it: the result is
        // then wrong, but every address formed from it stays within the head's rows
        col = min(max(blk_col[seg0 + tid], 0), a.nKt + (GATHER ? a.gather_rows / kBN : 0) - 1);
        quarters = (kind >> 1) & 15;
        full = kind & 1;
      }
      const int cnt = __popc(quarters);
      int incl = cnt;
      for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
      }
      if (lane == 63) s_wsum[wave] = incl;  // kSegTiles = 128: only waves 0 and 1 hold tiles
      __syncthreads();
      int at = incl - cnt + (wave == 1 ? s_wsum[0] : 0);
      while (quarters) {
        const int qq = __builtin_ctz(quarters);
        quarters &= quarters - 1;
        const bool gth = GATHER && col >= a.nKt;  // gathered tile: rows of the head's gathered copy (flag 4)
        const int key0 = gth ? min((col - a.nKt) * kBN + kBlkKeys * qq, a.gather_rows - kBlkKeys) : col * kBN + kBlkKeys * qq;
        const unsigned off_bits = (unsigned)((seg0 + tid - t0) * (kBM * 16) + 4 * qq);
        blk_list[at++] = make_uint2((unsigned)key0, off_bits | (unsigned)(full | (gth ? 4 : 0)) << 28);
      }
      const int total = s_wsum[0] + s_wsum[1];
      if (tid == 0) blk_list[total] = make_uint2(0u, 2u << 28);  // dummy: key 0, the item's first mask words, nothing kept
      __syncthreads();
      n_blk = __builtin_amdgcn_readfirstlane(total);
    };
    // K or V block -> ring slot: two 1 KiB copies per wave; every address is the head's base plus a
    // 32-bit byte offset (the host checks that a head's rows span less than 4 GiB). In the ragged case
    // a block that reaches past the sequence end redirects such keys (masked anyway) to the last row,
    // which keeps the slot finite.
    auto copy_blk = [&](auto slot_off, const unsigned char *g, unsigned stride2, unsigned lane_off, int chunk_xor, int key0,
                        unsigned blk_off, bool gathered) {
      constexpr int SO = decltype(slot_off)::value;
      if (!RAGGED || gathered || key0 + kBlkKeys <= a.S) {
        const unsigned o0 = lane_off + blk_off;
        lds_copy16<SO>(lds_kv, g, o0);
        lds_copy16<SO + 4096>(lds_kv, g, o0 + 16u * stride2);
      } else {
        const unsigned c = (unsigned)((pos ^ chunk_xor) << 4);
        lds_copy16<SO>(lds_kv, g, (unsigned)min(key0 + row0, a.S - 1) * stride2 + c);
        lds_copy16<SO + 4096>(lds_kv, g, (unsigned)min(key0 + 16 + row0, a.S - 1) * stride2 + c);
      }
    };
    auto copy_k = [&](const Blk &d, auto slot) {
      const bool gth = GATHER && (d.flags & 4) != 0;  // wave-uniform
      copy_blk(std::integral_constant<int, decltype(slot)::value * kBlkBytes>{}, gth ? kgg : kg, kss2, koff, row0 & 15, d.key0,
               (unsigned)d.key0 * kss2, gth);
    };
    auto copy_v = [&](const Blk &d, auto slot) {
      const bool gth = GATHER && (d.flags & 4) != 0;
      copy_blk(std::integral_constant<int, kVRing + decltype(slot)::value * kBlkBytes>{}, gth ? vgg : vg, vss2, voff, sub << 2, d.key0,
               (unsigned)d.key0 * vss2, gth);
    };
    // the block's mask word of every row of this wave (also issued for full and dummy blocks, so that
    // every iteration has the same number of copies in flight)
    const unsigned char *bits_row = reinterpret_cast<const unsigned char *>(tile_bits) + (int64_t)t0 * (kBM * 16);
    auto copy_bits = [&](const Blk &d, auto slot) {
      lds_copy4<decltype(slot)::value * 1024>(lds_bits, bits_row, boff + (unsigned)d.bits_off);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;

    // block i of the stream is described by d[i & 3]
    Blk d[4] = {};
    f32x16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[db][e] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;  // running max (raw logits) and this lane's part of the row sum
    unsigned seen = 0u;                     // FAST: union of the mask words of this lane's row, and whether a full
    int seen_full = 0;                      // tile was met: together "the row has a kept entry"

    if (t1 > t0) {
      // Q fragments: B operand of S^T = K Q^T. Chunk c covers dims 16c .. 16c+15; this lane holds dims
      // 16c + 8 hf .. + 7 of its query row.
      bf16x8 qf[8];
      {
        const __hip_bfloat16 *qp = q + wb * a.q_sb + whq * a.q_sh + (int64_t)qrow * a.q_ss + 8 * hf;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          u32x4 raw = {0u, 0u, 0u, 0u};
          if (qlive) raw = *reinterpret_cast<const u32x4 *>(qp + 16 * c);
          qf[c] = __builtin_bit_cast(bf16x8, raw);
        }
      }
      // one pass of the pipeline per segment of kSegTiles listed tiles (a query tile of c3 has at most 32;
      // the accumulators, the softmax state and the Q fragments carry over)
      for (int seg0 = t0; seg0 < t1; seg0 += kSegTiles) {
        if (seg0 > t0) __syncthreads();  // every wave is done with the previous list and with the rings
        expand(seg0, min(kSegTiles, t1 - seg0));
        d[0] = decode(list_read(0));
        d[1] = decode(list_read(1));
        d[2] = decode(list_read(2));
        cursor = 3;
        pre_raw = list_read(cursor);
        copy_k(d[0], I0{});
        copy_bits(d[0], I0{});
        copy_k(d[1], I1{});
        copy_bits(d[1], I1{});
        copy_k(d[2], I2{});
        copy_bits(d[2], I2{});
        copy_v(d[0], I0{});
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        // the Q fragments have arrived with that wait; passing them through an empty statement tells the
        // compiler so (it cannot see the wait, and would otherwise wait for every copy in flight at the
        // first use of a fragment in each iteration)
#pragma unroll
        for (int c = 0; c < 8; ++c) asm volatile("" : "+v"(qf[c]));
        __syncthreads();
        // S_b lives in sbuf[PH & 1] and S_{b+1} is written to the other one; P_b goes to pbuf[PH & 1] and
        // P_{b-1} is read from the other one, so nothing is copied between iterations
        f32x16 sbuf[2];
        unsigned pbuf[2][8];
#pragma unroll
        for (int e = 0; e < 16; ++e) sbuf[0][e] = -INFINITY;  // block -1 is a dummy
#pragma unroll
        for (int e = 0; e < 8; ++e) pbuf[1][e] = 0u;
        d[3].flags = 0;  // stands for block -1: the leading dummy must not end the loop
        // iteration b with (b + 1) % 4 == PH; returns true when the stream is finished
        auto step = [&](auto ph, auto partc) {
          constexpr int PH = decltype(ph)::value, PART = decltype(partc)::value;
          const int flag_cur = d[(PH + 3) & 3].flags;  // block b, whose descriptor is replaced now
          if constexpr (FAST) {

            // the bookkeeping of this iteration, dealt out over the segments of the product stream: the copies
            // only behind the last operand reads (segments 0 .. 3 issue those of segments 4 .. 7)
            auto bk = [&](auto, int x) {
              if (x == 2) d[(PH + 3) & 3] = decode(pre_raw);           // block b+4
              if (x == 4) copy_k(d[(PH + 3) & 3], std::integral_constant<int, (PH + 3) & 3>{});  // five copies per wave and iteration, always
              if (x == 5) copy_bits(d[(PH + 3) & 3], std::integral_constant<int, (PH + 3) & 3>{});
              if (x == 6) copy_v(d[(PH + 1) & 3], std::integral_constant<int, (PH + 1) & 3>{});  // block b+2
              if (x == 7) pre_raw = list_read(++cursor);               // block b+5 (a read past the list returns its dummy)
            };
            pipe_iter_seg<PH, PART>(lds, qf, oacc, sbuf[PH & 1], sbuf[(PH + 1) & 1], pbuf[(PH + 1) & 1], pbuf[PH & 1], l_run,
                                    seen, seen_full, d[PH].flags, bits_addr, c2, kbase, vbase, hf, bk);
            if (flag_cur & 2) return true;      // block b was the trailing dummy: P_{b-1} V_{b-1} is in
          } else {
            d[(PH + 3) & 3] = decode(pre_raw);           // block b+4
            copy_k(d[(PH + 3) & 3], std::integral_constant<int, (PH + 3) & 3>{});  // five copies per wave and iteration, always
            copy_bits(d[(PH + 3) & 3], std::integral_constant<int, (PH + 3) & 3>{});
            copy_v(d[(PH + 1) & 3], std::integral_constant<int, (PH + 1) & 3>{});  // block b+2
            pipe_iter<PH, FAST>(lds, qf, oacc, sbuf[PH & 1], sbuf[(PH + 1) & 1], pbuf[(PH + 1) & 1], pbuf[PH & 1], m_run,
                                l_run, seen, seen_full, d[PH].flags, bits_addr, c2, kbase, vbase, hf);
            if (flag_cur & 2) return true;      // block b was the trailing dummy: P_{b-1} V_{b-1} is in
            pre_raw = list_read(++cursor);      // block b+5, decoded at the start of the next iteration
          }
          // K_{b+2}, its mask words and V_b (issued two iterations ago) must have landed; the ten
          // youngest copies (this iteration's and the previous one's) may stay in flight
          // (wait and barrier as one statement: the library barrier would add a fence that waits for
          // everything in flight; the LDS rings are only written by the copies counted here)
          asm volatile("s_waitcnt vmcnt(10)\n\ts_barrier" ::: "memory");
          return false;
        };
        using PAll = std::integral_constant<int, kAll>;
        // block -1 (nothing to weigh, nothing to add) and block 0 (nothing to add yet) in front of the loop,
        // which therefore starts at phase 2
        if (!step(I0{}, std::integral_constant<int, FAST ? kChainOnly : kAll>{}) &&
            !step(I1{}, std::integral_constant<int, FAST ? kNoPV : kAll>{})) {
          while (true) {
            if (step(I2{}, PAll{})) break;
            if (step(I3{}, PAll{})) break;
            if (step(I0{}, PAll{})) break;
            if (step(I1{}, PAll{})) break;
          }
        }
      }
    }

    // finish: total sum over both half-waves, normalise, store. Accumulator e of block db is dim
    // 32 db + 8 (e / 4) + 4 hf + e % 4 of this lane's query.
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    if (FAST) {
      // a row with a kept entry whose sum of weights is zero, tiny, huge, infinite or NaN: its logits lie outside
      // what exp2 without a reference can carry (|logit * log2 e| of the order of 100)
      const bool bad = qlive && (seen != 0u || seen_full) && !(l_tot >= 0x1p-100f && l_tot <= 0x1p100f);
      if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) s_bad = 1;  // read by thread 0 after the loop's barrier
    }
    if (qlive) {
      __hip_bfloat16 *op = out + wb * a.o_sb + whq * a.o_sh + (int64_t)qrow * a.o_ss;
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
        lse[((int64_t)wb * a.Hq + whq) * a.S + qrow] =
            l_tot > 0.0f ? ((FAST ? 0.0f : m_run * c2) + log2f(l_tot)) * 0.6931471805599453f : -INFINITY;
    }
  }  // next work item
}

// Copies of the K and V rows of every head's matched columns (gather_idx, -1 = empty slot -> zeros) as
// [batch][hq][gather_rows] rows at the row stride of K (of V), so that a gathered tile is loaded like any other.
__global__ __launch_bounds__(256) void k_gather_kv(AttnArgs a, const __hip_bfloat16 *__restrict__ k,
                                                   const __hip_bfloat16 *__restrict__ v, const int *__restrict__ gather_idx,
                                                   __hip_bfloat16 *__restrict__ kgath, __hip_bfloat16 *__restrict__ vgath,
                                                   int *__restrict__ queue_next) {
  // (also resets the work queues of the attention kernel that follows: one launch less per call)
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < kCtlWords) queue_next[threadIdx.x] = 0;
  const int bh = blockIdx.y, b = bh / a.Hq, hq = bh % a.Hq, hkv = hq / (a.Hq / a.Hkv);
  const int s = blockIdx.x * 16 + (threadIdx.x >> 4), chunk = threadIdx.x & 15;
  if (s >= a.gather_rows) return;
  const int c = s < a.gather_stride ? gather_idx[(int64_t)hq * a.gather_stride + s] : -1;
  uint4 kv = make_uint4(0u, 0u, 0u, 0u), vv = kv;
  if (c >= 0 && c < a.S) {
    kv = *reinterpret_cast<const uint4 *>(k + b * a.k_sb + hkv * a.k_sh + (int64_t)c * a.k_ss + chunk * 8);
    vv = *reinterpret_cast<const uint4 *>(v + b * a.v_sb + hkv * a.v_sh + (int64_t)c * a.v_ss + chunk * 8);
  }
  const int64_t row = (int64_t)bh * a.gather_rows + s;
  *reinterpret_cast<uint4 *>(kgath + row * a.k_ss + chunk * 8) = kv;
  *reinterpret_cast<uint4 *>(vgath + row * a.v_ss + chunk * 8) = vv;
}

__global__ void k_zero_queues(int *queue_next) {
  if (threadIdx.x < kCtlWords) queue_next[threadIdx.x] = 0;
}

// Every work item onto the redo list, in the order the queues would hand them out (DAM_ATTN_RUNNING_REFERENCE:
// the caller asks for the variant with a running reference from the start).
__global__ void k_list_all_items(AttnArgs a, int *__restrict__ ctl, int2 *__restrict__ redo) {
  const int n_pairs = a.B * a.Hkv, per_pair = (a.Hq / a.Hkv) * a.nQt;
  const int rounds = (n_pairs + kXcd - 1) / kXcd * per_pair;
  int n_q[kXcd], total = 0;
  for (int x = 0; x < kXcd; ++x) {
    n_q[x] = (n_pairs - x + kXcd - 1) / kXcd * per_pair;  // items of queue x
    total += n_q[x];
  }
  for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < rounds * kXcd; e += gridDim.x * blockDim.x) {
    const int queue = e % kXcd, item = e / kXcd;
    if (item >= n_q[queue]) continue;
    int at = 0;  // valid entries before (item, queue) in round-robin order
    for (int x = 0; x < kXcd; ++x) at += min(n_q[x], item + (x < queue ? 1 : 0));
    redo[at] = make_int2(item, queue);
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) ctl[kRedoCount] = total;
}

int validate(const dam_attn_params *p, const void *q, const void *k, const void *v, const dam_mask_view *mk,
             const void *out) {
  if (!p || !q || !k || !v || !mk || !out) return DAM_ERR_INVALID_ARG;
  if (!mk->blk_row_ptr || !mk->blk_col || !mk->blk_kind || !mk->tile_bits) return DAM_ERR_INVALID_ARG;
  if (p->batch < 1 || p->hq < 1 || p->hkv < 1 || p->hq % p->hkv || p->seq < 1) return DAM_ERR_INVALID_ARG;
  if (p->tile_m < 64 || p->tile_n < 64 || p->tile_m % 64 || p->tile_n % 64) return DAM_ERR_INVALID_ARG;
  if (mk->gather_idx) {  // gathered column tiles (checked after the tile sizes: the test divides by tile_n)
    if (!mk->gather_cnt || mk->gather_stride < 1 || p->gather_rows < 0 || p->gather_rows % p->tile_n ||
        p->gather_rows > mk->gather_stride)
      return DAM_ERR_INVALID_ARG;
  } else if (p->gather_rows != 0) {
    return DAM_ERR_INVALID_ARG;
  }
  if (!(p->scale >= 0.0f)) return DAM_ERR_INVALID_ARG;
  if (p->flags & ~DAM_ATTN_RUNNING_REFERENCE) return DAM_ERR_INVALID_ARG;
  const int align = p->dtype == DAM_BF16 ? 8 : 4;
  const int64_t *sets[4] = {p->q_stride, p->k_stride, p->v_stride, p->o_stride};
  for (auto s : sets)
    for (int x = 0; x < 3; ++x)
      if (s[x] < 0 || s[x] % align) return DAM_ERR_INVALID_ARG;
  if (p->dtype == DAM_BF16) {
    if (p->head_dim != 128 || p->tile_m != 128 || p->tile_n != 128) return DAM_ERR_UNSUPPORTED;
    // the bf16 kernel addresses the rows of one K or V head with 32-bit byte offsets
    if ((int64_t)p->seq * p->k_stride[2] * 2 >= (int64_t(1) << 32) || (int64_t)p->seq * p->v_stride[2] * 2 >= (int64_t(1) << 32))
      return DAM_ERR_UNSUPPORTED;
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
  a.nKt = (p->seq + p->tile_n - 1) / p->tile_n;
  a.gather_rows = 0;
  a.gather_stride = 0;
  a.wpr = p->tile_n / 64;
  a.scale = p->scale > 0.0f ? p->scale : 1.0f / sqrtf((float)p->head_dim);
  a.q_sb = p->q_stride[0]; a.q_sh = p->q_stride[1]; a.q_ss = p->q_stride[2];
  a.k_sb = p->k_stride[0]; a.k_sh = p->k_stride[1]; a.k_ss = p->k_stride[2];
  a.v_sb = p->v_stride[0]; a.v_sh = p->v_stride[1]; a.v_ss = p->v_stride[2];
  a.o_sb = p->o_stride[0]; a.o_sh = p->o_stride[1]; a.o_ss = p->o_stride[2];
  return a;
}

}  // namespace

// bytes of the redo list: an int2 per (batch, query head, query tile), rounded up to 256
static size_t redo_bytes(const dam_attn_params *p) {
  const size_t items = (size_t)p->batch * p->hq * (size_t)((p->seq + p->tile_m - 1) / p->tile_m);
  return (items * sizeof(int2) + 255) / 256 * 256;
}

extern "C" size_t dam_sparse_attn_prefill_workspace(const dam_attn_params *p) {
  if (!p || p->batch < 1 || p->hkv < 1 || p->hq < 1 || p->seq < 1 || p->gather_rows < 0) return 0;
  if (p->dtype != DAM_BF16) return 0;
  if (p->hq % p->hkv || p->tile_m < 64) return 0;
  // the control words of the bf16 kernel (queue counters, redo list length and cursor), the redo list (one entry per
  // work item at most), then the gathered K and V copies (rows at the caches' strides)
  return kCtlBytes + redo_bytes(p) +
         (size_t)p->batch * p->hq * p->gather_rows * (size_t)(p->k_stride[2] + p->v_stride[2]) * sizeof(__hip_bfloat16);
}

extern "C" int dam_sparse_attn_prefill(const dam_attn_params *p, const void *q, const void *k, const void *v,
                                       const dam_mask_view *mk, void *out, float *lse, void *ws, size_t ws_bytes,
                                       void *stream_v) {
  const int bad = validate(p, q, k, v, mk, out);
  if (bad != DAM_OK) return bad;
  const size_t need = dam_sparse_attn_prefill_workspace(p);
  if (need && (!ws || ws_bytes < need)) return DAM_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream_v);
  AttnArgs a = make_args(p);
  if (mk->gather_idx) {
    a.gather_rows = p->gather_rows;
    a.gather_stride = mk->gather_stride;
  }
  const int blocks = work_blocks(a);
  if (p->dtype == DAM_F32) {
    // (passes of a query tile as separate workgroups while the launch stays small)
    const int rows_per_pass = 256 / (p->head_dim / 4), passes = (p->tile_m + rows_per_pass - 1) / rows_per_pass;
    const int spread = blocks * passes <= 16384 ? passes : 1;
    if (p->head_dim == 64)
      k_prefill_f32<64><<<dim3(blocks, spread), 256, 0, st>>>(a, (const float *)q, (const float *)k, (const float *)v, mk->blk_row_ptr,
                                               mk->blk_col, mk->blk_kind, mk->tile_bits, mk->gather_idx, (float *)out, lse);
    else
      k_prefill_f32<128><<<dim3(blocks, spread), 256, 0, st>>>(a, (const float *)q, (const float *)k, (const float *)v, mk->blk_row_ptr,
                                                mk->blk_col, mk->blk_kind, mk->tile_bits, mk->gather_idx, (float *)out, lse);
    return launch_status();
  }
  // (queried per call: the library keeps no state, and the device may differ from call to call)
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
    return DAM_ERR_DEVICE;
  int *ctl = static_cast<int *>(ws);
  int2 *redo = reinterpret_cast<int2 *>(static_cast<char *>(ws) + kCtlBytes);
  __hip_bfloat16 *kgath = reinterpret_cast<__hip_bfloat16 *>(static_cast<char *>(ws) + kCtlBytes + redo_bytes(p));
  __hip_bfloat16 *vgath = kgath + (size_t)p->batch * p->hq * a.gather_rows * (size_t)a.k_ss;
  if (a.gather_rows > 0)
    k_gather_kv<<<dim3((a.gather_rows + 15) / 16, p->batch * p->hq), 256, 0, st>>>(
        a, (const __hip_bfloat16 *)k, (const __hip_bfloat16 *)v, mk->gather_idx,
        kgath, vgath, ctl);
  else
    k_zero_queues<<<1, 64, 0, st>>>(ctl);
  const int persistent = std::min(blocks, 2 * n_cu);  // two workgroups fit a CU (registers and LDS)
  const bool ragged = p->seq % kBlkKeys != 0, gather = a.gather_rows > 0;
  using Kernel = void (*)(AttnArgs, const __hip_bfloat16 *, const __hip_bfloat16 *, const __hip_bfloat16 *, const int *,
                          const int *, const uint8_t *, const uint64_t *, __hip_bfloat16 *, float *, int *, int2 *,
                          const __hip_bfloat16 *, const __hip_bfloat16 *);
  static const Kernel kernels[2][4] = {
      {k_prefill_bf16_pipe<false, false, false>, k_prefill_bf16_pipe<true, false, false>,
       k_prefill_bf16_pipe<false, true, false>, k_prefill_bf16_pipe<true, true, false>},
      {k_prefill_bf16_pipe<false, false, true>, k_prefill_bf16_pipe<true, false, true>,
       k_prefill_bf16_pipe<false, true, true>, k_prefill_bf16_pipe<true, true, true>}};
  const int which = (ragged ? 1 : 0) + (gather ? 2 : 0);
  const bool reference_only = (p->flags & DAM_ATTN_RUNNING_REFERENCE) != 0;
  // first the softmax without a running maximum over every work item; then the variant with one over the items
  // the first pass put on the redo list (none for well-scaled inputs: its workgroups then leave at once)
  for (int fast = 1; fast >= 0; --fast) {
    // (idempotent; set on every call rather than remembered in a static)
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernels[fast][which]), hipFuncAttributeMaxDynamicSharedMemorySize,
                            kPipeLds) != hipSuccess)
      return DAM_ERR_DEVICE;
    if (fast && reference_only) {
      k_list_all_items<<<std::min((blocks + 255) / 256, 256), 256, 0, st>>>(a, ctl, redo);
      continue;
    }
    kernels[fast][which]<<<persistent, 256, kPipeLds, st>>>(a, (const __hip_bfloat16 *)q, (const __hip_bfloat16 *)k,
                                                            (const __hip_bfloat16 *)v, mk->blk_row_ptr, mk->blk_col,
                                                            mk->blk_kind, mk->tile_bits, (__hip_bfloat16 *)out, lse, ctl,
                                                            redo, kgath, vgath);
  }
  return launch_status();
}

extern "C" int dam_version(void) { return 1; }
