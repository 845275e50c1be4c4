// Grouped-query decode on the matrix cores (bf16, head_dim 128): the partial pass of
// dam_sparse_attn_decode_grouped for the common case.
//
// Paper (arXiv 2506.11104): Sec. 3 (scaled dot-product attention) with the mask of Sec. 4.3 applied
// as -inf before the softmax; the merged kept list is row p of the masks of a KV head's query heads.
//
// The path is HBM-bound (one 256-byte K row and one V row per listed key), but on the plain ALUs the
// arithmetic of G heads per row (dot products reduced across lanes, exponentials and weighted sums
// replicated over the lanes that share a row) took as long as the gather itself and overlapped with
// it only in part. Here the G query vectors of a (sequence, KV head) pair are the columns of the B
// operand of S^T = K Q^T (32 keys x 32 columns, G of them live) and of O^T += V^T P^T, exactly the
// products of the prefill kernel with the query heads in the place of query rows, so the arithmetic
// of a 32-key block shrinks to 16 matrix instructions and a 16-value softmax per lane.
//
// No barrier inside the loop: a wave owns every splits-th block of 32 list entries and two
// LDS slots of K and V rows (8 KiB each), filled by load-to-LDS copies whose row addresses come from
// the list. The entries themselves (key indices and member bits) are staged in LDS by the same kind
// of copy three blocks ahead, so that every vector-memory operation of the loop is one of these
// copies and the waits can be counted by hand. While block i is computed the copies of block i + 1
// are in flight; those of block i + 2 are issued as soon as block i has left its slot. Four waves
// per CU (LDS), each with 16 to 32 KiB in flight. The splits of a list are the waves of one workgroup
// when there are at most four (the workgroup merges them and stores the output), else workgroups of
// one wave each whose partial results go through the merge kernel.
#include <math.h>

#include "dam_internal.h"
#include "dam_mfma.h"

namespace {
using namespace dam;

constexpr int kBlk = 32;                   // keys per block
constexpr int kSlot = kBlk * 256;          // bytes of the K (or V) rows of a block
constexpr int kVSlots = 2 * kSlot;         // two K slots, then two V slots
constexpr int kEntries = 4 * kSlot;        // then four 256-byte slots of list entries
constexpr int kFix = kEntries + 4 * 256;   // PLAN: four 256-byte slots of plan-table words
constexpr int kLds = kFix + 4 * 256;

struct MfmaArgs {
  int B, Hq, Hkv, cap, splits, shared_lists;
  int fused;  // the splits of a list are the waves of one workgroup, which merges them itself and stores the result
  float scale;
  int64_t q_sb, q_sh, kv_sb, kv_sh, o_sb, o_sh;
  unsigned row_bytes;  // byte stride of a cache row
  int pos, n_flags;    // PLAN: position of the query row, length P of the pattern flags
};

// Four bytes per lane from a 64-bit address of the lane's own to LDS address lds_at + 4 * lane.
__device__ __forceinline__ void lds_copy4_at(unsigned lds_at, uint64_t addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" : : "s"(lds_at), "v"(addr) : "memory", "m0");
}

// (The register budget of two waves per SIMD, although LDS admits one: with all 512 registers on offer the
// compiler keeps the O accumulators in the accumulation registers for the products and in vector registers for
// the occasional rescaling, and moves all 64 of them both ways in every iteration.)
//
// PLAN: the list is a position-independent plan of a pattern mask (DAM_MASK_PATTERN_PLAN): an entry v < 0 is the
// diagonal -1 - v and stands for key pos + 1 + v, an entry v >= 0 is column v. A column entry serves the heads
// in member & ~table[pos - v] (the others reach that key through their diagonal already), and no head when the
// key does not exist yet (v > pos; a diagonal beyond pos likewise). The table byte of every column entry of a
// block is fetched into LDS by one more copy per block, issued as soon as the block's entries have landed, two
// blocks before its use, so that the loop still holds nothing but hand-counted copies.
//
// Up to four splits: they are the waves of one workgroup (each with LDS slots of its own; still no barrier inside the
// loop), and at the end wave 0 merges the partial results through LDS, normalises and stores the output: no merge
// launch. More splits: one wave per workgroup, partial results to the workspace for the merge kernel.
template <bool PLAN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_decode_group_mfma(
    MfmaArgs a, const __hip_bfloat16 *__restrict__ q, const __hip_bfloat16 *__restrict__ kc,
    const __hip_bfloat16 *__restrict__ vc, const int *__restrict__ kept_ptr, const int *__restrict__ kept_idx,
    const uint8_t *__restrict__ kept_member, const uint8_t *__restrict__ plan_table, float *__restrict__ part_o,
    float *__restrict__ part_ml, __hip_bfloat16 *__restrict__ out, float *__restrict__ lse) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_all[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  unsigned char *lds = lds_all + wave * kLds;  // this wave's slots
  const int n = lane & 31, hf = lane >> 5;     // column of the products (query head of the group), half-wave
  const int sub = lane >> 4, pos = lane & 15;  // copies: row within the instruction's four, 16-byte position
  const int G = a.Hq / a.Hkv;
  const int split = a.fused ? wave : (int)blockIdx.x % a.splits, pair = a.fused ? (int)blockIdx.x : (int)blockIdx.x / a.splits;
  const int b = pair / a.Hkv, hkv = pair % a.Hkv;
  const int list = a.shared_lists ? hkv : pair;
  const int lo = __builtin_amdgcn_readfirstlane(kept_ptr[list]), end = __builtin_amdgcn_readfirstlane(kept_ptr[list + 1]);
  const int n_blocks = (end - lo + kBlk - 1) / kBlk;
  // this wave's blocks are split, split + splits, ...: every wave gets its share of each run of the list
  const int nb = n_blocks > split ? (n_blocks - split + a.splits - 1) / a.splits : 0;
  const float c2 = a.scale * 1.4426950408889634f;
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds;

  f32x16 oacc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[db][e] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;  // reference of the weights (raw logits), this lane's part of their sum

  if (nb > 0) {
    const unsigned char *kg = reinterpret_cast<const unsigned char *>(kc + b * a.kv_sb + hkv * a.kv_sh);
    const unsigned char *vg = reinterpret_cast<const unsigned char *>(vc + b * a.kv_sb + hkv * a.kv_sh);
    const uint64_t idx_at = reinterpret_cast<uint64_t>(kept_idx), member_at = reinterpret_cast<uint64_t>(kept_member);
    auto entry0 = [&](int i) { return lo + (split + i * a.splits) * kBlk; };
    // Entries of local block i -> entry slot i & 3: lanes 0..31 fetch the key indices, lanes 32..40 the nine
    // aligned words that hold the block's 32 member bytes (the other lanes repeat the ninth). Entries past the
    // end of the list repeat its last one; their keys are masked below. An aligned word that holds a byte of
    // the array lies inside that byte's page, so the words at the array's two ends are safe to read.
    auto copy_entries = [&](int i) {
      const int e0 = entry0(i);
      const uint64_t first = (member_at + (unsigned)e0) & ~(uint64_t)3, last = (member_at + (unsigned)(end - 1)) & ~(uint64_t)3;
      const uint64_t addr = lane < 32 ? idx_at + 4ull * (unsigned)min(e0 + lane, end - 1)
                                      : min(first + 4u * (unsigned)min(lane - 32, 8), last);
      lds_copy4_at(__builtin_amdgcn_readfirstlane(lds_base + kEntries + (i & 3) * 256), addr);
    };
    // PLAN: the aligned word that holds table[pos - c] for every column entry c of local block i (its entries have
    // landed) -> fix slot i & 3, lane k < 32 for entry k; every other lane and entry fetches the table's first word
    const uint64_t table_at = reinterpret_cast<uint64_t>(plan_table) + (uint64_t)hkv * (unsigned)a.n_flags;
    auto table_index = [&](int v) { return (v >= 0 && v <= a.pos && a.pos - v < a.n_flags) ? a.pos - v : -1; };
    // (a block without a column entry needs no table word and issues no copy: the copy, when there is one, is older
    // than the block's sixteen row copies, which are all the waits below leave outstanding)
    auto copy_fix = [&](int i) {
      const unsigned char *entries = lds + kEntries + (i & 3) * 256;
      const int v = *reinterpret_cast<const int *>(entries + 4 * (lane & 31));
      const int t = lane < 32 ? table_index(v) : -1;
      if (__builtin_amdgcn_ballot_w64(t >= 0) == 0) return;
      const uint64_t addr = t >= 0 ? (table_at + (unsigned)t) & ~(uint64_t)3 : reinterpret_cast<uint64_t>(plan_table) & ~(uint64_t)3;
      lds_copy4_at(__builtin_amdgcn_readfirstlane(lds_base + kFix + (i & 3) * 256), addr);
    };
    // K and V rows of local block i -> slot i & 1: eight copies each; copy `it` moves rows 4 it .. 4 it + 3 of the
    // block, lane (sub, pos) the 16 bytes that belong at position pos of row 4 it + sub (the chunk permutations of
    // the prefill kernel: K chunk c of row r at position c ^ (r & 15), V chunk c at c ^ ((r & 3) << 2)).
    auto copy_rows = [&](int i) {
      const unsigned char *entries = lds + kEntries + (i & 3) * 256;
      const unsigned k_at = __builtin_amdgcn_readfirstlane(lds_base + (i & 1) * kSlot);
      const unsigned v_at = k_at + kVSlots;
      unsigned koff[8], voff[8];
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int r = 4 * it + sub;
        // (an index outside the cache is pulled to its nearest row: no address leaves the cache)
        int v = *reinterpret_cast<const int *>(entries + 4 * r);
        if (PLAN && v < 0) v += a.pos + 1;  // diagonal -1 - v: key pos - r
        // (PLAN: a pattern whose key does not exist yet is masked below; its row is taken from the keys that do, since
        // rows beyond the position may hold anything, and a NaN there would survive a zero weight)
        const int key = min(max(v, 0), PLAN ? min(a.pos, a.cap - 1) : a.cap - 1);
        // (row index and row stride are below 2^24: the 24-bit multiply runs at full rate, the 32-bit one does not)
        const unsigned row_at = __umul24((unsigned)key, a.row_bytes);
        koff[it] = row_at + ((pos ^ (r & 15)) << 4);
        voff[it] = row_at + ((pos ^ (sub << 2)) << 4);
      }
      lds_copy16_once<0 * 1024>(k_at, kg, koff[0]);
      lds_copy16_once<1 * 1024>(k_at, kg, koff[1]);
      lds_copy16_once<2 * 1024>(k_at, kg, koff[2]);
      lds_copy16_once<3 * 1024>(k_at, kg, koff[3]);
      lds_copy16_once<4 * 1024>(k_at, kg, koff[4]);
      lds_copy16_once<5 * 1024>(k_at, kg, koff[5]);
      lds_copy16_once<6 * 1024>(k_at, kg, koff[6]);
      lds_copy16_once<7 * 1024>(k_at, kg, koff[7]);
      lds_copy16_once<0 * 1024>(v_at, vg, voff[0]);
      lds_copy16_once<1 * 1024>(v_at, vg, voff[1]);
      lds_copy16_once<2 * 1024>(v_at, vg, voff[2]);
      lds_copy16_once<3 * 1024>(v_at, vg, voff[3]);
      lds_copy16_once<4 * 1024>(v_at, vg, voff[4]);
      lds_copy16_once<5 * 1024>(v_at, vg, voff[5]);
      lds_copy16_once<6 * 1024>(v_at, vg, voff[6]);
      lds_copy16_once<7 * 1024>(v_at, vg, voff[7]);
    };

    // Q fragments: B operand of S^T = K Q^T. Column n is query head n of the group (zero beyond the group);
    // chunk c covers dims 16 c .. 16 c + 15, this lane holds dims 16 c + 8 hf .. + 7.
    bf16x8 qf[8];
    {
      const __hip_bfloat16 *qp = q + b * a.q_sb + (int64_t)(hkv * G + min(n, G - 1)) * a.q_sh + 8 * hf;
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        u32x4 raw = {0u, 0u, 0u, 0u};
        if (n < G) raw = *reinterpret_cast<const u32x4 *>(qp + 16 * c);
        qf[c] = __builtin_bit_cast(bf16x8, raw);
      }
    }
    copy_entries(0);
    if (nb > 1) copy_entries(1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // (the Q fragments have arrived with that wait; the empty statement tells the compiler so)
#pragma unroll
    for (int c = 0; c < 8; ++c) asm volatile("" : "+v"(qf[c]));
    if (PLAN) {
      copy_fix(0);
      if (nb > 1) copy_fix(1);
    }
    if (nb > 2) copy_entries(2);
    copy_rows(0);
    if (nb > 1) copy_rows(1);

    // LDS byte offsets of this lane's operand fragments inside a slot (chunk pair 0, dim block 0; the others
    // differ by an XOR), as in the prefill kernel
    const int kbase = n * 256 + ((hf ^ (n & 15)) << 4);
    const int vbase = (4 * hf + ((n & 15) >> 2)) * 256 + (((n & 15) >> 2) << 6) + 32 * (n >> 4) + 8 * (n & 3);

    for (int i = 0; i < nb; ++i) {
      // The copies were issued in the order ... rows i, entries i + 2 (PLAN: table words i + 1), rows i + 1: block i's
      // rows and the entries of block i + 2 have landed once nothing but the sixteen copies of block i + 1's rows is
      // outstanding.
      if (i + 1 < nb) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      const unsigned char *ks = lds + (i & 1) * kSlot;
      const unsigned char *vs = ks + kVSlots;
      const unsigned char *entries = lds + kEntries + (i & 3) * 256;

      // which heads keep which key: lane k < 32 holds the member byte of key k of the block
      const int e0 = entry0(i);
      const int shift = (int)((member_at + (unsigned)e0) & 3);
      unsigned mem = lane < 32 && e0 + lane < end ? entries[128 + shift + lane] : 0u;
      if (PLAN) {
        const int v = *reinterpret_cast<const int *>(entries + 4 * (lane & 31));
        const bool exists = v < 0 ? a.pos + 1 + v >= 0 : v <= a.pos;
        const int t = table_index(v);
        unsigned covered = 0;  // heads that reach this column's key through a matched diagonal
        if (t >= 0) {
          const unsigned word = *reinterpret_cast<const unsigned *>(lds + kFix + (i & 3) * 256 + 4 * (lane & 31));
          covered = (word >> (8 * (int)((table_at + (unsigned)t) & 3))) & 0xFFu;
        }
        mem = exists ? mem & ~covered : 0u;
      }
      unsigned mine = 0;  // bit k: key k of the block is kept by this lane's head
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        if (x < G) {  // wave-uniform
          const unsigned kept_x = (unsigned)__ballot((mem >> x) & 1);
          if (n == x) mine = kept_x;
        }
      }
      if (n >= G) mine = 0;

      // S^T = K Q^T; accumulator e is key 8 (e / 4) + 4 hf + e % 4 and starts at 0 (kept) or -inf (masked)
      f32x16 s;
      mask_init(s, (int)~(mine >> (4 * hf)), std::make_integer_sequence<int, 16>{});
#pragma unroll
      for (int c = 0; c < 8; ++c)
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_read_b128(ks, kbase ^ (c << 5)), qf[c], s, 0, 0, 0);

      // online softmax, one head per lane pair (lane, lane ^ 32); the reference the weights are taken against
      // only moves when the maximum has grown past it by more than 8 in log2 units
      float mx = s[0];
#pragma unroll
      for (int e = 1; e < 16; ++e) mx = fmaxf(mx, s[e]);
      {
        const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
      }
      const float m_top = fmaxf(m_run, mx);
      const bool move = (m_top - m_run) * c2 > 8.0f;  // (-inf) - (-inf) is NaN: no move
      const float m_new = move ? m_top : m_run;
      const float m_ref = m_new == -INFINITY ? 0.0f : m_new;
      const float off = m_ref * c2;
      if (__ballot(move)) {
        const float corr = move ? __builtin_amdgcn_exp2f((m_run - m_ref) * c2) : 1.0f;  // old reference -inf: 0
        l_run *= corr;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[db][e] *= corr;
      }
      m_run = m_new;
      unsigned p[8];
      float psum = 0.0f;
      const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], c2, -off));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e + 1], c2, -off));
        p[e / 2] = pack_bf16(p0, p1);
        // the sum is taken over the rounded weights the P V product uses
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, p[e / 2]), ones, psum, false);
      }
      l_run += psum;

      // O^T += V^T P^T: accumulator e of dim block db is dim 32 db + 8 (e / 4) + 4 hf + e % 4
      typedef __attribute__((ext_vector_type(8))) short s16x8;
#pragma unroll
      for (int a2 = 0; a2 < 2; ++a2) {
        const u32x4 praw = {p[4 * a2], p[4 * a2 + 1], p[4 * a2 + 2], p[4 * a2 + 3]};
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const int va = vbase ^ (db << 6);
          const s16x4 r0 = lds_read_tr(vs, va + (a2 * 16) * 256);
          const s16x4 r1 = lds_read_tr(vs, va + (a2 * 16 + 8) * 256);
          const s16x8 vf = __builtin_shufflevector(r0, r1, 0, 1, 2, 3, 4, 5, 6, 7);
          oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf),
                                                             __builtin_bit_cast(bf16x8, praw), oacc[db], 0, 0, 0);
        }
      }
      // every LDS read of block i has returned (the products consumed them): its slots are free for block i + 2
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (i + 3 < nb) copy_entries(i + 3);
      if (PLAN && i + 2 < nb) copy_fix(i + 2);
      if (i + 2 < nb) copy_rows(i + 2);
    }
  }

  // partial results in the form the merge pass takes: reference in log2 units, sum, un-normalised O
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float m2 = m_run == -INFINITY ? -INFINITY : m_run * c2;
  if (a.fused) {
    // waves 1 .. splits - 1 hand their results to wave 0 through their own (now idle) slots: value e of lane l at
    // word 64 e + l (64 values of O, then the reference and the sum)
    float *mine_x = reinterpret_cast<float *>(lds);
    if (wave > 0) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) mine_x[(16 * db + e) * 64 + lane] = oacc[db][e];
      mine_x[64 * 64 + lane] = m2;
      mine_x[65 * 64 + lane] = l_tot;
    }
    __syncthreads();
    if (wave > 0) return;
    // the merge of the splits as the merge kernel does it: weights 2^(reference - largest reference)
    float M = m2;
    for (int sp = 1; sp < a.splits; ++sp) M = fmaxf(M, reinterpret_cast<const float *>(lds_all + sp * kLds)[64 * 64 + lane]);
    float L = 0.0f;
    if (M > -INFINITY) {
      const float w0 = exp2f(m2 - M);
      L = w0 * l_tot;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[db][e] *= w0;
      for (int sp = 1; sp < a.splits; ++sp) {
        const float *theirs = reinterpret_cast<const float *>(lds_all + sp * kLds);
        const float ws = exp2f(theirs[64 * 64 + lane] - M);
        L += ws * theirs[65 * 64 + lane];
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[db][e] += ws * theirs[(16 * db + e) * 64 + lane];
      }
    }
    if (n < G) {
      const float inv = L > 0.0f ? 1.0f / L : 0.0f;
      const int hq = hkv * G + n;
      __hip_bfloat16 *op = out + b * a.o_sb + hq * a.o_sh;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          uint2 pr;
          pr.x = pack_bf16(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv);
          pr.y = pack_bf16(oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv);
          *reinterpret_cast<uint2 *>(op + 32 * db + 8 * g + 4 * hf) = pr;
        }
      if (lse && hf == 0) lse[(int64_t)b * a.Hq + hq] = L > 0.0f ? (M + log2f(L)) * 0.6931471805599453f : -INFINITY;
    }
    return;
  }
  if (n < G) {
    const int64_t slot_out = ((int64_t)b * a.Hq + hkv * G + n) * a.splits + split;
    float *po = part_o + slot_out * 128;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<float4 *>(po + 32 * db + 8 * g + 4 * hf) =
            make_float4(oacc[db][4 * g], oacc[db][4 * g + 1], oacc[db][4 * g + 2], oacc[db][4 * g + 3]);
    if (hf == 0) {
      part_ml[slot_out * 2] = m2;
      part_ml[slot_out * 2 + 1] = l_tot;
    }
  }
}

}  // namespace

namespace dam {

bool decode_group_mfma_fits(const dam_decode_params *p) {
  if (p->dtype != DAM_BF16 || p->head_dim != 128) return false;
  if (p->hq / p->hkv > 8) return false;
  // row addresses are a base per (sequence, KV head) plus a 32-bit byte offset, the product of a row index and a
  // row stride of at most 24 bits each
  if (p->kv_capacity >= (1 << 24) || p->kv_stride[2] * 2 >= (1 << 24)) return false;
  return (uint64_t)p->kv_capacity * (uint64_t)p->kv_stride[2] * 2u < (1ull << 32);
}

bool decode_group_mfma_merges(int splits) { return splits <= 4; }

int launch_decode_group_mfma(const dam_decode_params *p, int splits, float scale, const void *q, const void *kc,
                             const void *vc, const int32_t *kept_ptr, const int32_t *kept_idx,
                             const uint8_t *kept_member, float *part_o, float *part_ml, void *out, float *lse,
                             hipStream_t st, const uint8_t *plan_table, int n_flags, int pos) {
  MfmaArgs a;
  a.B = p->batch; a.Hq = p->hq; a.Hkv = p->hkv; a.cap = p->kv_capacity; a.splits = splits;
  a.shared_lists = p->shared_lists != 0;
  a.scale = scale;
  a.q_sb = p->q_stride[0]; a.q_sh = p->q_stride[1];
  a.kv_sb = p->kv_stride[0]; a.kv_sh = p->kv_stride[1];
  a.o_sb = p->o_stride[0]; a.o_sh = p->o_stride[1];
  a.row_bytes = (unsigned)(p->kv_stride[2] * 2);
  a.pos = pos;
  a.n_flags = n_flags;
  a.fused = decode_group_mfma_merges(splits) ? 1 : 0;
  const int waves = a.fused ? splits : 1;
  const int blocks = a.fused ? p->batch * p->hkv : p->batch * p->hkv * splits;
  const size_t lds_bytes = (size_t)kLds * waves;
  const void *kernel = plan_table ? reinterpret_cast<const void *>(k_decode_group_mfma<true>)
                                  : reinterpret_cast<const void *>(k_decode_group_mfma<false>);
  // (more than the default limit of dynamic LDS with two or more waves; idempotent, set on every call)
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * kLds) != hipSuccess) return DAM_ERR_DEVICE;
  if (plan_table)
    k_decode_group_mfma<true><<<blocks, 64 * waves, lds_bytes, st>>>(
        a, static_cast<const __hip_bfloat16 *>(q), static_cast<const __hip_bfloat16 *>(kc),
        static_cast<const __hip_bfloat16 *>(vc), kept_ptr, kept_idx, kept_member, plan_table, part_o, part_ml,
        static_cast<__hip_bfloat16 *>(out), lse);
  else
    k_decode_group_mfma<false><<<blocks, 64 * waves, lds_bytes, st>>>(
        a, static_cast<const __hip_bfloat16 *>(q), static_cast<const __hip_bfloat16 *>(kc),
        static_cast<const __hip_bfloat16 *>(vc), kept_ptr, kept_idx, kept_member, nullptr, part_o, part_ml,
        static_cast<__hip_bfloat16 *>(out), lse);
  return DAM_OK;
}

}  // namespace dam
