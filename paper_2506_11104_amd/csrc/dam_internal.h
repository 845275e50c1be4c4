// Internal helpers shared by the HIP translation units of libdam.so (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "dam.h"

namespace dam {

constexpr int kWave = 64;  // CDNA wavefront width

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Converts the status of the launches enqueued so far into a dam_status.
inline int launch_status() { return hipGetLastError() == hipSuccess ? DAM_OK : DAM_ERR_DEVICE; }

// Carves consecutive 256-byte aligned regions out of one workspace allocation.
struct Carver {
  char *base;
  size_t off = 0;
  explicit Carver(void *p) : base(static_cast<char *>(p)) {}
  template <typename T>
  T *take(size_t n) {
    T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off = align_up(off + n * sizeof(T), 256);
    return p;
  }
};

// dam_capture.hip: argument check of a capture, bytes of its row log-sum-exp buffer, and the fused
// form that writes the true mask of one captured sequence (bit = probability >= threshold, the
// threshold given as the ordered fp32 key the mask builder uses).
int capture_validate(const dam_capture_params *p, const void *q, const void *k);
size_t capture_lse_bytes(const dam_capture_params *p);
void launch_capture_true_bits(const dam_capture_params *p, const void *q, const void *k, float *lse2,
                              const unsigned *theta_key, uint64_t *true_bits, hipStream_t stream);

// dam_decode_mfma.hip: the partial pass of the grouped-query decode on the matrix cores. `fits` says
// whether a call can take it (bf16, head_dim 128, at most 8 query heads per KV head, a head's cache rows
// within 4 GiB); the launch writes one (reference, sum, un-normalised O) triple per (sequence, query
// head, split) in the layout the merge pass of dam_decode.hip reads. plan_table != nullptr: the lists are a
// position-independent plan (DAM_MASK_PATTERN_PLAN) decoded at position pos; n_flags is the table's row length.
bool decode_group_mfma_fits(const dam_decode_params *p);
// true: the kernel merges the splits itself and stores the output (no merge pass, part_o / part_ml unused)
bool decode_group_mfma_merges(int splits);
int launch_decode_group_mfma(const dam_decode_params *p, int splits, float scale, const void *q, const void *kc,
                             const void *vc, const int32_t *kept_ptr, const int32_t *kept_idx,
                             const uint8_t *kept_member, float *part_o, float *part_ml, void *out, float *lse,
                             hipStream_t st, const uint8_t *plan_table = nullptr, int n_flags = 0, int pos = 0);

}  // namespace dam
