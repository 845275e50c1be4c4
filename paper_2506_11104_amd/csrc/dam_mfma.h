// Device helpers shared by the bf16 MFMA kernels (prefill and grouped decode): vector types, bf16
// packing, LDS operand reads, load-to-LDS copies and the mask-to-accumulator initialisation.
#pragma once
#include <hip/hip_bf16.h>
#include <hip/hip_runtime.h>

#include <utility>

namespace dam {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  const bf16x2 r = __builtin_convertvector((f32x2){lo, hi}, bf16x2);  // round to nearest even
  return __builtin_bit_cast(unsigned, r);
}

__device__ __forceinline__ bf16x8 lds_read_b128(const unsigned char *lds, int byte) {
  return *reinterpret_cast<const bf16x8 *>(lds + byte);
}

__device__ __forceinline__ s16x4 lds_read_tr(const unsigned char *lds, int byte) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4 *)(const_cast<unsigned char *>(lds + byte)));
}

// Load-to-LDS copies as inline assembly: lane L of the wave fetches `bytes` bytes from gbase + voff
// and writes them to LDS address m0 + L * bytes, m0 = lds_at + IMM. Written as assembly so that the
// compiler neither tracks them (it would make every later LDS read wait for all copies in flight) nor
// counts them: the kernel waits for them itself with explicit s_waitcnt vmcnt(n), and issues no other
// vector-memory loads inside the pipeline. gbase and lds_at are wave-uniform.
template <int IMM>
__device__ __forceinline__ void lds_copy16(unsigned lds_at, const void *gbase, unsigned voff) {
  asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
               :
               : "s"(lds_at), "n"(IMM), "v"(voff), "s"(gbase)
               : "memory", "scc", "m0");
}
// The same for rows that are read once: a non-temporal load, so that they stream past the caches.
template <int IMM>
__device__ __forceinline__ void lds_copy16_once(unsigned lds_at, const void *gbase, unsigned voff) {
  asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3 nt"
               :
               : "s"(lds_at), "n"(IMM), "v"(voff), "s"(gbase)
               : "memory", "scc", "m0");
}
template <int IMM>
__device__ __forceinline__ void lds_copy4(unsigned lds_at, const void *gbase, unsigned voff) {
  asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, %3"
               :
               : "s"(lds_at), "n"(IMM), "v"(voff), "s"(gbase)
               : "memory", "scc", "m0");
}

// 0 or -inf for bit POS of `inv` clear or set
template <int POS>
__device__ __forceinline__ float neg_inf_if_bit(int inv) {
  // (both instructions in one statement: after a statement of one instruction whose result is used at once
  // the compiler pads with a no-op)
  int field;
  asm("v_bfe_i32 %0, %1, %2, 1\n\tv_and_b32 %0, 0xff800000, %0" : "=&v"(field) : "v"(inv), "n"(POS));
  return __int_as_float(field);
}
template <int... E>
__device__ __forceinline__ void mask_init(f32x16 &s, int inv, std::integer_sequence<int, E...>) {
  ((s[E] = neg_inf_if_bit<8 * (E / 4) + E % 4>(inv)), ...);
}

}  // namespace dam
