// Accumulation registers (a0..a127) of the bf16 forward kernel, addressed BY NAME.
//
// The kernel runs two waves per SIMD, i.e. 256 registers per wave: 128 vector
// registers, which the compiler allocates as usual (score tiles, P, softmax state,
// addresses), and 128 accumulation registers, which this header owns completely:
//   a[0   .. 31 ]  the wave's Q fragments (MFMA B operand of S^T = K Q^T), 4 per k-step
//   a[32  .. 63 ]  8 slots of 4 registers: K / V^T fragments in flight between the
//                  LDS read that fills a slot and the MFMA that consumes it
//   a[64  .. 127]  the output accumulators O^T, 16 per 32-channel block
// Register numbers are template constants printed into the assembly text, so no copy
// between the register files can ever be inserted around a matrix instruction, and the
// LDS reads land directly where the matrix pipe takes its operands.  The compiler does
// not see these registers at all: it must not allocate any accumulation register itself
// in a translation unit that includes this header (the build step scans the generated
// assembly for that), and completion of the LDS reads is awaited explicitly with
// lds_wait<N>(): "at most N LDS operations issued after the one I need are outstanding".
// LDS operations complete in order, so a wait that names FEWER later operations than
// were really issued is always safe.
#pragma once
#include "moda_common.h"

namespace moda {

typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr int kAccQ = 0;      // first register of the Q fragments
constexpr int kAccSlot = 32;  // first register of the fragment slots
constexpr int kAccO = 64;     // first register of the output accumulators
constexpr int kSlots = 8;

// Tells the compiler how many accumulation registers the kernel needs (the register
// allocation of the launch is derived from the clobbers it sees).
__device__ __forceinline__ void reserve_acc_registers() { asm volatile("" ::: "a127"); }

// ---- Q fragment of k-step ST
template <int ST>
__device__ __forceinline__ void set_q(const i32x4& v) {
  asm volatile(
      "v_accvgpr_write_b32 a%c4, %0\n\tv_accvgpr_write_b32 a%c5, %1\n\t"
      "v_accvgpr_write_b32 a%c6, %2\n\tv_accvgpr_write_b32 a%c7, %3"
      :
      : "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "n"(kAccQ + 4 * ST), "n"(kAccQ + 4 * ST + 1),
        "n"(kAccQ + 4 * ST + 2), "n"(kAccQ + 4 * ST + 3));
}

// ---- LDS -> fragment slot.  `addr` is a byte address in LDS, OFF an immediate (< 64 KB).
// K fragment: 32 keys x 16 channels, one 128-bit read.
template <int SLOT, int OFF>
__device__ __forceinline__ void read_k_slot(int addr) {
  static_assert(OFF >= 0 && OFF < 65536 && SLOT >= 0 && SLOT < kSlots, "immediate offset");
  asm volatile("ds_read_b128 a[%c1:%c2], %0 offset:%c3"
               :
               : "v"(addr), "n"(kAccSlot + 4 * SLOT), "n"(kAccSlot + 4 * SLOT + 3), "n"(OFF)
               : "memory");
}
// V^T fragment: 16 keys x 32 channels, two transposing 64-bit reads ROWS8 bytes apart.
template <int SLOT, int OFF, int ROWS8>
__device__ __forceinline__ void read_v_slot(int addr) {
  static_assert(OFF >= 0 && OFF + ROWS8 < 65536 && SLOT >= 0 && SLOT < kSlots, "immediate offset");
  asm volatile("ds_read_b64_tr_b16 a[%c1:%c2], %0 offset:%c5\n\tds_read_b64_tr_b16 a[%c3:%c4], %0 offset:%c6"
               :
               : "v"(addr), "n"(kAccSlot + 4 * SLOT), "n"(kAccSlot + 4 * SLOT + 1),
                 "n"(kAccSlot + 4 * SLOT + 2), "n"(kAccSlot + 4 * SLOT + 3), "n"(OFF), "n"(OFF + ROWS8)
               : "memory");
}
template <int N>
__device__ __forceinline__ void lds_wait() {
  static_assert(N >= 0 && N < 16, "lgkmcnt immediate");
  asm volatile("s_waitcnt lgkmcnt(%c0)" : : "n"(N) : "memory");
}

// ---- S^T (vector registers) = / += K fragment (slot) x Q fragment (k-step ST)
template <int SLOT, int ST, bool INIT>
__device__ __forceinline__ void mfma_s(f32x16& s) {
  if constexpr (INIT)
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, a[%c1:%c2], a[%c3:%c4], 0"
                 : "=&v"(s)
                 : "n"(kAccSlot + 4 * SLOT), "n"(kAccSlot + 4 * SLOT + 3), "n"(kAccQ + 4 * ST),
                   "n"(kAccQ + 4 * ST + 3));
  else
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, a[%c1:%c2], a[%c3:%c4], %0"
                 : "+v"(s)
                 : "n"(kAccSlot + 4 * SLOT), "n"(kAccSlot + 4 * SLOT + 3), "n"(kAccQ + 4 * ST),
                   "n"(kAccQ + 4 * ST + 3));
}

// ---- O^T block OB += V^T fragment (slot) x P^T fragment (vector registers)
template <int OB, int SLOT>
__device__ __forceinline__ void mfma_o(const i32x4& p) {
  asm volatile("v_mfma_f32_32x32x16_bf16 a[%c1:%c2], a[%c3:%c4], %0, a[%c1:%c2]"
               :
               : "v"(p), "n"(kAccO + 16 * OB), "n"(kAccO + 16 * OB + 15), "n"(kAccSlot + 4 * SLOT),
                 "n"(kAccSlot + 4 * SLOT + 3));
}

// ---- single output registers
template <int R>
__device__ __forceinline__ void zero_acc() {
  asm volatile("v_accvgpr_write_b32 a%c0, 0" : : "n"(R));
}
template <int R>
__device__ __forceinline__ void write_acc(float x) {
  asm volatile("v_accvgpr_write_b32 a%c1, %0" : : "v"(x), "n"(R));
}
template <int R>
__device__ __forceinline__ void scale_acc(float f) {
  float t;
  asm volatile("v_accvgpr_read_b32 %0, a%c2\n\tv_mul_f32 %0, %0, %1\n\tv_accvgpr_write_b32 a%c2, %0"
               : "=&v"(t)
               : "v"(f), "n"(R));
}
template <int R>
__device__ __forceinline__ float read_acc() {
  float x;
  asm volatile("v_accvgpr_read_b32 %0, a%c1" : "=v"(x) : "n"(R));
  return x;
}

}  // namespace moda
