// Device helpers shared by the split-KV decode kernels of the Flash-LoRA-Attention library
// (bf16, gfx950): vector types, LDS reads, bf16 packing, lane-group exchanges and the
// hand-issued HBM -> LDS loads with their waits.
#pragma once

#include "lra_common.h"

namespace lra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

#ifdef LRA_TIMING
// Build-time instrumentation (never part of the shipped library): wall-clock stamps (100 MHz) of
// the phases of every wave, written to a buffer the test build passes in.
#define LRA_STAMP(k) do { unsigned long long t_; asm volatile("s_waitcnt lgkmcnt(0)\n\ts_memrealtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t_)); tt[k] = t_; } while (0)
#define LRA_STAMP_DECL unsigned long long tt[12] = {0,0,0,0,0,0,0,0,0,0,0,0}
#define LRA_STAMP_FLUSH() do { if (p.timing && lane == 0) { \
    unsigned long long* o_ = p.timing + ((static_cast<size_t>(blockIdx.z) * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 64 + wave * 16; \
    for (int i_ = 0; i_ < 12; ++i_) o_[i_] = tt[i_]; \
    o_[12] = __builtin_amdgcn_s_getreg((20) | (0 << 6) | ((4 - 1) << 11)); \
    o_[13] = __builtin_amdgcn_s_getreg((4) | (0 << 6) | ((32 - 1) << 11)); } } while (0)
#else
#define LRA_STAMP(k)
#define LRA_STAMP_DECL
#define LRA_STAMP_FLUSH()
#endif

#define LDS_AS(T, p) ((__attribute__((address_space(3))) T*)(p))
// Read-only int32 tables of a call, addressed as constant memory: wave-uniform reads stay
// scalar loads also after the hand-issued loads below, which the compiler must treat as
// statements that may write anywhere.
typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
#define CONST_I32(p) ((const_i32_ptr)(p))

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint4 lds_read16(const unsigned char* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ uint2 lds_read8(const unsigned char* p) { return *reinterpret_cast<const uint2*>(p); }

// ds_read_b64_tr_b16: inside every group of 16 lanes, lane i receives for e = 0..3
// element (i % 4) of the 8 bytes addressed by lane 4e + i/4.
__device__ __forceinline__ s16x4 lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_AS(s16x4, p));
}

__device__ __forceinline__ bf16x8 join_tr(s16x4 lo, s16x4 hi) {
  s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {  // one v_cvt_pk_bf16_f32
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Exchange between the four 16-lane groups of a wave (lanes l, l^16, l^32, l^48).
// v_permlane16_swap exchanges the odd 16-lane rows of its first register with the
// even rows of its second, v_permlane32_swap the upper half of the first with the
// lower half of the second.  Started from two copies of one value, the two
// registers afterwards hold, in every lane, the value and its partner's value.
// Written as inline assembly because the compiler's builtin for these
// instructions treats its two results as one and the same value.
__device__ __forceinline__ void permlane16_swap(float& x, float& y) {
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(x), "+v"(y));
}
__device__ __forceinline__ void permlane32_swap(float& x, float& y) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(x), "+v"(y));
}

__device__ __forceinline__ float max_over_lane_groups(float v) {
  float x = v, y = v;
  permlane16_swap(x, y);
  x = y = fmaxf(x, y);
  permlane32_swap(x, y);
  return fmaxf(x, y);
}

__device__ __forceinline__ float sum_over_lane_groups(float v) {
  float x = v, y = v;
  permlane16_swap(x, y);
  x = y = x + y;
  permlane32_swap(x, y);
  return x + y;
}

// Raw buffer resource over [base, base + bytes): loads past the end return zero
// and touch no memory.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, static_cast<int>(bytes), 0x00020000);
}

__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t rs, uint32_t voff, uint32_t soff) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, 0);
  return make_uint4(v[0], v[1], v[2], v[3]);
}

// The same kind of resource as four plain words, for the hand-issued loads below (the words
// are wave-uniform by construction; readfirstlane pins them to scalar registers).
__device__ __forceinline__ u32x4 make_rsrc_words(const void* base, uint32_t bytes) {
  auto uni = [](uint32_t v) { return static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(v))); };
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  return u32x4{uni(static_cast<uint32_t>(a)), uni(static_cast<uint32_t>(a >> 32) & 0xffffu), uni(bytes), 0x00020000u};
}

// 16 bytes per lane from the buffer straight into LDS at lds + lane*16 (the LDS base travels
// in M0; one wait state between the write of M0 and the load).  Issued as inline assembly
// and waited for by hand (wait_vm0): the compiler's own bookkeeping of such loads proved
// fragile - with other vector loads still outstanding it has placed the wait AFTER the
// first LDS reads of the tile.  Neither statement claims to touch memory (the compiler
// would then stop using scalar loads for the kernel's read-only tables); the ordering
// against the LDS reads of the tile comes from lds_fence() on both sides.
// STREAM = true marks the request non-temporal: K_base and V_base rows are read once per call, by
// one workgroup, and should not displace what other workgroups share (L, B_K, the partial states).
template <bool STREAM = false>
__device__ __forceinline__ void buf_load16_to_lds(u32x4 rs, unsigned char* lds, uint32_t voff, uint32_t soff) {
  const uint32_t lds_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(LDS_AS(unsigned char, lds)));
  if constexpr (STREAM)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen nt lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rs), "s"(soff)
                 : "m0");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rs), "s"(soff)
                 : "m0");
}
__device__ __forceinline__ void wait_vm0() { asm volatile("s_waitcnt vmcnt(0)"); }
// Compiler-level ordering point for the LDS traffic of one wave: no LDS access moves across
// it and LDS contents are taken as changed.  Emits no instruction.
__device__ __forceinline__ void lds_fence() { __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront"); }

constexpr uint32_t kOob = 0x80000000u;  // beyond any resource this kernel builds

// s_waitcnt vmcnt(N) with a compile-time N: at most N of this wave's vector-memory requests may
// still be outstanding afterwards (they retire in the order they were issued).
template <int N>
__device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N)); }

}  // namespace lra
