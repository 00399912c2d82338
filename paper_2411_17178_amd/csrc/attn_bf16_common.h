// Device helpers shared by the bf16 attention kernels (gfx950): vector typedefs, the
// transposing LDS read, lane-mask select, the cross-row maximum and the LDS / vmcnt
// primitives that must not wait for outstanding LDS-DMA loads.
#pragma once
#include "internal.h"

namespace lv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;
// constant address space: a load from a wave-uniform address becomes a scalar load
typedef const __attribute__((address_space(4))) uint64_t* const_u64_ptr;
typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;

constexpr float kFloor = -1.0e30f;   // initial softmax reference: keeps exp2 arguments finite
constexpr float kSlack = 6.0f;       // base-2 exponent by which a score may exceed the reference

__device__ inline bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ inline s16x4 lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
}

// keep `s` where the lane's bit of the wave-uniform `mask` is set, else -inf
// (inverse ballot: the SGPR pair becomes the select condition of one v_cndmask)
__device__ inline float mask_select(float s, uint64_t mask) {
  return __builtin_amdgcn_inverse_ballot_w64(mask) ? s : -INFINITY;
}

// max over the four lanes l, l^16, l^32, l^48: v_permlane32_swap exchanges the upper half
// of its first register with the lower half of its second, v_permlane16_swap the odd
// 16-lane rows of the first with the even rows of the second.  (The two results are
// copied into scalars before the float reinterpretation: a __builtin_bit_cast applied
// directly to an element of the returned vector reads element 0 for both.)
__device__ inline float max_across_rows(float x) {
  const unsigned u = __float_as_uint(x);
  auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const unsigned a0 = a[0], a1 = a[1];
  const unsigned v = __float_as_uint(fmaxf(__uint_as_float(a0), __uint_as_float(a1)));
  auto b = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  const unsigned b0 = b[0], b1 = b[1];
  return fmaxf(__uint_as_float(b0), __uint_as_float(b1));
}

// What every attention kernel checks before it reads anything else of the plan: the blob's
// header carries the magic and not the builder's error mark.  A zeroed, stale or half-built
// blob then makes the launch a no-op instead of a walk over garbage.  (Scalar loads: the
// header is the same for every workgroup.)
__device__ inline bool plan_usable(const Header* hdr) {
  const const_i32_ptr w = (const_i32_ptr)hdr;
  int magic_lo = w[0], magic_hi = w[1], err = w[offsetof(Header, error) / 4];
  asm volatile("" : "+s"(magic_lo), "+s"(magic_hi), "+s"(err));   // one round trip for the three words
  return magic_lo == (int32_t)(kMagic & 0xffffffffu) && magic_hi == (int32_t)(kMagic >> 32) && err != kErrBuilder;
}

// The bounds-checking build (-DLITEVAR_DEBUG_BOUNDS, a second library for tests and for chasing
// a suspected plan/kernel mismatch): every token that addresses a K/V row, every query row
// that addresses Q or O and every LDS offset taken from a step descriptor is compared with
// its limit before use; a value out of range is replaced by 0 and the plan's header is
// marked (litevar_plan_check then says so).  The normal build compiles the checks away.
__device__ inline int checked_index([[maybe_unused]] Header* hdr, int value, [[maybe_unused]] int limit) {
#ifdef LITEVAR_DEBUG_BOUNDS
  if ((unsigned)value >= (unsigned)limit) { hdr->error = kErrBounds; return 0; }
#endif
  return value;
}

// x = q n + r for a divisor n whose magic = floor(2^32 / n) came with the kernel arguments
// (n = 1: magic = 2^32 - 1): the estimate floor(x magic / 2^32) is the quotient or one below it
// for every x < 2^32, so one correction step makes it exact.
__device__ inline void divmod_by(uint32_t x, uint32_t n, uint32_t magic, int& q, int& r) {
  uint32_t qq = __umulhi(x, magic), rr = x - qq * n;
  if (rr >= n) { ++qq; rr -= n; }
  q = (int)qq; r = (int)rr;
}

template <int N> __device__ inline void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  // gfx9 encoding: vmcnt[3:0] in bits 3:0, vmcnt[5:4] in bits 15:14; expcnt/lgkmcnt left at max
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}

// N consecutive-stride LDS words (stride 32 bytes) written by earlier LDS-DMA loads of this
// wave whose completion the caller has already established.  Inline assembly, because the
// compiler would otherwise order these reads after a vmcnt(0) wait (it cannot know which
// DMA loads have landed) and so drain the prefetch queue.
template <int N> __device__ inline void lds_read_tokens(const int32_t* p, int (&t)[N]);
template <> __device__ inline void lds_read_tokens<4>(const int32_t* p, int (&t)[4]) {
  const unsigned a = (unsigned)(uintptr_t)(__attribute__((address_space(3))) const int32_t*)p;
  asm volatile("ds_read_b32 %0, %4\n\tds_read_b32 %1, %4 offset:32\n\t"
               "ds_read_b32 %2, %4 offset:64\n\tds_read_b32 %3, %4 offset:96\n\t"
               "s_waitcnt lgkmcnt(0)"
               : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]) : "v"(a) : "memory");
}
template <> __device__ inline void lds_read_tokens<8>(const int32_t* p, int (&t)[8]) {
  const unsigned a = (unsigned)(uintptr_t)(__attribute__((address_space(3))) const int32_t*)p;
  asm volatile("ds_read_b32 %0, %8\n\tds_read_b32 %1, %8 offset:32\n\t"
               "ds_read_b32 %2, %8 offset:64\n\tds_read_b32 %3, %8 offset:96\n\t"
               "ds_read_b32 %4, %8 offset:128\n\tds_read_b32 %5, %8 offset:160\n\t"
               "ds_read_b32 %6, %8 offset:192\n\tds_read_b32 %7, %8 offset:224\n\t"
               "s_waitcnt lgkmcnt(0)"
               : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]),
                 "=&v"(t[6]), "=&v"(t[7]) : "v"(a) : "memory");
}

// LDS accesses of the loader wave that must not wait for its outstanding LDS-DMA loads
// (the compiler orders ordinary LDS accesses after vmcnt(0) once a DMA load is pending)
__device__ inline void lds_store_i32_nowait(int32_t* p, int v) {
  const unsigned a = (unsigned)(uintptr_t)(__attribute__((address_space(3))) int32_t*)p;
  asm volatile("ds_write_b32 %0, %1" : : "v"(a), "v"(v) : "memory");
}
__device__ inline int lds_load_i32_nowait(const int32_t* p) {   // waits for LDS only, not for vector memory
  const unsigned a = (unsigned)(uintptr_t)(__attribute__((address_space(3))) const int32_t*)p;
  int v;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(a) : "memory");
  return v;
}
template <int NW> __device__ inline int lds_min_progress(const int32_t* p) {
  static_assert(NW == 4 || NW == 8, "progress words are read four at a time");
  const unsigned a = (unsigned)(uintptr_t)(__attribute__((address_space(3))) const int32_t*)p;
  typedef __attribute__((ext_vector_type(4))) int i32x4;
  i32x4 x, y;
  if constexpr (NW == 8) {
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:16\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(x), "=&v"(y) : "v"(a) : "memory");
  } else {
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(x) : "v"(a) : "memory");
    y = x;
  }
  const int m0 = min(min(x[0], x[1]), min(x[2], x[3])), m1 = min(min(y[0], y[1]), min(y[2], y[3]));
  return min(m0, m1);
}

}  // namespace lv
