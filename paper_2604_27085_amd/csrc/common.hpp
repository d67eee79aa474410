// Shared device/host helpers for the gfx950 kernels (wave64, bf16 MFMA).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define RP_DEV __device__ __forceinline__

// Launch with a clean error slate: hipGetLastError() after the launch must report this launch, not an error another
// library left behind earlier on this thread.
#define RP_LAUNCH(...)               \
  do {                               \
    (void)hipGetLastError();         \
    hipLaunchKernelGGL(__VA_ARGS__); \
  } while (0)

static RP_DEV float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
static RP_DEV float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
static RP_DEV float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// round-to-nearest-even float -> bf16 bit pattern
static RP_DEV uint32_t f32_to_bf16_bits(float f) {
  bf16 h = (bf16)f;
  return (uint32_t)__builtin_bit_cast(unsigned short, h);
}
static RP_DEV uint32_t pack_bf16x2(float lo, float hi) {   // one v_cvt_pk_bf16_f32 (round to nearest even)
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}


static RP_DEV f32x16 mfma32(const uint4& a, const uint4& b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

static RP_DEV float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
static RP_DEV float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Blocks are handed to the 8 XCDs round-robin; remap so that consecutive logical ids share an XCD (and its L2).
static RP_DEV int xcd_remap(int pid, int nblk) {
  const int q = nblk >> 3, r = nblk & 7;
  const int xcd = pid & 7, local = pid >> 3;
  return xcd * q + (xcd < r ? xcd : r) + local;
}
