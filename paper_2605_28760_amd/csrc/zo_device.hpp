// Device-side helpers shared by the gfx950 kernels: the counter-based factor
// generator (Philox4x32-10 + Box-Muller; the paper's "directions regenerated
// from a seed", Sec. 2.2 / taxonomy table, with N(0,1) entries as in Sec. 3.3),
// bf16 conversion, and the MFMA fragment types.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t bf16_t;  // storage type of a bfloat16 value

constexpr int kWave = 64;

// ---- sequence kinds written by the batch preparation kernel ----------------
constexpr int kKindForeground = -2;  // candidate id -1: base weights only
constexpr int kKindCentre = -1;      // candidate without a probe: bank only

// ---- Philox4x32-10 ----------------------------------------------------------
__device__ __forceinline__ uint4 philox4x32_10(uint4 c, uint2 k) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)M0 * c.x, p1 = (uint64_t)M1 * c.z;   // one 32 x 32 -> 64 multiply each
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    c = make_uint4(hi1 ^ c.y ^ k.x, lo1, hi0 ^ c.w ^ k.y, lo0);
    k.x += W0;
    k.y += W1;
  }
  return c;
}

__device__ __forceinline__ uint4 factor_block(uint64_t seed, uint32_t tensor_id, uint64_t q) {
  return philox4x32_10(make_uint4((uint32_t)q, (uint32_t)(q >> 32), tensor_id, 0u),
                       make_uint2((uint32_t)seed, (uint32_t)(seed >> 32)));
}

// u(w) = (2 (w >> 9) + 1) 2^-24: exact in fp32.  Box-Muller on (wa, wb):
// z0 = rho cos(2 pi u_b), z1 = rho sin(2 pi u_b), rho = sqrt(-2 ln u_a).  The hardware's own logarithm (base
// 2), square root, and sine / cosine (which take their argument in revolutions, so the angle is u_b itself
// and needs no range reduction) serve: over all 2^23 uniforms the generator can produce, rho is within
// 1.4e-7 (relative) and the sine and cosine within 1.3e-7 (absolute) of the exact values, the same as
// the library routines, at a third of their instructions.
__device__ __forceinline__ void box_muller(uint32_t wa, uint32_t wb, float& z0, float& z1) {
  const float ua = (float)(((wa >> 9) << 1) | 1u) * 0x1p-24f;
  const float ub = (float)(((wb >> 9) << 1) | 1u) * 0x1p-24f;
  constexpr float kMinus2Ln2 = -1.3862943611198906f;
  const float rho = __builtin_amdgcn_sqrtf(kMinus2Ln2 * __builtin_amdgcn_logf(ua));
  z0 = rho * __builtin_amdgcn_cosf(ub);
  z1 = rho * __builtin_amdgcn_sinf(ub);
}

// Standard normal for flat index e of the stream (seed, tensor_id).
__device__ __forceinline__ float factor_normal(uint64_t seed, uint32_t tensor_id, uint64_t e) {
  const uint4 w = factor_block(seed, tensor_id, e >> 2);
  const bool second = (e & 2) != 0;
  float z0, z1;
  box_muller(second ? w.z : w.x, second ? w.w : w.y, z0, z1);
  return (e & 1) ? z1 : z0;
}

// ---- bfloat16 ------------------------------------------------------------------
__device__ __forceinline__ bf16_t f32_to_bf16(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ float bf16_round(float x) { return bf16_to_f32(f32_to_bf16(x)); }
// Two fp32 -> packed bf16 (round to nearest even) with the gfx950 conversion instruction.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 16-byte global load of 8 bf16 values as an MFMA operand fragment.
__device__ __forceinline__ bf16x8 load_frag(const bf16_t* p) {
  return *reinterpret_cast<const bf16x8*>(p);
}
__device__ __forceinline__ bf16x8 zero_frag() {
  u32x4 z = {0u, 0u, 0u, 0u};
  return __builtin_bit_cast(bf16x8, z);
}

}  // namespace zo
