// Device-side basics shared by all kernels: storage types, MFMA policy, small helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16;
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));

#define PE_DEV __device__ __forceinline__

// ---------------------------------------------------------------------------
// Storage helpers
// ---------------------------------------------------------------------------
template <typename T> PE_DEV float to_f(T v) { return (float)v; }
template <typename T> PE_DEV T from_f(float v) { return (T)v; }

// 16-byte vector of storage elements
template <typename T> struct Vec16;
template <> struct Vec16<bf16> { static constexpr int N = 8; typedef bf16x8 type; };
template <> struct Vec16<float> { static constexpr int N = 4; typedef f32x4 type; };

// 1 / (1 + 2^(-x log2 e)) with the hardware exponential and reciprocal (about 1 ulp each): four instructions;
// the correctly rounded division alone is a ten-instruction sequence.  2^(+large) = inf gives exactly 0.
PE_DEV float sigmoidf_(float x) { return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(x * -1.4426950408889634f)); }

// ---------------------------------------------------------------------------
// MFMA policy.  One 32x32 output tile per wave-instruction.
//   Operand A: lane l holds A[row = l%32][k = (l/32)*KP + 0..KP-1]
//   Operand B: lane l holds B[k = (l/32)*KP + 0..KP-1][col = l%32]
//   Accumulator element a (0..15) of lane l: row = 8*(a/4) + 4*(l/32) + a%4, col = l%32
// bf16 uses v_mfma_f32_32x32x16_bf16 (KP = 8, 16 contraction steps per instruction),
// fp32 uses v_mfma_f32_32x32x2_f32 (KP = 1, 2 steps per instruction).
// ---------------------------------------------------------------------------
template <typename T> struct Mma;
template <> struct Mma<bf16> {
  static constexpr int KP = 8;
  static constexpr int KSTEP = 16;
  typedef bf16x8 frag;
  static PE_DEV void mma(f32x16& acc, frag a, frag b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
  }
  static PE_DEV frag load(const bf16* p) { return *reinterpret_cast<const bf16x8*>(p); }
  static PE_DEV frag zero() { frag f; for (int i = 0; i < 8; i++) f[i] = (bf16)0.0f; return f; }
};
template <> struct Mma<float> {
  static constexpr int KP = 1;
  static constexpr int KSTEP = 2;
  typedef float frag;
  static PE_DEV void mma(f32x16& acc, frag a, frag b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
  }
  static PE_DEV frag load(const float* p) { return *p; }
  static PE_DEV frag zero() { return 0.0f; }
};

// row index inside a 32x32 accumulator tile held by (lane group g = lane/32, element a)
PE_DEV int acc_row(int g, int a) { return 8 * (a >> 2) + 4 * g + (a & 3); }

PE_DEV float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
PE_DEV float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Host-side launch check used by all launchers.
#define PE_LAUNCH_CHECK() (hipGetLastError())
