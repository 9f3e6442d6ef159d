// Device side of the seeded input generator (test and bench infrastructure; not part of libflux).
//
// Bit-for-bit the same function of (key, counter) as synth.py: splitmix64 hash -> two 24-bit
// uniforms -> Box-Muller with a hand-written ln (atanh series on the reduced mantissa; reciprocal by
// Newton), square root (Newton on rsqrt) and cos (Taylor polynomial on one quadrant), using only
// single fp32 add / subtract / multiply roundings in a fixed order.
// This file must be compiled with -ffp-contract=off so that no multiply-add pair is fused.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

__device__ __forceinline__ uint64_t hash_u64(uint64_t key, uint64_t counter) {
  uint64_t z = counter * 0x9E3779B97F4A7C15ull + key;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// 1/d for d in (1.7, 2.5): Newton on d/4, multiplies and adds only
__device__ __forceinline__ float recip_1p7_2p5(float d) {
  const float dq = __fmul_rn(d, 0.25f);
  float y = __fsub_rn((float)(48.0 / 17.0), __fmul_rn((float)(32.0 / 17.0), dq));
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float e = __fsub_rn(1.0f, __fmul_rn(dq, y));
    y = __fadd_rn(y, __fmul_rn(y, e));
  }
  return __fmul_rn(y, 0.25f);
}

// sqrt(x) for x >= 0 as x * rsqrt(x): bit-level first guess, four Newton steps on rsqrt
__device__ __forceinline__ float sqrt_newton(float x) {
  float y = __uint_as_float(0x5F3759DFu - (__float_as_uint(x) >> 1));
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float t = __fmul_rn(x, y);
    t = __fmul_rn(t, y);
    t = __fsub_rn(1.5f, __fmul_rn(0.5f, t));
    y = __fmul_rn(y, t);
  }
  return __fmul_rn(x, y);
}

__device__ __forceinline__ float normal_f32(uint64_t key, uint64_t counter) {
  const uint64_t h = hash_u64(key, counter);
  const uint32_t k1 = (uint32_t)(h >> 40);
  const uint32_t k2 = (uint32_t)(h >> 16) & 0xFFFFFFu;
  // -ln(u1), u1 = (k1 + 1) / 2^24
  const float x = (float)(k1 + 1u);
  const uint32_t bits = __float_as_uint(x);
  int e = (int)(bits >> 23) - 127;
  float m = __uint_as_float((bits & 0x7FFFFFu) | 0x3F800000u);
  const bool big = m > 1.41421354f;
  m = big ? __fmul_rn(m, 0.5f) : m;
  e += big ? 1 : 0;
  const float s = __fmul_rn(__fsub_rn(m, 1.0f), recip_1p7_2p5(__fadd_rn(m, 1.0f)));
  const float s2 = __fmul_rn(s, s);
  float p = (float)(2.0 / 9.0);
  p = __fadd_rn(__fmul_rn(p, s2), (float)(2.0 / 7.0));
  p = __fadd_rn(__fmul_rn(p, s2), (float)(2.0 / 5.0));
  p = __fadd_rn(__fmul_rn(p, s2), (float)(2.0 / 3.0));
  p = __fadd_rn(__fmul_rn(p, s2), 2.0f);
  const float ln_m = __fmul_rn(s, p);
  float neg_ln = __fsub_rn(__fmul_rn((float)(24 - e), 0.6931471805599453f), ln_m);
  neg_ln = fmaxf(neg_ln, 0.0f);
  const float r = sqrt_newton(__fadd_rn(neg_ln, neg_ln));
  // cos(2 pi u2), u2 = k2 / 2^24
  const uint32_t quad = k2 >> 22;
  const float theta = __fmul_rn((float)(k2 & 0x3FFFFFu), (float)(1.5707963267948966 / 4194304.0));
  const float t2 = __fmul_rn(theta, theta);
  float sp = (float)(-1.0 / 39916800.0);
  sp = __fadd_rn(__fmul_rn(sp, t2), (float)(1.0 / 362880.0));
  sp = __fadd_rn(__fmul_rn(sp, t2), (float)(-1.0 / 5040.0));
  sp = __fadd_rn(__fmul_rn(sp, t2), (float)(1.0 / 120.0));
  sp = __fadd_rn(__fmul_rn(sp, t2), (float)(-1.0 / 6.0));
  sp = __fadd_rn(__fmul_rn(sp, t2), 1.0f);
  const float sin_t = __fmul_rn(theta, sp);
  float cp = (float)(1.0 / 479001600.0);
  cp = __fadd_rn(__fmul_rn(cp, t2), (float)(-1.0 / 3628800.0));
  cp = __fadd_rn(__fmul_rn(cp, t2), (float)(1.0 / 40320.0));
  cp = __fadd_rn(__fmul_rn(cp, t2), (float)(-1.0 / 720.0));
  cp = __fadd_rn(__fmul_rn(cp, t2), (float)(1.0 / 24.0));
  cp = __fadd_rn(__fmul_rn(cp, t2), -0.5f);
  cp = __fadd_rn(__fmul_rn(cp, t2), 1.0f);
  const float c = quad == 0 ? cp : (quad == 1 ? -sin_t : (quad == 2 ? -cp : sin_t));
  return __fmul_rn(r, c);
}

__device__ __forceinline__ uint32_t bf16_rne(float f) {
  uint32_t b = __float_as_uint(f);
  b = b + 0x7FFFu + ((b >> 16) & 1u);
  return b >> 16;
}

struct FillArgs {
  uint16_t* out;
  long long n0, n1, n2, n3;     // logical shape, n3 contiguous and a multiple of 8
  long long s0, s1, s2;         // element strides of the first three axes
  uint64_t key, counter0;
  const float* scale;           // optional, indexed along scale_axis
  int scale_axis;
};

__global__ __launch_bounds__(256) void fill_normal_bf16_kernel(FillArgs a) {
  const long long groups_per_row = a.n3 / 8;
  const long long total = a.n0 * a.n1 * a.n2 * groups_per_row;
  const long long step = (long long)gridDim.x * blockDim.x;
  for (long long gidx = (long long)blockIdx.x * blockDim.x + threadIdx.x; gidx < total; gidx += step) {
    const long long c8 = gidx % groups_per_row;
    long long r = gidx / groups_per_row;
    const long long i2 = r % a.n2; r /= a.n2;
    const long long i1 = r % a.n1;
    const long long i0 = r / a.n1;
    const uint64_t flat = (uint64_t)(((i0 * a.n1 + i1) * a.n2 + i2) * a.n3 + c8 * 8);
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float z0 = normal_f32(a.key, a.counter0 + flat + 2 * j);
      float z1 = normal_f32(a.key, a.counter0 + flat + 2 * j + 1);
      if (a.scale) {
        if (a.scale_axis == 3) {
          z0 = __fmul_rn(z0, a.scale[c8 * 8 + 2 * j]);
          z1 = __fmul_rn(z1, a.scale[c8 * 8 + 2 * j + 1]);
        } else {
          const float sc = a.scale[a.scale_axis == 0 ? i0 : (a.scale_axis == 1 ? i1 : i2)];
          z0 = __fmul_rn(z0, sc);
          z1 = __fmul_rn(z1, sc);
        }
      }
      w[j] = bf16_rne(z0) | (bf16_rne(z1) << 16);
    }
    *(u32x4*)(a.out + i0 * a.s0 + i1 * a.s1 + i2 * a.s2 + c8 * 8) = u32x4{w[0], w[1], w[2], w[3]};
  }
}

}  // namespace

// Fill a (possibly strided) 4-D bf16 tensor with scale * N(0,1); element (i0,i1,i2,i3) takes
// counter counter0 + row-major flat index in the LOGICAL shape.  Returns a hipError_t value.
extern "C" int synth_fill_normal_bf16(void* out, long long n0, long long n1, long long n2, long long n3,
                                      long long s0, long long s1, long long s2, unsigned long long key,
                                      unsigned long long counter0, const float* scale, int scale_axis,
                                      void* stream) {
  if (!out || n0 <= 0 || n1 <= 0 || n2 <= 0 || n3 <= 0 || (n3 & 7) || ((uintptr_t)out & 15)) return (int)hipErrorInvalidValue;
  if ((s0 | s1 | s2) & 7) return (int)hipErrorInvalidValue;
  if (scale_axis < 0 || scale_axis > 3) return (int)hipErrorInvalidValue;
  FillArgs a{(uint16_t*)out, n0, n1, n2, n3, s0, s1, s2, key, counter0, scale, scale_axis};
  const long long total = n0 * n1 * n2 * (n3 / 8);
  long long blocks = (total + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(fill_normal_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}
