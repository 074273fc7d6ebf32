// Device twin of reference_np.py: the same seeded input streams, generated in HBM.
// INPUTS only (gradient streams, initial parameters); none of the gradient path's arithmetic.
//
//   Philox4x32-10, key = (seed, tag), counter = (c0, mb_id, iter, kind)
//   kind 0 Gaussian: c0 = i >> 2, element i takes lane i & 3;  kind 1 Student-t(3): c0 = i
//   u = odd 24-bit numerator / 2^24; Box-Muller on (u0,u1) and (u2,u3)
//   value = fp32(scale * z)   or   fp32(scale * z0 / sqrt((z1^2 + z2^2 + z3^2) / 3))
//
// ln, cos, sin follow the fixed fp64 operation sequences of the NumPy file (+, -, *, /, sqrt,
// each correctly rounded, nothing fused: this file is compiled with -ffp-contract=off), so the
// two sides return the same bits.
#include <hip/hip_runtime.h>
#include <stdint.h>

#pragma clang fp contract(off)

namespace {

struct Words {
  uint32_t x[4];
};

__device__ inline Words philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  Words w = {{c0, c1, c2, c3}};
  return w;
}

__device__ inline uint32_t numerator(uint32_t x) { return ((x >> 9) << 1) | 1u; }

// ln(n / 2^24), n odd in [1, 2^24)
__device__ inline double ln_u(uint32_t n) {
  int e = 31 - __clz(n);
  double m = (double)n / (double)(1u << e);  // [1, 2), exact
  if (m > 1.4142135623730951) {
    m = m * 0.5;
    e += 1;
  }
  const double s = (m - 1.0) / (m + 1.0);
  const double s2 = s * s;
  double acc = 2.0 / 25.0;
  acc = acc * s2 + 2.0 / 23.0;
  acc = acc * s2 + 2.0 / 21.0;
  acc = acc * s2 + 2.0 / 19.0;
  acc = acc * s2 + 2.0 / 17.0;
  acc = acc * s2 + 2.0 / 15.0;
  acc = acc * s2 + 2.0 / 13.0;
  acc = acc * s2 + 2.0 / 11.0;
  acc = acc * s2 + 2.0 / 9.0;
  acc = acc * s2 + 2.0 / 7.0;
  acc = acc * s2 + 2.0 / 5.0;
  acc = acc * s2 + 2.0 / 3.0;
  acc = acc * s2 + 2.0;
  return (double)(e - 24) * 0.6931471805599453 + s * acc;
}

// cos and sin of 2 pi n / 2^24, n odd in [1, 2^24)
__device__ inline void cos_sin_2pi_u(uint32_t n, double *c, double *s) {
  const int q = (int)(n >> 22);
  int r = (int)(n & ((1u << 22) - 1));
  const bool flip = r > (1 << 21);
  if (flip) r = (1 << 22) - r;
  const double th = ((double)r * (1.0 / 4194304.0)) * 1.5707963267948966;
  const double t2 = th * th;
  double sp = 1.0 / 355687428096000.0;
  sp = sp * t2 + -1.0 / 1307674368000.0;
  sp = sp * t2 + 1.0 / 6227020800.0;
  sp = sp * t2 + -1.0 / 39916800.0;
  sp = sp * t2 + 1.0 / 362880.0;
  sp = sp * t2 + -1.0 / 5040.0;
  sp = sp * t2 + 1.0 / 120.0;
  sp = sp * t2 + -1.0 / 6.0;
  sp = sp * t2 + 1.0;
  sp = sp * th;
  double cp = -1.0 / 6402373705728000.0;
  cp = cp * t2 + 1.0 / 20922789888000.0;
  cp = cp * t2 + -1.0 / 87178291200.0;
  cp = cp * t2 + 1.0 / 479001600.0;
  cp = cp * t2 + -1.0 / 3628800.0;
  cp = cp * t2 + 1.0 / 40320.0;
  cp = cp * t2 + -1.0 / 720.0;
  cp = cp * t2 + 1.0 / 24.0;
  cp = cp * t2 + -1.0 / 2.0;
  cp = cp * t2 + 1.0;
  const double c1 = flip ? sp : cp;
  const double s1 = flip ? cp : sp;
  *c = q == 0 ? c1 : (q == 1 ? -s1 : (q == 2 ? -c1 : s1));
  *s = q == 0 ? s1 : (q == 1 ? c1 : (q == 2 ? -s1 : -c1));
}

__device__ inline void four_normals(const Words &w, double z[4]) {
  double c, s;
  const double ra = sqrt(-2.0 * ln_u(numerator(w.x[0])));
  cos_sin_2pi_u(numerator(w.x[1]), &c, &s);
  z[0] = ra * c;
  z[1] = ra * s;
  const double rb = sqrt(-2.0 * ln_u(numerator(w.x[2])));
  cos_sin_2pi_u(numerator(w.x[3]), &c, &s);
  z[2] = rb * c;
  z[3] = rb * s;
}

__device__ inline uint16_t bf16_rne(float x) {
  const uint32_t b = __builtin_bit_cast(uint32_t, x);
  if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((b >> 16) | 0x40u);  // a NaN stays a NaN
  return (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}

__device__ inline void put(float *out, size_t i, float v) { out[i] = v; }
__device__ inline void put(uint16_t *out, size_t i, float v) { out[i] = bf16_rne(v); }

// One thread per group of four consecutive elements (Gaussian) starting at a multiple of four.
template <typename T>
__global__ __launch_bounds__(256) void k_normal(T *out, size_t start, size_t n, uint32_t seed, uint32_t tag,
                                                uint32_t mb_id, uint32_t iter, double scale) {
  const size_t q0 = start >> 2, q1 = (start + n + 3) >> 2;
  for (size_t q = q0 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; q < q1; q += (size_t)gridDim.x * blockDim.x) {
    double z[4];
    four_normals(philox4x32_10((uint32_t)q, mb_id, iter, 0u, seed, tag), z);
#pragma unroll
    for (int l = 0; l < 4; ++l) {
      const size_t i = q * 4 + l;
      if (i >= start && i < start + n) put(out, i - start, (float)(scale * z[l]));
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void k_student_t3(T *out, size_t start, size_t n, uint32_t seed, uint32_t tag,
                                                    uint32_t mb_id, uint32_t iter, double scale) {
  for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += (size_t)gridDim.x * blockDim.x) {
    const size_t i = start + k;
    double z[4];
    four_normals(philox4x32_10((uint32_t)i, mb_id, iter, 1u, seed, tag), z);
    const double den = sqrt(((z[1] * z[1] + z[2] * z[2]) + z[3] * z[3]) / 3.0);
    put(out, k, (float)((scale * z[0]) / den));
  }
}

}  // namespace

extern "C" {

// Fill out[0..n) (device; fp32 if !bf16 else bf16 bit patterns) with stream elements
// start .. start+n-1.  kind 0 Gaussian, 1 Student-t(3).  Asynchronous on `stream`.
// The element index goes into one 32-bit counter word: the Gaussian stream packs four elements per counter
// (indices below 2^34), the Student-t stream one (below 2^32).
// Returns 0, -1 on a bad argument, -4 on a HIP error.
int synth_fill(void *out, int bf16, uint64_t start, uint64_t n, uint32_t seed, uint32_t tag, uint32_t mb_id,
               uint32_t iter, double scale, int kind, void *stream) {
  if (!out || (kind != 0 && kind != 1) || start + n > (kind == 0 ? 1ull << 34 : 1ull << 32)) return -1;
  if (n == 0) return 0;
  hipStream_t s = (hipStream_t)stream;
  const size_t work = kind == 0 ? ((start + n + 3) >> 2) - (start >> 2) : n;
  size_t blocks = (work + 255) / 256;
  if (blocks > 65536 * 16) blocks = 65536 * 16;
  if (kind == 0) {
    if (bf16)
      hipLaunchKernelGGL(k_normal<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, s, (uint16_t *)out, (size_t)start, (size_t)n, seed, tag, mb_id, iter, scale);
    else
      hipLaunchKernelGGL(k_normal<float>, dim3((unsigned)blocks), dim3(256), 0, s, (float *)out, (size_t)start, (size_t)n, seed, tag, mb_id, iter, scale);
  } else {
    if (bf16)
      hipLaunchKernelGGL(k_student_t3<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, s, (uint16_t *)out, (size_t)start, (size_t)n, seed, tag, mb_id, iter, scale);
    else
      hipLaunchKernelGGL(k_student_t3<float>, dim3((unsigned)blocks), dim3(256), 0, s, (float *)out, (size_t)start, (size_t)n, seed, tag, mb_id, iter, scale);
  }
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
