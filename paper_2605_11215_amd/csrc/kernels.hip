// gfx950 kernels of the gradient path.  Every step is an elementwise stream over flat fp32
// buffers, bound by HBM bandwidth, so the design is the same everywhere: one 128-bit load or
// store per lane per access (a wavefront moves 1 KiB of consecutive bytes per instruction),
// one-wavefront workgroups with one tile each (a finished wavefront frees its slot at once; measured
// 4 % faster than four-wavefront groups), U independent vectors in flight per lane before the first
// use, 64-bit element indices (a shard can exceed 2^32 bytes), no LDS (no element is used twice) and
// no atomics (the sums have a fixed order).  Ranges that do not start or end on a 16-byte boundary
// get their ragged ends from a few lanes of workgroup 0.
#include "kernels.h"

#include <type_traits>

namespace recover {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

Tuning &tuning() {
  static Tuning t;
  return t;
}

// A range [begin, end) of elements split into a ragged head, nvec aligned 4-element vectors
// starting at element vbegin, and a ragged tail.
struct Span {
  size_t begin, end, vbegin, nvec;
};

static Span make_span(size_t begin, size_t end) {
  Span s;
  s.begin = begin;
  s.end = end;
  size_t vb = (begin + 3) & ~size_t(3);
  if (vb > end) vb = end;
  s.vbegin = vb;
  s.nvec = (end - vb) / 4;
  return s;
}

// Element index of the k-th ragged element (head first, then tail), or end if k is past them.
__device__ inline size_t ragged_index(const Span &sp, unsigned k) {
  size_t head = sp.vbegin - sp.begin;
  if (k < head) return sp.begin + k;
  size_t i = sp.vbegin + sp.nvec * 4 + (k - head);
  return i < sp.end ? i : sp.end;
}

template <bool NT, typename T>
__device__ inline T ld(const T *p) {
  if (NT) return __builtin_nontemporal_load(p);
  return *p;
}
template <bool NT, typename T>
__device__ inline void st(T *p, T v) {
  if (NT)
    __builtin_nontemporal_store(v, p);
  else
    *p = v;
}

__device__ inline float bf16_to_f32(uint32_t h) { return __builtin_bit_cast(float, h << 16); }

// Four gradient elements of vector i, widened to fp32.
template <bool NT>
__device__ inline f32x4 load_grad(const float *g, size_t i) {
  return ld<NT>(reinterpret_cast<const f32x4 *>(g) + i);
}
template <bool NT>
__device__ inline f32x4 load_grad(const uint16_t *g, size_t i) {
  u32x2 w = ld<NT>(reinterpret_cast<const u32x2 *>(g) + i);
  f32x4 r;
  r.x = __builtin_bit_cast(float, w.x << 16);
  r.y = __builtin_bit_cast(float, w.x & 0xFFFF0000u);
  r.z = __builtin_bit_cast(float, w.y << 16);
  r.w = __builtin_bit_cast(float, w.y & 0xFFFF0000u);
  return r;
}
__device__ inline float load_grad1(const float *g, size_t i) { return g[i]; }
__device__ inline float load_grad1(const uint16_t *g, size_t i) { return bf16_to_f32(g[i]); }

// ---------------------------------------------------------------------------------------------
// accumulate: acc[i] = acc[i] + widen(g[i]);  FIRST: acc[i] = (+0) + widen(g[i])
// ---------------------------------------------------------------------------------------------
template <typename G, int T, int U, bool NT, bool FIRST, bool SNAP>
__global__ __launch_bounds__(T) void k_accumulate(float *__restrict__ acc, float *__restrict__ snap,
                                                  const G *__restrict__ g, Span sp, size_t ntiles, int xcd_chunked) {
  f32x4 *a4 = reinterpret_cast<f32x4 *>(acc + sp.vbegin);
  f32x4 *s4 = SNAP ? reinterpret_cast<f32x4 *>(snap + sp.vbegin) : nullptr;
  const G *gv = g + sp.vbegin;
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
  size_t first = blockIdx.x, stride = gridDim.x;
  if (xcd_chunked) {  // grid = 8 * ceil(ntiles / 8): one tile per workgroup, XCD x owns the x-th eighth
    first = size_t(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    stride = ntiles;
  }
  for (size_t tile = first; tile < ntiles; tile += stride) {
    const size_t base = tile * size_t(T * U) + threadIdx.x;
    f32x4 x[U], a[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) ok[u] = base + size_t(T) * u < sp.nvec;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) x[u] = load_grad<NT>(gv, base + size_t(T) * u);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) a[u] = FIRST ? zero : ld<NT>(a4 + base + size_t(T) * u);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (ok[u]) {
        const f32x4 r = a[u] + x[u];
        st<NT>(a4 + base + size_t(T) * u, r);
        if (SNAP) st<NT>(s4 + base + size_t(T) * u, r);
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < 8) {
    const size_t i = ragged_index(sp, threadIdx.x);
    if (i < sp.end) {
      const float r = (FIRST ? 0.f : acc[i]) + load_grad1(g, i);
      acc[i] = r;
      if (SNAP) snap[i] = r;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// accumulate for several replicas in one launch (blockIdx.y = pair index): same arithmetic per pair
// as k_accumulate; for shards so small that the launch, not HBM, bounds a single accumulate.
// ---------------------------------------------------------------------------------------------
template <typename G, int T, bool NT>
__global__ __launch_bounds__(T) void k_accumulate_many(AccumulateManyArgs a, Span sp) {
  const int pair = blockIdx.y;
  float *acc = a.acc[pair];
  const G *g = static_cast<const G *>(a.grad[pair]);
  const bool first = a.first[pair] != 0;
  const size_t i = size_t(blockIdx.x) * T + threadIdx.x;
  if (i < sp.nvec) {
    f32x4 *a4 = reinterpret_cast<f32x4 *>(acc + sp.vbegin) + i;
    const f32x4 x = load_grad<NT>(g + sp.vbegin, i);
    f32x4 av = {0.f, 0.f, 0.f, 0.f};
    if (!first) av = ld<NT>(a4);
    st<NT>(a4, av + x);
  }
  if (blockIdx.x == 0 && threadIdx.x < 8) {
    const size_t e = ragged_index(sp, threadIdx.x);
    if (e < sp.end) acc[e] = (first ? 0.f : acc[e]) + load_grad1(g, e);
  }
}

// ---------------------------------------------------------------------------------------------
// copy (snapshot and restore): dst[i] = src[i]
// ---------------------------------------------------------------------------------------------
template <int T, int U, bool NT>
__global__ __launch_bounds__(T) void k_copy(float *__restrict__ dst, const float *__restrict__ src, Span sp,
                                                   size_t ntiles) {
  f32x4 *d4 = reinterpret_cast<f32x4 *>(dst + sp.vbegin);
  const f32x4 *s4 = reinterpret_cast<const f32x4 *>(src + sp.vbegin);
  for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const size_t base = tile * size_t(T * U) + threadIdx.x;
    f32x4 x[U];
    if (base + size_t(T) * (U - 1) < sp.nvec) {
#pragma unroll
      for (int u = 0; u < U; ++u) x[u] = ld<NT>(s4 + base + size_t(T) * u);
#pragma unroll
      for (int u = 0; u < U; ++u) st<NT>(d4 + base + size_t(T) * u, x[u]);
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const size_t i = base + size_t(T) * u;
        if (i < sp.nvec) st<NT>(d4 + i, ld<NT>(s4 + i));
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < 8) {
    const size_t i = ragged_index(sp, threadIdx.x);
    if (i < sp.end) dst[i] = src[i];
  }
}

// ---------------------------------------------------------------------------------------------
// reduce: out[i] = ((src0[i] + src1[i]) + ...) / divisor, ascending contributor order; in-place mode
// also stores the undivided sum to every sum_dst buffer.  A workgroup walks the contributors one
// after the other over its whole tile (U consecutive 4 KiB rows per contributor), two contributors'
// loads in flight at a time, so each of its bursts reads one buffer contiguously; every element's
// adds stay strictly left to right.
// ---------------------------------------------------------------------------------------------
template <int T, int U, bool NT, bool INPLACE>
__global__ __launch_bounds__(T) void k_reduce(ReduceArgs a, Span sp, size_t ntiles) {
  f32x4 *o4 = reinterpret_cast<f32x4 *>(a.out + sp.vbegin);
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
  for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const size_t base = tile * size_t(T * U) + threadIdx.x;
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) ok[u] = base + size_t(T) * u < sp.nvec;
    f32x4 sum[U];
#pragma unroll
    for (int u = 0; u < U; ++u) sum[u] = zero;
    int r = 0;
    if (a.n_src > 0) {
      const f32x4 *s0 = reinterpret_cast<const f32x4 *>(a.src[0] + sp.vbegin) + base;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) sum[u] = ld<NT>(s0 + size_t(T) * u);
      r = 1;
    }
    for (; r + 1 < a.n_src; r += 2) {
      const f32x4 *s0 = reinterpret_cast<const f32x4 *>(a.src[r] + sp.vbegin) + base;
      const f32x4 *s1 = reinterpret_cast<const f32x4 *>(a.src[r + 1] + sp.vbegin) + base;
      f32x4 t0[U], t1[U];
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) t0[u] = ld<NT>(s0 + size_t(T) * u);
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) t1[u] = ld<NT>(s1 + size_t(T) * u);
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) sum[u] = (sum[u] + t0[u]) + t1[u];
    }
    if (r < a.n_src) {
      const f32x4 *s0 = reinterpret_cast<const f32x4 *>(a.src[r] + sp.vbegin) + base;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) sum[u] = sum[u] + ld<NT>(s0 + size_t(T) * u);
    }
    if (INPLACE) {
      for (int d = 0; d < a.n_sum_dst; ++d) {
        f32x4 *dd = reinterpret_cast<f32x4 *>(a.sum_dst[d] + sp.vbegin) + base;
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (ok[u]) st<NT>(dd + size_t(T) * u, sum[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (ok[u]) {
        f32x4 q;
        q.x = sum[u].x / a.divisor;
        q.y = sum[u].y / a.divisor;
        q.z = sum[u].z / a.divisor;
        q.w = sum[u].w / a.divisor;
        st<NT>(o4 + base + size_t(T) * u, q);
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < 8) {
    const size_t i = ragged_index(sp, threadIdx.x);
    if (i < sp.end) {
      float sum = 0.f;
      for (int r = 0; r < a.n_src; ++r) sum = (r == 0) ? a.src[r][i] : sum + a.src[r][i];
      if (INPLACE)
        for (int d = 0; d < a.n_sum_dst; ++d) a.sum_dst[d][i] = sum;
      a.out[i] = sum / a.divisor;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// AdamW (decoupled weight decay), fp32 state:
//   p *= decay_mul;  m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g g;
//   p -= step_size * m / (sqrt(v) * inv_sqrt_bc2 + eps)
// with decay_mul = 1 - lr wd, step_size = lr / (1 - b1^t), inv_sqrt_bc2 = 1 / sqrt(1 - b2^t)
// prepared in double on the host.
// ---------------------------------------------------------------------------------------------
__global__ void k_adam_prologue(StepState *st, float lr, float beta1, float beta2, float eps, float weight_decay) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    double p1 = st->step ? st->beta1_pow : 1.0, p2 = st->step ? st->beta2_pow : 1.0;
    st->args = next_adam_args(p1, p2, lr, beta1, beta2, eps, weight_decay);
    st->beta1_pow = p1;
    st->beta2_pow = p2;
    st->step = st->step + 1;
  }
}

// The fused multiply-adds are written out so that every kernel that inlines this function rounds
// in the same places.
__device__ inline void adam1(float &p, float &m, float &v, float g, const AdamArgs &h) {
#pragma clang fp contract(off)
  m = __builtin_fmaf(h.beta1, m, h.one_minus_beta1 * g);
  v = __builtin_fmaf(h.beta2, v, h.one_minus_beta2 * (g * g));
  const float denom = __builtin_fmaf(sqrtf(v), h.inv_sqrt_bc2, h.eps);
  p = __builtin_fmaf(-h.step_size, m / denom, p * h.decay_mul);
}

__device__ inline uint32_t f32_to_bf16_rne(float x) {
  uint32_t b = __builtin_bit_cast(uint32_t, x);
  return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

template <int T, int U, bool NT, bool BF16OUT>
__global__ __launch_bounds__(T) void k_adamw(float *__restrict__ p, float *__restrict__ m,
                                                    float *__restrict__ v, const float *__restrict__ g,
                                                    uint16_t *__restrict__ pb, size_t n, AdamArgs h_arg,
                                                    const AdamArgs *h_dev, size_t ntiles) {
  const AdamArgs h = h_dev ? *h_dev : h_arg;
  const size_t nvec = n / 4;
  f32x4 *p4 = reinterpret_cast<f32x4 *>(p), *m4 = reinterpret_cast<f32x4 *>(m), *v4 = reinterpret_cast<f32x4 *>(v);
  const f32x4 *g4 = reinterpret_cast<const f32x4 *>(g);
  u32x2 *b2 = reinterpret_cast<u32x2 *>(pb);
  for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const size_t base = tile * size_t(T * U) + threadIdx.x;
    f32x4 gv[U], pv[U], mv[U], vv[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) ok[u] = base + size_t(T) * u < nvec;
    // one buffer after the other, U consecutive rows each
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) gv[u] = ld<NT>(g4 + base + size_t(T) * u);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) pv[u] = ld<NT>(p4 + base + size_t(T) * u);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) mv[u] = ld<NT>(m4 + base + size_t(T) * u);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) vv[u] = ld<NT>(v4 + base + size_t(T) * u);
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int l = 0; l < 4; ++l) {
        float pp = pv[u][l], mm = mv[u][l], v1 = vv[u][l];
        adam1(pp, mm, v1, gv[u][l], h);
        pv[u][l] = pp;
        mv[u][l] = mm;
        vv[u][l] = v1;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) st<NT>(p4 + base + size_t(T) * u, pv[u]);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) st<NT>(m4 + base + size_t(T) * u, mv[u]);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) st<NT>(v4 + base + size_t(T) * u, vv[u]);
    if (BF16OUT) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (ok[u]) {
          u32x2 w;
          w.x = f32_to_bf16_rne(pv[u].x) | (f32_to_bf16_rne(pv[u].y) << 16);
          w.y = f32_to_bf16_rne(pv[u].z) | (f32_to_bf16_rne(pv[u].w) << 16);
          st<NT>(b2 + base + size_t(T) * u, w);
        }
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < 4) {
    const size_t i = nvec * 4 + threadIdx.x;
    if (i < n) {
      float pp = p[i], mm = m[i], vv = v[i];
      adam1(pp, mm, vv, g[i], h);
      p[i] = pp;
      m[i] = mm;
      v[i] = vv;
      if (BF16OUT) pb[i] = (uint16_t)f32_to_bf16_rne(pp);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// fused reduce + AdamW: the contributor sum of k_reduce, its division, and the update of k_adamw in
// one pass; the gradient goes to HBM only if WRITE_GRAD.  4 R_c + 24 (+4) bytes per element.
// ---------------------------------------------------------------------------------------------
template <int T, bool NT, bool WRITE_GRAD, bool BF16OUT>
__global__ __launch_bounds__(T) void k_reduce_adamw(ReduceArgs a, float *__restrict__ p, float *__restrict__ m,
                                                    float *__restrict__ v, uint16_t *__restrict__ pb, Span sp,
                                                    AdamArgs h_arg, const AdamArgs *h_dev) {
  const AdamArgs h = h_dev ? *h_dev : h_arg;
  const size_t i = size_t(blockIdx.x) * T + threadIdx.x;
  if (i < sp.nvec) {
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    int r = 0;
    if (a.n_src > 0) {
      sum = ld<NT>(reinterpret_cast<const f32x4 *>(a.src[0] + sp.vbegin) + i);
      r = 1;
    }
    for (; r + 1 < a.n_src; r += 2) {
      const f32x4 t0 = ld<NT>(reinterpret_cast<const f32x4 *>(a.src[r] + sp.vbegin) + i);
      const f32x4 t1 = ld<NT>(reinterpret_cast<const f32x4 *>(a.src[r + 1] + sp.vbegin) + i);
      sum = (sum + t0) + t1;
    }
    if (r < a.n_src) sum = sum + ld<NT>(reinterpret_cast<const f32x4 *>(a.src[r] + sp.vbegin) + i);
    f32x4 *p4 = reinterpret_cast<f32x4 *>(p + sp.vbegin) + i;
    f32x4 *m4 = reinterpret_cast<f32x4 *>(m + sp.vbegin) + i;
    f32x4 *v4 = reinterpret_cast<f32x4 *>(v + sp.vbegin) + i;
    f32x4 pv = ld<NT>(p4), mv = ld<NT>(m4), vv = ld<NT>(v4), q;
#pragma unroll
    for (int l = 0; l < 4; ++l) {
      q[l] = sum[l] / a.divisor;
      float pp = pv[l], mm = mv[l], v1 = vv[l];
      adam1(pp, mm, v1, q[l], h);
      pv[l] = pp;
      mv[l] = mm;
      vv[l] = v1;
    }
    st<NT>(p4, pv);
    st<NT>(m4, mv);
    st<NT>(v4, vv);
    if (WRITE_GRAD) st<NT>(reinterpret_cast<f32x4 *>(a.out + sp.vbegin) + i, q);
    if (BF16OUT) {
      u32x2 w;
      w.x = f32_to_bf16_rne(pv.x) | (f32_to_bf16_rne(pv.y) << 16);
      w.y = f32_to_bf16_rne(pv.z) | (f32_to_bf16_rne(pv.w) << 16);
      st<NT>(reinterpret_cast<u32x2 *>(pb + sp.vbegin) + i, w);
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < 8) {
    const size_t e = ragged_index(sp, threadIdx.x);
    if (e < sp.end) {
      float sum = 0.f;
      for (int r = 0; r < a.n_src; ++r) sum = (r == 0) ? a.src[r][e] : sum + a.src[r][e];
      const float q = sum / a.divisor;
      float pp = p[e], mm = m[e], v1 = v[e];
      adam1(pp, mm, v1, q, h);
      p[e] = pp;
      m[e] = mm;
      v[e] = v1;
      if (WRITE_GRAD) a.out[e] = q;
      if (BF16OUT) pb[e] = (uint16_t)f32_to_bf16_rne(pp);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// compare (verification support, off the timed path): bitwise mismatch count, max |x - ref|,
// max |ref|, NaN count and two position-weighted 64-bit checksums of two fp32 buffers, without
// moving them to the host.  Each lane folds its elements, a wavefront folds its 64 lanes with
// cross-lane shuffles, one lane per wavefront adds to the result with integer atomics (sums and
// maxima of integers do not depend on the order, so the result is reproducible).
// ---------------------------------------------------------------------------------------------
__device__ inline uint64_t wave_sum_u64(uint64_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}
__device__ inline uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const uint32_t o = (uint32_t)__shfl_xor((int)v, d, 64);
    v = o > v ? o : v;
  }
  return v;
}

__global__ __launch_bounds__(256) void k_compare_clear(CompareResult *out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    out->n_mismatch = out->n_nan = out->checksum_x = out->checksum_ref = 0;
    out->max_abs_diff_bits = out->max_abs_ref_bits = 0;
  }
}

__global__ __launch_bounds__(256) void k_compare(const float *__restrict__ x, const float *__restrict__ ref, size_t n,
                                                 CompareResult *out) {
  uint64_t mism = 0, nans = 0, cx = 0, cr = 0;
  uint32_t mdiff = 0, mref = 0;  // bit patterns of non-negative floats order like the floats
  for (size_t i = size_t(blockIdx.x) * 256 + threadIdx.x; i < n; i += size_t(gridDim.x) * 256) {
    const float a = x[i], b = ref[i];
    const uint32_t ab = __builtin_bit_cast(uint32_t, a), bb = __builtin_bit_cast(uint32_t, b);
    mism += ab != bb;
    cx += uint64_t(ab) * (2 * uint64_t(i) + 1);
    cr += uint64_t(bb) * (2 * uint64_t(i) + 1);
    if (a != a || b != b) {
      nans += 1;
    } else {
      const uint32_t d = __builtin_bit_cast(uint32_t, __builtin_fabsf(a - b));
      const uint32_t r = bb & 0x7FFFFFFFu;
      mdiff = d > mdiff ? d : mdiff;
      mref = r > mref ? r : mref;
    }
  }
  mism = wave_sum_u64(mism);
  nans = wave_sum_u64(nans);
  cx = wave_sum_u64(cx);
  cr = wave_sum_u64(cr);
  mdiff = wave_max_u32(mdiff);
  mref = wave_max_u32(mref);
  if ((threadIdx.x & 63) == 0) {
    atomicAdd(reinterpret_cast<unsigned long long *>(&out->n_mismatch), (unsigned long long)mism);
    atomicAdd(reinterpret_cast<unsigned long long *>(&out->n_nan), (unsigned long long)nans);
    atomicAdd(reinterpret_cast<unsigned long long *>(&out->checksum_x), (unsigned long long)cx);
    atomicAdd(reinterpret_cast<unsigned long long *>(&out->checksum_ref), (unsigned long long)cr);
    atomicMax(&out->max_abs_diff_bits, mdiff);
    atomicMax(&out->max_abs_ref_bits, mref);
  }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
static bool grid_for(size_t nvec, int T, int U, unsigned *grid, size_t *ntiles) {
  size_t tiles = (nvec + size_t(T) * U - 1) / (size_t(T) * U);
  *ntiles = tiles;
  size_t g = tiles ? tiles : 1;
  int cap = tuning().grid_cap;
  if (cap > 0 && g > size_t(cap)) g = size_t(cap);
  if (g > 0x7FFFFFFFull) return false;
  *grid = (unsigned)g;
  return true;
}

template <int V>
using Int = std::integral_constant<int, V>;

// Calls f(Int<T>, Int<U>, bool_constant<NT>) for the run-time launch shape.
template <typename F>
static void with_shape(int T, int U, bool NT, F &&f) {
  auto with_u = [&](auto t, auto nt) {
    switch (U) {
      case 2: f(t, Int<2>{}, nt); break;
      case 4: f(t, Int<4>{}, nt); break;
      default: f(t, Int<1>{}, nt); break;
    }
  };
  auto with_nt = [&](auto t) {
    if (NT)
      with_u(t, std::true_type{});
    else
      with_u(t, std::false_type{});
  };
  if (T == 256)
    with_nt(Int<256>{});
  else
    with_nt(Int<64>{});
}

hipError_t launch_accumulate(float *acc, float *snap, const void *grad, bool grad_is_bf16, bool first, size_t begin,
                             size_t end, hipStream_t s) {
  if (begin >= end) return hipSuccess;
  const Span sp = make_span(begin, end);
  const int Uv = tuning().vecs_per_thread, Tv = tuning().threads;
  unsigned grid;
  size_t ntiles;
  if (!grid_for(sp.nvec, Tv, Uv, &grid, &ntiles)) return hipErrorInvalidConfiguration;
  const int xc = tuning().xcd_chunked && tuning().grid_cap == 0 && ntiles >= 64 ? 1 : 0;
  if (xc) grid = (unsigned)(((ntiles + 7) / 8) * 8);
  with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
    constexpr int T = decltype(t)::value, U = decltype(u)::value;
    constexpr bool NT = decltype(nt)::value;
    auto go = [&](auto gptr, auto is_first, auto with_snap) {
      using GT = std::remove_cv_t<std::remove_pointer_t<decltype(gptr)>>;
      hipLaunchKernelGGL((k_accumulate<GT, T, U, NT, decltype(is_first)::value, decltype(with_snap)::value>), dim3(grid),
                         dim3(T), 0, s, acc, snap, gptr, sp, ntiles, xc);
    };
    auto pick = [&](auto gptr) {
      if (first) {
        if (snap) go(gptr, std::true_type{}, std::true_type{});
        else go(gptr, std::true_type{}, std::false_type{});
      } else {
        if (snap) go(gptr, std::false_type{}, std::true_type{});
        else go(gptr, std::false_type{}, std::false_type{});
      }
    };
    if (grad_is_bf16)
      pick(static_cast<const uint16_t *>(grad));
    else
      pick(static_cast<const float *>(grad));
  });
  return hipGetLastError();
}

hipError_t launch_accumulate_many(const AccumulateManyArgs &a, int n_pairs, bool grad_is_bf16, size_t begin, size_t end,
                                  hipStream_t s) {
  if (begin >= end || n_pairs <= 0) return hipSuccess;
  const Span sp = make_span(begin, end);
  const size_t tiles = (sp.nvec + 63) / 64;
  if (tiles > 0x7FFFFFFFull || n_pairs > kMaxReplicas) return hipErrorInvalidConfiguration;
  const dim3 grid(tiles ? (unsigned)tiles : 1u, (unsigned)n_pairs);
  const bool nt = tuning().nontemporal;
  if (grad_is_bf16) {
    if (nt) hipLaunchKernelGGL((k_accumulate_many<uint16_t, 64, true>), grid, dim3(64), 0, s, a, sp);
    else hipLaunchKernelGGL((k_accumulate_many<uint16_t, 64, false>), grid, dim3(64), 0, s, a, sp);
  } else {
    if (nt) hipLaunchKernelGGL((k_accumulate_many<float, 64, true>), grid, dim3(64), 0, s, a, sp);
    else hipLaunchKernelGGL((k_accumulate_many<float, 64, false>), grid, dim3(64), 0, s, a, sp);
  }
  return hipGetLastError();
}

hipError_t launch_copy(float *dst, const float *src, size_t begin, size_t end, hipStream_t s) {
  if (begin >= end) return hipSuccess;
  const Span sp = make_span(begin, end);
  const int Uv = tuning().copy_vecs, Tv = tuning().threads;
  unsigned grid;
  size_t ntiles;
  if (!grid_for(sp.nvec, Tv, Uv, &grid, &ntiles)) return hipErrorInvalidConfiguration;
  with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
    constexpr int T = decltype(t)::value, U = decltype(u)::value;
    constexpr bool NT = decltype(nt)::value;
    hipLaunchKernelGGL((k_copy<T, U, NT>), dim3(grid), dim3(T), 0, s, dst, src, sp, ntiles);
  });
  return hipGetLastError();
}

hipError_t launch_reduce(const ReduceArgs &a, size_t begin, size_t end, hipStream_t s) {
  if (begin >= end) return hipSuccess;
  const Span sp = make_span(begin, end);
  const int Uv = tuning().reduce_vecs, Tv = tuning().threads;
  unsigned grid;
  size_t ntiles;
  if (!grid_for(sp.nvec, Tv, Uv, &grid, &ntiles)) return hipErrorInvalidConfiguration;
  const bool inplace = a.n_sum_dst > 0;
  with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
    constexpr int T = decltype(t)::value, U = decltype(u)::value;
    constexpr bool NT = decltype(nt)::value;
    if (inplace)
      hipLaunchKernelGGL((k_reduce<T, U, NT, true>), dim3(grid), dim3(T), 0, s, a, sp, ntiles);
    else
      hipLaunchKernelGGL((k_reduce<T, U, NT, false>), dim3(grid), dim3(T), 0, s, a, sp, ntiles);
  });
  return hipGetLastError();
}

hipError_t launch_adam_prologue(StepState *st, float lr, float beta1, float beta2, float eps, float weight_decay,
                                hipStream_t s) {
  hipLaunchKernelGGL(k_adam_prologue, dim3(1), dim3(64), 0, s, st, lr, beta1, beta2, eps, weight_decay);
  return hipGetLastError();
}

hipError_t launch_adamw(float *p, float *m, float *v, const float *g, uint16_t *p_bf16, size_t n, const AdamArgs &h,
                        const AdamArgs *device_args, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const int Uv = tuning().adamw_vecs, Tv = tuning().threads;
  unsigned grid;
  size_t ntiles;
  if (!grid_for(n / 4, Tv, Uv, &grid, &ntiles)) return hipErrorInvalidConfiguration;
  with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
    constexpr int T = decltype(t)::value, U = decltype(u)::value;
    constexpr bool NT = decltype(nt)::value;
    if (p_bf16)
      hipLaunchKernelGGL((k_adamw<T, U, NT, true>), dim3(grid), dim3(T), 0, s, p, m, v, g, p_bf16, n, h, device_args,
                         ntiles);
    else
      hipLaunchKernelGGL((k_adamw<T, U, NT, false>), dim3(grid), dim3(T), 0, s, p, m, v, g, p_bf16, n, h, device_args,
                         ntiles);
  });
  return hipGetLastError();
}

hipError_t launch_reduce_adamw(const ReduceArgs &a, float *p, float *m, float *v, uint16_t *p_bf16, bool write_grad,
                               size_t begin, size_t end, const AdamArgs &h, const AdamArgs *device_args,
                               hipStream_t s) {
  if (begin >= end) return hipSuccess;
  const Span sp = make_span(begin, end);
  const size_t tiles = (sp.nvec + 63) / 64;  // one tile per one-wavefront workgroup, no grid cap
  if (tiles > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
  const unsigned grid = tiles ? (unsigned)tiles : 1u;
  auto go = [&](auto nt, auto wg, auto bf) {
    hipLaunchKernelGGL((k_reduce_adamw<64, decltype(nt)::value, decltype(wg)::value, decltype(bf)::value>), dim3(grid),
                       dim3(64), 0, s, a, p, m, v, p_bf16, sp, h, device_args);
  };
  auto with_bf = [&](auto nt, auto wg) {
    if (p_bf16) go(nt, wg, std::true_type{});
    else go(nt, wg, std::false_type{});
  };
  auto with_wg = [&](auto nt) {
    if (write_grad) with_bf(nt, std::true_type{});
    else with_bf(nt, std::false_type{});
  };
  if (tuning().nontemporal) with_wg(std::true_type{});
  else with_wg(std::false_type{});
  return hipGetLastError();
}

hipError_t launch_compare(const float *x, const float *ref, size_t n, CompareResult *out, hipStream_t s) {
  hipLaunchKernelGGL(k_compare_clear, dim3(1), dim3(256), 0, s, out);
  if (n > 0) {
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(k_compare, dim3((unsigned)blocks), dim3(256), 0, s, x, ref, n, out);
  }
  return hipGetLastError();
}

}  // namespace recover
