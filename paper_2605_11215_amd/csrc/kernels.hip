// gfx950 kernels of the gradient path.  Every step is an elementwise stream over flat fp32
// buffers, bound by HBM bandwidth, so the design is the same everywhere: one 128-bit load or
// store per lane per access (a wavefront moves 1 KiB of consecutive bytes per instruction),
// one-wavefront workgroups with one tile each (a finished wavefront frees its slot at once; measured
// 4 % faster than four-wavefront groups), U independent vectors in flight per lane before the first
// use, 64-bit element indices (a shard can exceed 2^32 bytes), no LDS (no element is used twice) and
// no atomics (the sums have a fixed order).  Ranges that do not start or end on a 16-byte boundary
// get their ragged ends from a few lanes of workgroup 0.
//
// Every kernel body exists twice, selected by a wavefront-uniform test: FULL tiles (all but at most
// the last one) run without any per-lane bounds test, so all their loads are issued back to back
// before the first wait; the last, partial tile masks each access.  Raw bf16 words are widened only
// after every load of the tile has been issued (widening right after the load would put a wait
// between the gradient load and the accumulator load).
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

using True = std::true_type;
using False = std::false_type;

// Runs body(True) on a full tile and body(False) on the partial one; `full` is wavefront-uniform.
template <typename F>
__device__ inline void on_tile(bool full, F &&body) {
  if (full)
    body(True{});
  else
    body(False{});
}

__device__ inline float bf16_to_f32(uint32_t h) { return __builtin_bit_cast(float, h << 16); }

// Four gradient elements as they lie in memory (fp32: one 128-bit vector; bf16: one 64-bit vector),
// and their fp32 values.
template <typename G>
struct Grad4;
template <>
struct Grad4<float> {
  typedef f32x4 raw;
  __device__ static inline f32x4 widen(raw w) { return w; }
};
template <>
struct Grad4<uint16_t> {
  typedef u32x2 raw;
  __device__ static inline f32x4 widen(raw w) {
    f32x4 r;
    r.x = __builtin_bit_cast(float, w.x << 16);
    r.y = __builtin_bit_cast(float, w.x & 0xFFFF0000u);
    r.z = __builtin_bit_cast(float, w.y << 16);
    r.w = __builtin_bit_cast(float, w.y & 0xFFFF0000u);
    return r;
  }
};
__device__ inline float load_grad1(const float *g, size_t i) { return g[i]; }
__device__ inline float load_grad1(const uint16_t *g, size_t i) { return bf16_to_f32(g[i]); }

// ---------------------------------------------------------------------------------------------
// accumulate: acc[i] = acc[i] + widen(g[i]);  FIRST: acc[i] = (+0) + widen(g[i])
// ---------------------------------------------------------------------------------------------
template <typename G, int T, int U, bool NT, bool FIRST, bool SNAP>
__device__ inline void accumulate_tiles(float *__restrict__ acc, float *__restrict__ snap, const G *__restrict__ g,
                                        const Span &sp, size_t first, size_t stride, size_t ntiles) {
  typedef typename Grad4<G>::raw Raw;
  f32x4 *a4 = reinterpret_cast<f32x4 *>(acc + sp.vbegin);
  f32x4 *s4 = SNAP ? reinterpret_cast<f32x4 *>(snap + sp.vbegin) : nullptr;
  const Raw *g4 = reinterpret_cast<const Raw *>(g + sp.vbegin);
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
  for (size_t tile = first; tile < ntiles; tile += stride) {
    const size_t base = tile * size_t(T * U) + threadIdx.x;
    on_tile((tile + 1) * size_t(T * U) <= sp.nvec, [&](auto full) {
      constexpr bool FULL = decltype(full)::value;
      Raw x[U];
      f32x4 a[U];
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; ++u) ok[u] = FULL || base + size_t(T) * u < sp.nvec;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) x[u] = ld<NT>(g4 + base + size_t(T) * u);
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) a[u] = FIRST ? zero : ld<NT>(a4 + base + size_t(T) * u);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (ok[u]) {
          const f32x4 r = a[u] + Grad4<G>::widen(x[u]);
          st<NT>(a4 + base + size_t(T) * u, r);
          if (SNAP) st<NT>(s4 + base + size_t(T) * u, r);
        }
      }
    });
  }
}

template <typename G, int T, int U, bool NT, bool FIRST, bool SNAP>
__global__ __launch_bounds__(T) void k_accumulate(float *__restrict__ acc, float *__restrict__ snap,
                                                  const G *__restrict__ g, Span sp, size_t ntiles, int xcd_chunked) {
  size_t first = blockIdx.x, stride = gridDim.x;
  if (xcd_chunked) {  // grid = 8 * ceil(ntiles / 8): one tile per workgroup, XCD x owns the x-th eighth
    first = size_t(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    stride = ntiles;
  }
  accumulate_tiles<G, T, U, NT, FIRST, SNAP>(acc, snap, g, sp, first, stride, ntiles);
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
  const size_t ntiles = (sp.nvec + T - 1) / T;
  if (a.first[pair])
    accumulate_tiles<G, T, 1, NT, true, false>(acc, nullptr, g, sp, blockIdx.x, gridDim.x, ntiles);
  else
    accumulate_tiles<G, T, 1, NT, false, false>(acc, nullptr, g, sp, blockIdx.x, gridDim.x, ntiles);
  if (blockIdx.x == 0 && threadIdx.x < 8) {
    const size_t e = ragged_index(sp, threadIdx.x);
    if (e < sp.end) acc[e] = (a.first[pair] ? 0.f : acc[e]) + load_grad1(g, e);
  }
}

// ---------------------------------------------------------------------------------------------
// copy (snapshot and restore): dst[i] = src[i]
// ---------------------------------------------------------------------------------------------
template <int T, int U, bool NT>
__device__ inline void copy_tiles(float *__restrict__ dst, const float *__restrict__ src, const Span &sp, size_t ntiles) {
  f32x4 *d4 = reinterpret_cast<f32x4 *>(dst + sp.vbegin);
  const f32x4 *s4 = reinterpret_cast<const f32x4 *>(src + sp.vbegin);
  for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const size_t base = tile * size_t(T * U) + threadIdx.x;
    on_tile((tile + 1) * size_t(T * U) <= sp.nvec, [&](auto full) {
      constexpr bool FULL = decltype(full)::value;
      f32x4 x[U];
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; ++u) ok[u] = FULL || base + size_t(T) * u < sp.nvec;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) x[u] = ld<NT>(s4 + base + size_t(T) * u);
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) st<NT>(d4 + base + size_t(T) * u, x[u]);
    });
  }
  if (blockIdx.x == 0 && threadIdx.x < 8) {
    const size_t i = ragged_index(sp, threadIdx.x);
    if (i < sp.end) dst[i] = src[i];
  }
}

template <int T, int U, bool NT>
__global__ __launch_bounds__(T) void k_copy(float *__restrict__ dst, const float *__restrict__ src, Span sp,
                                            size_t ntiles) {
  copy_tiles<T, U, NT>(dst, src, sp, ntiles);
}

// copy for several buffer pairs in one launch (blockIdx.y = pair): a snapshot or a rewind of every
// survivor without a launch per replica.
template <int T, int U, bool NT>
__global__ __launch_bounds__(T) void k_copy_many(CopyManyArgs a, Span sp, size_t ntiles) {
  copy_tiles<T, U, NT>(a.dst[blockIdx.y], a.src[blockIdx.y], sp, ntiles);
}

// ---------------------------------------------------------------------------------------------
// reduce: out[i] = ((src0[i] + src1[i]) + ...) / divisor, ascending contributor order; in-place mode
// also stores the undivided sum to every sum_dst buffer.  A workgroup walks the contributors one
// after the other over its whole tile (U consecutive 1 KiB rows per contributor), two contributors'
// loads in flight at a time, so each of its bursts reads one buffer contiguously; every element's
// adds stay strictly left to right.
// ---------------------------------------------------------------------------------------------
// sum[u] = contributor sum of the tile's vectors, for the lanes with ok[u].
template <int T, int U, bool NT>
__device__ inline void contributor_sum(const ReduceArgs &a, const Span &sp, size_t base, const bool (&ok)[U],
                                       f32x4 (&sum)[U]) {
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
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
}

template <int T, int U, bool NT, bool INPLACE>
__global__ __launch_bounds__(T) void k_reduce(ReduceArgs a, Span sp, size_t ntiles) {
  f32x4 *o4 = reinterpret_cast<f32x4 *>(a.out + sp.vbegin);
  for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const size_t base = tile * size_t(T * U) + threadIdx.x;
    on_tile((tile + 1) * size_t(T * U) <= sp.nvec, [&](auto full) {
      constexpr bool FULL = decltype(full)::value;
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; ++u) ok[u] = FULL || base + size_t(T) * u < sp.nvec;
      f32x4 sum[U];
      contributor_sum<T, U, NT>(a, sp, base, ok, sum);
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
    });
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

// Round to nearest even; a NaN stays a NaN (quiet bit set) instead of being carried into Inf or zero by
// the rounding increment.
__device__ inline uint32_t f32_to_bf16_rne(float x) {
  uint32_t b = __builtin_bit_cast(uint32_t, x);
  if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (b >> 16) | 0x40u;
  return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}
__device__ inline u32x2 pack_bf16x4(f32x4 p) {
  u32x2 w;
  w.x = f32_to_bf16_rne(p.x) | (f32_to_bf16_rne(p.y) << 16);
  w.y = f32_to_bf16_rne(p.z) | (f32_to_bf16_rne(p.w) << 16);
  return w;
}

// Loads p, m, v of the tile, applies the update with gradient gv, stores p, m, v (and the bf16 copy).
template <int T, int U, bool NT, bool BF16OUT>
__device__ inline void adam_tile(f32x4 *__restrict__ p4, f32x4 *__restrict__ m4, f32x4 *__restrict__ v4,
                                 u32x2 *__restrict__ b2, size_t base, const bool (&ok)[U], const f32x4 (&gv)[U],
                                 const AdamArgs &h) {
  f32x4 pv[U], mv[U], vv[U];
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
    if (ok[u]) {
#pragma unroll
      for (int l = 0; l < 4; ++l) {
        float pp = pv[u][l], mm = mv[u][l], v1 = vv[u][l];
        adam1(pp, mm, v1, gv[u][l], h);
        pv[u][l] = pp;
        mv[u][l] = mm;
        vv[u][l] = v1;
      }
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
    for (int u = 0; u < U; ++u)
      if (ok[u]) st<NT>(b2 + base + size_t(T) * u, pack_bf16x4(pv[u]));
  }
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
    on_tile((tile + 1) * size_t(T * U) <= nvec, [&](auto full) {
      constexpr bool FULL = decltype(full)::value;
      bool ok[U];
      f32x4 gv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) ok[u] = FULL || base + size_t(T) * u < nvec;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) gv[u] = ld<NT>(g4 + base + size_t(T) * u);
      adam_tile<T, U, NT, BF16OUT>(p4, m4, v4, b2, base, ok, gv, h);
    });
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
// fused reduce + AdamW: the contributor sum of k_reduce (same walk, same order), its division, and the
// update of k_adamw in one pass; the gradient goes to HBM only if WRITE_GRAD.  4 R_c + 24 (+4) bytes
// per element.
// ---------------------------------------------------------------------------------------------
template <int T, int U, bool NT, bool WRITE_GRAD, bool BF16OUT>
__global__ __launch_bounds__(T) void k_reduce_adamw(ReduceArgs a, float *__restrict__ p, float *__restrict__ m,
                                                    float *__restrict__ v, uint16_t *__restrict__ pb, Span sp,
                                                    AdamArgs h_arg, const AdamArgs *h_dev, size_t ntiles) {
  const AdamArgs h = h_dev ? *h_dev : h_arg;
  f32x4 *p4 = reinterpret_cast<f32x4 *>(p + sp.vbegin), *m4 = reinterpret_cast<f32x4 *>(m + sp.vbegin);
  f32x4 *v4 = reinterpret_cast<f32x4 *>(v + sp.vbegin), *o4 = reinterpret_cast<f32x4 *>(a.out + sp.vbegin);
  u32x2 *b2 = reinterpret_cast<u32x2 *>(pb + sp.vbegin);
  for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const size_t base = tile * size_t(T * U) + threadIdx.x;
    on_tile((tile + 1) * size_t(T * U) <= sp.nvec, [&](auto full) {
      constexpr bool FULL = decltype(full)::value;
      bool ok[U];
#pragma unroll
      for (int u = 0; u < U; ++u) ok[u] = FULL || base + size_t(T) * u < sp.nvec;
      f32x4 sum[U];
      contributor_sum<T, U, NT>(a, sp, base, ok, sum);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        sum[u].x = sum[u].x / a.divisor;
        sum[u].y = sum[u].y / a.divisor;
        sum[u].z = sum[u].z / a.divisor;
        sum[u].w = sum[u].w / a.divisor;
      }
      adam_tile<T, U, NT, BF16OUT>(p4, m4, v4, b2, base, ok, sum, h);
      if (WRITE_GRAD) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (ok[u]) st<NT>(o4 + base + size_t(T) * u, sum[u]);
      }
    });
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
    } else if (ab != bb) {  // equal bits differ by nothing (also for two equal infinities, whose difference is a NaN)
      const uint32_t d = __builtin_bit_cast(uint32_t, __builtin_fabsf(a - b));  // +Inf for opposite infinities
      const uint32_t r = bb & 0x7FFFFFFFu;
      mdiff = d > mdiff ? d : mdiff;
      mref = r > mref ? r : mref;
    } else {
      const uint32_t r = bb & 0x7FFFFFFFu;
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

// Dynamic LDS bytes per workgroup that leave room for `waves` wavefronts of T-lane workgroups on a CU
// (160 KiB of LDS each); 0 = no limit.  The kernels never touch the allocation.
static unsigned lds_share(int waves, int T) {
  const int per_wg = T / 64;
  if (waves <= 0 || waves >= 32) return 0;
  int wgs = waves / per_wg;
  if (wgs < 1) wgs = 1;
  unsigned b = (163840u / (unsigned)wgs) & ~255u;
  return b > 65536u ? 65536u : b;
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
  const Shape sh = tuning().shape[grad_is_bf16 ? (first ? kAccFirstBf16 : kAccRmwBf16) : (first ? kAccFirstF32 : kAccRmwF32)];
  const int Uv = sh.vecs, Tv = tuning().threads;
  const unsigned lds = lds_share(sh.waves, Tv);
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
                         dim3(T), lds, s, acc, snap, gptr, sp, ntiles, xc);
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
  const Shape sh = tuning().shape[kCopy];
  const int Uv = sh.vecs, Tv = tuning().threads;
  unsigned grid;
  size_t ntiles;
  if (!grid_for(sp.nvec, Tv, Uv, &grid, &ntiles)) return hipErrorInvalidConfiguration;
  with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
    constexpr int T = decltype(t)::value, U = decltype(u)::value;
    constexpr bool NT = decltype(nt)::value;
    hipLaunchKernelGGL((k_copy<T, U, NT>), dim3(grid), dim3(T), lds_share(sh.waves, T), s, dst, src, sp, ntiles);
  });
  return hipGetLastError();
}

hipError_t launch_copy_many(const CopyManyArgs &a, int n_pairs, size_t begin, size_t end, hipStream_t s) {
  if (begin >= end || n_pairs <= 0) return hipSuccess;
  if (n_pairs > kMaxReplicas) return hipErrorInvalidConfiguration;
  const Span sp = make_span(begin, end);
  const Shape sh = tuning().shape[kCopy];
  const int Uv = sh.vecs, Tv = tuning().threads;
  unsigned grid;
  size_t ntiles;
  if (!grid_for(sp.nvec, Tv, Uv, &grid, &ntiles)) return hipErrorInvalidConfiguration;
  with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
    constexpr int T = decltype(t)::value, U = decltype(u)::value;
    constexpr bool NT = decltype(nt)::value;
    hipLaunchKernelGGL((k_copy_many<T, U, NT>), dim3(grid, (unsigned)n_pairs), dim3(T), lds_share(sh.waves, T), s, a, sp,
                       ntiles);
  });
  return hipGetLastError();
}

hipError_t launch_reduce(const ReduceArgs &a, size_t begin, size_t end, hipStream_t s) {
  if (begin >= end) return hipSuccess;
  const Span sp = make_span(begin, end);
  const Shape sh = tuning().shape[kReduce];
  const int Uv = sh.vecs, Tv = tuning().threads;
  unsigned grid;
  size_t ntiles;
  if (!grid_for(sp.nvec, Tv, Uv, &grid, &ntiles)) return hipErrorInvalidConfiguration;
  const bool inplace = a.n_sum_dst > 0;
  with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
    constexpr int T = decltype(t)::value, U = decltype(u)::value;
    constexpr bool NT = decltype(nt)::value;
    const unsigned lds = lds_share(sh.waves, T);
    if (inplace)
      hipLaunchKernelGGL((k_reduce<T, U, NT, true>), dim3(grid), dim3(T), lds, s, a, sp, ntiles);
    else
      hipLaunchKernelGGL((k_reduce<T, U, NT, false>), dim3(grid), dim3(T), lds, s, a, sp, ntiles);
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
  const Shape sh = tuning().shape[kAdamw];
  const int Uv = sh.vecs, Tv = tuning().threads;
  unsigned grid;
  size_t ntiles;
  if (!grid_for(n / 4, Tv, Uv, &grid, &ntiles)) return hipErrorInvalidConfiguration;
  with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
    constexpr int T = decltype(t)::value, U = decltype(u)::value;
    constexpr bool NT = decltype(nt)::value;
    const unsigned lds = lds_share(sh.waves, T);
    if (p_bf16)
      hipLaunchKernelGGL((k_adamw<T, U, NT, true>), dim3(grid), dim3(T), lds, s, p, m, v, g, p_bf16, n, h, device_args,
                         ntiles);
    else
      hipLaunchKernelGGL((k_adamw<T, U, NT, false>), dim3(grid), dim3(T), lds, s, p, m, v, g, p_bf16, n, h, device_args,
                         ntiles);
  });
  return hipGetLastError();
}

hipError_t launch_reduce_adamw(const ReduceArgs &a, float *p, float *m, float *v, uint16_t *p_bf16, bool write_grad,
                               size_t begin, size_t end, const AdamArgs &h, const AdamArgs *device_args,
                               hipStream_t s) {
  if (begin >= end) return hipSuccess;
  const Span sp = make_span(begin, end);
  const Shape sh = tuning().shape[kReduceAdamw];
  const int Uv = sh.vecs, Tv = tuning().threads;
  unsigned grid;
  size_t ntiles;
  if (!grid_for(sp.nvec, Tv, Uv, &grid, &ntiles)) return hipErrorInvalidConfiguration;
  with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
    constexpr int T = decltype(t)::value, U = decltype(u)::value;
    constexpr bool NT = decltype(nt)::value;
    const unsigned lds = lds_share(sh.waves, T);
    auto go = [&](auto wg, auto bf) {
      hipLaunchKernelGGL((k_reduce_adamw<T, U, NT, decltype(wg)::value, decltype(bf)::value>), dim3(grid), dim3(T), lds,
                         s, a, p, m, v, p_bf16, sp, h, device_args, ntiles);
    };
    auto with_bf = [&](auto wg) {
      if (p_bf16) go(wg, std::true_type{});
      else go(wg, std::false_type{});
    };
    if (write_grad) with_bf(std::true_type{});
    else with_bf(std::false_type{});
  });
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
