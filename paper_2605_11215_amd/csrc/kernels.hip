// gfx950 kernels of the gradient path.  Every step is an elementwise stream over flat fp32
// buffers, bound by HBM bandwidth, so the design is the same everywhere: one 128-bit load or
// store per lane per access (a wavefront moves 1 KiB of consecutive bytes per instruction),
// one-wavefront workgroups with ONE tile each (a finished wavefront frees its slot at once; measured
// 4 % faster than four-wavefront groups), U independent vectors in flight per lane before the first
// use, 64-bit element indices (a shard can exceed 2^32 elements), no LDS (no element is used twice) and
// no atomics (the sums have a fixed order).
//
// A wavefront moves only a few KiB in its whole life, so its prologue counts: the kernels take
// pointers that the host has already advanced to the first aligned vector, and a vector count;
// there is no tile loop, no range arithmetic and no ragged-end code in them.  Ranges that do not
// start or end on a 16-byte boundary get their (at most six) ragged elements from a second,
// eight-lane launch of a scalar kernel.  Every kernel body exists twice, selected by a
// wavefront-uniform test: full tiles (all but the last) run without per-lane bounds tests, so all
// their loads are issued back to back before the first wait; the last, partial tile masks each
// access.  Raw bf16 words are widened only after every load of the tile has been issued.
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
static bool ragged(const Span &sp) { return sp.vbegin != sp.begin || sp.vbegin + sp.nvec * 4 != sp.end; }

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

// The calling workgroup's tile: index of its lane's first vector, and whether the whole tile lies inside
// [0, nvec) (wavefront-uniform).  T * U vectors per tile, lane l takes vectors base + T * u.
template <int T, int U>
__device__ inline size_t tile_base(size_t nvec, bool *full) {
  const size_t t0 = size_t(blockIdx.x) * (T * U);
  *full = t0 + T * U <= nvec;
  return t0 + threadIdx.x;
}
// Runs body(True) on a full tile and body(False) on the partial one.
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
// a4, s4, g4 point at the first aligned vector of the range.
// ---------------------------------------------------------------------------------------------
template <typename G, int T, int U, bool NT, bool FIRST, bool SNAP>
__device__ inline void accumulate_tile(f32x4 *__restrict__ a4, f32x4 *__restrict__ s4,
                                       const typename Grad4<G>::raw *__restrict__ g4, size_t nvec) {
  typedef typename Grad4<G>::raw Raw;
  bool full;
  const size_t base = tile_base<T, U>(nvec, &full);
  on_tile(full, [&](auto is_full) {
    constexpr bool FULL = decltype(is_full)::value;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    Raw x[U];
    f32x4 a[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) ok[u] = FULL || base + size_t(T) * u < nvec;
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

template <typename G, int T, int U, bool NT, bool FIRST, bool SNAP>
__global__ __launch_bounds__(T) void k_accumulate(f32x4 *__restrict__ a4, f32x4 *__restrict__ s4,
                                                  const typename Grad4<G>::raw *__restrict__ g4, size_t nvec) {
  accumulate_tile<G, T, U, NT, FIRST, SNAP>(a4, s4, g4, nvec);
}

template <typename G, bool FIRST, bool SNAP>
__global__ __launch_bounds__(64) void k_accumulate_ragged(float *__restrict__ acc, float *__restrict__ snap,
                                                          const G *__restrict__ g, Span sp) {
  const size_t i = ragged_index(sp, threadIdx.x);
  if (threadIdx.x < 8 && i < sp.end) {
    const float r = (FIRST ? 0.f : acc[i]) + load_grad1(g, i);
    acc[i] = r;
    if (SNAP) snap[i] = r;
  }
}

// accumulate for several replicas in one launch (blockIdx.y = pair index): same arithmetic per pair;
// for shards so small that the launch, not HBM, bounds a single accumulate.  Lanes 0..7 of the first
// workgroup of a pair also take the pair's ragged elements.
template <typename G, int T, bool NT>
__global__ __launch_bounds__(T) void k_accumulate_many(AccumulateManyArgs a, Span sp) {
  typedef typename Grad4<G>::raw Raw;
  const int pair = blockIdx.y;
  float *acc = a.acc[pair];
  const G *g = static_cast<const G *>(a.grad[pair]);
  f32x4 *a4 = reinterpret_cast<f32x4 *>(acc + sp.vbegin);
  const Raw *g4 = reinterpret_cast<const Raw *>(g + sp.vbegin);
  if (a.first[pair])
    accumulate_tile<G, T, 1, NT, true, false>(a4, nullptr, g4, sp.nvec);
  else
    accumulate_tile<G, T, 1, NT, false, false>(a4, nullptr, g4, sp.nvec);
  if (blockIdx.x == 0 && threadIdx.x < 8) {
    const size_t e = ragged_index(sp, threadIdx.x);
    if (e < sp.end) acc[e] = (a.first[pair] ? 0.f : acc[e]) + load_grad1(g, e);
  }
}

// ---------------------------------------------------------------------------------------------
// copy (snapshot and restore): dst[i] = src[i]
// ---------------------------------------------------------------------------------------------
template <int T, int U, bool NT>
__device__ inline void copy_tile(f32x4 *__restrict__ d4, const f32x4 *__restrict__ s4, size_t nvec) {
  bool full;
  const size_t base = tile_base<T, U>(nvec, &full);
  on_tile(full, [&](auto is_full) {
    constexpr bool FULL = decltype(is_full)::value;
    f32x4 x[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) ok[u] = FULL || base + size_t(T) * u < nvec;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) x[u] = ld<NT>(s4 + base + size_t(T) * u);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) st<NT>(d4 + base + size_t(T) * u, x[u]);
  });
}

// RESTORE only names the instantiation (snapshot or rewind), so that a kernel trace tells the two apart.
template <int T, int U, bool NT, bool RESTORE>
__global__ __launch_bounds__(T) void k_copy(f32x4 *__restrict__ d4, const f32x4 *__restrict__ s4, size_t nvec) {
  copy_tile<T, U, NT>(d4, s4, nvec);
}

// copy for several buffer pairs in one launch (blockIdx.y = pair): a snapshot or a rewind of every
// survivor without a launch per replica; lanes 0..7 of a pair's first workgroup take its ragged elements.
template <int T, int U, bool NT, bool RESTORE>
__global__ __launch_bounds__(T) void k_copy_many(CopyManyArgs a, Span sp) {
  float *dst = a.dst[blockIdx.y];
  const float *src = a.src[blockIdx.y];
  copy_tile<T, U, NT>(reinterpret_cast<f32x4 *>(dst + sp.vbegin), reinterpret_cast<const f32x4 *>(src + sp.vbegin), sp.nvec);
  if (blockIdx.x == 0 && threadIdx.x < 8) {
    const size_t i = ragged_index(sp, threadIdx.x);
    if (i < sp.end) dst[i] = src[i];
  }
}

__global__ __launch_bounds__(64) void k_copy_ragged(float *__restrict__ dst, const float *__restrict__ src, Span sp) {
  const size_t i = ragged_index(sp, threadIdx.x);
  if (threadIdx.x < 8 && i < sp.end) dst[i] = src[i];
}

// ---------------------------------------------------------------------------------------------
// reduce: out[i] = ((src0[i] + src1[i]) + ...) / divisor, ascending contributor order; in-place mode
// also stores the undivided sum to every sum_dst buffer.  A wavefront walks the contributors one after
// the other over its tile, so each of its bursts reads one buffer contiguously; every element's adds
// stay strictly left to right.  The pointers in ReduceArgs are the buffers' bases; `first` is the
// element index of the range's first aligned vector.
// ---------------------------------------------------------------------------------------------
// sum[u] = contributor sum of the tile's vectors, for the lanes with ok[u].  D = contributors whose loads
// a wavefront has in flight at a time: 1 (each load waits for the one before: the least data in flight
// per wavefront, best with many resident wavefronts) or 2 (pairs).  The order of the adds is the same.
template <int T, int U, bool NT, int D>
__device__ inline void contributor_sum(const ReduceArgs &a, size_t first, size_t base, const bool (&ok)[U],
                                       f32x4 (&sum)[U]) {
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int u = 0; u < U; ++u) sum[u] = zero;
  int r = 0;
  if (a.n_src > 0) {
    const f32x4 *s0 = reinterpret_cast<const f32x4 *>(a.src[0] + first) + base;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) sum[u] = ld<NT>(s0 + size_t(T) * u);
    r = 1;
  }
  if (D == 1) {
#pragma clang loop unroll(disable)
    for (; r < a.n_src; ++r) {
      const f32x4 *s0 = reinterpret_cast<const f32x4 *>(a.src[r] + first) + base;
      f32x4 t0[U];
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) t0[u] = ld<NT>(s0 + size_t(T) * u);
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) sum[u] = sum[u] + t0[u];
      asm volatile("" ::: "memory");  // the next contributor's load is issued after this one has arrived
    }
    return;
  }
  for (; r + 1 < a.n_src; r += 2) {
    const f32x4 *s0 = reinterpret_cast<const f32x4 *>(a.src[r] + first) + base;
    const f32x4 *s1 = reinterpret_cast<const f32x4 *>(a.src[r + 1] + first) + base;
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
    const f32x4 *s0 = reinterpret_cast<const f32x4 *>(a.src[r] + first) + base;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) sum[u] = sum[u] + ld<NT>(s0 + size_t(T) * u);
  }
}

template <int T, int U, bool NT, bool INPLACE, int D>
__global__ __launch_bounds__(T) void k_reduce(ReduceArgs a, size_t first, size_t nvec) {
  bool full;
  const size_t base = tile_base<T, U>(nvec, &full);
  on_tile(full, [&](auto is_full) {
    constexpr bool FULL = decltype(is_full)::value;
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) ok[u] = FULL || base + size_t(T) * u < nvec;
    f32x4 sum[U];
    contributor_sum<T, U, NT, D>(a, first, base, ok, sum);
    if (INPLACE) {
      for (int d = 0; d < a.n_sum_dst; ++d) {
        f32x4 *dd = reinterpret_cast<f32x4 *>(a.sum_dst[d] + first) + base;
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (ok[u]) st<NT>(dd + size_t(T) * u, sum[u]);
      }
    }
    f32x4 *o4 = reinterpret_cast<f32x4 *>(a.out + first) + base;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (ok[u]) {
        f32x4 q;
        q.x = sum[u].x / a.divisor;
        q.y = sum[u].y / a.divisor;
        q.z = sum[u].z / a.divisor;
        q.w = sum[u].w / a.divisor;
        st<NT>(o4 + size_t(T) * u, q);
      }
    }
  });
}

template <bool INPLACE>
__global__ __launch_bounds__(64) void k_reduce_ragged(ReduceArgs a, Span sp) {
  const size_t i = ragged_index(sp, threadIdx.x);
  if (threadIdx.x < 8 && i < sp.end) {
    float sum = 0.f;
    for (int r = 0; r < a.n_src; ++r) sum = (r == 0) ? a.src[r][i] : sum + a.src[r][i];
    if (INPLACE)
      for (int d = 0; d < a.n_sum_dst; ++d) a.sum_dst[d][i] = sum;
    a.out[i] = sum / a.divisor;
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

// Device pointers of the optimiser state, advanced to the range's first aligned vector.
struct AdamPtrs {
  f32x4 *p4, *m4, *v4;
  u32x2 *b2;  // bf16 copy of the parameters or nullptr
};

// The tile's p, m, v.
template <int U>
struct AdamTile {
  f32x4 pv[U], mv[U], vv[U];
};
template <int T, int U, bool NT>
__device__ inline void adam_load(const AdamPtrs &s, size_t base, const bool (&ok)[U], AdamTile<U> &x) {
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (ok[u]) x.pv[u] = ld<NT>(s.p4 + base + size_t(T) * u);
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (ok[u]) x.mv[u] = ld<NT>(s.m4 + base + size_t(T) * u);
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (ok[u]) x.vv[u] = ld<NT>(s.v4 + base + size_t(T) * u);
}
// Applies the update with gradient gv to the loaded tile and stores p, m, v (and the bf16 copy).
template <int T, int U, bool NT, bool BF16OUT>
__device__ inline void adam_update_store(const AdamPtrs &s, size_t base, const bool (&ok)[U], AdamTile<U> &x,
                                         const f32x4 (&gv)[U], const AdamArgs &h) {
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (ok[u]) {
#pragma unroll
      for (int l = 0; l < 4; ++l) {
        float pp = x.pv[u][l], mm = x.mv[u][l], v1 = x.vv[u][l];
        adam1(pp, mm, v1, gv[u][l], h);
        x.pv[u][l] = pp;
        x.mv[u][l] = mm;
        x.vv[u][l] = v1;
      }
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (ok[u]) st<NT>(s.p4 + base + size_t(T) * u, x.pv[u]);
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (ok[u]) st<NT>(s.m4 + base + size_t(T) * u, x.mv[u]);
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (ok[u]) st<NT>(s.v4 + base + size_t(T) * u, x.vv[u]);
  if (BF16OUT) {
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) st<NT>(s.b2 + base + size_t(T) * u, pack_bf16x4(x.pv[u]));
  }
}

// DEV: the step's constants are read from device memory (written by k_adam_prologue) instead of the
// kernel arguments; a template parameter so that the argument path keeps its constants in scalar registers.
template <int T, int U, bool NT, bool BF16OUT, bool DEV>
__global__ __launch_bounds__(T) void k_adamw(AdamPtrs s, const f32x4 *__restrict__ g4, size_t nvec, AdamArgs h_arg,
                                             const AdamArgs *__restrict__ h_dev) {
  const AdamArgs h = DEV ? *h_dev : h_arg;
  bool full;
  const size_t base = tile_base<T, U>(nvec, &full);
  on_tile(full, [&](auto is_full) {
    constexpr bool FULL = decltype(is_full)::value;
    bool ok[U];
    f32x4 gv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) ok[u] = FULL || base + size_t(T) * u < nvec;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ok[u]) gv[u] = ld<NT>(g4 + base + size_t(T) * u);
    AdamTile<U> x;
    adam_load<T, U, NT>(s, base, ok, x);
    adam_update_store<T, U, NT, BF16OUT>(s, base, ok, x, gv, h);
  });
}

// The ragged elements of a range (at most three before its first aligned vector and three after its last), one per lane.
__global__ __launch_bounds__(64) void k_adamw_ragged(float *__restrict__ p, float *__restrict__ m, float *__restrict__ v,
                                                     const float *__restrict__ g, uint16_t *__restrict__ pb, Span sp,
                                                     AdamArgs h_arg, const AdamArgs *h_dev) {
  const AdamArgs h = h_dev ? *h_dev : h_arg;
  const size_t i = ragged_index(sp, threadIdx.x);
  if (threadIdx.x < 8 && i < sp.end) {
    float pp = p[i], mm = m[i], vv = v[i];
    adam1(pp, mm, vv, g[i], h);
    p[i] = pp;
    m[i] = mm;
    v[i] = vv;
    if (pb) pb[i] = (uint16_t)f32_to_bf16_rne(pp);
  }
}

// ---------------------------------------------------------------------------------------------
// fused reduce + AdamW: the contributor sum of k_reduce (same walk, same order), its division, and the
// update of k_adamw in one pass; the gradient goes to HBM only if WRITE_GRAD.  4 R_c + 24 (+4) bytes
// per element.  Launched for up to tuning().one_pass_max contributors (see launch_reduce_adamw).
// ---------------------------------------------------------------------------------------------
template <int T, int U, bool NT, bool WRITE_GRAD, bool BF16OUT, int D, bool DEV>
__global__ __launch_bounds__(T) void k_reduce_adamw(ReduceArgs a, AdamPtrs s, size_t first, size_t nvec, AdamArgs h_arg,
                                                    const AdamArgs *__restrict__ h_dev) {
  const AdamArgs h = DEV ? *h_dev : h_arg;
  bool full;
  const size_t base = tile_base<T, U>(nvec, &full);
  on_tile(full, [&](auto is_full) {
    constexpr bool FULL = decltype(is_full)::value;
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) ok[u] = FULL || base + size_t(T) * u < nvec;
    f32x4 sum[U];
    AdamTile<U> x;
    contributor_sum<T, U, NT, D>(a, first, base, ok, sum);
    adam_load<T, U, NT>(s, base, ok, x);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      sum[u].x = sum[u].x / a.divisor;
      sum[u].y = sum[u].y / a.divisor;
      sum[u].z = sum[u].z / a.divisor;
      sum[u].w = sum[u].w / a.divisor;
    }
    adam_update_store<T, U, NT, BF16OUT>(s, base, ok, x, sum, h);
    if (WRITE_GRAD) {
      f32x4 *o4 = reinterpret_cast<f32x4 *>(a.out + first) + base;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) st<NT>(o4 + size_t(T) * u, sum[u]);
    }
  });
}

template <bool WRITE_GRAD>
__global__ __launch_bounds__(64) void k_reduce_adamw_ragged(ReduceArgs a, float *__restrict__ p, float *__restrict__ m,
                                                            float *__restrict__ v, uint16_t *__restrict__ pb, Span sp,
                                                            AdamArgs h_arg, const AdamArgs *h_dev) {
  const AdamArgs h = h_dev ? *h_dev : h_arg;
  const size_t e = ragged_index(sp, threadIdx.x);
  if (threadIdx.x < 8 && e < sp.end) {
    float sum = 0.f;
    for (int r = 0; r < a.n_src; ++r) sum = (r == 0) ? a.src[r][e] : sum + a.src[r][e];
    const float q = sum / a.divisor;
    float pp = p[e], mm = m[e], v1 = v[e];
    adam1(pp, mm, v1, q, h);
    p[e] = pp;
    m[e] = mm;
    v[e] = v1;
    if (WRITE_GRAD) a.out[e] = q;
    if (pb) pb[e] = (uint16_t)f32_to_bf16_rne(pp);
  }
}

// ---------------------------------------------------------------------------------------------
// compare (verification support, off the timed path): bitwise mismatch count, max |x - ref|,
// max |ref|, NaN count and two position-weighted 64-bit checksums of two fp32 buffers, without
// moving them to the host.  Each lane folds its elements, a wavefront folds its 64 lanes with
// cross-lane shuffles, the wavefronts of a workgroup fold through LDS, and one lane per workgroup adds to the result
// with integer atomics (sums and maxima of integers do not depend on the order, so the result is reproducible).
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

struct CompareFold {
  uint64_t mism = 0, nans = 0, cx = 0, cr = 0;
  uint32_t mdiff = 0, mref = 0;  // bit patterns of non-negative floats order like the floats
  __device__ inline void take(float a, float b, size_t i) {
    const uint32_t ab = __builtin_bit_cast(uint32_t, a), bb = __builtin_bit_cast(uint32_t, b);
    cx += uint64_t(ab) * (2 * uint64_t(i) + 1);
    cr += uint64_t(bb) * (2 * uint64_t(i) + 1);
    take_no_checksum(a, b);
  }
  // Four consecutive elements 4 v .. 4 v + 3: their weights are 8 v + 1, + 3, + 5, + 7, so the weighted sum is
  // (8 v + 1)(b0 + b1 + b2 + b3) + 2 (b1 + 2 b2 + 3 b3) modulo 2^64: one wide multiply per vector and buffer.
  __device__ inline void take4(const f32x4 &a, const f32x4 &b, size_t v) {
    const uint64_t w = 8 * uint64_t(v) + 1;
    uint64_t sa = 0, ta = 0, sb = 0, tb = 0;
#pragma unroll
    for (int l = 0; l < 4; ++l) {
      const float al = a[l], bl = b[l];  // by value: a bit cast applied to the vector-element lvalue reads element 0
      const uint64_t ab = __builtin_bit_cast(uint32_t, al), bb = __builtin_bit_cast(uint32_t, bl);
      sa += ab;
      ta += uint64_t(l) * ab;
      sb += bb;
      tb += uint64_t(l) * bb;
      take_no_checksum(al, bl);
    }
    cx += w * sa + 2 * ta;
    cr += w * sb + 2 * tb;
  }
  __device__ inline void take_no_checksum(float a, float b) {
    const uint32_t ab = __builtin_bit_cast(uint32_t, a), bb = __builtin_bit_cast(uint32_t, b);
    mism += ab != bb;
    if (a != a || b != b) {
      nans += 1;
    } else {
      const uint32_t r = bb & 0x7FFFFFFFu;
      mref = r > mref ? r : mref;
      if (ab != bb) {  // equal bits differ by nothing (also two equal infinities, whose difference is a NaN)
        const uint32_t d = __builtin_bit_cast(uint32_t, __builtin_fabsf(a - b));  // +Inf for opposite infinities
        mdiff = d > mdiff ? d : mdiff;
      }
    }
  }
};

// Two streams read with 128-bit loads, nothing written but six atomics per wavefront.
__global__ __launch_bounds__(256) void k_compare(const float *__restrict__ x, const float *__restrict__ ref, size_t n,
                                                 CompareResult *out) {
  CompareFold f;
  const size_t nvec = n / 4;
  const f32x4 *x4 = reinterpret_cast<const f32x4 *>(x), *r4 = reinterpret_cast<const f32x4 *>(ref);
  for (size_t v = size_t(blockIdx.x) * 256 + threadIdx.x; v < nvec; v += size_t(gridDim.x) * 256) {
    const f32x4 a = __builtin_nontemporal_load(x4 + v), b = __builtin_nontemporal_load(r4 + v);
    f.take4(a, b, v);
  }
  if (blockIdx.x == 0 && threadIdx.x < 4) {
    const size_t i = nvec * 4 + threadIdx.x;
    if (i < n) f.take(x[i], ref[i], i);
  }
  const uint64_t mism = wave_sum_u64(f.mism), nans = wave_sum_u64(f.nans), cx = wave_sum_u64(f.cx), cr = wave_sum_u64(f.cr);
  const uint32_t mdiff = wave_max_u32(f.mdiff), mref = wave_max_u32(f.mref);
  // The four wavefronts of the workgroup fold through LDS, so the six atomics (all workgroups hit the same six
  // words, which serialises them) are issued once per workgroup.
  __shared__ uint64_t part64[4][4];
  __shared__ uint32_t part32[4][2];
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    part64[wave][0] = mism;
    part64[wave][1] = nans;
    part64[wave][2] = cx;
    part64[wave][3] = cr;
    part32[wave][0] = mdiff;
    part32[wave][1] = mref;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint64_t t[4] = {0, 0, 0, 0};
    uint32_t m0 = 0, m1 = 0;
    for (int w = 0; w < 4; ++w) {
      for (int k = 0; k < 4; ++k) t[k] += part64[w][k];
      m0 = part32[w][0] > m0 ? part32[w][0] : m0;
      m1 = part32[w][1] > m1 ? part32[w][1] : m1;
    }
    atomicAdd(reinterpret_cast<unsigned long long *>(&out->n_mismatch), (unsigned long long)t[0]);
    atomicAdd(reinterpret_cast<unsigned long long *>(&out->n_nan), (unsigned long long)t[1]);
    atomicAdd(reinterpret_cast<unsigned long long *>(&out->checksum_x), (unsigned long long)t[2]);
    atomicAdd(reinterpret_cast<unsigned long long *>(&out->checksum_ref), (unsigned long long)t[3]);
    atomicMax(&out->max_abs_diff_bits, m0);
    atomicMax(&out->max_abs_ref_bits, m1);
  }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
// One tile of T * U vectors per workgroup.
static bool grid_for(size_t nvec, int T, int U, unsigned *grid) {
  const size_t tiles = (nvec + size_t(T) * U - 1) / (size_t(T) * U);
  if (tiles > 0x7FFFFFFFull) return false;
  *grid = (unsigned)tiles;
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
  const Shape sh = tuning().shape[snap ? (grad_is_bf16 ? kAccSnapBf16 : kAccSnapF32)
                                       : grad_is_bf16 ? (first ? kAccFirstBf16 : kAccRmwBf16) : (first ? kAccFirstF32 : kAccRmwF32)];
  const int Uv = sh.vecs, Tv = tuning().threads;
  const unsigned lds = lds_share(sh.waves, Tv);
  unsigned grid;
  if (!grid_for(sp.nvec, Tv, Uv, &grid)) return hipErrorInvalidConfiguration;
  f32x4 *a4 = reinterpret_cast<f32x4 *>(acc + sp.vbegin);
  f32x4 *s4 = snap ? reinterpret_cast<f32x4 *>(snap + sp.vbegin) : nullptr;
  auto pick = [&](auto gptr) {  // gptr: typed base of the gradient
    using GT = std::remove_cv_t<std::remove_pointer_t<decltype(gptr)>>;
    using Raw = typename Grad4<GT>::raw;
    const Raw *g4 = reinterpret_cast<const Raw *>(gptr + sp.vbegin);
    auto go = [&](auto is_first, auto with_snap) {
      constexpr bool F = decltype(is_first)::value, SN = decltype(with_snap)::value;
      if (grid)
        with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
          hipLaunchKernelGGL((k_accumulate<GT, decltype(t)::value, decltype(u)::value, decltype(nt)::value, F, SN>),
                             dim3(grid), dim3(decltype(t)::value), lds, s, a4, s4, g4, sp.nvec);
        });
      if (ragged(sp)) hipLaunchKernelGGL((k_accumulate_ragged<GT, F, SN>), dim3(1), dim3(64), 0, s, acc, snap, gptr, sp);
    };
    if (first) {
      if (snap) go(std::true_type{}, std::true_type{});
      else go(std::true_type{}, std::false_type{});
    } else {
      if (snap) go(std::false_type{}, std::true_type{});
      else go(std::false_type{}, std::false_type{});
    }
  };
  if (grad_is_bf16)
    pick(static_cast<const uint16_t *>(grad));
  else
    pick(static_cast<const float *>(grad));
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

hipError_t launch_copy(float *dst, const float *src, size_t begin, size_t end, bool restore, hipStream_t s) {
  if (begin >= end) return hipSuccess;
  const Span sp = make_span(begin, end);
  const Shape sh = tuning().shape[kCopy];
  const int Uv = sh.vecs, Tv = tuning().threads;
  unsigned grid;
  if (!grid_for(sp.nvec, Tv, Uv, &grid)) return hipErrorInvalidConfiguration;
  if (grid)
    with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
      constexpr int T = decltype(t)::value, U = decltype(u)::value;
      f32x4 *d4 = reinterpret_cast<f32x4 *>(dst + sp.vbegin);
      const f32x4 *s4 = reinterpret_cast<const f32x4 *>(src + sp.vbegin);
      if (restore)
        hipLaunchKernelGGL((k_copy<T, U, decltype(nt)::value, true>), dim3(grid), dim3(T), lds_share(sh.waves, T), s, d4, s4,
                           sp.nvec);
      else
        hipLaunchKernelGGL((k_copy<T, U, decltype(nt)::value, false>), dim3(grid), dim3(T), lds_share(sh.waves, T), s, d4, s4,
                           sp.nvec);
    });
  if (ragged(sp)) hipLaunchKernelGGL(k_copy_ragged, dim3(1), dim3(64), 0, s, dst, src, sp);
  return hipGetLastError();
}

hipError_t launch_copy_many(const CopyManyArgs &a, int n_pairs, size_t begin, size_t end, bool restore, hipStream_t s) {
  if (begin >= end || n_pairs <= 0) return hipSuccess;
  if (n_pairs > kMaxReplicas) return hipErrorInvalidConfiguration;
  const Span sp = make_span(begin, end);
  const Shape sh = tuning().shape[kCopy];
  const int Uv = sh.vecs, Tv = tuning().threads;
  unsigned grid;
  if (!grid_for(sp.nvec, Tv, Uv, &grid)) return hipErrorInvalidConfiguration;
  if (!grid) grid = 1;  // the ragged elements ride on workgroup 0 of every pair
  with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
    constexpr int T = decltype(t)::value, U = decltype(u)::value;
    if (restore)
      hipLaunchKernelGGL((k_copy_many<T, U, decltype(nt)::value, true>), dim3(grid, (unsigned)n_pairs), dim3(T),
                         lds_share(sh.waves, T), s, a, sp);
    else
      hipLaunchKernelGGL((k_copy_many<T, U, decltype(nt)::value, false>), dim3(grid, (unsigned)n_pairs), dim3(T),
                         lds_share(sh.waves, T), s, a, sp);
  });
  return hipGetLastError();
}

hipError_t launch_reduce(const ReduceArgs &a, size_t begin, size_t end, hipStream_t s) {
  if (begin >= end) return hipSuccess;
  const Span sp = make_span(begin, end);
  const Shape sh = tuning().shape[kReduce];
  const int Uv = sh.vecs, Tv = tuning().threads;
  unsigned grid;
  if (!grid_for(sp.nvec, Tv, Uv, &grid)) return hipErrorInvalidConfiguration;
  const bool inplace = a.n_sum_dst > 0;
  if (grid)
    with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
      constexpr int T = decltype(t)::value, U = decltype(u)::value;
      constexpr bool NT = decltype(nt)::value;
      const unsigned lds = lds_share(sh.waves, T);
      auto go = [&](auto ip, auto d) {
        hipLaunchKernelGGL((k_reduce<T, U, NT, decltype(ip)::value, decltype(d)::value>), dim3(grid), dim3(T), lds, s, a,
                           sp.vbegin, sp.nvec);
      };
      auto with_d = [&](auto ip) {
        if (sh.depth == 1) go(ip, Int<1>{});
        else go(ip, Int<2>{});
      };
      if (inplace) with_d(std::true_type{});
      else with_d(std::false_type{});
    });
  if (ragged(sp)) {
    if (inplace) hipLaunchKernelGGL(k_reduce_ragged<true>, dim3(1), dim3(64), 0, s, a, sp);
    else hipLaunchKernelGGL(k_reduce_ragged<false>, dim3(1), dim3(64), 0, s, a, sp);
  }
  return hipGetLastError();
}

// Library-owned step states (4 KiB per GPU, held until the process ends).  In host code the array's name is
// only a handle for hipGetSymbolAddress; kernels get the resolved device address as an argument.
static __device__ __align__(256) StepState scratch[kStaticStepSlots];

hipError_t static_step_state(int slot, StepState **out) {
  constexpr int kMaxDevices = 64;
  static StepState *base[kMaxDevices] = {};
  if (slot < 0 || slot >= kStaticStepSlots) return hipErrorInvalidValue;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!base[dev]) {
    StepState *p = nullptr;
    e = hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    base[dev] = p;
  }
  *out = base[dev] + slot;
  return hipSuccess;
}

__global__ void k_clear_step_state(StepState *st) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    st->step = 0;
    st->beta1_pow = 1.0;
    st->beta2_pow = 1.0;
    st->args = AdamArgs{};
    st->reserved = 0;
  }
}

hipError_t launch_clear_step_state(StepState *st, hipStream_t s) {
  hipLaunchKernelGGL(k_clear_step_state, dim3(1), dim3(64), 0, s, st);
  return hipGetLastError();
}

hipError_t launch_adam_prologue(StepState *st, float lr, float beta1, float beta2, float eps, float weight_decay,
                                hipStream_t s) {
  hipLaunchKernelGGL(k_adam_prologue, dim3(1), dim3(64), 0, s, st, lr, beta1, beta2, eps, weight_decay);
  return hipGetLastError();
}

static AdamPtrs adam_ptrs(float *p, float *m, float *v, uint16_t *p_bf16, size_t first) {
  AdamPtrs q;
  q.p4 = reinterpret_cast<f32x4 *>(p + first);
  q.m4 = reinterpret_cast<f32x4 *>(m + first);
  q.v4 = reinterpret_cast<f32x4 *>(v + first);
  q.b2 = p_bf16 ? reinterpret_cast<u32x2 *>(p_bf16 + first) : nullptr;
  return q;
}

hipError_t launch_adamw(float *p, float *m, float *v, const float *g, uint16_t *p_bf16, size_t begin, size_t end,
                        const AdamArgs &h, const AdamArgs *device_args, hipStream_t s) {
  if (begin >= end) return hipSuccess;
  const Span sp = make_span(begin, end);
  const Shape sh = tuning().shape[kAdamw];
  const int Uv = sh.vecs, Tv = tuning().threads;
  unsigned grid;
  if (!grid_for(sp.nvec, Tv, Uv, &grid)) return hipErrorInvalidConfiguration;
  const AdamPtrs q = adam_ptrs(p, m, v, p_bf16, sp.vbegin);
  if (grid)
    with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
      constexpr int T = decltype(t)::value, U = decltype(u)::value;
      constexpr bool NT = decltype(nt)::value;
      const unsigned lds = lds_share(sh.waves, T);
      const f32x4 *g4 = reinterpret_cast<const f32x4 *>(g + sp.vbegin);
      auto go = [&](auto bf, auto dev) {
        hipLaunchKernelGGL((k_adamw<T, U, NT, decltype(bf)::value, decltype(dev)::value>), dim3(grid), dim3(T), lds, s, q,
                           g4, sp.nvec, h, device_args);
      };
      auto with_dev = [&](auto bf) {
        if (device_args) go(bf, std::true_type{});
        else go(bf, std::false_type{});
      };
      if (p_bf16) with_dev(std::true_type{});
      else with_dev(std::false_type{});
    });
  if (ragged(sp)) hipLaunchKernelGGL(k_adamw_ragged, dim3(1), dim3(64), 0, s, p, m, v, g, p_bf16, sp, h, device_args);
  return hipGetLastError();
}

hipError_t launch_reduce_adamw(const ReduceArgs &a, float *p, float *m, float *v, uint16_t *p_bf16, bool write_grad,
                               size_t begin, size_t end, const AdamArgs &h, const AdamArgs *device_args,
                               hipStream_t s) {
  if (begin >= end) return hipSuccess;
  if (a.n_src > tuning().one_pass_max) {
    if (hipError_t he = launch_reduce(a, begin, end, s)) return he;
    return launch_adamw(p, m, v, a.out, p_bf16, begin, end, h, device_args, s);
  }
  const Span sp = make_span(begin, end);
  const Shape sh = tuning().shape[kReduceAdamw];
  const int Uv = sh.vecs, Tv = tuning().threads;
  unsigned grid;
  if (!grid_for(sp.nvec, Tv, Uv, &grid)) return hipErrorInvalidConfiguration;
  const AdamPtrs q = adam_ptrs(p, m, v, p_bf16, sp.vbegin);
  if (grid)
    with_shape(Tv, Uv, tuning().nontemporal, [&](auto t, auto u, auto nt) {
      constexpr int T = decltype(t)::value, U = decltype(u)::value;
      constexpr bool NT = decltype(nt)::value;
      const unsigned lds = lds_share(sh.waves, T);
      auto go = [&](auto wg, auto bf, auto d, auto dev) {
        hipLaunchKernelGGL((k_reduce_adamw<T, U, NT, decltype(wg)::value, decltype(bf)::value, decltype(d)::value,
                                           decltype(dev)::value>),
                           dim3(grid), dim3(T), lds, s, a, q, sp.vbegin, sp.nvec, h, device_args);
      };
      auto with_dev = [&](auto wg, auto bf, auto d) {
        if (device_args) go(wg, bf, d, std::true_type{});
        else go(wg, bf, d, std::false_type{});
      };
      auto with_d = [&](auto wg, auto bf) {
        if (sh.depth == 1) with_dev(wg, bf, Int<1>{});
        else with_dev(wg, bf, Int<2>{});
      };
      auto with_bf = [&](auto wg) {
        if (p_bf16) with_d(wg, std::true_type{});
        else with_d(wg, std::false_type{});
      };
      if (write_grad) with_bf(std::true_type{});
      else with_bf(std::false_type{});
    });
  if (ragged(sp)) {
    if (write_grad)
      hipLaunchKernelGGL(k_reduce_adamw_ragged<true>, dim3(1), dim3(64), 0, s, a, p, m, v, p_bf16, sp, h, device_args);
    else
      hipLaunchKernelGGL(k_reduce_adamw_ragged<false>, dim3(1), dim3(64), 0, s, a, p, m, v, p_bf16, sp, h, device_args);
  }
  return hipGetLastError();
}

hipError_t launch_compare(const float *x, const float *ref, size_t n, CompareResult *out, hipStream_t s) {
  hipLaunchKernelGGL(k_compare_clear, dim3(1), dim3(256), 0, s, out);
  if (n > 0) {
    size_t blocks = (n / 4 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 256 * 4) blocks = 256 * 4;  // four workgroups of four wavefronts per CU
    hipLaunchKernelGGL(k_compare, dim3((unsigned)blocks), dim3(256), 0, s, x, ref, n, out);
  }
  return hipGetLastError();
}

}  // namespace recover
