// Internal launch interface between the host bookkeeping (recover_host.cpp) and the gfx950
// kernels (kernels.hip).  All pointers are device pointers; [begin, end) are element indices
// into flat buffers; every launcher returns a hipError_t and never synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace recover {

constexpr int kMaxReplicas = 64;

// Kernel classes with a launch shape of their own (index of Tuning::shape).
enum KernelClass {
  kAccFirstF32 = 0,  // accumulate, first microbatch (no read of acc), fp32 gradient
  kAccRmwF32,        // accumulate, read-modify-write, fp32 gradient
  kAccFirstBf16,
  kAccRmwBf16,
  kCopy,             // snapshot / restore
  kReduce,
  kAdamw,
  kReduceAdamw,
  kAccSnapF32,       // accumulate with the second store to the snapshot (first or read-modify-write)
  kAccSnapBf16,
  kNumClasses
};

// vecs: 128-bit vectors each lane keeps in flight per stream {1, 2, 4}.
// waves: wavefronts resident per CU, 0 = as many as the hardware takes (32).  HBM efficiency falls once
// much more than ~48 KiB of loads per CU are outstanding (measured: the read latency at the memory
// interface and the L2's read-credit stalls rise, the launch takes 7-13 % more GPU cycles), so the kernels
// that keep several KiB per wavefront outstanding run faster with fewer resident wavefronts.  The limit is
// imposed by giving every workgroup a share of the CU's 160 KiB of LDS that it never touches.
// depth (reduce kernels only): contributors whose loads a wavefront has in flight at a time {1, 2}.
struct Shape {
  int vecs, waves, depth;
};

struct Tuning {
  int threads = 64;     // lanes per workgroup: 64 (one wavefront) or 256
  int nontemporal = 1;  // streaming cache hints on loads and stores
  // The one-pass reduce+AdamW kernel is used up to this many contributors; beyond it the same call launches the
  // reduction and then the update (same bits, 8 more bytes per element).  Measured on 100 M elements: the three
  // state stores at the end of a long contributor walk cost more than their bytes, and the more the longer the
  // walk (one pass against two kernels: 1.08 / 1.20 ms at 12 contributors, 2.44 / 2.45 at 32, 3.59 / 3.39 at 48,
  // 4.62 / 4.38 at 64, whatever the store's cache policy, one or three store streams, state loaded before or
  // after the walk).
  int one_pass_max = 32;
  // Defaults from sweeps on the four large benchmark workloads (one vector per lane everywhere).
  Shape shape[kNumClasses] = {
      {1, 0, 0},   // kAccFirstF32
      {1, 0, 0},   // kAccRmwF32
      {1, 0, 0},   // kAccFirstBf16
      {1, 0, 0},   // kAccRmwBf16
      {1, 0, 0},   // kCopy
      {1, 14, 2},  // kReduce: contributors in pairs, 14 wavefronts per CU
      {1, 10, 0},  // kAdamw: four loads per wavefront outstanding, 10 wavefronts per CU
      {1, 12, 2},  // kReduceAdamw
      {1, 16, 0},  // kAccSnapF32
      {1, 28, 0},  // kAccSnapBf16
  };
};
Tuning &tuning();

struct ReduceArgs {
  const float *src[kMaxReplicas];  // contributors, ascending replica index
  float *sum_dst[kMaxReplicas];    // buffers that also receive the undivided sum (in-place mode)
  int n_src;
  int n_sum_dst;
  float *out;
  float divisor;
};

// Device-side layout of recover_compare_result (include/recover.h); the two maxima are kept as the bit
// patterns of non-negative floats.
struct CompareResult {
  uint64_t n_mismatch, n_nan, checksum_x, checksum_ref;
  uint32_t max_abs_diff_bits, max_abs_ref_bits;
};
hipError_t launch_compare(const float *x, const float *ref, size_t n, CompareResult *out, hipStream_t s);

struct AccumulateManyArgs {
  float *acc[kMaxReplicas];
  const void *grad[kMaxReplicas];
  unsigned char first[kMaxReplicas];  // 1: this replica's first microbatch of the iteration (overwrite)
};
hipError_t launch_accumulate_many(const AccumulateManyArgs &a, int n_pairs, bool grad_is_bf16, size_t begin, size_t end,
                                  hipStream_t s);

// snap != nullptr: the new accumulator value is stored to snap as well (accumulate + snapshot in one pass)
hipError_t launch_accumulate(float *acc, float *snap, const void *grad, bool grad_is_bf16, bool first, size_t begin,
                             size_t end, hipStream_t s);
// restore only selects the kernel's name (snapshot or rewind) for traces
hipError_t launch_copy(float *dst, const float *src, size_t begin, size_t end, bool restore, hipStream_t s);

// dst[i][begin, end) = src[i][begin, end) for n_pairs buffer pairs in one launch.
struct CopyManyArgs {
  float *dst[kMaxReplicas];
  const float *src[kMaxReplicas];
};
hipError_t launch_copy_many(const CopyManyArgs &a, int n_pairs, size_t begin, size_t end, bool restore, hipStream_t s);
hipError_t launch_reduce(const ReduceArgs &a, size_t begin, size_t end, hipStream_t s);
// Per-step constants of AdamW: decay_mul = 1 - lr wd, step_size = lr / (1 - beta1^t),
// inv_sqrt_bc2 = 1 / sqrt(1 - beta2^t).
struct AdamArgs {
  float decay_mul, beta1, one_minus_beta1, beta2, one_minus_beta2, step_size, inv_sqrt_bc2, eps;
};

// The constants of the NEXT step from the running products beta1^t, beta2^t (updated in place), in
// double, with nothing fused, so that the host and the device arrive at the same bits.
__host__ __device__ inline AdamArgs next_adam_args(double &beta1_pow, double &beta2_pow, float lr, float beta1,
                                                   float beta2, float eps, float weight_decay) {
#pragma clang fp contract(off)
  beta1_pow = beta1_pow * (double)beta1;
  beta2_pow = beta2_pow * (double)beta2;
  const double bc1 = 1.0 - beta1_pow, bc2 = 1.0 - beta2_pow;
  AdamArgs a;
  const double lw = (double)lr * (double)weight_decay;
  a.decay_mul = (float)(1.0 - lw);
  a.beta1 = beta1;
  a.one_minus_beta1 = (float)(1.0 - (double)beta1);
  a.beta2 = beta2;
  a.one_minus_beta2 = (float)(1.0 - (double)beta2);
  a.step_size = (float)((double)lr / bc1);
  a.inv_sqrt_bc2 = (float)(1.0 / sqrt(bc2));
  a.eps = eps;
  return a;
}

// Optional device-resident step state (64 bytes, caller-owned, zero-filled before the first step): the
// step count and the running products live on the device, so a captured graph of an iteration advances
// them on every replay.
struct StepState {
  uint64_t step;
  double beta1_pow, beta2_pow;
  AdamArgs args;
  uint64_t reserved;
};
static_assert(sizeof(StepState) == 64, "StepState is 64 bytes");

// Step states owned by the library, for callers that cannot allocate device memory: kStaticStepSlots
// slots of one StepState each in a file-scope device array (every GPU holds its own copy).  Gives the
// address of slot `slot` on the CURRENT device; the symbol is resolved once per device.
constexpr int kStaticStepSlots = 64;
hipError_t static_step_state(int slot, StepState **out);
// Zero-fills *st with a one-thread kernel (no memset node, so the call can be captured into a graph).
hipError_t launch_clear_step_state(StepState *st, hipStream_t s);

// Advances *st by one step and stores that step's constants in st->args (one thread).
hipError_t launch_adam_prologue(StepState *st, float lr, float beta1, float beta2, float eps, float weight_decay,
                                hipStream_t s);

// device_args != nullptr: the kernel reads its constants from device memory instead of `h`.
// Elements [begin, end) of all five buffers.
hipError_t launch_adamw(float *p, float *m, float *v, const float *g, uint16_t *p_bf16, size_t begin, size_t end,
                        const AdamArgs &h, const AdamArgs *device_args, hipStream_t s);

// One pass up to tuning().one_pass_max contributors, else launch_reduce into a.out followed by launch_adamw.

hipError_t launch_reduce_adamw(const ReduceArgs &a, float *p, float *m, float *v, uint16_t *p_bf16, bool write_grad,
                               size_t begin, size_t end, const AdamArgs &h, const AdamArgs *device_args, hipStream_t s);

}  // namespace recover
