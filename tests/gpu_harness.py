"""Helpers of the GPU parity tests: an adapter that lets the shared driver feed the HIP
library, sampling of element indices for shards too large for the CPU oracle, and the
error measures of the parity bar."""
import numpy as np

from paper_2605_11215_amd import binding as B
from paper_2605_11215_amd import synth
from paper_2605_11215_amd.synth import reference_np as S


def view_hip(s):
    q = s.query()
    return dict(alive=[r for r in range(s.W) if q["role"][r] != B.ROLE_DEAD], target=q["target"],
                contributed=q["contributed"], loop_bound=q["loop_bound"], role=q["role"], epoch=q["epoch"])


class HipEngine:
    """Forwards the driver's calls to a Shard; gradients may be NumPy arrays (uploaded) or
    device tensors."""

    def __init__(self, shard, bf16=False):
        import torch
        self.torch, self.s, self.bf16 = torch, shard, bf16
        self._keep = []

    def __getattr__(self, k):
        return getattr(self.s, k)

    def accumulate_many(self, replicas, ids, grads):
        return self.s.accumulate_many(replicas, ids, [self._device(g) for g in grads])

    def accumulate(self, r, mb, g, tb=0, te=None, snapshot=False):
        return self.s.accumulate(r, mb, self._device(g), tb, te, snapshot=snapshot)

    def _device(self, g):
        torch = self.torch
        if isinstance(g, np.ndarray):
            if self.bf16:
                h = torch.from_numpy(S.f32_to_bf16_bits(g).view(np.int16)).cuda().view(torch.bfloat16)
            else:
                h = torch.from_numpy(g).cuda()
            if h.numel() < 8:
                h = torch.cat([h, torch.zeros(8, dtype=h.dtype, device=h.device)])
            g = h
        return g


def device_grad_source(cfg, buf):
    """grad_of(t, mb) that regenerates the microbatch gradient into the one device buffer `buf`
    (stream-ordered with the accumulate that consumes it)."""
    def grad_of(t, mb):
        return synth.fill_device(buf, cfg["seed"], S.TAG_GRAD, mb, t, cfg["scale"], cfg["kind"])
    return grad_of


def sampled_grad_source(cfg, idx):
    """grad_of(t, mb) for the oracle: the same stream at the sampled indices, as fp32 values
    (bf16-rounded when the workload feeds bf16 gradients)."""
    cache = {}

    def grad_of(t, mb):
        if (t, mb) not in cache:
            if len(cache) > 256:
                cache.clear()
            v = S.values(idx, cfg["seed"], S.TAG_GRAD, mb, t, cfg["scale"], cfg["kind"])
            if cfg["bf16"]:
                v = S.bf16_bits_to_f32(S.f32_to_bf16_bits(v))
            cache[(t, mb)] = v
        return cache[(t, mb)]
    return grad_of


def sample_indices(off, n_random, seed, edge=64, windows=()):
    """Per tensor: its first and last `edge` elements, a share of n_random random ones, and the part of
    every contiguous window (start, length) that falls inside it.  Returns (sorted unique global indices,
    offsets of the sampled shard)."""
    rng = np.random.default_rng(seed)
    N = off[-1]
    idx, soff = [], [0]
    for b in range(len(off) - 1):
        lo, hi = off[b], off[b + 1]
        n = hi - lo
        if n <= 2 * edge + 16:
            pick = np.arange(lo, hi)
        else:
            k = max(8, int(n_random * n / max(N, 1)))
            parts = [np.arange(lo, lo + edge), np.arange(hi - edge, hi), rng.integers(lo, hi, k)]
            for w0, wn in windows:
                a, z = max(lo, w0), min(hi, w0 + wn)
                if a < z:
                    parts.append(np.arange(a, z))
            pick = np.unique(np.concatenate(parts))
        idx.append(pick)
        soff.append(soff[-1] + len(pick))
    return np.concatenate(idx).astype(np.int64), soff


def contiguous_windows(N, n_windows, length, seed):
    """Windows of `length` consecutive elements: across the element whose fp32 byte offset is 2^32 and the one
    at 2^31 (where 32-bit byte offsets would wrap), at both ends of the shard, and at random odd starts, so
    that whole workgroup tiles, their borders and tensor borders are compared, not isolated elements."""
    rng = np.random.default_rng(seed)
    starts = [0, max(0, N - length)]
    for e in (1 << 30, 1 << 29):
        if e + length // 2 < N:
            starts.append(e - length // 2)
    while len(starts) < n_windows:
        starts.append(int(rng.integers(0, max(1, N - length))) | 1)
    return [(s0, length) for s0 in starts[:n_windows]]


def gather(t, idx_dev):
    """Values of the flat device tensor t at the device index tensor, as a NumPy array."""
    return t[idx_dev].cpu().numpy()


def max_rel(x, ref):
    """Max-norm relative error: max|x - ref| / max|ref|."""
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.max(np.abs(ref))
    return float(np.max(np.abs(x - ref)) / den) if den > 0 else float(np.max(np.abs(x - ref)))


def assert_adamw_elementwise(before, g, t, hp, got, ref):
    """Every element of the AdamW state against the fp64 step `ref` = (p, m, v) computed from the same fp32
    inputs `before` = (p, m, v) and gradient g, with bounds that follow the kernel's roundings (u = 2^-23):
      exp_avg     product, fused multiply-add, rounded constant 1 - beta1: <= 1.5 u of the terms' size
                  |beta1 m| + |(1 - beta1) g|; gate 2 u of it (the result itself may cancel)
      exp_avg_sq  g g, its product with the rounded 1 - beta2, fused multiply-add: <= 2 u v; gate 3 u v
      param       p (1 - lr wd) and the final fused multiply-add: <= 1.5 u |p|; the update inherits exp_avg's
                  error and adds sqrt, two rounded constants, a fused multiply-add and the divide: <= 4.5 u of
                  the update's size; gate 2 u |p| + 8 u |step_size| (|beta1 m| + |(1 - beta1) g|) / denominator.
    A per-element defect on a small-magnitude entry, invisible to a max-norm bar, fails these."""
    u = 2.0 ** -23
    tiny = 1e-44
    p0, m0, _ = [np.asarray(x, np.float64) for x in before]
    g = np.asarray(g, np.float64)
    p, m, v = [np.asarray(x, np.float64) for x in ref]
    gp, gm, gv = [np.asarray(x, np.float64) for x in got]
    b1, b2 = hp["beta1"], hp["beta2"]
    scale_m = np.abs(b1 * m0) + np.abs((1.0 - b1) * g)
    bad = np.abs(gm - m) > 2 * u * scale_m + tiny
    assert not bad.any(), "exp_avg: %d elements off, worst %g" % (bad.sum(), np.max(np.abs(gm - m) / (scale_m + tiny)))
    bad = np.abs(gv - v) > 3 * u * v + tiny
    assert not bad.any(), "exp_avg_sq: %d elements off" % bad.sum()
    denom = np.sqrt(v / (1.0 - b2 ** t)) + hp["eps"]
    upd = hp["lr"] / (1.0 - b1 ** t) * scale_m / denom
    bound = u * (2 * np.abs(p0) + 8 * upd) + tiny
    bad = np.abs(gp - p) > bound
    assert not bad.any(), "param: %d elements off, worst %g of its bound" % (bad.sum(), np.max(np.abs(gp - p) / bound))


def bits_equal(a, b):
    return np.array_equal(np.asarray(a, np.float32).view(np.uint32), np.asarray(b, np.float32).view(np.uint32))
