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


def sample_indices(off, n_random, seed, edge=64):
    """Per tensor: its first and last `edge` elements plus a share of n_random random ones.
    Returns (sorted unique global indices, offsets of the sampled shard)."""
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
            pick = np.unique(np.concatenate([np.arange(lo, lo + edge), np.arange(hi - edge, hi),
                                             rng.integers(lo, hi, k)]))
        idx.append(pick)
        soff.append(soff[-1] + len(pick))
    return np.concatenate(idx).astype(np.int64), soff


def gather(t, idx_dev):
    """Values of the flat device tensor t at the device index tensor, as a NumPy array."""
    return t[idx_dev].cpu().numpy()


def max_rel(x, ref):
    """Max-norm relative error: max|x - ref| / max|ref|."""
    x = np.asarray(x, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.max(np.abs(ref))
    return float(np.max(np.abs(x - ref)) / den) if den > 0 else float(np.max(np.abs(x - ref)))


def bits_equal(a, b):
    return np.array_equal(np.asarray(a, np.float32).view(np.uint32), np.asarray(b, np.float32).view(np.uint32))
