"""The five synthetic workloads (shapes, seeds, failure schedules) used by the benchmark and
the GPU parity tests.  Each stands in for one GPU's parameter shard of the named model;
gradients come from the seeded streams in paper_2605_11215_amd.synth, never from a dataset.

Failure schedules: {iteration: {replica: n}} = the replica crashes having accumulated n
microbatches of that iteration; the survivors learn of it at the synchronisation point.
Iterations, replicas and offsets count from 0."""
from paper_2605_11215_amd.synth import reference_np as S


def offsets(shapes):
    off = [0]
    for s in shapes:
        n = 1
        for d in (s if isinstance(s, tuple) else (s,)):
            n *= d
        off.append(off[-1] + n)
    return off


def gpt2_small_shapes():
    """148 tensors, 123,589,632 elements: embedding, then 12 layers of q,k,v,o (768x768),
    fc (768x3072), proj (3072x768) and six 768-vectors, then three final 768-vectors."""
    shapes = [(50257, 768)]
    for _ in range(12):
        shapes += [(768, 768)] * 4 + [(768, 3072), (3072, 768)] + [768] * 6
    shapes += [768] * 3
    return shapes


def llama3_8b_hsdp8_shapes():
    """One GPU's 1/8 share under 8-way HSDP: 4 layers of 2x(4096x4096), 2x(1024x4096),
    2x(4096x14336), 1x(14336x4096), plus embedding and head rows 128256/8 = 16032."""
    shapes = []
    for _ in range(4):
        shapes += [(4096, 4096)] * 2 + [(1024, 4096)] * 2 + [(4096, 14336)] * 2 + [(14336, 4096)]
    shapes += [(16032, 4096)] * 2
    return shapes


def attrition_shapes():
    return ([(2048, 2048)] * 4 + [(2048, 8192)] * 2) * 2


def llama70b_split16_shapes():
    """37 layers of the 70B-like tensors split 1/16 row-wise."""
    layer = [(512, 8192)] * 2 + [(64, 8192)] * 2 + [(512, 28672)] + [(1792, 8192)] * 2
    return layer * 37


CONFIGS = {
    1: dict(name="tiny", W=4, G=2, off=[0, 1048576], bf16=False, scale=1e-3, kind=S.KIND_NORMAL, seed=1, iters=3,
            schedule={1: {2: 1}}),
    2: dict(name="gpt2-small-shard", W=8, G=4, off=offsets(gpt2_small_shapes()), bf16=False, scale=1e-3,
            kind=S.KIND_NORMAL, seed=1, iters=5, schedule={2: {3: 2, 6: 2}}),
    3: dict(name="llama3-8b-hsdp8-shard", W=8, G=8, off=offsets(llama3_8b_hsdp8_shapes()), bf16=True, scale=5e-4,
            kind=S.KIND_NORMAL, seed=1, iters=4, schedule={t: {2 * t + 1: t + 1} for t in range(4)},
            fidelity=True),
    4: dict(name="heavy-attrition", W=64, G=2, off=offsets(attrition_shapes()), bf16=False, scale=1e-3,
            kind=S.KIND_NORMAL, seed=1, iters=16, schedule={t: {2 * t: 1, 2 * t + 1: 1} for t in range(16)},
            snapshot_every=True),
    5: dict(name="mixed-precision-stress", W=4, G=4, off=offsets(llama70b_split16_shapes()), bf16=True, scale=1e-3,
            kind=S.KIND_STUDENT_T3, seed=1, iters=4, schedule=None),
}

assert len(CONFIGS[2]["off"]) - 1 == 148 and CONFIGS[2]["off"][-1] == 123589632
assert len(CONFIGS[3]["off"]) - 1 == 30 and CONFIGS[3]["off"][-1] == 1003749376
assert len(CONFIGS[4]["off"]) - 1 == 12 and CONFIGS[4]["off"][-1] == 100663296
assert len(CONFIGS[5]["off"]) - 1 == 259 and CONFIGS[5]["off"][-1] == 1978662912
