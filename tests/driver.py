"""Iteration drivers of the tests.  The oracle is driven by its OWN statement of Alg. 1
(oracle/loop.py); the HIP library by the caller loop of its package
(paper_2605_11215_amd/loop.py).  `run_iteration` picks by the engine it is handed, so a test
writes the same line for both sides while the two loops share no code; tests/test_loops.py checks
that they issue the same calls."""
from oracle.loop import run_iteration as oracle_iteration
from oracle.proto import Proto
from paper_2605_11215_amd.loop import HP, run_iteration as library_iteration, eng_committed_ids  # noqa: F401


def view_oracle(p):
    """State view of a Proto (or of anything that keeps its bookkeeping in `.world`)."""
    w = p.world
    return dict(alive=w.alive(), target=list(w.target), contributed=list(w.contributed),
                loop_bound=w.loop_bound, role=list(w.role), epoch=w.eps)


def run_iteration(eng, view, t, grad_of, W_init, dying=None, fidelity_k=0, snapshot_every=False, hp=HP,
                  on_sync=None, fuse=False, batch=False):
    if isinstance(eng, Proto):
        assert W_init == eng.world.W_init and on_sync is None
        return oracle_iteration(eng, t, grad_of, dying=dying, reduced_before_failure=fidelity_k,
                                snapshot_every=snapshot_every, hp=hp)
    return library_iteration(eng, view, t, grad_of, W_init, dying=dying, fidelity_k=fidelity_k,
                             snapshot_every=snapshot_every, hp=hp, on_sync=on_sync, fuse=fuse, batch=batch)
