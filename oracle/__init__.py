"""CPU oracle for the ReCoVer data-parallel numeric path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, independent statement of what the
path computes, written from the paper (Sec. 4.2, Sec. 4.3, Alg. 1, 2, 4-8, the boundary-step
walk-through appendix and the proof-sketch appendix).  It shares no code with the HIP
library and never imports it.  Only the test-suite, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product path never does.

Modules
  policy  integer versatile-workload policy (Alg. 6, 7, 8; Record step of Alg. 2)
  proto   step-by-step simulator of one replica set on NumPy arrays (Alg. 1, 2, 5)
  brute   the definition of the iteration gradient: (1/B) * sum over committed microbatches
  adamw   textbook decoupled-weight-decay Adam step in fp64

Pins (see tests/test_oracle_*.py): the printed W=32, G=8 example; Eq. 1 on exhaustive
sweeps; minimality of G_ext and G_cur by counting up; proto == brute on small inputs;
constant-gradient closed form; restore == never accumulated; AdamW against
torch.optim.AdamW (fp64, CPU) and the first-step closed form.  No function here is
"parity unpinned" except the identity of the boundary minors (only their number is
printed by the paper) and the failure schedules of the synthetic configs, which are free
choices and not results.
"""
