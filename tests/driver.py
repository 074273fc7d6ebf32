"""The caller's side of Alg. 1 lives in the package (paper_2605_11215_amd/loop.py) because the
attrition report uses it too; the tests import it from here."""
from paper_2605_11215_amd.loop import HP, run_iteration, view_oracle, eng_committed_ids  # noqa: F401
