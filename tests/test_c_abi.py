"""include/recover.h is valid C99 and the library is usable from plain C: a C program runs the
paper's printed W=32, G=8 example through the ABI on a host-only context (no GPU work) and its
output is compared with the golden values.  CPU only."""
import os
import subprocess

from tests.test_oracle_policy import load_golden

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
PKG = os.path.join(ROOT, "paper_2605_11215_amd")


def test_header_is_c99_and_the_walkthrough_runs_from_c(tmp_path):
    exe = str(tmp_path / "walkthrough")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(HERE, "c_abi_walkthrough.c"), "-o", exe, "-L", PKG, "-lrecover",
                    "-Wl,-rpath," + PKG, "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    got = {}
    for line in out.splitlines():
        k, v = [x.strip() for x in line.split("=")]
        got[k] = int(v) if v.lstrip("-").isdigit() else v
    g = load_golden()
    for k in ("B", "W_cur_after_first", "C_cur", "at_boundary", "G_ext", "n_bdry", "loop_bound_after",
              "majors_extended", "restore_mode_first", "G_cur", "n_maj", "R_cur", "n_min", "n_ms", "n_mi", "minor_is",
              "minor_spare_is", "at_boundary_second", "loop_bound_second", "restore_mode_second", "promoted_second"):
        assert got[k] == g[k], (k, got.get(k), g[k])
    assert got["boundary_minors_at_8"] == g["n_bdry"]
