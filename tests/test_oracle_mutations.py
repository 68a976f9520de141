"""Do the oracle's pins notice a plausible mistake?  Each case plants ONE mistake in a copy of
oracle/jacobi_oracle.c - a dropped term, a wrong sign, index or constant, a residual of the wrong grid, a halo
copied from the wrong cell - builds it, and runs tests/test_oracle_pins.py against it in a subprocess: the pins
must FAIL.  The unchanged copy must pass.  CPU only; the mistakes are planted in the oracle, never in the GPU
path.  (Every mutant stays inside its arrays: a pin has to catch it, not a crash.)"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = os.path.join(ROOT, "oracle", "jacobi_oracle.c")

F64 = "DEFINE_ORACLE(double, f64, 0.25, (1.0 / 6.0), 4.0, 6.0)"
F32 = "DEFINE_ORACLE(float, f32, 0.25f, (1.0f / 6.0f), 4.0f, 6.0f)"
WE = "T we = A[i * P + (j - 1)] + A[i * P + (j + 1)];"
SN = "T sn = A[(i - 1) * P + j] + A[(i + 1) * P + j];"
ZZ = "T zz = A[c - Q] + A[c + Q];"
YY = "T yy = A[c - P] + A[c + P];"

# (name, text to find, which occurrence, replacement)
MUTANTS = [
    ("update2d_wrong_index", SN, 0, "T sn = A[(i - 1) * P + j] + A[(i + 1) * P + j + 1];"),
    ("update2d_dropped_east", WE, 0, "T we = A[i * P + (j - 1)] + A[i * P + (j - 1)];"),
    ("update2d_north_for_west", WE, 0, "T we = A[(i - 1) * P + j] + A[i * P + (j + 1)];"),
    ("update2d_sign", "B[i * P + j] = QUARTER * (we + sn);", 0, "B[i * P + j] = QUARTER * (we - sn);"),
    ("update2d_centre_weight", "B[i * P + j] = QUARTER * (we + sn);", 0, "B[i * P + j] = QUARTER * (we + sn) + QUARTER * A[i * P + j];"),
    ("update3d_y_for_z", ZZ, 0, "T zz = A[c - Q] + A[c + P];"),
    ("update3d_dropped_z", "B[c] = SIXTH * ((xx + yy) + zz);", 0, "B[c] = SIXTH * ((xx + yy) + yy);"),
    ("update3d_sign", "B[c] = SIXTH * ((xx + yy) + zz);", 0, "B[c] = SIXTH * ((xx - yy) + zz);"),
    ("update3d_dropped_south", YY, 0, "T yy = A[c - P] + A[c - P];"),
    ("residual2d_wrong_centre", "T r = (we + sn) - FOUR * A[i * P + j];", 0, "T r = (we + sn) - FOUR * A[i * P + j + 1];"),
    ("residual2d_sign", "T r = (we + sn) - FOUR * A[i * P + j];", 0, "T r = (we + sn) + FOUR * A[i * P + j];"),
    ("residual2d_dropped_east", WE, 1, "T we = A[i * P + (j - 1)] + A[i * P + (j - 1)];"),
    ("residual2d_no_square", "acc += (long double)r * (long double)r;", 0, "acc += (long double)r;"),
    ("residual2d_no_sqrt", "return (double)sqrtl(acc);", 0, "return (double)acc;"),
    ("residual3d_four_for_six", "T r = ((xx + yy) + zz) - SIX * A[c];", 0, "T r = ((xx + yy) + zz) - FOUR * A[c];"),
    ("residual3d_dropped_up", ZZ, 1, "T zz = A[c - Q] + A[c - Q];"),
    ("residual3d_no_sqrt", "return (double)sqrtl(acc);", 1, "return (double)acc;"),
    ("run_residual_one_iteration_early", "k % res_every == 0 && res_out", 0, "(k + 1) % res_every == 0 && res_out"),
    ("run_residual_of_the_older_grid", "oracle_residual2d_##SUF(src, Ny, Nx)", 0, "oracle_residual2d_##SUF(dst, Ny, Nx)"),
    ("tiled_y_halo_from_wrong_row", "b[(k * py + 0) * px + j] = n[(k * py + by) * px + j];", 0,
     "b[(k * py + 0) * px + j] = n[(k * py + by - 1) * px + j];"),
    ("tiled_x_halo_from_wrong_column", "b[(k * py + i) * px + bx + 1] = n[(k * py + i) * px + 1];", 0,
     "b[(k * py + i) * px + bx + 1] = n[(k * py + i) * px + 2];"),
    ("tiled_z_halo_from_wrong_plane", "b[((bz + 1) * py + i) * px + j] = n[(1 * py + i) * px + j];", 0,
     "b[((bz + 1) * py + i) * px + j] = n[(2 * py + i) * px + j];"),
    ("f64_quarter", F64, 0, F64.replace("0.25,", "0.2,")),
    ("f64_sixth", F64, 0, F64.replace("(1.0 / 6.0)", "(1.0 / 5.0)")),
    ("f64_sixth_truncated", F64, 0, F64.replace("(1.0 / 6.0)", "0.16666666")),
    ("f64_four", F64, 0, F64.replace("4.0,", "3.0,")),
    ("f64_six", F64, 0, F64.replace("6.0)", "5.0)")),
    ("f32_quarter", F32, 0, F32.replace("0.25f,", "0.2f,")),
    ("f32_sixth", F32, 0, F32.replace("(1.0f / 6.0f)", "(1.0f / 5.0f)")),
    ("f32_sixth_truncated", F32, 0, F32.replace("(1.0f / 6.0f)", "0.1666f")),
    ("f32_four", F32, 0, F32.replace("4.0f,", "3.0f,")),
    ("f32_six", F32, 0, F32.replace("6.0f)", "5.0f)")),
    ("f32_six_is_four", F32, 0, F32.replace("6.0f)", "4.0f)")),
]


def nth_replace(text, find, n, repl):
    pos = -1
    for _ in range(n + 1):
        pos = text.find(find, pos + 1)
        assert pos >= 0, f"pattern not found ({n + 1} times): {find}"
    return text[:pos] + repl + text[pos + len(find):]


def pins_pass(src_path):
    # the copy must BUILD (with the oracle's own flags): a mutant is to be caught by a pin, not by the compiler
    subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
                    "-Werror", "-o", os.path.splitext(src_path)[0] + ".so", src_path, "-lm"], check=True)
    env = dict(os.environ, JACOBI_ORACLE_SRC=src_path, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode in (0, 1), r.stdout[-2000:] + r.stderr[-2000:]      # 1 = a pin failed; anything else is an accident
    return r.returncode == 0


def test_unchanged_copy_passes_the_pins(tmp_path):
    path = tmp_path / "oracle_copy.c"
    path.write_text(open(SOURCE).read())
    assert pins_pass(str(path))


@pytest.mark.parametrize("name,find,n,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_a_planted_mistake(tmp_path, name, find, n, repl):
    text = open(SOURCE).read()
    assert text.count(find) > n
    path = tmp_path / f"{name}.c"
    path.write_text(nth_replace(text, find, n, repl))
    assert not pins_pass(str(path)), f"mutant {name} survived every pin"
