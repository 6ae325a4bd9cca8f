"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's sources (a
dropped term, a flipped sign, a wrong constant, a swapped operand), compiles the copy, and runs the
pin files of that component against it: at least one pin must fail.  CPU only; nothing here
touches the GPU path, and the in-tree oracle is never modified."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle")

PHILOX = ["tests/test_oracle_philox.py"]
PONG = ["tests/test_oracle_pong.py", "tests/test_oracle_pixels.py"]
BODY = ["tests/test_oracle_body.py"]
NEWTON = ["tests/test_oracle_body_newton.py"]
CART = ["tests/test_oracle_cartpole.py"]

# (name, source file, text as it stands, text with the mistake, pin files to run)
MUTANTS = [
    ("philox: multipliers swapped", "philox.cpp",
     "const uint64_t pa = (uint64_t)kMulA * (uint64_t)c0;", "const uint64_t pa = (uint64_t)kMulB * (uint64_t)c0;", PHILOX),
    ("philox: nine rounds", "philox.cpp", "round < 10", "round < 9", PHILOX),
    ("philox: key bumped before the first round too", "philox.cpp", "if (round > 0) {", "if (round >= 0) {", PHILOX),
    ("philox: hi and lo words exchanged", "philox.cpp",
     "const uint32_t n1 = lo_b;", "const uint32_t n1 = lo_a;", PHILOX),
    ("uniform: 23 bits instead of 24", "philox.cpp",
     "float oracle_u01(uint32_t w) { return (float)(w >> 8) * 5.9604644775390625e-8f; }",
     "float oracle_u01(uint32_t w) { return (float)(w >> 9) * 5.9604644775390625e-8f; }", PHILOX + PONG),
    ("pong: wall mirror keeps vy", "pong.cpp",
     "if (e->by < 0.0f) { e->by = -e->by; e->vy = -e->vy; }", "if (e->by < 0.0f) { e->by = -e->by; }", PONG),
    ("pong: opponent one unit faster", "pong.cpp", "OPP_SPEED = 3.0f", "OPP_SPEED = 4.0f", PONG),
    ("pong: reward signs exchanged", "pong.cpp",
     "if (e->bx < 0.0f) { reward = 1.0f; e->sa += 1; }", "if (e->bx < 0.0f) { reward = -1.0f; e->sa += 1; }", PONG),
    ("pong: spin measured from the paddle top", "pong.cpp",
     "e->vy = 0.2f * ((e->by + 1.0f) - (e->pa + 8.0f));", "e->vy = 0.2f * ((e->by + 1.0f) - (e->pa));", PONG),
    ("pong: serve one unit off centre", "pong.cpp", "SERVE_X = 79.0f", "SERVE_X = 80.0f", PONG),
    ("pixels: touching edges count as overlap", "pong.cpp",
     "if (left < FIELD_W * (float)(c + 1) && right > FIELD_W * (float)c &&",
     "if (left <= FIELD_W * (float)(c + 1) && right >= FIELD_W * (float)c &&", PONG),
    ("body: bias force sign", "body.cpp",
     "h[j] += m * (k.J[0][j] * k.jdqd[0] + k.J[1][j] * k.jdqd[1]);",
     "h[j] -= m * (k.J[0][j] * k.jdqd[0] + k.J[1][j] * k.jdqd[1]);", BODY),
    ("body: rod inertia about the end", "body.cpp",
     "LINK_LEN[i] * LINK_LEN[i] / 12.0", "LINK_LEN[i] * LINK_LEN[i] / 3.0", BODY),
    ("body: gravity pushes up", "body.cpp",
     "Qg[j] += k.J[1][j] * (-m * P.gravity);", "Qg[j] += k.J[1][j] * (m * P.gravity);", BODY),
    ("body: contact damper sign", "body.cpp",
     "fn = -P.contact_k * k.pos[1] - P.contact_c * k.vel[1];", "fn = -P.contact_k * k.pos[1] + P.contact_c * k.vel[1];", BODY),
    ("body: friction pushes along the motion", "body.cpp", "ft = -want;", "ft = want;", BODY),
    ("body: limit projection keeps the coupling column", "body.cpp",
     "for (int k = 0; k < NQ; ++k) { M[j][k] = 0; M[k][j] = 0; }", "for (int k = 0; k < NQ; ++k) { M[j][k] = 0; }", BODY),
    ("body: reward takes the last substep's velocity", "body.cpp",
     "R reward = vx_sum / (R)P.substeps - (R)0.1 * cost;", "R reward = e->v[0] - (R)0.1 * cost;", BODY),
    ("body: action cost of the unclipped action", "body.cpp",
     "cost += a[j] * a[j];", "cost += a_in[j] * a_in[j];", BODY),
    ("body: fifth action reuses a word of stream 0", "body.cpp",
     "a[4] = (R)(-1.0f + 2.0f * oracle_u01(w1[0]));", "a[4] = (R)(-1.0f + 2.0f * oracle_u01(w0[0]));", BODY),
    ("body: non-finite step keeps its reward", "body.cpp",
     "    info->done = 1;\n    reward = 0;\n", "    info->done = 1;\n", BODY),
    ("body: non-finite step counted as an episode", "body.cpp",
     "if (info.nonfinite) st->nonfinite += 1;\n      else if (info.done) {",
     "if (info.nonfinite) st->nonfinite += 1;\n      if (info.done) {", BODY),
    ("body: non-finite state re-initialised with this step's draws", "body.cpp",
     "info->fin_len = e->ep_len + 1;\n    reset_env(P, e, seed, env, step + 1);",
     "info->fin_len = e->ep_len + 1;\n    reset_env(P, e, seed, env, step);", BODY),
    ("body: storage rounding skips the velocities", "body.cpp",
     "e->q[j] = (R)(float)e->q[j]; e->v[j] = (R)(float)e->v[j];", "e->q[j] = (R)(float)e->q[j];", BODY),
    ("newton: velocity-product term dropped from the reference", "body.cpp",
     "rows->aref[i] = -b * jv - k * kin.pos[1] - (kin.jdqd[1] + smu * kin.jdqd[0]);",
     "rows->aref[i] = -b * jv - k * kin.pos[1];", NEWTON),
    ("newton: both pyramid edges on the same side", "body.cpp",
     "const R smu = e == 0 ? P.friction_mu : -P.friction_mu;", "const R smu = P.friction_mu;", NEWTON),
    ("newton: right-hand side without the row weight", "body.cpp",
     "g[x] += rows.D[i] * rows.aref[i] * rows.J[i][x];", "g[x] += rows.aref[i] * rows.J[i][x];", NEWTON),
    ("newton: limit rows damp the wrong way", "body.cpp",
     "rows->aref[i] = -b * (sign * v[j]);", "rows->aref[i] = b * (sign * v[j]);", NEWTON),
    ("cartpole: angular acceleration sign", "cartpole.cpp",
     "*thacc = (9.8f * s - c * temp) / denom;", "*thacc = (9.8f * s + c * temp) / denom;", CART),
    ("cartpole: pole inertia factor", "cartpole.cpp", "(4.0f / 3.0f)", "(1.0f / 3.0f)", CART),
    ("cartpole: velocity updated before the position", "cartpole.cpp",
     "e->x = e->x + 0.02f * e->xd;\n  e->xd = e->xd + 0.02f * xacc;",
     "e->xd = e->xd + 0.02f * xacc;\n  e->x = e->x + 0.02f * e->xd;", CART),
]


@pytest.fixture(scope="module")
def build_mod():
    import importlib.util
    spec = importlib.util.spec_from_file_location("build_oracle", os.path.join(ORACLE, "build_oracle.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


@pytest.mark.parametrize("name,src,good,bad,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(tmp_path, build_mod, name, src, good, bad, pins):
    for f in build_mod.SOURCES:
        shutil.copy(os.path.join(ORACLE, f), tmp_path / f)
    text = (tmp_path / src).read_text()
    assert text.count(good) == 1, "the source no longer contains this line exactly once: %r" % good
    (tmp_path / src).write_text(text.replace(good, bad))
    lib = build_mod.build(force=True, src_dir=str(tmp_path), out=str(tmp_path / "liboracle_mutant.so"))
    env = dict(os.environ, MI355ENV_ORACLE_LIB=lib)
    # the golden trajectory digest is itself a pin of the Pong oracle
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + pins,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode != 0, "every pin passed with this mistake planted: %s\n%s" % (name, r.stdout[-400:])
    assert " failed" in r.stdout or " error" in r.stdout, r.stdout[-400:]


def test_control_an_unchanged_copy_passes_every_pin(tmp_path, build_mod):
    """The same machinery with no mistake planted: the copy must pass, so a failure above is the
    mistake's doing and not the harness's."""
    for f in build_mod.SOURCES:
        shutil.copy(os.path.join(ORACLE, f), tmp_path / f)
    lib = build_mod.build(force=True, src_dir=str(tmp_path), out=str(tmp_path / "liboracle_copy.so"))
    env = dict(os.environ, MI355ENV_ORACLE_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"]
                       + PHILOX + PONG + BODY + NEWTON + CART,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-800:]
