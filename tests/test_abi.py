"""The C-ABI library loads and exports every symbol include/mi355env.h declares (CPU only: no
kernel is launched; the argument checks exercised here return before any HIP call)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mi355env.h")


@pytest.fixture(scope="module")
def L():
    from paper_2603_12145_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2603_12145_amd import build
        build.build(force=True)
    return binding.lib()


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(env_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = _declared()
    assert {"env_create", "env_reset", "env_step", "env_rollout", "env_stats", "env_get_state",
            "env_set_state", "env_destroy"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_every_tuning_symbol_is_exported(L):
    text = open(os.path.join(ROOT, "include", "mi355env_tuning.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(mi355env_[a-z_]+)\s*\(", text)))
    assert len(names) == 21, names
    for n in names:
        assert hasattr(L, n), n
    assert L.mi355env_tune_paged_stores(9) == -1 and L.mi355env_tune_paged_stores(2) == 0
    assert L.mi355env_tune_rollout(100, 1) == -1 and L.mi355env_tune_rollout(0, 1) == 0
    assert L.mi355env_tune_step_kernel(3) == -1 and L.mi355env_tune_step_kernel(1) == 0


def test_dims_and_strings(L):
    from paper_2603_12145_amd import binding as b
    assert b.env_obs_dim(b.ENV_PONG) == 8
    assert b.env_obs_dim(b.ENV_PONG_PIXELS) == 4 * 84 * 84
    assert b.env_obs_dim(b.ENV_BODY) == 17
    assert b.env_obs_dim(b.ENV_CARTPOLE) == 4 and b.env_action_dim(b.ENV_CARTPOLE) == 1
    assert b.env_obs_dim(99) == b.ENV_E_ARG
    assert b.env_action_dim(b.ENV_PONG) == 1 and b.env_action_dim(b.ENV_BODY) == 6
    for code in (0, -1, -2, -3, -4, -5, -6, -99):
        assert isinstance(b.env_strerror(code), str) and b.env_strerror(code)


def test_argument_errors_without_gpu(L):
    from paper_2603_12145_amd import binding as b
    h = C.c_void_p()
    assert L.env_create(None, 0, 64, 0, None, None) == b.ENV_E_ARG
    assert L.env_create(C.byref(h), 7, 64, 0, None, None) == b.ENV_E_ARG
    assert L.env_create(C.byref(h), 0, 0, 0, None, None) == b.ENV_E_ARG
    assert L.env_create(C.byref(h), 0, -5, 0, None, None) == b.ENV_E_ARG
    assert L.env_create(C.byref(h), 0, (1 << 30) + 1, 0, None, None) == b.ENV_E_ARG
    bad = b.env_config_t(struct_size=2)
    assert L.env_create(C.byref(h), 0, 64, 0, C.byref(bad), None) == b.ENV_E_ARG
    assert h.value is None
    assert L.env_reset(None, None) == b.ENV_E_ARG
    assert L.env_set_stream(None, None) == b.ENV_E_ARG
    odd = b.env_config_t(struct_size=C.sizeof(b.env_config_t), step_counter=7)
    assert L.env_create(C.byref(h), 0, 64, 0, C.byref(odd), None) == b.ENV_E_ARG
    dev = b.env_config_t(struct_size=C.sizeof(b.env_config_t), armature=-1, joint_damping=-1,
                         friction_mu=-1, obs_scaling=b.ENV_OBS_NORMALIZED)
    assert L.env_create(C.byref(h), b.ENV_PONG_PIXELS, 64, 0, C.byref(dev), None) == b.ENV_E_UNSUPPORTED
    assert L.env_step(None, None, None, None, None) == b.ENV_E_ARG
    assert L.env_rollout(None, 5, None, None, None, None) == b.ENV_E_ARG
    assert L.env_stats(None, None, 0) == b.ENV_E_ARG
    assert L.env_state_bytes(None) == 0
    assert L.env_get_state(None, None, 0) == b.ENV_E_ARG
    assert L.env_set_state(None, None, 0) == b.ENV_E_ARG
    L.env_destroy(None)


def test_binding_struct_layout_matches_header():
    from paper_2603_12145_amd import binding as b
    assert C.sizeof(b.env_config_t) == 48
    assert C.sizeof(b.env_stats_t) == 48
    hdr = open(HEADER).read()
    cfg = re.search(r"typedef struct env_config_t \{(.*?)\} env_config_t;", hdr, re.S).group(1)
    cfg = re.sub(r"/\*.*?\*/", "", cfg, flags=re.S)
    names = re.findall(r"\b(\w+)\s*;", cfg)
    assert names == [n for n, _ in b.env_config_t._fields_]
    st = re.search(r"typedef struct env_stats_t \{(.*?)\} env_stats_t;", hdr, re.S).group(1)
    st = re.sub(r"/\*.*?\*/", "", st, flags=re.S)
    assert re.findall(r"\b(\w+)\s*;", st) == [n for n, _ in b.env_stats_t._fields_]


def test_the_headers_are_plain_c(tmp_path):
    # the boundary is a C ABI: both headers compile as C99 (and as C++11) on their own
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no C compiler")
    src = tmp_path / "use_headers.c"
    src.write_text('#include "mi355env.h"\n#include "mi355env_tuning.h"\n'
                   "int main(void) { env_config_t c; env_stats_t s; (void)c; (void)s; return ENV_OK; }\n")
    inc = os.path.join(ROOT, "include")
    for cmd in (["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only"],
                ["g++", "-std=c++11", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++"]):
        if shutil.which(cmd[0]):
            subprocess.run(cmd + ["-I", inc, str(src)], check=True)
