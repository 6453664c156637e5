"""CPU-side checks of the C ABI: the library loads, exports what include/mpe.h declares, and
rejects bad arguments on the host before touching the device.  No compute calls."""
import ctypes as C
import os
import re

import pytest

from paper_2311_10090_amd import binding
from paper_2311_10090_amd.binding import MpeConfig, MPE_EINVAL, MPE_EHIP, MPE_OK

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2311_10090_amd.build import build
        build(force=True)
    return binding.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mpe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mpe_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS), names
    for n in names:
        assert getattr(lib, n) is not None


def test_config_struct_matches_header():
    # 5 int32 + 8 float + 3 int32 + 1 float + 2 int32 + 4 float, no padding
    assert C.sizeof(binding._CConfig) == 23 * 4
    text = open(os.path.join(ROOT, "include", "mpe.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} mpe_config;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(int32_t|float)\s+([a-z_]+);", body)
    assert [f[1] for f in fields] == [f[0] for f in binding._CConfig._fields_]
    ctype = {"int32_t": C.c_int32, "float": C.c_float}
    assert [ctype[f[0]] for f in fields] == [f[1] for f in binding._CConfig._fields_]


@pytest.mark.parametrize("bad", [
    dict(num_envs=0), dict(num_runs=0), dict(num_agents=0), dict(num_agents=11, num_landmarks=11),
    dict(num_landmarks=2), dict(max_episode_steps=0), dict(dt=0.0), dict(mass=-1.0),
    dict(contact_margin=0.0), dict(damping=1.5), dict(hidden=32), dict(weight_dtype=7),
    dict(dt=float("nan")), dict(accel=float("inf")), dict(num_envs=1 << 20, num_runs=1 << 11),
    dict(reward_mode=2), dict(reward_mode=1, local_ratio=1.5), dict(reward_mode=1, local_ratio=float("nan")),
    dict(scenario=2), dict(scenario=1, num_agents=4, num_landmarks=2, num_adversaries=0),
    dict(scenario=1, num_agents=4, num_landmarks=2, num_adversaries=4),
    dict(scenario=1, num_agents=4, num_landmarks=3, num_adversaries=3),      # shape that is not built
    dict(scenario=1, num_agents=5, num_landmarks=2, num_adversaries=3),
    dict(scenario=1, num_agents=4, num_landmarks=2, num_adversaries=3, adv_max_speed=0.0),
    dict(scenario=1, num_agents=4, num_landmarks=2, num_adversaries=3, good_max_speed=float("nan")),
    dict(scenario=1, num_agents=4, num_landmarks=2, num_adversaries=3, adv_radius=-0.1),
])
def test_bad_config_is_rejected_on_host(lib, bad):
    cfg = MpeConfig(**bad).to_c()
    h = C.c_void_p()
    rc = lib.mpe_create(C.byref(cfg), C.byref(h))
    assert rc == MPE_EINVAL
    assert h.value is None
    assert len(lib.mpe_last_error()) > 0


def test_null_arguments(lib):
    h = C.c_void_p()
    assert lib.mpe_create(None, C.byref(h)) == MPE_EINVAL
    cfg = MpeConfig().to_c()
    assert lib.mpe_create(C.byref(cfg), None) == MPE_EINVAL
    assert lib.mpe_destroy(None) == MPE_OK
    assert lib.mpe_obs_dim(None) == MPE_EINVAL
    assert lib.mpe_reset(None, 0, None, None) == MPE_EINVAL
    assert lib.mpe_step(None, None, None, None, None, None) == MPE_EINVAL
    assert lib.mpe_rollout(None, 1, None, None, None, None, None, None) == MPE_EINVAL
    assert lib.mpe_set_policy(None, None, None, None, None, None, None, None) == MPE_EINVAL
    assert lib.mpe_set_critic(None, None, None, None, None, None, None, None) == MPE_EINVAL
    assert lib.mpe_rollout_ac(None, 1, None, None, None, None, None, None, None, None, None) == MPE_EINVAL
    assert lib.mpe_get_state(None, None, None, None, None, None, None) == MPE_EINVAL
    assert lib.mpe_set_state(None, None, None, None, None, 0, 0, None) == MPE_EINVAL
    assert b"NULL" in lib.mpe_last_error()


def test_valid_config_without_device_fails_cleanly(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a device is present; covered by the gpu tests")
    cfg = MpeConfig().to_c()
    h = C.c_void_p()
    rc = lib.mpe_create(C.byref(cfg), C.byref(h))
    assert rc == MPE_EHIP and h.value is None
    assert b"allocation failed" in lib.mpe_last_error()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2311_10090_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle", src, flags=re.M), f
                assert "liboracle" not in src and "orc_" not in src, f


def _expected_valid(c):
    """The validity rules of include/mpe.h, restated from the header's text."""
    import math
    fin = math.isfinite
    if c["num_envs"] < 1 or c["num_runs"] < 1 or not (1 <= c["num_agents"] <= 10):
        return False
    if c["scenario"] not in (0, 1):
        return False
    if c["scenario"] == 0 and c["num_landmarks"] != c["num_agents"]:
        return False
    if c["scenario"] == 1:
        if not (1 <= c["num_adversaries"] < c["num_agents"]):
            return False
        shape = (c["num_agents"], c["num_landmarks"], c["num_agents"] - c["num_adversaries"])
        if shape not in ((4, 2, 1), (2, 1, 1), (3, 0, 1), (6, 2, 2), (5, 2, 1), (8, 2, 2), (10, 3, 2)):
            return False
        if not (fin(c["adv_radius"]) and c["adv_radius"] >= 0 and fin(c["adv_accel"])):
            return False
        if not (fin(c["adv_max_speed"]) and c["adv_max_speed"] > 0 and fin(c["good_max_speed"]) and c["good_max_speed"] > 0):
            return False
    if c["num_envs"] * c["num_runs"] > 2 ** 30 or c["max_episode_steps"] < 1:
        return False
    for k in ("dt", "mass", "contact_margin"):
        if not (fin(c[k]) and c[k] > 0):
            return False
    if not (fin(c["damping"]) and 0 <= c["damping"] <= 1):
        return False
    for k in ("accel", "contact_force", "agent_radius", "landmark_radius"):
        if not fin(c[k]):
            return False
    if c["agent_radius"] < 0 or c["landmark_radius"] < 0:
        return False
    if c["hidden"] not in (0, 64, 128) or c["weight_dtype"] not in (0, 1) or c["reward_mode"] not in (0, 1):
        return False
    if c["reward_mode"] == 1 and not (fin(c["local_ratio"]) and 0 <= c["local_ratio"] <= 1):
        return False
    return True


def test_random_configs_are_accepted_or_refused_as_the_header_says(lib):
    import torch
    from hypothesis import given, settings, strategies as st
    if torch.cuda.is_available():
        pytest.skip("valid configs would allocate device memory; the host rules are checked without a device")
    small = st.integers(-1, 12)
    fl = st.one_of(st.floats(-1.0, 2.0, width=32), st.sampled_from([float("nan"), float("inf"), 0.0, 1.0, 0.1]))
    wild = dict(
        num_envs=st.sampled_from([0, 1, 64, 1 << 20]), num_agents=small, num_landmarks=small,
        num_runs=st.sampled_from([0, 1, 3, 1 << 11]), max_episode_steps=st.sampled_from([0, 1, 25]),
        dt=fl, damping=fl, mass=fl, accel=fl, agent_radius=fl, landmark_radius=fl, contact_force=fl, contact_margin=fl,
        hidden=st.sampled_from([0, 32, 64, 128]), weight_dtype=st.sampled_from([0, 1, 2]),
        reward_mode=st.sampled_from([0, 1, 2]), local_ratio=fl, scenario=st.sampled_from([0, 1, 2]),
        num_adversaries=small, adv_radius=fl, adv_accel=fl, adv_max_speed=fl, good_max_speed=fl)
    bases = [dict(), dict(scenario=1, num_agents=4, num_landmarks=2, num_adversaries=3),
             dict(scenario=1, num_agents=6, num_landmarks=2, num_adversaries=4), dict(num_agents=10, num_landmarks=10),
             dict(reward_mode=1, local_ratio=0.25)]
    # a valid base config with zero to three fields replaced by arbitrary values
    cfgs = st.tuples(st.sampled_from(bases),
                     st.lists(st.sampled_from(sorted(wild)), min_size=0, max_size=3, unique=True).flatmap(
                         lambda ks: st.fixed_dictionaries({k: wild[k] for k in ks})))

    seen = {True: 0, False: 0}

    @settings(max_examples=600, deadline=None, derandomize=True)
    @given(cfgs)
    def check(pair):
        c = dict(pair[0])
        c.update(pair[1])
        cc = MpeConfig(**c).to_c()
        h = C.c_void_p()
        rc = lib.mpe_create(C.byref(cc), C.byref(h))
        valid = _expected_valid({k: getattr(cc, k) for k, _ in binding._CConfig._fields_})
        seen[valid] += 1
        assert rc == (MPE_EHIP if valid else MPE_EINVAL), (c, lib.mpe_last_error())
        assert h.value is None

    check()
    assert seen[True] > 20 and seen[False] > 100


def test_header_is_plain_c_and_links_from_a_c_program(lib, tmp_path):
    """include/mpe.h compiles as C99 with a C compiler (no C++ types in the boundary), every declared
    entry point links, and a host-side refusal works from a program that is not Python."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if not gcc:
        pytest.skip("no C compiler")
    names = declared_symbols()
    refs = "\n".join("  p[%d] = (fn)%s;" % (i, n) for i, n in enumerate(names))
    src = tmp_path / "use_mpe.c"
    src.write_text("""#include <stdio.h>
#include <string.h>
#include "mpe.h"
typedef void (*fn)(void);
int main(void) {
  fn p[%d];
  mpe_config cfg;
  mpe_env* env = NULL;
  int rc;
%s
  if (sizeof(mpe_config) != 92) return 10;
  memset(&cfg, 0, sizeof cfg);          /* num_envs = 0: refused on the host */
  rc = mpe_create(&cfg, &env);
  if (rc != MPE_EINVAL || env != NULL) return 11;
  if (strstr(mpe_last_error(), "num_envs") == NULL) return 12;
  if (mpe_destroy(NULL) != MPE_OK && mpe_destroy(NULL) != MPE_EINVAL) return 13;
  printf("%%d symbols, %%s\\n", (int)(sizeof p / sizeof p[0]), p[0] ? "ok" : "null");
  return 0;
}
""" % (len(names), refs))
    exe = tmp_path / "use_mpe"
    libdir = os.path.dirname(binding.LIB_PATH)
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                        str(src), "-o", str(exe), "-L", libdir, "-l:libmpe.so", "-Wl,-rpath," + libdir],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert "%d symbols, ok" % len(names) in r.stdout


def test_bench_source_hash_ignores_comments_and_layout_but_not_code():
    """bench.py reports the committed counter figures only while the kernel sources hash to the value stored
    with them: the hash must not move with a comment or a blank, and must move with the code."""
    import importlib.util
    import os
    spec = importlib.util.spec_from_file_location("bench_for_hash", os.path.join(os.path.dirname(os.path.dirname(__file__)), "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    a = 'int f(int x) {  // adds one\n  /* block\n comment */ return x + 1;\n}\nconst char* s = "// kept /* kept */";\n'
    b = 'int f(int x) { return x + 1; }\n\n\nconst char* s = "// kept /* kept */";   // trailing\n'
    c = 'int f(int x) { return x + 2; }\nconst char* s = "// kept /* kept */";\n'
    d = 'int f(int x) { return x + 1; }\nconst char* s = "// kept /* lost */";\n'
    assert bench._code_only(a) == bench._code_only(b)
    assert bench._code_only(a) != bench._code_only(c) and bench._code_only(a) != bench._code_only(d)
    assert len(bench.kernel_source_hash()) == 64
