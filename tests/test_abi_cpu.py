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
    assert b"hipMalloc" in lib.mpe_last_error()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2311_10090_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle", src, flags=re.M), f
                assert "liboracle" not in src and "orc_" not in src, f
