"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and its
host-side checks (configuration, pointers, alignment, call order) answer with the documented codes."""
import ctypes
import os
import re

import pytest

import paper_2108_13976_amd as wd
from paper_2108_13976_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "wd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(wd_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = wd.load_library()
    names = declared_symbols()
    assert {"wd_create", "wd_reset", "wd_sample", "wd_step", "wd_destroy", "wd_query_layout"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_offers_the_same_names():
    for n in declared_symbols():
        assert callable(getattr(binding, n)), n


def good_config(**over):
    kw = dict(num_envs=4, num_agents=10, num_taggers=2, grid_size=8, episode_length=20)
    kw.update(over)
    return binding.make_config(**kw)


def fake_buffers(base=0x10000, stride=0x1000):
    # never dereferenced: wd_create only checks for NULL and alignment
    return binding.wd_buffers(*[base + stride * i for i in range(len(binding.BUFFER_NAMES))])


def test_layout_query_matches_the_documented_formulas():
    lay = wd.wd_query_layout(good_config(num_envs=2000, num_agents=1000, num_taggers=100, grid_size=100, episode_length=500))
    assert lay.obs_dim == 21
    assert lay.per_agent_elems == 2_000_000 and lay.obs_elems == 42_000_000
    assert lay.per_env_elems == 2000 and lay.probs_elems == 10_000_000
    assert lay.bytes_per_iteration == 2_000_000 * 140 + 24 * 2000
    assert wd.wd_query_layout(good_config(obs_mode=wd.WD_OBS_FULL)).obs_dim == 5 + 4 * 10


@pytest.mark.parametrize("over", [
    dict(num_envs=0), dict(num_agents=1), dict(num_agents=40000), dict(num_taggers=0), dict(num_taggers=10),
    dict(grid_size=0), dict(grid_size=40000), dict(num_actions=4), dict(episode_length=0), dict(obs_mode=2),
    dict(obs_k=10), dict(obs_k=-1), dict(env_offset=-1), dict(tag_reward=float("nan")),
])
def test_bad_configurations_are_rejected(over):
    with pytest.raises(wd.WdError) as ei:
        wd.wd_query_layout(good_config(**over))
    assert ei.value.status == binding.WD_E_CONFIG
    with pytest.raises(wd.WdError) as ei:
        wd.wd_create(good_config(**over), fake_buffers())
    assert ei.value.status == binding.WD_E_CONFIG


@pytest.mark.parametrize("over", [
    dict(num_agents=32768, num_taggers=3000, grid_size=100),               # tables of one env beyond a workgroup's LDS
    dict(num_agents=20000, num_taggers=100, grid_size=30000, tag_r2=50),   # the same with 64-bit keys
    dict(num_agents=9000, num_taggers=100, grid_size=300, obs_mode=binding.WD_OBS_FULL),
    dict(num_agents=9000, num_taggers=100, grid_size=300, obs_k=17),
])
def test_valid_configurations_without_a_kernel_are_refused(over):
    """Sizes the header allows but no kernel of this build covers: WD_E_UNSUPPORTED from wd_create
    (before anything is allocated), while the layout query still answers."""
    cfg = good_config(**over)
    assert wd.wd_query_layout(cfg).obs_dim > 0
    with pytest.raises(wd.WdError) as ei:
        wd.wd_create(cfg, fake_buffers())
    assert ei.value.status == binding.WD_E_UNSUPPORTED


def test_struct_size_is_checked():
    cfg = good_config()
    cfg.struct_size = 8
    with pytest.raises(wd.WdError) as ei:
        wd.wd_query_layout(cfg)
    assert ei.value.status == binding.WD_E_CONFIG


def test_null_and_misaligned_buffers():
    bufs = fake_buffers()
    bufs.obs = None
    with pytest.raises(wd.WdError) as ei:
        wd.wd_create(good_config(), bufs)
    assert ei.value.status == binding.WD_E_NULL
    bufs = fake_buffers()
    bufs.reward = bufs.reward + 64
    with pytest.raises(wd.WdError) as ei:
        wd.wd_create(good_config(), bufs)
    assert ei.value.status == binding.WD_E_ALIGN
    lib = wd.load_library()
    assert lib.wd_create(None, None, None) == binding.WD_E_NULL
    assert lib.wd_step(None) == binding.WD_E_NULL
    assert lib.wd_destroy(None) == binding.WD_E_NULL
    assert lib.wd_reset(None, 0) == binding.WD_E_NULL


def test_call_order_is_enforced_before_any_launch():
    h = wd.wd_create(good_config(), fake_buffers())
    for call in (lambda: wd.wd_step(h), lambda: wd.wd_sample(h, 0x20000), lambda: wd.wd_iterate(h, 0x20000),
                 lambda: wd.wd_rollout(h, 0x20000, 4, 3), lambda: wd.wd_reset(h, wd.WD_RESET_DONE)):
        with pytest.raises(wd.WdError) as ei:
            call()
        assert ei.value.status == binding.WD_E_STATE
    with pytest.raises(wd.WdError) as ei:
        wd.wd_reset(h, 7)
    assert ei.value.status == binding.WD_E_CONFIG
    with pytest.raises(wd.WdError) as ei:
        wd.wd_sample(h, 0)
    assert ei.value.status == binding.WD_E_NULL
    # wd_rollout checks its own arguments before the call order
    for ring_len, k in ((0, 1), (1, 0), (-3, 2)):
        with pytest.raises(wd.WdError) as ei:
            wd.wd_rollout(h, 0x20000, ring_len, k)
        assert ei.value.status == binding.WD_E_CONFIG
    with pytest.raises(wd.WdError) as ei:
        wd.wd_rollout(h, 0, 1, 1)
    assert ei.value.status == binding.WD_E_NULL
    with pytest.raises(wd.WdError) as ei:
        wd.wd_rollout(h, 0x20000, 1, 1, binding.wd_rollout_buffers(0x30000, 0x30004, None, None))
    assert ei.value.status == binding.WD_E_ALIGN
    assert wd.wd_get_step(h) == 0
    wd.wd_set_step(h, 2**40 + 3)
    assert wd.wd_get_step(h) == 2**40 + 3
    assert wd.wd_last_error(h) == ""
    wd.wd_destroy(h)


def test_status_texts():
    assert wd.wd_strerror(0) == "ok"
    texts = {wd.wd_strerror(s) for s in range(-7, 1)}
    assert len(texts) == 8 and wd.wd_strerror(-99) == "unknown status"


def test_static_entry_point_checks_its_arguments_before_any_launch():
    lib = wd.load_library()
    assert lib.wd_iterate_static(None, None, None, 0) == binding.WD_E_NULL
    bufs = fake_buffers()
    with pytest.raises(wd.WdError) as ei:
        wd.wd_iterate_static(good_config(num_agents=1), bufs, 0x40000, 0)
    assert ei.value.status == binding.WD_E_CONFIG
    with pytest.raises(wd.WdError) as ei:
        wd.wd_iterate_static(good_config(num_agents=12), bufs, 0x40004, 0)  # probs: 16-byte alignment with N % 4 == 0
    assert ei.value.status == binding.WD_E_ALIGN
    # 160 envs of 8192 agents (large-env layout): work tables of about 25 MB, beyond the static array
    big = binding.make_config(160, 8192, 512, 512, 10)
    with pytest.raises(wd.WdError) as ei:
        wd.wd_iterate_static(big, bufs, 0x40000, 0)
    assert ei.value.status == binding.WD_E_SCRATCH
    assert "static scratch" in wd.wd_strerror(binding.WD_E_SCRATCH)


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    with pytest.raises(FileNotFoundError):
        binding.load_library(str(tmp_path / "libwd.so"))
    monkeypatch.undo()
    wd.load_library()


# ---------------------------------------------------------------- continuous Tag (include/wdc.h)
def declared_continuous_symbols():
    text = open(os.path.join(ROOT, "include", "wdc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(wdc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_continuous_symbol():
    lib = wd.load_library()
    names = declared_continuous_symbols()
    assert {"wdc_create", "wdc_reset", "wdc_sample", "wdc_step", "wdc_iterate", "wdc_destroy",
            "wdc_query_layout"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
        assert callable(getattr(binding, n)), n


def test_continuous_layout_and_rejections():
    lay = binding.wdc_query_layout(binding.make_cconfig(2000, 5, 1, 500))
    assert lay.obs_dim == 32 and lay.agent_elems == 10_000 and lay.action_elems == 20_000
    assert lay.obs_elems == 320_000 and lay.env_elems == 2000 and lay.probs_elems == 100_000
    assert lay.bytes_per_iteration == 10_000 * (40 + 20 + 20 + 8 + 4 + 128) + 24 * 2000
    good = dict(num_envs=4, num_agents=6, num_taggers=2, episode_length=20)
    for over in (dict(num_envs=0), dict(num_agents=1), dict(num_agents=1025), dict(num_taggers=0),
                 dict(num_taggers=6), dict(num_headings=6), dict(num_headings=0), dict(num_headings=8192),
                 dict(episode_length=0), dict(obs_k=9), dict(obs_k=6), dict(obs_k=-1), dict(world_size=0.0),
                 dict(world_size=float("nan")), dict(accel=-1.0), dict(tag_reward=float("inf")), dict(env_offset=-2)):
        with pytest.raises(wd.WdError) as ei:
            binding.wdc_query_layout(binding.make_cconfig(**{**good, **over}))
        assert ei.value.status == binding.WD_E_CONFIG, over
    cfg = binding.make_cconfig(**good)
    cfg.struct_size = 12
    with pytest.raises(wd.WdError) as ei:
        binding.wdc_query_layout(cfg)
    assert ei.value.status == binding.WD_E_CONFIG
    bufs = binding.wdc_buffers(*[0x10000 + 0x1000 * i for i in range(len(binding.CBUFFER_NAMES))])
    bufs.obs = 0
    with pytest.raises(wd.WdError) as ei:
        binding.wdc_create(binding.make_cconfig(**good), bufs)
    assert ei.value.status == binding.WD_E_NULL
    bufs.obs = 0x20010
    with pytest.raises(wd.WdError) as ei:
        binding.wdc_create(binding.make_cconfig(**good), bufs)
    assert ei.value.status == binding.WD_E_ALIGN
    lib = wd.load_library()
    assert lib.wdc_reset(None, 0) == binding.WD_E_NULL and lib.wdc_step(None) == binding.WD_E_NULL
    assert lib.wdc_iterate(None, None) == binding.WD_E_NULL and lib.wdc_destroy(None) == binding.WD_OK
