"""The C-ABI library loads, exports every symbol the header declares, and its host-side
argument checks work without a GPU (no kernel is launched here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "evo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text)
    return sorted(set(names))


def test_header_symbols_are_exported():
    from paper_2202_05008_amd import _lib
    lib = _lib.load()
    declared = _declared()
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(lib, name), "library does not export %s" % name
    assert sorted(_lib.EXPORTS) == declared, "binding and header disagree"
    assert lib.evo_version().decode().startswith("evo-gfx950")


def test_host_side_argument_checks():
    from paper_2202_05008_amd import _lib, api
    lib = _lib.load()
    cfg = api.make_pgpe_config(P=676, pop_max=64)
    assert lib.pgpe_workspace_bytes(C.byref(cfg)) >= 64 * 12
    h = C.c_void_p()
    rc = lib.pgpe_create(C.byref(h), C.byref(cfg), None, None, None, None, None, None)
    assert rc == -1 and b"non-null" in lib.evo_last_error()
    bad = api.make_pgpe_config(P=10, pop_max=63)
    assert lib.pgpe_workspace_bytes(C.byref(bad)) == 0
    fake = C.c_void_p(0x1000)
    rc = lib.pgpe_create(C.byref(h), C.byref(bad), fake, fake, fake, fake, None, fake)
    assert rc == -1 and b"pop_max" in lib.evo_last_error()
    rule1 = api.make_pgpe_config(P=10, pop_max=8, sigma_rule=1)
    rc = lib.pgpe_create(C.byref(h), C.byref(rule1), fake, fake, fake, fake, None, fake)
    assert rc == -1 and b"aux" in lib.evo_last_error()
    rc = lib.pgpe_create(C.byref(h), C.byref(cfg), fake, fake, fake, fake, None, fake)
    assert rc == 0 and h.value
    # tell before ask, odd pop, pop above pop_max, bad dtype: all rejected before any launch
    assert lib.pgpe_tell(h, fake, None) == -2
    assert lib.pgpe_ask(h, 1, 63, fake, 0, None) == -1
    assert lib.pgpe_ask(h, 1, 66, fake, 0, None) == -1
    assert lib.pgpe_ask(h, 1, 64, fake, 7, None) == -1
    assert lib.pgpe_ask(h, 1, 64, C.c_void_p(0x1004), 0, None) == -1
    t = C.c_uint32()
    assert lib.pgpe_get_generation(h, C.byref(t)) == 0 and t.value == 1
    assert lib.pgpe_set_generation(h, 0) == -1
    assert lib.pgpe_destroy(h) == 0


def test_policy_and_task_descriptions():
    from paper_2202_05008_amd import api
    from workloads import CONFIGS
    for name in ("cfg1", "cfg3", "cfg4"):
        c = CONFIGS[name]
        pd = api.make_policy_desc(api.EVO_POLICY_MLP, c.dims, c.acts, c.dtype)
        assert api.policy_param_count(pd) == c.P
    c = CONFIGS["cfg2"]
    pd = api.make_policy_desc(api.EVO_POLICY_CONVNET, (28,) + tuple(c.dims))
    assert api.policy_param_count(pd) == 9098 == c.P
    with pytest.raises(api.EvoError):
        api.policy_param_count(api.make_policy_desc(api.EVO_POLICY_CONVNET, (30, 8, 16, 10)))
    with pytest.raises(api.EvoError):
        api.policy_param_count(api.make_policy_desc(api.EVO_POLICY_MLP, (4, 0, 2), (0, 0)))
    td = api.make_task_desc(api.EVO_TASK_CLASSIFY, B=512)
    pd1 = api.make_policy_desc(api.EVO_POLICY_MLP, (16, 32, 4), (1, 0))
    assert api.rollout_workspace_bytes(td, pd1, 64) >= 64 * 8 * 4
    assert api.rollout_workspace_bytes(api.make_task_desc(api.EVO_TASK_SPHERE, P=8), None, 4) >= 16
    assert api.rollout_workspace_bytes(api.make_task_desc(api.EVO_TASK_CARTPOLE), pd1, 4) == 0
    # the ConvNet's workspace also holds the shared batch converted once for all members (4 KB per image)
    pdc = api.make_policy_desc(api.EVO_POLICY_CONVNET, (28, 8, 16, 10))
    tdc = api.make_task_desc(api.EVO_TASK_CLASSIFY, B=1024)
    need = api.rollout_workspace_bytes(tdc, pdc, 256)
    assert need >= 1024 * 4096 + 256 * 4 and need % 256 == 0 and need <= api.rollout_static_scratch_bytes()


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2202_05008_amd import _lib
    monkeypatch.setattr(_lib, "_lib", None)
    monkeypatch.setattr(_lib, "LIB_PATH", "/nonexistent/libevo_gfx950.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        _lib.load()
