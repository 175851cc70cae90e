"""The C-ABI library loads without a GPU and exports every function include/*.h declares;
argument validation that needs no device is exercised too."""
import ctypes as C
import glob
import os
import re

import pytest

from paper_2411_05894_amd import binding as sv
from sssd_synth import MODEL_SHAPES

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    for path in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
        names += re.findall(r"\b(sssd_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert len(names) >= 15
    lib = sv.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/ but not exported"


def test_sizes_and_config_validation_without_gpu():
    cfg = sv.make_config(MODEL_SHAPES["8b"], 1, 16, 2048 + 17)
    kv, ws, pk = sv.sssd_verify_sizes(cfg)
    assert kv == 2 * 32 * 8 * 2080 * 128 * 2            # K and V, 32 layers, rows padded to 32
    assert pk == 15009316864                            # every 8B matrix, bf16, no padding needed
    assert ws > 0
    bad = sv.make_config(MODEL_SHAPES["8b"], 1, 16, 2048 + 17)
    bad.head_dim = 96
    assert sv.lib().sssd_verify_sizes(C.byref(bad), None, None, None) == sv.SSSD_EINVAL
    bad = sv.make_config(MODEL_SHAPES["8b"], 1, 40, 4096)
    assert sv.lib().sssd_verify_sizes(C.byref(bad), None, None, None) == sv.SSSD_EINVAL
    assert sv.lib().sssd_verify_sizes(None, None, None, None) == sv.SSSD_EINVAL
    tiny = sv.make_config(MODEL_SHAPES["tiny"], 1, 4, 512)
    _, _, pk = sv.sssd_verify_sizes(tiny)
    assert pk > 3424256                                 # ffn = 688 is padded to 704 columns


def test_null_handles_are_rejected():
    lib = sv.lib()
    assert lib.sssd_verify_step(None, 1, 0, None, None, None, None, None) == sv.SSSD_EINVAL
    assert lib.sssd_kv_rollback(None, 1, None, None, None, None) == sv.SSSD_EINVAL
    assert lib.sssd_verify_destroy(None) == sv.SSSD_EINVAL
    assert lib.sssd_verify_sync(None, None) == sv.SSSD_EINVAL
    assert "capacity" in sv.strerror(sv.SSSD_ECAPACITY)
    assert lib.sssd_op_packed_weight_bytes(4096, 4096) == 4096 * 4096 * 2
    assert lib.sssd_op_packed_weight_bytes(256, 688) == 256 * 704 * 2


def test_plan_check_covers_every_step_of_a_configuration_without_gpu():
    """sssd_verify_plan_check (host only): every (B, k) inside the configuration fits the buffers
    sssd_verify_sizes asks for; anything beyond the configuration is a capacity error."""
    lib = sv.lib()
    for shape, mb, mk, ms in (("tiny", 8, 31, 260), ("8b", 32, 16, 4113), ("70b", 16, 8, 2057)):
        cfg = sv.make_config(MODEL_SHAPES[shape], mb, mk, ms)
        for B in range(1, mb + 1):
            for k in range(mk + 1):
                assert lib.sssd_verify_plan_check(C.byref(cfg), B, k) == sv.SSSD_OK, (shape, B, k)
        assert lib.sssd_verify_plan_check(C.byref(cfg), mb + 1, 0) == sv.SSSD_ECAPACITY
        assert lib.sssd_verify_plan_check(C.byref(cfg), 1, mk + 1) == sv.SSSD_ECAPACITY
        assert lib.sssd_verify_plan_check(C.byref(cfg), 0, 0) == sv.SSSD_EINVAL
    assert lib.sssd_verify_plan_check(None, 1, 0) == sv.SSSD_EINVAL
