"""Host-side checks that need no GPU: the library loads, exports exactly what the header
declares, and fails cleanly when no device is present."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def gv():
    import paper_1903_00757_amd as gv

    if not os.path.exists(gv.LIB_PATH):
        from paper_1903_00757_amd import build

        build.build()
    gv.load()
    return gv


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gvhot.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gv_[a-z_]+)\s*\(", text)))


def test_every_declared_entry_point_is_exported(gv):
    names = declared_functions()
    assert len(names) >= 19
    lib = ctypes.CDLL(gv.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(gv.EXPORTS) == names  # the binding covers the same set, under the same names
    for name in names:
        assert callable(getattr(gv, name))


def test_config_struct_layout_matches_header(gv):
    # the header's field order and natural alignment give a 64-byte struct
    assert ctypes.sizeof(gv.binding.gv_config) == 64
    assert gv.binding.gv_config.total_samples.offset == 24
    assert gv.binding.gv_config.device.offset == 48
    assert ctypes.sizeof(gv.binding.gv_stats) == 64


def test_argument_errors_need_no_device(gv):
    import torch

    with pytest.raises(gv.GvError) as e:
        gv.gv_create(dim=100, num_neg=1, total_samples=10, pool_capacity=10)
    assert e.value.code == gv.GV_EINVAL and "dim" in str(e.value)
    for bad in (dict(num_neg=0), dict(num_neg=6), dict(total_samples=0), dict(pool_capacity=0), dict(mode=7),
                dict(lr0=float("nan")), dict(neg_weight=-1.0)):
        kw = dict(dim=128, num_neg=1, total_samples=10, pool_capacity=10)
        kw.update(bad)
        with pytest.raises(gv.GvError) as e:
            gv.gv_create(**kw)
        assert e.value.code == gv.GV_EINVAL, bad
    if not torch.cuda.is_available():
        with pytest.raises(gv.GvError) as e:
            gv.gv_create(dim=128, num_neg=1, total_samples=10, pool_capacity=10)
        assert e.value.code == gv.GV_EHIP  # loud failure, no CPU fallback
    lib = gv.load()
    assert lib.gv_sync(None) == gv.GV_EINVAL
    assert lib.gv_train_pool(None) == gv.GV_EINVAL
    lib.gv_destroy(None)


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_1903_00757_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
