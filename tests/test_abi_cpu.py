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
    # the header's field order and natural alignment give an 80-byte struct (76 bytes of fields)
    assert ctypes.sizeof(gv.binding.gv_config) == 80
    assert gv.binding.gv_config.total_samples.offset == 24
    assert gv.binding.gv_config.device.offset == 48
    assert gv.binding.gv_config.pool_slots.offset == 64 and gv.binding.gv_config.partitions.offset == 68
    assert gv.binding.gv_config.track_loss.offset == 72
    assert ctypes.sizeof(gv.binding.gv_stats) == 96 and gv.binding.gv_stats.train_loss_sum.offset == 80
    # constants of the header and of the binding agree
    text = open(os.path.join(ROOT, "include", "gvhot.h")).read()
    assert float(re.search(r"#define GV_NEG_WEIGHT_DEFAULT \((-?[0-9.]+)f\)", text).group(1)) == gv.GV_NEG_WEIGHT_DEFAULT
    assert int(re.search(r"#define GV_MAX_POOL_SLOTS (\d+)", text).group(1)) == gv.GV_MAX_POOL_SLOTS
    assert int(re.search(r"#define GV_MAX_PARTITIONS (\d+)", text).group(1)) == gv.GV_MAX_PARTITIONS
    assert re.search(r"GV_SCHEDULE_AUTO = (\d+)", text).group(1) == str(gv.GV_SCHEDULE_AUTO)
    assert re.search(r"#define GV_STATIC_SCRATCH_WORDS \(1u << (\d+)\)", text).group(1) == "22" and \
        gv.GV_STATIC_SCRATCH_WORDS == 1 << 22


def test_argument_errors_need_no_device(gv):
    import torch

    with pytest.raises(gv.GvError) as e:
        gv.gv_create(dim=100, num_neg=1, total_samples=10, pool_capacity=10)
    assert e.value.code == gv.GV_EINVAL and "dim" in str(e.value)
    for bad in (dict(num_neg=0), dict(num_neg=6), dict(total_samples=0), dict(pool_capacity=0), dict(mode=7),
                dict(lr0=float("nan")), dict(neg_weight=-2.0), dict(neg_weight=float("inf")), dict(pool_slots=1),
                dict(pool_slots=17), dict(schedule=3), dict(partitions=1), dict(partitions=65)):
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


def test_auc_is_the_rank_statistic_with_shared_ranks(gv):
    """gv_auc needs no device: brute force over all pairs (a tie counts one half), including heavy ties."""
    import numpy as np

    rng = np.random.default_rng(3)
    for num_pos, num_neg, levels in [(1, 1, 2), (7, 5, 3), (200, 300, 4), (500, 400, 10**6), (50, 1, 2)]:
        pos = (rng.integers(levels, size=num_pos) / levels + (0.1 if levels > 100 else 0.0)).astype(np.float32)
        neg = (rng.integers(levels, size=num_neg) / levels).astype(np.float32)
        wins = (pos[:, None] > neg[None, :]).sum() + 0.5 * (pos[:, None] == neg[None, :]).sum()
        assert abs(gv.gv_auc(pos, neg) - wins / (num_pos * num_neg)) < 1e-12
    assert gv.gv_auc([2.0, 3.0], [0.0, 1.0]) == 1.0 and gv.gv_auc([0.0], [1.0, 2.0]) == 0.0
    assert gv.gv_auc([1.0, 1.0], [1.0]) == 0.5
    for bad in (([], [1.0]), ([1.0], []), ([float("nan")], [1.0]), ([1.0], [float("inf")])):
        with pytest.raises(gv.GvError) as e:
            gv.gv_auc(*bad)
        assert e.value.code == gv.GV_EINVAL


def test_host_producer_rejects_an_ill_formed_adjacency(gv):
    """gv_augment checks the adjacency where its walks touch it and reports instead of reading out of bounds."""
    import numpy as np

    offsets = np.array([0, 2, 4, 6], dtype=np.uint64)  # triangle
    adj = np.array([1, 2, 0, 2, 0, 1], dtype=np.uint32)
    pairs, walks = gv.gv_augment(offsets, adj, seed=1, count=500, threads=2)
    assert pairs.max() < 3 and walks == 3
    for broken_offsets, broken_adj in [
        (offsets, np.array([1, 2, 0, 7, 0, 1], dtype=np.uint32)),                  # entry >= n
        (np.array([0, 2, 2, 4], dtype=np.uint64), np.array([1, 2, 0, 1], dtype=np.uint32)),  # reachable empty row
        (np.array([1, 2, 4, 6], dtype=np.uint64), adj),                               # does not start at 0
    ]:
        with pytest.raises(gv.GvError) as e:
            gv.gv_augment(broken_offsets, broken_adj, seed=1, count=500, threads=2)
        assert e.value.code == gv.GV_EINVAL
    # a window far wider than the walk, up to the largest value: no overflow in the pair loop
    wide, _ = gv.gv_augment(offsets, adj, seed=1, walk_length=3, window=7, count=60, shuffle=gv.GV_SHUFFLE_NONE)
    assert wide.shape == (60, 2)


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_1903_00757_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
