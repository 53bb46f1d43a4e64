"""CPU-side checks of the C ABI: the library loads, exports every function the header
declares, and rejects bad arguments / ill-typed layer lists before touching a device."""
import ctypes as ct
import os
import re

import pytest

from paper_2012_12544_amd import binding as B
from stage_inputs import configs as C

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    names = set()
    for h in ("bapipe_stage.h", "bapipe_plan.h"):
        src = open(os.path.join(ROOT, "include", h)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(bapipe_[a-z0-9_]+)\s*\(", src))
    return sorted(names)


def test_library_exports_every_declared_function():
    lib = B.load()
    names = header_functions()
    assert len(names) >= 17
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_struct_sizes_match_the_header_layout():
    assert ct.sizeof(B.LayerDesc) == 12 * 4
    assert ct.sizeof(B.LayerProfile) == 2 * 8 + 3 * 8
    assert B.StageOpts.hip_stream.offset % 8 == 0 and ct.sizeof(B.Allocator) == 24


def _create(stage, **over):
    st = dict(stage, **over)
    return B.bapipe_stage_create(st["layers"], st["micro_batch"], st["n_micro"], B.make_opts(st))


def test_create_rejects_bad_arguments_without_a_device():
    stage = C.tiny_stage(c=4, hw=8, micro_batch=2, n_micro=2)
    with pytest.raises(B.BapipeError) as e:
        _create(stage, micro_batch=0)
    assert e.value.status == B.E_INVALID
    with pytest.raises(B.BapipeError) as e:
        _create(stage, dtype=7)
    assert e.value.status == B.E_INVALID
    with pytest.raises(B.BapipeError) as e:
        _create(stage, stage_index=3, n_stages=2)
    assert e.value.status == B.E_INVALID
    lib = B.load()
    assert lib.bapipe_stage_create(None, 1, 1, 1, None, None) == B.E_INVALID
    assert lib.bapipe_stage_step(None, 0.1) == B.E_INVALID
    assert lib.bapipe_stage_forward(None, 0, None, None) == B.E_INVALID
    lib.bapipe_stage_destroy(None)


def test_create_type_checks_the_layer_list():
    stage = C.tiny_stage(c=4, hw=8, micro_batch=2, n_micro=2)
    bad = [dict(L) for L in stage["layers"]]
    bad[1]["cin"] = 5                                  # channel mismatch
    with pytest.raises(B.BapipeError) as e:
        _create(stage, layers=bad)
    assert e.value.status == B.E_SHAPE and "layer 1" in str(e.value)
    bad = [dict(L) for L in stage["layers"]]
    bad[1]["src0"] = 2                                 # consumer before producer
    with pytest.raises(B.BapipeError) as e:
        _create(stage, layers=bad)
    assert e.value.status == B.E_SHAPE
    bad = [dict(L) for L in stage["layers"]]
    bad[2]["pad"] = 2                                  # a window may not lie wholly in the padding
    with pytest.raises(B.BapipeError) as e:
        _create(stage, layers=bad)
    assert e.value.status == B.E_UNSUPPORTED
    bad = [dict(L) for L in stage["layers"]] + [dict(stage["layers"][0], src0=-1)]
    with pytest.raises(B.BapipeError) as e:            # dangling output of layer 2
        _create(stage, layers=bad)
    assert e.value.status == B.E_SHAPE
    cls = C.vgg16_classifier(c=4, hw=3, hidden=8, classes=5, micro_batch=2, n_micro=2)
    bad = [dict(L) for L in cls["layers"]]
    bad[1]["cin"] = 35
    with pytest.raises(B.BapipeError) as e:
        _create(cls, layers=bad)
    assert e.value.status == B.E_SHAPE
