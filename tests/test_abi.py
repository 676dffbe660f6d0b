"""CPU-only checks of the C ABI: the library loads, exports every function the header
declares, and validates its arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2605_16341_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "orthdion.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(orthdion_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    lib = b.load()
    names = declared_functions()
    assert "orthdion_create" in names and "orthdion_step" in names and len(names) >= 10
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(b.EXPORTS) == names


def test_create_validates_shapes_and_config():
    ok = b.orthdion_create([(256, 256), (64, 128)], 16, b.ORTHDION_F32, b.ORTHDION_F32)
    assert b.orthdion_workspace_bytes(ok) > 0
    b.orthdion_destroy(ok)
    bad_shapes = [((250, 256), 16), ((256, 250), 16), ((256, 256), 12), ((256, 256), 0), ((32, 64), 40),
                  ((64, 32), 40), ((0, 8), 8)]
    for shape, r in bad_shapes:
        with pytest.raises(b.OrthDionError) as e:
            b.orthdion_create([shape], r, b.ORTHDION_BF16, b.ORTHDION_BF16)
        assert e.value.status == b.ORTHDION_E_BAD_SHAPE, (shape, r)
    # leading dimension smaller than n / not a multiple of 8
    for lds in ([(120, 128, 128)], [(128, 132, 128)]):
        with pytest.raises(b.OrthDionError) as e:
            b.orthdion_create([(64, 128)], 16, 1, 1, lds=lds)
        assert e.value.status == b.ORTHDION_E_BAD_SHAPE
    for kw in (dict(mu=1.5), dict(mu=-0.1), dict(mu=float("nan")), dict(lr=float("inf")), dict(variant=7),
               dict(ef=3), dict(precision=9), dict(groups=3), dict(groups=-1)):
        with pytest.raises(b.OrthDionError) as e:
            b.orthdion_create([(64, 64)], 8, 1, 1, **kw)
        assert e.value.status == b.ORTHDION_E_INVALID_ARG, kw
    with pytest.raises(b.OrthDionError) as e:
        b.orthdion_create([(64, 64)], 8, 5, 1)
    assert e.value.status == b.ORTHDION_E_INVALID_ARG
    with pytest.raises(b.OrthDionError) as e:
        b.orthdion_create([], 8, 1, 1)
    assert e.value.status == b.ORTHDION_E_INVALID_ARG


def test_null_arguments_are_reported():
    lib = b.load()
    assert lib.orthdion_create(None, None, 1, None) == b.ORTHDION_E_NULL_PTR
    h = ctypes.c_void_p()
    assert lib.orthdion_create(ctypes.byref(h), None, 1, None) == b.ORTHDION_E_NULL_PTR
    assert lib.orthdion_set_lr(None, 0.1) == b.ORTHDION_E_NULL_PTR
    assert lib.orthdion_destroy(None) == b.ORTHDION_E_NULL_PTR
    assert lib.orthdion_workspace_bytes(None) == 0


def test_step_rejects_bad_buffers_before_launching():
    h = b.orthdion_create([(64, 64)], 8, 1, 1)
    need = b.orthdion_workspace_bytes(h)
    fake = 1 << 20           # a 16-byte aligned, never dereferenced "device address"
    with pytest.raises(b.OrthDionError) as e:
        b.orthdion_step(h, [fake], [fake], [fake], [fake], 0, need)
    assert e.value.status == b.ORTHDION_E_NULL_PTR
    with pytest.raises(b.OrthDionError) as e:
        b.orthdion_step(h, [fake], [fake], [fake], [fake], fake, need - 1)
    assert e.value.status == b.ORTHDION_E_WORKSPACE_TOO_SMALL
    with pytest.raises(b.OrthDionError) as e:
        b.orthdion_step(h, [fake], [fake], [fake], [fake], fake + 8, need)
    assert e.value.status == b.ORTHDION_E_MISALIGNED
    with pytest.raises(b.OrthDionError) as e:
        b.orthdion_step(h, [fake + 4], [fake], [fake], [fake], fake, need)
    assert e.value.status == b.ORTHDION_E_MISALIGNED
    with pytest.raises(b.OrthDionError) as e:
        b.orthdion_step(h, [fake], [0], [fake], [fake], fake, need)
    assert e.value.status == b.ORTHDION_E_NULL_PTR
    with pytest.raises(b.OrthDionError) as e:
        b.orthdion_get_info(h, 1)
    assert e.value.status == b.ORTHDION_E_NO_STEP
    b.orthdion_destroy(h)


def test_setters_and_layout():
    shapes = [(256, 512), (128, 128), (256, 512)]
    h = b.orthdion_create(shapes, 32, 1, 1)
    b.orthdion_set_lr(h, 0.5)
    b.orthdion_set_mu(h, 0.0)
    b.orthdion_set_variant(h, b.ORTHDION_COLNORM)
    for bad in (lambda: b.orthdion_set_mu(h, 2.0), lambda: b.orthdion_set_lr(h, float("nan")),
                lambda: b.orthdion_set_variant(h, 4)):
        with pytest.raises(b.OrthDionError):
            bad()
    need = b.orthdion_workspace_bytes(h)
    seen = []
    for i, (m, n) in enumerate(shapes):
        lay = b.orthdion_workspace_layout(h, i)
        sizes = {"P": m * 32 * 4, "R": n * 32 * 4, "T_P1": 32 * 32 * 4, "T_P2": 32 * 32 * 4, "T_Q1": 32 * 32 * 4,
                 "T_Q2": 32 * 32 * 4}
        for key, nbytes in sizes.items():
            assert lay[key] % 16 == 0 and lay[key] + nbytes <= need
            seen.append((lay[key], lay[key] + nbytes))
    seen.sort()
    for (a0, a1), (b0, b1) in zip(seen, seen[1:]):
        assert a1 <= b0, "debug regions overlap"
    with pytest.raises(b.OrthDionError):
        b.orthdion_workspace_layout(h, 3)
    assert "shape" in b.orthdion_strerror(b.ORTHDION_E_BAD_SHAPE)
    assert b.orthdion_strerror(0) == "ok"
    b.orthdion_destroy(h)


def test_workspace_grows_with_the_set():
    one = b.orthdion_create([(512, 512)], 64, 1, 1)
    two = b.orthdion_create([(512, 512)] * 40, 64, 1, 1)      # more than one launch batch
    assert b.orthdion_workspace_bytes(two) > 30 * b.orthdion_workspace_bytes(one) // 2
    b.orthdion_destroy(one)
    b.orthdion_destroy(two)


def test_binding_phase_and_diagnostic_names_follow_the_header():
    """The binding's name lists are in the header's enum order and of its length."""
    import re
    from paper_2605_16341_amd import binding
    text = open(os.path.join(os.path.dirname(__file__), "..", "include", "orthdion.h")).read()
    phases = re.findall(r"ORTHDION_PHASE_([A-Z_]+)\s*=\s*(\d+)", text)
    assert [name.lower() for name, _ in phases] == binding.PHASES
    assert [int(v) for _, v in phases] == list(range(len(phases)))
    assert int(re.search(r"ORTHDION_NPHASE\s*=\s*(\d+)", text).group(1)) == len(binding.PHASES)
    assert int(re.search(r"ORTHDION_NDIAG\s*=\s*(\d+)", text).group(1)) == len(binding.DIAG)


def test_groups_follow_the_size_of_the_set():
    """Host-side planning of orthdion_config.groups: the library takes two groups for several
    matrices of 2^26 to 2^29 elements in all, one otherwise; a caller's 2 needs at least two launch
    batches; the workspace never shrinks with the choice."""
    from paper_2605_16341_amd import synth

    def groups(shapes, r, asked):
        h = b.orthdion_create(shapes, r, b.ORTHDION_BF16, b.ORTHDION_BF16, groups=asked)
        got, ws = b.orthdion_get_groups(h), b.orthdion_workspace_bytes(h)
        b.orthdion_destroy(h)
        return got, ws

    c3, c4 = synth.WORKLOADS["C3"], synth.WORKLOADS["C4"]
    assert groups(c4.shapes, c4.r, 0)[0] == 2 and groups(c4.shapes, c4.r, 1)[0] == 1
    assert groups(c3.shapes, c3.r, 0)[0] == 1 and groups(c3.shapes, c3.r, 2)[0] == 2
    assert groups([(8192, 8192)], 256, 0)[0] == 1 and groups([(8192, 8192)], 256, 2)[0] == 1      # one batch
    assert groups([(8192, 8192)] * 3, 256, 2)[0] == 1                                             # still one batch
    small = [(256, 128), (128, 512), (96, 96)]
    assert groups(small, 32, 0)[0] == 1 and groups(small, 32, 2)[0] == 2
    assert groups(small, 32, 2)[1] >= groups(small, 32, 1)[1]
    assert b.load().orthdion_get_groups(None) == 0
