"""The C-ABI library on the host: it loads, exports every symbol the header declares,
and rejects bad arguments before touching the GPU.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

import paper_1905_04374_amd as mb

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "mbulyan.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+)?(?:char|int)\s*\*?\s*(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert len(names) >= 19 and "mbulyan_aggregate" in names and "coordwise_trimmed_avg" in names
    for name in names:
        assert hasattr(mb.lib, name), f"{name} declared in mbulyan.h but not exported"
    assert sorted(mb.EXPORTS) == names


def test_library_is_in_tree():
    assert os.path.dirname(mb.LIB_PATH) == os.path.dirname(os.path.abspath(mb.__file__))
    assert "gfx950" in mb.version()


@pytest.mark.parametrize("n,f,mode,expect", [
    (11, 2, 0, (7, 3)), (11, 2, 1, (5, 1)), (39, 9, 0, (21, 3)), (39, 9, 1, (19, 1)),
    (51, 12, 0, (27, 3)), (64, 15, 0, (34, 4)), (9, 1, 1, (5, 3)), (3, 0, 0, (3, 3)),
])
def test_params(n, f, mode, expect):
    assert mb.mbulyan_params(n, f, mode) == expect


@pytest.mark.parametrize("args,status", [
    ((10, 2, 0), mb.MB_EPRECOND), ((2, 0, 0), mb.MB_EPRECOND), ((0, 0, 0), mb.MB_EINVAL),
    ((11, -1, 0), mb.MB_EINVAL), ((11, 2, 7), mb.MB_EINVAL), ((65, 0, 0), mb.MB_EUNSUPPORTED),
])
def test_params_errors(args, status):
    with pytest.raises(mb.MBulyanError) as e:
        mb.mbulyan_params(*args)
    assert e.value.status == status


def test_workspace_bytes():
    small = mb.mbulyan_workspace_bytes(11, 1000)
    big = mb.mbulyan_workspace_bytes(64, 10 ** 9)
    assert 0 < small < big < 64 << 20 and small % 256 == 0 and big % 256 == 0
    with pytest.raises(mb.MBulyanError):
        mb.mbulyan_workspace_bytes(65, 10)


def test_strerror_and_codes():
    for s in range(6):
        assert mb.lib.mbulyan_strerror(s)
    assert b"4f+3" in mb.lib.mbulyan_strerror(mb.MB_EPRECOND)


def test_bad_arguments_are_rejected_on_the_host():
    """Null pointers, bad sizes and violated preconditions return before any HIP call."""
    lib = mb.lib
    one = C.c_void_p(256)   # never dereferenced: every call below fails validation first
    assert lib.mbulyan_aggregate(None, 11, 2, 100, one, None, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate(one, 11, 2, 100, None, None, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate(one, 10, 2, 100, one, None, None) == mb.MB_EPRECOND
    assert lib.mbulyan_aggregate(one, 11, 2, 0, one, None, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate(one, 65, 0, 10, one, None, None) == mb.MB_EUNSUPPORTED
    assert lib.mbulyan_aggregate_ex(one, 11, 2, 100, 99, 0, 0, 0, one, None, None, 0, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_ex(one, 11, 2, 100, 100, 0, 12, 0, one, None, None, 0, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_ex(one, 11, 2, 100, 100, 0, 5, 6, one, None, None, 0, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_ex(one, 11, 2, 100, 100, 0, 0, 0, one, None, one, 16, None) == mb.MB_EWORKSPACE
    assert lib.mbulyan_aggregate_ex(one, 11, 2, 100, 100, 0, 0, 0, one, None, C.c_void_p(257), 1 << 30,
                                    None) == mb.MB_EWORKSPACE
    assert lib.pairwise_sqdist(one, 11, 100, 100, None, 0, 0, None, 0, None) == mb.MB_EINVAL
    assert lib.pairwise_sqdist(one, 11, 100, 100, one, 0, 9, None, 0, None) == mb.MB_EINVAL
    assert lib.krum_scores(None, 11, 2, None, one, None) == mb.MB_EINVAL
    assert lib.multikrum_select(one, 11, 2, 0, one, None, None, None) == mb.MB_EINVAL
    assert lib.multikrum_select(one, 11, 2, 12, one, None, None, None) == mb.MB_EINVAL
    assert lib.coordwise_trimmed_avg(one, 11, 100, 100, one, 7, 8, None, one, None) == mb.MB_EINVAL
    assert lib.coordwise_trimmed_avg(one, 11, 100, 100, None, 7, 3, None, one, None) == mb.MB_EINVAL
    assert lib.multikrum_aggregate(one, 6, 2, 100, 100, one, None, None, 0, None) == mb.MB_EPRECOND
    assert lib.coordwise_median(one, 11, 100, 100, None, None) == mb.MB_EINVAL
    # the entry point that allocates nothing: same checks, and n beyond what its static array is sized for
    assert lib.mbulyan_aggregate_noalloc(one, 65, 0, 100, 100, 0, one, None, None) == mb.MB_EUNSUPPORTED
    assert lib.mbulyan_aggregate_noalloc(one, 10, 2, 100, 100, 0, one, None, None) == mb.MB_EPRECOND
    assert lib.mbulyan_aggregate_noalloc(one, 11, 2, 100, 99, 0, one, None, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_noalloc(one, 11, 2, 100, 100, 0, None, None, None) == mb.MB_EINVAL
    # gradients in host memory: the same checks before anything is allocated
    assert lib.mbulyan_aggregate_host(None, 0, 11, 2, 100, 100, 0, 50, one, None, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_host(one, 0, 10, 2, 100, 100, 0, 50, one, None, None) == mb.MB_EPRECOND
    assert lib.mbulyan_aggregate_host(one, 7, 11, 2, 100, 100, 0, 50, one, None, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_host(one, 0, 11, 2, 100, 100, 0, 0, one, None, None) == mb.MB_EINVAL
    assert lib.mbulyan_aggregate_fp16(one, 10, 2, 100, 100, 0, 0, 0, one, None, None, 0, None) == mb.MB_EPRECOND
    assert lib.pairwise_sqdist_fp16(one, 11, 100, 100, None, 0, None, 0, None) == mb.MB_EINVAL
    assert lib.mbulyan_set_dist_algo(5) == mb.MB_EINVAL
    assert lib.mbulyan_set_dist_algo(0) == mb.MB_OK
