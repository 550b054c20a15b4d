"""Host logic of the per-call / per-thread kernel-variant options (no GPU needed): validation, the
one-knob setters, and that the defaults of one host thread are invisible to another."""
import ctypes
import threading

import pytest

from paper_2209_06979_amd import binding as mc


@pytest.fixture(autouse=True)
def _reset():
    mc.set_thread_options(None)
    yield
    mc.set_thread_options(None)


def _fields(o):
    return {n: getattr(o, n) for n, _ in mc.Options._fields_}


def test_init_is_all_automatic():
    o = mc.Options(1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11)
    mc.lib.mc_options_init(ctypes.byref(o))
    assert set(_fields(o).values()) == {0}
    assert set(_fields(mc.get_thread_options()).values()) == {0}


@pytest.mark.parametrize("field,good,bad", [
    ("spmm_row_tile_bytes", [0, 64, 128, 256], [32, 100, -64, 512]),
    ("spmm_waves", [0, 1, 2, 4, 8], [3, 16, -1]),
    ("spmm_stages", [0, 1, 2], [3, -1]),
    ("spmm_splitting", [0, -1, 1], [-2, 2]),
    ("spmm_slab", [-1, 0, 1], [2, -2]),
    ("spmm_slab_waves", [0, 1, 8, 15], [16, -1]),
    ("spmm_slab_panels", [0, 1, 2, 4], [3, 8, -1]),
    ("sddmm_waves", [0, -1, 1, 2, 4, 8], [3, 16, -2]),
    ("softmax_variant", [0, 1, 2], [3, -1]),
    ("attention_mode", [0, 1, 2, 3, 4, 5, 6], [7, -1]),
    ("spmm_merge", [-1, 0, 1], [2, -2]),
])
def test_validation_of_every_field(field, good, bad):
    for v in good:
        o = mc.Options()
        setattr(o, field, v)
        mc.set_thread_options(o)
        assert getattr(mc.get_thread_options(), field) == v
    keep = _fields(mc.get_thread_options())
    for v in bad:
        o = mc.Options()
        setattr(o, field, v)
        with pytest.raises(mc.MagicubeError) as e:
            mc.set_thread_options(o)
        assert e.value.status == mc.MC_EINVAL
        assert _fields(mc.get_thread_options()) == keep      # a rejected struct changes nothing


def test_one_knob_setters_fill_the_thread_defaults():
    mc.set_spmm_variant(64, 4)
    mc.set_spmm_stages(1)
    mc.set_spmm_splitting(False)
    mc.set_sddmm_variant(0)          # this setter's convention: 0 = the direct-load kernel
    mc.set_softmax_variant(2)
    mc.set_attention_mode(3)
    o = mc.get_thread_options()
    assert _fields(o) == dict(spmm_row_tile_bytes=64, spmm_waves=4, spmm_stages=1, spmm_splitting=-1, spmm_slab=0,
                              spmm_slab_waves=0, spmm_slab_panels=0, sddmm_waves=-1, softmax_variant=2, attention_mode=3,
                              spmm_merge=0)
    mc.set_sddmm_variant(-1)         # -1 = automatic
    mc.set_spmm_splitting(True)
    assert mc.get_thread_options().sddmm_waves == 0 and mc.get_thread_options().spmm_splitting == 0
    for call in (lambda: mc.set_spmm_variant(96, 0), lambda: mc.set_spmm_variant(0, 3), lambda: mc.set_spmm_stages(0),
                 lambda: mc.set_sddmm_variant(5), lambda: mc.set_attention_mode(9), lambda: mc.set_softmax_variant(-1)):
        with pytest.raises(mc.MagicubeError):
            call()
    assert mc.get_thread_options().spmm_row_tile_bytes == 64       # failed setters left everything as it was


def test_defaults_are_per_thread():
    mc.set_spmm_variant(128, 2)
    seen = {}

    def other():
        seen["initial"] = _fields(mc.get_thread_options())
        mc.set_attention_mode(1)
        mc.set_spmm_variant(256, 8)
        seen["own"] = _fields(mc.get_thread_options())

    t = threading.Thread(target=other)
    t.start()
    t.join()
    assert set(seen["initial"].values()) == {0}                     # a new thread starts at automatic
    assert seen["own"]["attention_mode"] == 1 and seen["own"]["spmm_row_tile_bytes"] == 256
    mine = mc.get_thread_options()
    assert (mine.spmm_row_tile_bytes, mine.spmm_waves, mine.attention_mode) == (128, 2, 0)


def test_null_arguments():
    assert mc.lib.mc_get_thread_options(None) == mc.MC_EINVAL
    mc.lib.mc_options_init(None)                                    # ignored
    assert mc.lib.mc_set_thread_options(None) == mc.MC_OK           # NULL = automatic
