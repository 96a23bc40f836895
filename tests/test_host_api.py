"""CPU-side checks of the C boundary: the library loads, exports what the header declares,
and its host-only planning calls agree with the oracle.  No GPU compute here."""
import ctypes
import os
import re

import pytest

import paper_2303_01675_amd as kf
from oracle import schedule as sch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(kf.library_path()):
        from paper_2303_01675_amd import build
        build.build()
    return kf.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "kfkb.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*|int|size_t|double)\s+(\w+)\s*\(", header, flags=re.M)
    assert len(names) >= 30
    raw = ctypes.CDLL(kf.library_path())
    for n in names:
        assert hasattr(raw, n), "missing export: " + n


def test_schedule_matches_oracle(lib):
    for M in range(1, 14):
        for k in range(1, M + 1):
            for w in range(0, 5):
                assert kf.kfkb_schedule(k, M, w) == sch.kfkb_order(k, M, w), (k, M, w)
                assert kf.kfkb_peak_live(k, M, w) == sch.peak_live(sch.kfkb_order(k, M, w))
    assert kf.kfkb_schedule(2, 32, 0)[:6] == [("F", 0), ("F", 1), ("B", 0), ("B", 1), ("F", 2), ("F", 3)]


def test_schedule_errors(lib):
    for args in [(0, 4, 0), (5, 4, 0), (1, 0, 0), (1, 4, -1)]:
        with pytest.raises(kf.KfkbError) as e:
            kf.kfkb_schedule(*args)
        assert e.value.code == -1


def test_memory_model_matches_oracle(lib):
    for (L, b, T, H, h, F, eb) in [(2, 2, 64, 128, 4, 512, 4), (6, 4, 1024, 1024, 16, 4096, 2),
                                   (6, 2, 2048, 2048, 16, 8192, 2), (4, 1, 2048, 4096, 32, 16384, 2),
                                   (2, 1, 4096, 8192, 64, 32768, 2)]:
        assert kf.kfkb_activation_bytes_per_microbatch(L, b, T, H, h, F, eb) == \
            sch.activation_bytes_per_microbatch(L, b, T, H, h, F, eb)
        assert kf.kfkb_activation_bytes_per_microbatch(L, b, T, H, h, F, eb, recompute=1) == \
            sch.activation_bytes_per_microbatch(L, b, T, H, h, F, eb, recompute=True)


def test_calls_before_init_fail_cleanly(lib):
    kf.stage_destroy()
    for fn, args in [(kf.stage_forward, (0,)), (kf.stage_backward, (0,)), (kf.run_kFkB, (1, 1, 0)),
                     (kf.stage_zero_grads, ()), (kf.stage_sync, ())]:
        with pytest.raises(kf.KfkbError) as e:
            fn(*args)
        assert e.value.code == -2
    assert kf.stage_param_count() == 0 and kf.stage_workspace_bytes(1) == 0


def test_receive_list_mode_is_checked_and_returned(lib):
    assert kf.kfkb_set_inputs_ahead(0) == 2          # the default is "by k"
    assert kf.kfkb_set_inputs_ahead(1) == 0
    assert kf.kfkb_set_inputs_ahead(2) == 1
    for bad in (-1, 3):
        with pytest.raises(kf.KfkbError) as e:
            kf.kfkb_set_inputs_ahead(bad)
        assert e.value.code == -1
    assert kf.kfkb_set_inputs_ahead(2) == 2


def test_mid_tile_setter_is_checked(lib):
    assert kf.kfkb_set_mid_tiles(0) == 1             # default: where the shape rates best
    assert kf.kfkb_set_mid_tiles(2, 75) == 0
    for bad in ((-1, 90), (3, 90), (1, 0), (1, 101)):
        with pytest.raises(kf.KfkbError) as e:
            kf.kfkb_set_mid_tiles(*bad)
        assert e.value.code == -1
    assert kf.kfkb_set_mid_tiles(1) == 2


def test_sixteen_bit_attention_refuses_samples_beyond_its_32_bit_offsets(lib):
    """The 16-bit attention kernels address the rows of one sample with 32-bit byte offsets: T * 3H * 2 < 2 GiB is
    checked before any launch (host-side; nothing runs)."""
    for fn, args in ((kf.kfkb_op_attention_fwd, (kf.BF16, None, None, None, 1, 65536, 8192, 64, 1)),
                     (kf.kfkb_op_attention_bwd, (kf.BF16, None, None, None, None, None, None, 1, 65536, 8192, 64, 1))):
        with pytest.raises(kf.KfkbError) as e:
            fn(*args)
        assert e.value.code == -1 and "2 GiB" in str(e.value)
