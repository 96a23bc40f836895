"""Host-only check of the library's list schedule for S virtual stages against the oracle's (no GPU compute)."""
import os

import pytest

import paper_2303_01675_amd as kf
from oracle import pipeline as pl


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(kf.library_path()):
        from paper_2303_01675_amd import build
        build.build()
    return kf.load_library()


def test_list_schedule_equals_the_oracle(lib):
    n = 0
    for S in range(1, 7):
        for M in range(1, 13):
            for k in range(1, M + 1):
                assert kf.kfkb_pipeline_schedule(S, k, M) == pl.list_schedule(S, k, M), (S, k, M)
                n += 1
    assert n > 400
    assert kf.kfkb_pipeline_schedule(8, 4, 32) == pl.list_schedule(8, 4, 32)


def test_bad_arguments(lib):
    for S, k, M in [(0, 1, 4), (2, 0, 4), (2, 5, 4), (2, 1, 0)]:
        with pytest.raises(kf.KfkbError) as e:
            kf.kfkb_pipeline_schedule(S, k, M)
        assert e.value.code == -1
    assert kf.stage_pipeline_bytes(2, 4) == 0          # no stage yet
    with pytest.raises(kf.KfkbError):
        kf.run_pipeline_kFkB(1)                          # nothing bound
