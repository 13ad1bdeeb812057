"""Host logic of the bf16 GEMM's launch schedule: tile coverage of every grid the library would build (no GPU)."""
import itertools

import pytest

from paper_2603_13289_amd import binding as rc


def test_every_tile_is_covered_exactly_once_on_the_workload_shapes():
    shapes = [(m, n, k, swiglu) for m in (33, 256, 1024, 1025, 1088, 1089, 1639, 3687, 5120, 7373, 36864)
              for (n, k, swiglu) in ((6144, 4096, False), (4096, 4096, False), (14336, 4096, True), (4096, 14336, False),
                                     (27648, 5120, True), (5120, 27648, False), (7168, 5120, False))]
    for (m, n, k, swiglu), tile, ws in itertools.product(shapes, (5, 6, 7), (True, False)):
        if tile == 7 and (swiglu or n % 192):
            continue
        err, nb = rc.rc_gemm_plan_check(m, n, k, swiglu, tile, 256, ws)
        assert err == 0, (m, n, k, swiglu, tile, ws, nb)
        assert nb > 0


@pytest.mark.parametrize("n_cus", [256, 304, 64, 8])
def test_coverage_over_a_sweep_of_row_counts(n_cus):
    """All row counts around the tile and round boundaries, ragged last tile rows of every height."""
    for n, k, swiglu in ((2048, 256, False), (16384, 128, False), (8192, 64, True), (384, 1024, False)):
        for m in list(range(1, 600)) + list(range(1000, 1300, 7)) + [4095, 4096, 4097, 4160, 4161]:
            for tile in (5, 6, 7):
                if tile == 7 and (swiglu or n % 192):
                    continue
                err, _ = rc.rc_gemm_plan_check(m, n, k, swiglu, tile, n_cus, True)
                assert err == 0, (m, n, k, swiglu, tile, n_cus)


def test_thin_tiles_are_used_for_a_one_row_remainder():
    """1024 + 1 rows against a wide N: the schedule with the thin last tile row needs fewer workgroups than
    five full tile rows would."""
    rc.rc_tune_set(rc.RC_TUNE_GEMM_THIN_TILES, 0)
    try:
        err0, nb_plain = rc.rc_gemm_plan_check(1025, 14336, 4096, True, 5, 256, True)
    finally:
        rc.rc_tune_set(rc.RC_TUNE_GEMM_THIN_TILES, 1)
    err1, nb_thin = rc.rc_gemm_plan_check(1025, 14336, 4096, True, 5, 256, True)
    assert err0 == 0 and err1 == 0
    assert nb_thin != nb_plain


def test_coverage_without_the_xcd_regrouping():
    rc.rc_tune_set(rc.RC_TUNE_GEMM_XCD_REMAP, 0)
    try:
        for m in (1, 255, 257, 1025, 1088, 1639, 5120):
            for (n, k, swiglu) in ((6144, 4096, False), (14336, 4096, True), (4096, 14336, False)):
                for tile in (5, 6, 7):
                    if tile == 7 and (swiglu or n % 192):
                        continue
                    assert rc.rc_gemm_plan_check(m, n, k, swiglu, tile, 256, True)[0] == 0, (m, n, k, tile)
    finally:
        rc.rc_tune_set(rc.RC_TUNE_GEMM_XCD_REMAP, 1)


def test_bad_arguments():
    assert rc.rc_gemm_plan_check(0, 64, 64, False, 5)[0] == -1
    assert rc.rc_gemm_plan_check(64, 64, 100, False, 5)[0] == -1
    assert rc.rc_gemm_plan_check(64, 64, 64, False, 4)[0] == -1
