"""Host logic of the library, no GPU: which select path serves which shape, and that the sizes
a plan hands to the kernels fit together (a grid or a capacity that does not match what a
kernel assumes is how a GPU gets faulted).  Through the C ABI of the built library
(bts_testing_plan)."""
import pytest

import workloads as wl

ONE_WORKGROUP, DENSE, SINGLE_PASS, THREE_LAUNCH = 0, 1, 2, 3


def plan(rows, d, K):
    from paper_2209_15203_amd import binding
    return binding.testing_plan(rows, d, K)


@pytest.mark.parametrize("name,up,dn", [
    ("C1", THREE_LAUNCH, THREE_LAUNCH),       # a few million coordinates, K = 1049
    ("C2", SINGLE_PASS, SINGLE_PASS),         # K = 1 % of d: too many for the three-launch select
    ("C3", SINGLE_PASS, SINGLE_PASS),
    ("C4", SINGLE_PASS, SINGLE_PASS),
    ("C5", SINGLE_PASS, SINGLE_PASS),
])
def test_default_paths_of_the_five_configurations(name, up, dn):
    cfg = wl.CONFIGS[name]
    assert plan(cfg.N, cfg.d, cfg.K_up)["path"] == up
    assert plan(1, cfg.d, cfg.K_dn)["path"] == dn


def test_default_paths_by_shape():
    assert plan(64, 8192, 82)["path"] == ONE_WORKGROUP
    assert plan(3, 100, 1)["path"] == ONE_WORKGROUP
    assert plan(4, 8193, 9)["path"] == THREE_LAUNCH
    assert plan(20, 29_034, 30)["path"] == THREE_LAUNCH          # the paper's smallest model
    assert plan(100, 242_762, 243)["path"] == SINGLE_PASS        # 2.4e7 coordinates a call
    assert plan(20, 20_040_522, 20_041)["path"] == SINGLE_PASS
    assert plan(1, 20_040_522, 20_041)["path"] == SINGLE_PASS    # a lone row from 8e6
    assert plan(1, 5_000_000, 5_000)["path"] == DENSE            # a lone row below 8e6, K > 3072
    assert plan(4, 1 << 20, (1 << 20) // 32)["path"] == DENSE    # K > d / 64
    assert plan(4, 1 << 20, 1 << 20)["path"] == DENSE            # K = d
    assert plan(2, 3_000_000, 4000)["path"] == DENSE             # small call, K > 3072
    assert plan(7, 50_000, 0)["path"] == DENSE                   # K = 0: no select at all


SHAPES = [(r, d, K) for r in (1, 2, 16, 64, 100, 256)
          for d in (65_536, 70_001, 262_147, 1 << 20, 4_194_304, 11_173_962, 25_557_032,
                    110_000_000, (1 << 32) - 1)
          for K in (1, 17, d // 100_000 + 1, d // 1000, d // 64)]


@pytest.mark.parametrize("rows,d,K", SHAPES)
def test_single_pass_plan_fits_together(rows, d, K):
    p = plan(rows, d, K)
    if not p["single_pass_possible"]:
        assert K == 0 or d < 65_536 or K * 64 > d
        return
    chunks = (d + 511) // 512 + 1                 # a row may straddle one more 512-chunk
    assert p["dir_entries"] == p["tiles"] * 64 >= chunks
    assert p["lists"] == 64
    assert 1 <= p["sample_stride"] <= max(1, (d // 256) // 64)
    assert p["sample_target"] >= 48
    assert p["waves_per_simd"] in (3, 5, 6)
    # the lists hold the candidates a sampled bound aims at (up to 2 x target x stride) and
    # those a handed-on bound aims at, twice over
    assert p["rank_next"] > K
    total_cap = p["list_cap"] * p["lists"]
    assert total_cap >= 4 * p["sample_target"] * p["sample_stride"]
    assert total_cap >= 2 * p["rank_next"]
    assert p["list_cap"] < (1 << 31)


@pytest.mark.parametrize("rows,d,K", [(r, d, K) for r in (1, 4, 20, 100)
                                      for d in (8193, 29_034, 242_762, 1 << 20, 1 << 22, (1 << 22) + 1)
                                      for K in (1, 30, 1049, 8192, 8193)])
def test_three_launch_plan_fits_together(rows, d, K):
    p = plan(rows, d, K)
    ok = 1 <= K <= 8192 and K * 64 <= d and 8192 < d <= (1 << 22) and rows * d <= (1 << 25)
    assert bool(p["three_launch_possible"]) == ok
    if not ok:
        return
    chunks = (d + 511) // 512 + 1
    assert p["three_launch_dir_entries"] == p["three_launch_tiles"] * 64 >= chunks
    assert p["three_launch_tiles"] <= 256
    # a list can take every coordinate of the chunks that append to it: no overflow
    assert p["three_launch_cap"] == p["three_launch_dir_entries"] // 64 * 512
    assert 1 <= p["three_launch_hist_blocks"] <= 64
    assert 1 <= p["three_launch_blocks"]


def test_plan_rejects_bad_shapes():
    from paper_2209_15203_amd import binding
    for rows, d, K in ((0, 100, 1), (1, 0, 0), (1, 1 << 32, 1), (1, 100, 101)):
        with pytest.raises(binding.BtsError):
            binding.testing_plan(rows, d, K)
