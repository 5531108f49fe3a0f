"""The fitting step behind the GEMM cost model, on a synthetic timing table with known parameters."""
import numpy as np

from paper_1702_03192_amd import binding as mt
from paper_1702_03192_amd import tune


def test_every_configuration_name_parses():
    for name in mt.gemm_configs():
        bm, bn, occ = tune._config_geometry(name)
        assert bm % 32 == 0 and bn % 32 == 0 and 1 <= occ <= 4
        assert name.startswith(f"{bm}x{bn}x")


def test_tile_units_charge_the_workgroup_left_alone():
    assert tune.tile_units(4, 2, 4) == 4.0                       # whole rounds
    assert tune.tile_units(3, 2, 4) == 2 + 1 / 0.85              # two together, one alone
    assert tune.tile_units(1, 2, 4) == 1 / 0.85
    assert tune.tile_units(4, 3, 4) == 3 + 1 / 0.92              # alone after a round of three
    assert tune.tile_units(5, 3, 4) == 5.0                       # two left over run at the full rate
    assert tune.tile_units(3, 1, 8) == 3.0                       # 8-wave workgroups fill the SIMDs alone


def test_fit_recovers_planted_parameters():
    names = mt.gemm_configs()
    planted = {}
    table = {}
    for c, name in enumerate(names):
        bm, bn, occ = tune._config_geometry(name)
        for op in (0, 1):
            eff, round_s = 0.6 + 0.02 * c + 0.01 * op, (2.0 + c + 0.5 * op) * 1e-6
            planted[(c, op)] = (eff, round_s)
            for m in tune.SIZES:
                for n in tune.SIZES:
                    for k in (64, 512, 4096):
                        tiles = -(-m // bm) * -(-n // bn)
                        per_cu = -(-tiles // 256)
                        units = tune.tile_units(per_cu, occ, tune._config_waves(name))
                        t = units * 2.0 * bm * bn * k / (tune.PEAK_PER_CU * eff) + -(-per_cu // occ) * round_s + 3e-6
                        table.setdefault((op, m, n, k), {})[(c, 1)] = t
    fitted = tune.fit_table(table, names)
    for key, (eff, round_s) in planted.items():
        got = fitted[key]
        assert got is not None and got[2] >= 4
        assert abs(got[0] - eff) < 1e-6 and abs(got[1] - round_s) < 1e-10
        assert got[4] < 1e-9
