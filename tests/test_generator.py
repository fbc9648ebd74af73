"""Host generator: the counter RNG against its published known answers, the noise law against
its definition, and determinism."""
import numpy as np
import pytest
from scipy import stats

from gen.bf16 import bf16_bits_to_f32, f32_to_bf16_bits
from gen.configs import BF16, CONFIGS, F32
from gen.host import HostGenerator, philox4x32
from gen.tables import build_table
from gen.trajectory import Trajectory


def test_philox4x32_10_known_answers():
    # known-answer vectors distributed with the reference implementation of
    # Salmon et al., "Parallel random numbers: as easy as 1, 2, 3" (SC'11)
    kat = [
        ([0, 0, 0, 0], [0, 0], [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]),
        ([0xFFFFFFFF] * 4, [0xFFFFFFFF] * 2, [0x408F276D, 0x41C83B0E, 0xA20BC7C6, 0x6D5451FD]),
        ([0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344], [0xA4093822, 0x299F31D0],
         [0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1]),
    ]
    for ctr, key, want in kat:
        assert philox4x32(ctr, key).tolist() == want


def test_tables_are_monotone_quantiles():
    for kind in ("normal", "student3"):
        t = build_table(kind, 1.0)
        assert np.all(np.diff(t[:1665]) < 0) and abs(t[1664]) < 1e-6
    t = build_table("normal", 1.0)
    assert abs(t[0] - (-stats.norm.ppf(0.5 / 2 ** 32))) < 1e-5


@pytest.mark.parametrize("cid,kind", [(1, "normal"), (5, "student3")])
def test_noise_follows_its_law(cid, kind):
    cfg = CONFIGS[cid].replace(V=200_000)
    tr = Trajectory(cfg)
    g = HostGenerator(cfg, np.full_like(tr.target, -1), tr.rival * 0 - 1)
    pos = np.arange(cfg.gen_start, cfg.gen_start + 5)
    z = np.zeros(cfg.B * cfg.L, np.float32)
    x = g.rows(3, pos, z, z).astype(np.float64).reshape(-1) / cfg.noise_scale
    dist = stats.norm if kind == "normal" else stats.t(3)
    ks = stats.kstest(x, dist.cdf)
    assert ks.statistic < 0.004, ks
    # tail: empirical count above the 1e-4 upper quantile
    q = dist.ppf(1 - 1e-4)
    assert 60 <= np.sum(x > q) <= 145


def test_rows_are_pure_functions_of_their_coordinates():
    cfg = CONFIGS[2].replace(V=5000)
    tr = Trajectory(cfg)
    g1 = HostGenerator(cfg, tr.target, tr.rival, threads=1)
    g4 = HostGenerator(cfg, tr.target, tr.rival, threads=4)
    T, R = tr.planted(7)
    pos = np.array([64, 65, 200, 319])
    a = g1.rows(7, pos, T, R).copy()
    b = g4.rows(7, pos[::-1].copy(), T, R)[::-1]
    np.testing.assert_array_equal(a, b)
    c = g1.rows(8, pos, T, R)
    assert np.mean(a == c) < 0.05
    # bf16 rows are the RNE rounding of the fp32 rows
    f = HostGenerator(cfg.replace(dtype=F32), tr.target, tr.rival).rows(7, pos, T, R)
    np.testing.assert_array_equal(f32_to_bf16_bits(f), a)
    # planted target: row minus noise equals T at the target, 0 elsewhere
    g0 = HostGenerator(cfg.replace(dtype=F32), np.full_like(tr.target, -1), np.full_like(tr.rival, -1))
    noise = g0.rows(7, pos, T, R).copy()
    for k, p in enumerate(pos):
        d = f[k] - noise[k]
        assert np.count_nonzero(d) <= 1
        assert f[k, tr.target[p]] == np.float32(noise[k, tr.target[p]] + T[p])


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -2.5, 3.0e38], np.float32)
    h = f32_to_bf16_bits(x)
    back = bf16_bits_to_f32(h)
    assert back[0] == 1.0 and back[1] == 1.0            # tie -> even
    assert back[2] == 1.0078125 and back[3] == 1.015625  # above half / tie -> even (up)
    assert back[4] == -2.5
