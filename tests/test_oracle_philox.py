"""Pins for the oracle's counter-based generator and its element mapping (CPU only)."""
import os
import shutil
import subprocess
import sys

import numpy as np
import pytest

from oracle import qsync_oracle as orc
from tests import bigint_ref as ref

HERE = os.path.dirname(os.path.abspath(__file__))


def _ctr_array(values):
    return np.array([[(v >> (32 * j)) & 0xFFFFFFFF for j in range(4)] for v in values], dtype=np.uint32)


def test_philox_matches_bigint_rederivation():
    rng = np.random.default_rng(11)
    for key in [(0, 0), (1, 0), (0xDEADBEEF, 0x12345678), (0xFFFFFFFF, 0xFFFFFFFF)]:
        ctrs = [int.from_bytes(rng.bytes(16), "little") for _ in range(300)] + [0, 1, (1 << 128) - 1, 1 << 64]
        got = orc.philox4x32_10(_ctr_array(ctrs), key)
        for c, g in zip(ctrs, got):
            want = ref.philox4x32_10([(c >> (32 * j)) & 0xFFFFFFFF for j in range(4)], list(key))
            assert list(map(int, g)) == want


def test_philox_published_known_answers():
    """The generator's standard check vectors (tests/golden/philox4x32_10_known_answers.txt)."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_known_answers.txt")
    rows = [ln for ln in open(path).read().splitlines() if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for ln in rows:
        ctr, key, want = [[int(w, 16) for w in part.split()] for part in ln.split("|")]
        got = orc.philox4x32_10(np.array([ctr], dtype=np.uint32), (key[0], key[1]))
        assert [int(v) for v in got.reshape(-1)] == want, ln


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not found")
def test_philox_matches_rocrand_host_engine(tmp_path):
    """Library pin: rocRAND's host-callable Philox4x32-10 engine produces the same blocks."""
    exe = tmp_path / "rocrand_philox_host"
    src = os.path.join(HERE, "helpers", "rocrand_philox_host.cpp")
    subprocess.run(["hipcc", "--cuda-host-only", "-O1", "-o", str(exe), src], check=True,
                   stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    for seed, subs, first, count in [(1, 0, 0, 64), (0x0123456789ABCDEF, 0, (1 << 40) + 5, 64),
                                     (7, 3, (1 << 32) - 8, 32), (0xFFFFFFFFFFFFFFFF, 0xFFFFFFFF00000001, 12345, 16)]:
        out = subprocess.run([str(exe), str(seed), str(subs), str(first), str(count)], check=True,
                             capture_output=True, text=True).stdout.split()
        want = np.array(list(map(int, out)), dtype=np.uint32).reshape(count, 4)
        ctrs = [(subs << 64) | (first + i) for i in range(count)]
        got = orc.philox4x32_10(_ctr_array(ctrs), (seed & 0xFFFFFFFF, seed >> 32))
        np.testing.assert_array_equal(got, want)


def test_draw_mapping_and_offset_carry():
    # element i -> block offset + i//8, 16-bit slot i%8 (word (i%8)//2, low half first)
    for seed, offset, n in [(1, 0, 37), (2**63 + 5, 123456789012345, 64), (9, 2**64 - 2, 40), (3, 2**64 + 7, 9)]:
        got = orc.sr_draws(seed, offset, n)
        want = [ref.draw16(seed, offset, i) for i in range(n)]
        assert list(map(int, got)) == want


def test_draws_do_not_depend_on_length_and_offset_shifts_by_groups():
    a = orc.sr_draws(5, 100, 1000)
    b = orc.sr_draws(5, 100, 64)
    np.testing.assert_array_equal(a[:64], b)
    c = orc.sr_draws(5, 103, 64)
    np.testing.assert_array_equal(a[24:88], c)          # three groups of eight later


def test_draws_uniform_chi_square():
    n = 1 << 20
    u = orc.sr_draws(2024, 0, n).astype(np.int64)
    counts = np.bincount(u >> 8, minlength=256)         # 256 equiprobable cells on the high byte
    chi2 = ((counts - n / 256) ** 2 / (n / 256)).sum()
    assert 150 < chi2 < 380                             # 255 d.o.f.: mean 255, sd 22.6
    low = np.bincount(u & 0xFF, minlength=256)
    chi2_low = ((low - n / 256) ** 2 / (n / 256)).sum()
    assert 150 < chi2_low < 380
    # neighbouring draws of a block are uncorrelated
    r = np.corrcoef(u[0::2], u[1::2])[0, 1]
    assert abs(r) < 5e-3
