"""Pins of the page-accounting oracle: the paper's Fig. 3 worked example, Table 1 and the
F_mem figure of Sec. 3.1, and a byte-level brute force of "which pages does a set of loaded
expert ranges touch"."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import pool


def test_fig3_worked_example(golden_fig3):
    g = golden_fig3
    E_max, e0, e1 = g["E_max"], g["e_0"], g["e_1"]
    page = 1 << 20
    expert = g["expert_pages_times_2"] * page // 2                  # 1.5 pages per expert
    M = 4                                                            # even, so Delta_0 is page aligned
    vt = pool.VirtualTensorPages(M + 2 * E_max, expert, page)
    base_pages = vt.load(0, M)
    assert len(base_pages) == M * 3 // 2
    new0 = vt.load(M, e0)
    assert len(new0) == g["pages_adapter_0"]                         # 3 pages under 2 experts
    delta1 = M + E_max
    assert (delta1 * expert) % page != 0                             # second adapter starts mid-page
    new1 = vt.load(delta1, e1)
    assert len(new1) == 2                                            # 1.5 pages of data, one half-filled page
    # padding slots [Delta_0+e_0, Delta_0+E_max) and [Delta_1+e_1, ...) own no page of their own
    pad_lo, pad_hi = (M + e0) * expert, delta1 * expert
    fully_pad = [q for q in range(pad_lo // page, pad_hi // page) if q * page >= pad_lo and (q + 1) * page <= pad_hi]
    assert fully_pad and not set(fully_pad) & set(vt.mapped_pages())
    assert vt.mapped_bytes() == (len(base_pages) + 3 + 2) * page
    # evict in reverse: everything returns
    assert sorted(vt.unload(delta1)) == sorted(new1)
    assert sorted(vt.unload(M)) == sorted(new0)
    assert vt.mapped_pages() == sorted(base_pages)


def test_shared_boundary_page_is_refcounted():
    page, expert = 4096, 6144                                        # 1.5 pages
    vt = pool.VirtualTensorPages(8, expert, page)
    a = vt.load(0, 3)                                                # bytes [0, 18432) -> pages 0..4 (page 4 half)
    b = vt.load(3, 1)                                                # bytes [18432, 24576) -> pages 4, 5
    assert a == [0, 1, 2, 3, 4] and b == [5] and vt.shared_pages() == [4]
    assert vt.unload(0) == [0, 1, 2, 3]                              # page 4 survives for its neighbour
    assert vt.mapped_pages() == [4, 5]
    assert vt.unload(3) == [4, 5] and vt.mapped_pages() == []


@pytest.mark.parametrize("seed", range(5))
def test_mapped_pages_equal_byte_level_cover(seed):
    rng = np.random.default_rng(seed)
    page, expert, P = 64, int(rng.integers(20, 200)), 40
    vt = pool.VirtualTensorPages(P, expert, page)
    touched = np.zeros(P * expert, dtype=bool)
    live = {}
    for _ in range(30):
        if live and rng.random() < 0.4:
            s0 = list(live)[int(rng.integers(len(live)))]
            vt.unload(s0); live.pop(s0)
        else:
            s0 = int(rng.integers(0, P)); n = int(rng.integers(0, 5))
            if s0 + n > P or any(not (s0 + n <= a or a + m <= s0) or s0 == a for a, m in live.items()):
                continue
            vt.load(s0, n); live[s0] = n
        touched[:] = False
        for a, m in live.items():
            touched[a * expert:(a + m) * expert] = True
        cover = sorted({int(b) // page for b in np.nonzero(touched)[0]})
        assert vt.mapped_pages() == cover


def _layers_with(mx, total, L):
    """Any per-layer expert counts with the given maximum and sum (S_i depends on nothing else)."""
    e = [mx] + [0] * (L - 1)
    rest = total - mx
    for l in range(1, L):
        take = min(mx, rest)
        e[l] = take
        rest -= take
    assert rest == 0
    return e


def test_table1_sparsity_and_fmem(golden_table1):
    L, M, E_max = 26, 64, 13
    per_adapter = []
    for name, mx, avg, s_printed in golden_table1:
        total = round(avg * L)
        assert abs(total / L - avg) < 0.005, name                    # the printed average is k/26
        e = _layers_with(mx, total, L)
        S = pool.adapter_sparsity(e)
        assert S == 1 - Fraction(total, L * mx)
        assert abs(float(S) - s_printed) <= 0.0051, (name, float(S), s_printed)
        per_adapter.append(e)
    assert max(mx for _, mx, _, _ in golden_table1) == E_max         # "smallest feasible E_max = 13"
    e_li = [[per_adapter[i][l] for i in range(len(per_adapter))] for l in range(L)]
    F = float(pool.fragmentation_factor(M, len(per_adapter), E_max, e_li))
    assert abs(F - 1.51) <= 0.01, F                                   # paper prints 1.51; table gives 1.502


def test_sparsity_closed_forms():
    assert pool.adapter_sparsity([5, 5, 5]) == 0                     # fully dense adapter
    assert pool.adapter_sparsity([4, 0, 0, 0]) == Fraction(3, 4)
    assert pool.fragmentation_factor(8, 2, 3, [[3, 3]]) == 1         # no padding, no fragmentation
    assert pool.fragmentation_factor(8, 2, 3, [[0, 0]]) == Fraction(14, 8)
