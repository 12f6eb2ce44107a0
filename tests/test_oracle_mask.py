"""Pins for the oracle's mask and index maps (CPU only).

Each check ties oracle/ksa_oracle.c to something outside itself: hand-derived masks,
a set-form generator written literally from Eq. 1 / Eq. 3, closed-form counts, and the
partition property the paper states for chunk-granular sliding.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import ksa_oracle as O


# --------------------------------------------------------------------------------------
# An independent, literal construction: build the augmented token list of Eq. 1 as a
# Python list, then each row's visible SET from the two ranges of Eq. 3.
# --------------------------------------------------------------------------------------
def literal_sequence(n, c, m):
    seq = []
    for j in range(n // c):
        seq += [("t", j * c + r) for r in range(c)]
        seq += [("s", j, u) for u in range(m)]
    return seq


def literal_visible_sets(n, c, m, Cw, self_only=False):
    seq = literal_sequence(n, c, m)
    where = {tok: a for a, tok in enumerate(seq)}
    rows = []
    for tok in seq:
        if tok[0] == "t":
            i = tok[1]
            first_chunk = max(0, i // c - Cw)
            vis = {where[("t", t)] for t in range(first_chunk * c, i + 1)}
            vis |= {where[("s", j, u)] for j in range(0, i // c - Cw) for u in range(m)}
        else:
            _, j, u = tok
            vis = {where[("t", t)] for t in range(j * c, (j + 1) * c)}
            vis |= {where[("s", j, uu)] for uu in (range(u, u + 1) if self_only else range(0, u + 1))}
        rows.append(vis)
    return rows


def read_golden(path):
    with open(path) as f:
        lines = [ln.strip() for ln in f if ln.strip()]
    n, c, m, Cw = map(int, lines[0].split())
    rows = [list(map(int, ln.split(":")[1].split())) for ln in lines[1:]]
    return (n, c, m, Cw), np.array(rows, dtype=np.uint8)


@pytest.mark.parametrize("name", ["mask_n8_c2_m1_C1.txt", "mask_n8_c4_m2_C1.txt", "mask_n6_c2_m1_C0.txt"])
def test_hand_derived_masks(golden_dir, name):
    (n, c, m, Cw), want = read_golden(os.path.join(golden_dir, name))
    got = O.mask(n, c, m, Cw)
    assert got.shape == want.shape
    assert np.array_equal(got, want)


SMALL_SHAPES = [(n, c, m, Cw)
                for c in (1, 2, 3, 4, 8)
                for m in (0, 1, 2, 4)
                for J in (1, 2, 3, 5, 8)
                for Cw in (0, 1, 2, 3, 9)
                for n in (J * c,)
                if n <= 64]


def test_predicate_equals_literal_sets_exhaustively():
    checked = 0
    for (n, c, m, Cw) in SMALL_SHAPES:
        for flags in (0, O.FLAG_SUMMARY_SELF_ONLY):
            got = O.mask(n, c, m, Cw, flags)
            sets = literal_visible_sets(n, c, m, Cw, self_only=bool(flags))
            want = np.zeros_like(got)
            for a, vis in enumerate(sets):
                want[a, sorted(vis)] = 1
            assert np.array_equal(got, want), (n, c, m, Cw, flags)
            checked += 1
    assert checked > 500


def test_index_maps_match_literal_sequence():
    for (n, c, m) in [(8, 2, 1), (8, 4, 2), (512, 64, 8), (12, 3, 0), (30, 5, 3)]:
        seq = literal_sequence(n, c, m)
        maps = O.index_maps(n, c, m)
        assert O.aug_len(n, c, m) == len(seq)
        for a, tok in enumerate(seq):
            assert maps["aug_is_summary"][a] == (tok[0] == "s")
            assert maps["aug_chunk"][a] == (tok[1] // c if tok[0] == "t" else tok[1])
            if tok[0] == "t":
                assert maps["text_to_aug"][tok[1]] == a
                assert maps["position_ids"][a] == tok[1]
            else:
                assert maps["summary_to_aug"][tok[1] * m + tok[2]] == a
                # summary position id = its chunk's last text token's (section 2.2.1, first bullet)
                assert maps["position_ids"][a] == tok[1] * c + c - 1


def test_aug_len_and_bad_shapes():
    assert O.aug_len(10, 4, 1) == 12      # two whole chunks with a summary each, two text tokens of the third
    assert O.aug_len(8, 0, 1) == -1
    assert O.aug_len(8, 4, -1) == -1
    assert O.aug_len(0, 4, 1) == 0
    assert O.aug_len(131072, 64, 8) == 147456   # L = n + n/k with k = 8 (section 2.3)


# --------------------------------------------------------------------------------------
# Closed-form counts.  Text row (chunk j, slot r): min(j,C)*c + r + 1 text keys and
# max(0, j-C)*m summary keys.  Summary row (chunk j, ordinal u): c + u + 1.
# --------------------------------------------------------------------------------------
def closed_form_row_count(a, c, m, Cw):
    j, r = divmod(a, c + m)
    if r < c:
        return min(j, Cw) * c + r + 1 + max(0, j - Cw) * m
    return c + (r - c) + 1


def closed_form_total(n, c, m, Cw):
    J = n // c
    text = sum(min(j, Cw) * c * c + c * (c + 1) // 2 + max(0, j - Cw) * m * c for j in range(J))
    summ = J * (m * c + m * (m + 1) // 2)
    return text + summ


@pytest.mark.parametrize("shape", [(512, 64, 8, 1), (256, 16, 2, 2), (64, 8, 1, 3), (64, 8, 1, 0), (96, 8, 4, 20)])
def test_row_counts_match_closed_form(shape):
    n, c, m, Cw = shape
    M = O.mask(n, c, m, Cw)
    for a in range(M.shape[0]):
        assert int(M[a].sum()) == closed_form_row_count(a, c, m, Cw), (shape, a)
    assert int(M.sum()) == closed_form_total(n, c, m, Cw)


def test_live_element_totals_of_the_benchmark_shapes():
    # Tiny is brute-forced above via (512, 64, 8, 1); the larger ones only by closed form plus
    # sampled rows of the oracle's mask.
    assert closed_form_total(512, 64, 8, 1) == 60448
    assert closed_form_total(4096, 64, 8, 1) == 1426176
    assert closed_form_total(32768, 128, 16, 1) == 73175040
    assert closed_form_total(131072, 64, 8, 1) == 1085936128
    rng = np.random.default_rng(0)
    n, c, m, Cw = 131072, 64, 8, 1
    for a in rng.integers(0, O.aug_len(n, c, m), size=12):
        assert int(O.mask_row(int(a), n, c, m, Cw).sum()) == closed_form_row_count(int(a), c, m, Cw)


def test_mask_is_causal_and_diagonal_is_live():
    for (n, c, m, Cw) in [(64, 8, 2, 1), (48, 4, 4, 0), (40, 8, 1, 9)]:
        M = O.mask(n, c, m, Cw)
        assert np.array_equal(np.triu(M, 1), np.zeros_like(M))   # never a future position
        assert np.all(np.diag(M) == 1)                           # every token sees itself


def test_clean_partition_of_past_chunks():
    """Section 2.2.2: each past chunk is either fully in the window (all its text visible, none of
    its summaries) or fully outside (none of its text, all of its summaries)."""
    for (n, c, m, Cw) in [(64, 8, 1, 1), (64, 8, 2, 0), (96, 8, 4, 3), (64, 4, 2, 2)]:
        M = O.mask(n, c, m, Cw)
        maps = O.index_maps(n, c, m)
        J = n // c
        for i in range(n):
            aq = maps["text_to_aug"][i]
            for jk in range(i // c):
                text_cols = maps["text_to_aug"][jk * c:(jk + 1) * c]
                sum_cols = maps["summary_to_aug"][jk * m:(jk + 1) * m]
                t_all, t_any = M[aq, text_cols].all(), M[aq, text_cols].any()
                s_all, s_any = M[aq, sum_cols].all(), M[aq, sum_cols].any()
                assert (t_all and not s_any) or (s_all and not t_any), (n, c, m, Cw, i, jk)
            # nothing of a future chunk
            for jk in range(i // c + 1, J):
                assert not M[aq, jk * (c + m):(jk + 1) * (c + m)].any()


def test_special_cases_of_the_mask():
    n = 32
    tril = np.tril(np.ones((n, n), np.uint8))
    # one chunk, no summaries -> dense causal
    assert np.array_equal(O.mask(n, n, 0, 0), tril)
    # no summaries, window covering every earlier chunk -> dense causal
    assert np.array_equal(O.mask(n, 4, 0, 7), tril)
    assert np.array_equal(O.mask(n, 4, 0, 100), tril)
    # no summaries, C previous chunks (Eq. 2): key i' visible iff (i//c - C)*c <= i' <= i
    for c, Cw in itertools.product((2, 4, 8), (0, 1, 2)):
        want = np.array([[1 if max(0, i // c - Cw) * c <= ik <= i else 0 for ik in range(n)] for i in range(n)],
                        np.uint8)
        assert np.array_equal(O.mask(n, c, 0, Cw), want)


# --------------------------------------------------------------------------------------
# An incomplete last chunk (n not a multiple of c): it has text positions only.  Visibility depends on positions at
# or before the query alone, so everything about the shorter sequence must be the leading part of the same thing for
# the sequence extended to whole chunks, which the tests above pin.
# --------------------------------------------------------------------------------------
RAGGED = [(7, 2, 1, 1), (9, 4, 2, 1), (100, 64, 8, 1), (70, 64, 8, 0), (150, 20, 5, 2), (45, 8, 1, 3), (5, 8, 1, 1)]


@pytest.mark.parametrize("shape", RAGGED)
@pytest.mark.parametrize("flags", [0, 1])
def test_ragged_mask_is_the_leading_block_of_the_whole_chunk_mask(shape, flags):
    n, c, m, C = shape
    n_up = (n + c - 1) // c * c
    L = O.aug_len(n, c, m)
    assert L == (n // c) * (c + m) + n % c
    big = O.mask(n_up, c, m, C, flags)
    assert np.array_equal(O.mask(n, c, m, C, flags), big[:L, :L])
    maps, maps_up = O.index_maps(n, c, m), O.index_maps(n_up, c, m)
    for key in ("aug_chunk", "aug_is_summary", "position_ids"):
        assert np.array_equal(maps[key], maps_up[key][:L]), key
    assert np.array_equal(maps["text_to_aug"], maps_up["text_to_aug"][:n])
    assert np.array_equal(maps["summary_to_aug"], maps_up["summary_to_aug"][:(n // c) * m])
    assert not maps["aug_is_summary"][L - (n % c):].any()      # the tail is text


def test_ragged_mask_of_the_worked_example(golden_dir):
    """The first ten rows and columns of the printed-by-hand example (n = 8, c = 2, m = 1, C = 1) are the mask of
    n = 7: t6 is the only position of the last chunk."""
    (n, c, m, Cw), gold = read_golden(os.path.join(golden_dir, "mask_n8_c2_m1_C1.txt"))
    assert (n, c, m, Cw) == (8, 2, 1, 1)
    assert np.array_equal(O.mask(7, 2, 1, 1), gold[:10, :10])
