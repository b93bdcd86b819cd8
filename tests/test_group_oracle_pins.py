"""Pins for the query-tile grouping oracle (paper Sec. 4.2): definitions written a second time, brute force over
all groupings on tiny masks, and structured masks whose best grouping is known."""
import itertools

import numpy as np
import pytest

from oracle import grouping as GR


def rand_bits(rng, QB, G, density=0.4):
    return rng.random((QB, G)) < density


def csr_of(bits3):
    S, QB, G = bits3.shape
    indptr, idx = [0], []
    for s in range(S):
        for i in range(QB):
            ids = np.flatnonzero(bits3[s, i]).astype(np.int32)
            idx.append(ids)
            indptr.append(indptr[-1] + ids.size)
    return np.asarray(indptr, np.int64), np.concatenate(idx) if idx else np.zeros(0, np.int32)


def test_distance_is_the_symmetric_difference():
    rng = np.random.default_rng(0)
    b = rand_bits(rng, 6, 37)
    for i in range(6):
        assert GR.distance(b[i], b[i]) == 0
        for j in range(6):
            A, B = set(np.flatnonzero(b[i])), set(np.flatnonzero(b[j]))
            assert GR.distance(b[i], b[j]) == len(A ^ B) == len(A) + len(B) - 2 * len(A & B) == GR.distance(b[j], b[i])


def greedy_by_hand(bits, R):
    """The heuristic of Sec. 4.2 once more, with explicit loops and sets."""
    QB, G = bits.shape
    sets = [set(int(x) for x in np.flatnonzero(bits[i])) for i in range(QB)]
    ungrouped = list(range(QB))
    out = []
    while ungrouped:
        c = ungrouped[0]
        ungrouped = ungrouped[1:]
        group = [c]
        for _ in range(R - 1):
            if not ungrouped:
                break
            best = None
            for j in ungrouped:
                dj = len(sets[c] ^ sets[j])
                if best is None or dj < best[0]:
                    best = (dj, j)          # ascending j: the first minimum wins ties
            group.append(best[1])
            ungrouped.remove(best[1])
        out.append(group)
    return out


@pytest.mark.parametrize("QB,G,R", [(8, 20, 4), (9, 33, 2), (12, 16, 4), (7, 10, 8), (16, 64, 8)])
def test_greedy_matches_second_implementation(QB, G, R):
    rng = np.random.default_rng(QB * 7 + R)
    b = rand_bits(rng, QB, G)
    assert GR.group_greedy_xor(b, R) == greedy_by_hand(b, R)


def all_groupings(QB, R):
    """Every partition of range(QB) into groups of R (QB a multiple of R), every choice of representative."""
    def parts(items):
        if not items:
            yield []
            return
        first, rest = items[0], items[1:]
        for others in itertools.combinations(rest, R - 1):
            left = [x for x in rest if x not in others]
            for p in parts(left):
                yield [[first] + list(others)] + p
    for p in parts(list(range(QB))):
        for reps in itertools.product(*[range(R)] * len(p)):
            yield [[g[r]] + [x for t, x in enumerate(g) if t != r] for g, r in zip(p, reps)]


@pytest.mark.parametrize("QB,R", [(4, 2), (6, 2), (6, 3), (8, 4)])
def test_objective_against_brute_force(QB, R):
    rng = np.random.default_rng(QB + R)
    b = rand_bits(rng, QB, 12)
    best = min(sum(len(set(np.flatnonzero(b[g[0]])) ^ set(np.flatnonzero(b[i]))) for g in gr for i in g)
               for gr in all_groupings(QB, R))
    greedy = GR.group_greedy_xor(b, R)
    assert sorted(x for g in greedy for x in g) == list(range(QB)) and all(len(g) == R for g in greedy)
    assert GR.objective(b, greedy) >= best                      # a heuristic: never below the optimum ...
    cons = GR.group_consecutive(QB, R)
    assert GR.objective(b, cons) >= best


def test_structured_mask_is_grouped_perfectly():
    # tile i repeats pattern i mod 3: the greedy grouping with R = 4 puts equal patterns together (objective 0),
    # consecutive grouping mixes the three patterns
    rng = np.random.default_rng(3)
    pats = rand_bits(rng, 3, 48, 0.3)
    b = np.stack([pats[i % 3] for i in range(12)])
    g = GR.group_greedy_xor(b, 4)
    assert g == [[0, 3, 6, 9], [1, 4, 7, 10], [2, 5, 8, 11]] and GR.objective(b, g) == 0
    assert GR.objective(b, GR.group_consecutive(12, 4)) > 0
    for members in g:
        ids, memb = GR.union_and_membership(b, members)
        assert np.array_equal(ids, np.flatnonzero(b[members[0]])) and np.all(memb == 0b1111)


def test_union_and_membership_and_csr_form():
    rng = np.random.default_rng(4)
    S, QB, G, R = 2, 10, 21, 4
    b3 = rng.random((S, QB, G)) < 0.3
    indptr, indices = csr_of(b3)
    assert np.array_equal(GR.tile_bitmaps(indptr, indices, S, QB, G), b3)
    for mode in ("consecutive", "xor"):
        tiles, up, ui, um = GR.grouped_mask(indptr, indices, S, QB, G, R, mode)
        NG = 3
        assert tiles.shape == (S * NG, R) and up.size == S * NG + 1 and up[-1] == ui.size == um.size
        for s in range(S):
            seen = []
            for g in range(NG):
                row = tiles[s * NG + g]
                members = [int(x) for x in row if x >= 0]
                assert list(row[:len(members)]) == members and len(members) == (R if g < NG - 1 else QB - R * (NG - 1))
                seen += members
                ids = ui[up[s * NG + g]:up[s * NG + g + 1]]
                memb = um[up[s * NG + g]:up[s * NG + g + 1]]
                assert np.all(np.diff(ids) > 0) and np.all(memb > 0)
                assert set(ids.tolist()) == set(np.flatnonzero(b3[s, members].any(axis=0)).tolist())
                for t, m in enumerate(members):
                    assert np.array_equal(ids[(memb >> t) & 1 == 1], np.flatnonzero(b3[s, m]))
                assert np.all(memb >> len(members) == 0)
            assert sorted(seen) == list(range(QB))
        if mode == "consecutive":
            assert np.array_equal(tiles[:NG].ravel()[:QB], np.arange(QB))


def objective_by_sets(sets, groups):
    """Eq. (1) once more from its definition: for every group, the key blocks selected by exactly one of
    (representative, member), counted over the group's members (the representative is the group's first tile)."""
    total = 0
    for g in groups:
        rep = sets[g[0]]
        for i in g:
            total += sum(1 for x in rep | sets[i] if (x in rep) != (x in sets[i]))
    return total


@pytest.mark.parametrize("QB,G,R,seed", [(8, 20, 4, 0), (12, 33, 3, 1), (16, 64, 8, 2), (9, 17, 2, 3), (10, 25, 4, 4)])
def test_objective_equals_the_definition_on_arbitrary_groupings(QB, G, R, seed):
    # random groupings with a random tile (mostly not the lowest-numbered, not the first in index order) as
    # representative, groups of uneven size included: the value must EQUAL the set-based sum, not just bound it
    rng = np.random.default_rng(100 + seed)
    b = rand_bits(rng, QB, G)
    sets = [set(int(x) for x in np.flatnonzero(b[i])) for i in range(QB)]
    for _ in range(20):
        perm = [int(x) for x in rng.permutation(QB)]
        groups = [perm[s:s + R] for s in range(0, QB, R)]
        assert GR.objective(b, groups) == objective_by_sets(sets, groups)
    # hand-checkable case: rows {0,1}, {1,2}, {5}; group [2,0,1] with tile 2 as representative:
    # d(2,2) + d(2,0) + d(2,1) = 0 + 3 + 3; with tile 0 as representative: 0 + 2 + 3
    hb = np.zeros((3, 6), dtype=bool)
    hb[0, [0, 1]] = True
    hb[1, [1, 2]] = True
    hb[2, 5] = True
    assert GR.objective(hb, [[2, 0, 1]]) == 6
    assert GR.objective(hb, [[0, 1, 2]]) == 5
    assert GR.objective(hb, [[0, 1], [2]]) == 2
    assert GR.objective(hb, [[1], [2, 0]]) == 3


def test_objective_pin_catches_planted_mistakes():
    # the pins above must tell the definition from near misses: last tile as representative, pairs counted
    # twice, union instead of symmetric difference, distance to the previous member instead of the representative
    rng = np.random.default_rng(7)
    b = rand_bits(rng, 12, 30)
    sets = [set(int(x) for x in np.flatnonzero(b[i])) for i in range(12)]
    wrong = {
        "last tile as representative": lambda bits, groups: sum(GR.distance(bits[g[-1]], bits[i]) for g in groups for i in g),
        "every pair counted": lambda bits, groups: sum(GR.distance(bits[j], bits[i]) for g in groups for j in g for i in g),
        "union instead of xor": lambda bits, groups: sum(int(np.count_nonzero(bits[g[0]] | bits[i])) for g in groups for i in g),
        "chain of neighbours": lambda bits, groups: sum(GR.distance(bits[g[max(t - 1, 0)]], bits[g[t]])
                                                         for g in groups for t in range(len(g))),
    }
    for name, fn in wrong.items():
        caught = False
        for trial in range(20):
            perm = [int(x) for x in rng.permutation(12)]
            groups = [perm[s:s + 4] for s in range(0, 12, 4)]
            if fn(b, groups) != objective_by_sets(sets, groups):
                caught = True
                break
        assert caught, name
