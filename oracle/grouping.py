"""ORACLE -- test infrastructure, not product.

Grouping of query tiles that attend to similar sets of key blocks (paper Sec. 4.2 "Grouping
Query Tiles Attending to Similar Sets of Keys/Values"), in plain numpy / Python:

  * distance d(i, j) = number of key blocks selected by exactly one of the query tiles i, j;
  * objective of Eq. (1): sum over groups of the distances of the members to the group's
    representative tile;
  * the greedy heuristic the section describes: the first query tile not yet grouped becomes a
    representative and takes the R - 1 ungrouped tiles closest to it;
  * "merge-consecutive" (Sec. 5): groups of R consecutive query tiles;
  * what a group loads: the union of its members' key blocks, and for every key block of the
    union the set of members that selected it.

Readings (the paper is silent): grouping never crosses a (batch, head) slice; equal distances
are ordered by ascending tile index; a group lists its representative first and then its
members by (distance, index); if the number of tiles is not a multiple of R the last group is
short.  Results are STRICT: a member attends only to its own key blocks, the union decides
what is loaded, not what is attended.
"""
import numpy as np


def tile_bitmaps(indptr, indices, slices, QB, G):
    """Boolean [slices, QB, G]: tile (s, i) selects key block g."""
    b = np.zeros((slices, QB, G), dtype=bool)
    for w in range(slices * QB):
        s, i = divmod(w, QB)
        b[s, i, indices[indptr[w]:indptr[w + 1]]] = True
    return b


def distance(bi, bj):
    """d(i, j) of Sec. 4.2: key blocks selected by exactly one of the two tiles."""
    return int(np.count_nonzero(np.logical_xor(bi, bj)))


def group_consecutive(QB, R):
    return [list(range(g, min(g + R, QB))) for g in range(0, QB, R)]


def group_greedy_xor(bits, R):
    """Greedy grouping of one slice.  bits: bool [QB, G].  Returns groups (lists of tile ids, representative first)."""
    QB = bits.shape[0]
    free = list(range(QB))
    groups = []
    while free:
        c = free.pop(0)
        ranked = sorted(free, key=lambda j: (distance(bits[c], bits[j]), j))
        take = ranked[:R - 1]
        for j in take:
            free.remove(j)
        groups.append([c] + take)
    return groups


def objective(bits, groups):
    """Eq. (1) with the first tile of each group as its representative."""
    return sum(distance(bits[g[0]], bits[i]) for g in groups for i in g)


def union_and_membership(bits, group):
    """Key blocks any member selects (ascending) and, per such key block, a bit mask of the members that select it."""
    sel = bits[group]                                  # [len(group), G]
    ids = np.flatnonzero(sel.any(axis=0)).astype(np.int32)
    memb = np.zeros(ids.size, dtype=np.uint8)
    for t in range(len(group)):
        memb |= (sel[t, ids].astype(np.uint8) << t)
    return ids, memb


def grouped_mask(indptr, indices, slices, QB, G, R, mode):
    """Whole-problem grouping: mode "consecutive" or "xor".

    Returns (group_tiles int32 [slices*NG, R] with -1 padding, u_indptr int64, u_indices int32, u_memb uint8),
    tile ids being local to the slice.
    """
    bits = tile_bitmaps(indptr, indices, slices, QB, G)
    NG = (QB + R - 1) // R
    tiles = np.full((slices * NG, R), -1, dtype=np.int32)
    u_indptr = [0]
    u_idx, u_mem = [], []
    for s in range(slices):
        groups = group_consecutive(QB, R) if mode == "consecutive" else group_greedy_xor(bits[s], R)
        assert len(groups) == NG
        for g, members in enumerate(groups):
            tiles[s * NG + g, :len(members)] = members
            ids, memb = union_and_membership(bits[s], members)
            u_idx.append(ids)
            u_mem.append(memb)
            u_indptr.append(u_indptr[-1] + ids.size)
    return (tiles, np.asarray(u_indptr, dtype=np.int64),
            np.concatenate(u_idx).astype(np.int32) if u_idx else np.zeros(0, np.int32),
            np.concatenate(u_mem).astype(np.uint8) if u_mem else np.zeros(0, np.uint8))
