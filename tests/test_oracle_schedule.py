"""Pins for oracle/schedule.py: everything here is checked against the definitions of Sec. 3.1.1
(Hamiltonian, arc-disjoint), the properties proved in Sec. 3.2.2 (accessibility, zero-copy), the
placement equations of Sec. 3.2.3 and the counting facts the paper states, by brute force."""
import hashlib
import json
import os
from itertools import combinations, permutations

import pytest

from oracle import schedule as sch

NS = [8, 12, 16, 20, 24, 28, 32, 48, 64]


def arcs_of(ring):
    n = len(ring)
    return [(ring[j], ring[(j + 1) % n]) for j in range(n)]


# ---------------------------------------------------------------- Sec. 3.1.1 / 3.1.2
@pytest.mark.parametrize("n", NS)
def test_rings_are_hamiltonian_and_arc_disjoint(n):
    rings = sch.hamilton_rings(n)
    assert len(rings) == n - 1                      # n-1 cycles, Sec. 3.1.2
    seen = set()
    for ring in rings:
        assert sorted(ring) == list(range(n))       # visits every vertex exactly once
        for a in arcs_of(ring):
            assert a[0] != a[1]
            assert a not in seen                    # eq. (2): E_i and E_j disjoint
            seen.add(a)
    assert len(seen) == n * (n - 1)                 # all n(n-1) links are used
    assert sch.is_decomposition(rings)


@pytest.mark.parametrize("n", NS)
def test_removed_arcs_form_the_last_ring(n):
    """Algorithm 1: the arc taken out of each of the n-2 cycles on 0..n-2 must chain into one
    Hamiltonian path starting at vertex n-2; together with vertex n-1 it is the last ring."""
    rings = sch.hamilton_rings(n)
    last = rings[-1]
    assert last[0] == n - 2 and last[-1] == n - 1
    for i in range(n - 2):
        ring = rings[i]
        assert ring[-1] == n - 1
        # the arc closing ring i without vertex n-1 appears on the last ring
        assert (ring[n - 2], ring[0]) in arcs_of(last)


def test_zigzag_sequence_has_distinct_differences():
    for m in range(2, 66, 2):
        z = sch.zigzag_sequence(m)
        assert sorted(z) == list(range(m))
        diffs = [(z[t + 1] - z[t]) % m for t in range(m - 1)]
        assert sorted(diffs) == list(range(1, m))   # row-complete Latin square property


def test_get_path_is_row_complete_latin_square():
    m = 6
    paths = sch.get_path(m)
    for col in range(m):
        assert sorted(p[col] for p in paths) == list(range(m))
    ordered_pairs = [(p[t], p[t + 1]) for p in paths for t in range(m - 1)]
    assert len(set(ordered_pairs)) == m * (m - 1)   # every ordered pair is adjacent exactly once


def test_domain_of_algorithm_1():
    for n in (2, 3, 5, 6, 7, 9, 10, 14):
        with pytest.raises(ValueError):
            sch.hamilton_rings(n)


def test_validator_rejects_planted_mistakes():
    rings = sch.hamilton_rings(8)
    assert sch.is_decomposition(rings)
    bad = [list(r) for r in rings]
    bad[2][1], bad[2][2] = bad[2][2], bad[2][1]     # still Hamiltonian, arcs now collide
    assert not sch.is_decomposition(bad)
    bad = [list(r) for r in rings]
    bad[0][3] = bad[0][4]                           # not a permutation
    assert not sch.is_decomposition(bad)
    assert not sch.is_decomposition(rings[:-1])
    # the plain ring 0->1->...->n-1 repeated is not a decomposition either
    assert not sch.is_decomposition([list(range(8))] * 7)


def test_wrong_shift_breaks_the_decomposition(monkeypatch):
    """The shift table of Algorithm 1 matters: any other rotation of cycle 0 is caught."""
    good = sch.hamilton_rings(8)
    n = 8
    nxt = sch.hub_cycles(n - 2)[0]
    cyc0 = [n - 2]
    while nxt[cyc0[-1]] != n - 2:
        cyc0.append(nxt[cyc0[-1]])
    for wrong in (0, 2, 3):
        row0 = [cyc0[(j + wrong) % (n - 1)] for j in range(n - 1)] + [n - 1]
        assert not sch.is_decomposition([row0] + good[1:])


# ---------------------------------------------------------------- n = 4 stand-in (reading R7)
def test_k4_has_no_decomposition_and_standin_is_least_overlap():
    cycles = [[0] + list(p) for p in permutations([1, 2, 3])]
    assert len(cycles) == 6
    assert sch.count_disjoint_triples_k4() == 0
    best = None
    for t in combinations(cycles, 3):
        load = sch.arc_loads(list(t))
        key = (max(load.values()), sum(c - 1 for c in load.values()))
        best = key if best is None or key < best else best
    rings = sch.hamilton_rings(4)
    assert rings == [[0, 1, 2, 3], [0, 1, 3, 2], [0, 2, 3, 1]]
    load = sch.arc_loads(rings)
    assert (max(load.values()), sum(c - 1 for c in load.values())) == best == (2, 2)
    assert len(load) == 10                          # 12 arcs, 2 unused
    for ring in rings:
        assert sorted(ring) == [0, 1, 2, 3]


# ---------------------------------------------------------------- Algorithm 2
@pytest.mark.parametrize("n", [8, 16, 32])
def test_routing_tables(n):
    rings = sch.hamilton_rings(n)
    out_m, in_m = sch.out_mapping(rings), sch.in_mapping(rings)
    for u in range(n):
        assert out_m[u][u] == -1 and in_m[u][u] == -1
        assert sorted(out_m[u][v] for v in range(n) if v != u) == list(range(n - 1))
        assert sorted(in_m[u][v] for v in range(n) if v != u) == list(range(n - 1))
        for v in range(n):
            assert in_m[u][v] == out_m[v][u]
            if u != v:
                i = out_m[u][v]
                assert (u, v) in arcs_of(rings[i])


# ---------------------------------------------------------------- Sec. 3.2.2 / Fig. 4
@pytest.mark.parametrize("n", [4, 8, 12, 16, 32])
def test_simulation_matches_closed_form_and_properties(n):
    rings = sch.hamilton_rings(n)
    m = n - 1
    held = sch.simulate_allgather(rings)
    assert len(held) == n                                            # n compute iterations
    for rank in range(n):
        table = sch.arrival_table(rings, rank)
        assert table == [held[s][rank] for s in range(n)]
        assert table[0] == [rank] * m                                # step 0 is local
        for i in range(m):                                           # accessibility
            assert sorted(table[s][i] for s in range(n)) == list(range(n))
    for s in range(n):                                               # zero-copy: one live copy
        for i in range(m):
            assert sorted(held[s][rank][i] for rank in range(n)) == list(range(n))


def test_every_link_carries_one_subchunk_per_step():
    """Full link utilisation (Sec. 3.2.2) versus 1/(n-1) for a single ring (Sec. 1)."""
    n = 8
    rings = sch.hamilton_rings(n)
    per_step = [a for ring in rings for a in arcs_of(ring)]
    assert len(per_step) == len(set(per_step)) == n * (n - 1)
    single_ring_links = n
    assert abs(single_ring_links / (n * (n - 1)) - 1 / 7) < 1e-12    # about 14.3 %
    assert n * (n - 1) == 56                                         # 56 KV chunks for K_8 (Sec. 5.4)


def test_k_8x2_link_counts():
    """Sec. 3.1.3: in the K_{8x2} scheme each node has 7*8=56 internal links and 8*8=64 links to
    the other node, hence about 64 GB/s vs 6.3 GB/s per link; (8-K_8-8)^2 has 50 GB/s."""
    rings = sch.hamilton_rings(16)
    arcs = [a for ring in rings for a in arcs_of(ring)]
    intra0 = sum(1 for u, v in arcs if u < 8 and v < 8)
    cross01 = sum(1 for u, v in arcs if u < 8 and v >= 8)
    assert (intra0, cross01) == (56, 64)
    assert round(7200 / (intra0 * 2)) == 64
    assert abs(800 / (cross01 * 2) - 6.25) < 1e-12
    assert 800 / (8 * 2) == 50


# ---------------------------------------------------------------- Sec. 3.1.3 (m-K_m-m)^u scheme
MULTINODE = [(2, 2), (4, 2), (8, 2), (8, 3), (8, 4), (6, 5), (16, 2), (32, 2)]


@pytest.mark.parametrize("m", [2, 4, 6, 8, 10, 16, 32])
def test_node_paths_decompose_k_m(m):
    assert sch.is_path_decomposition(sch.get_path(m))
    bad = sch.get_path(m)
    bad[0] = list(reversed(bad[0]))                                  # a reversed path repeats arcs of others
    assert m == 2 or not sch.is_path_decomposition(bad)


@pytest.mark.parametrize("m,u", MULTINODE)
def test_multinode_scheme_properties(m, u):
    """Sec. 3.1.3 from the rings alone: Hamiltonian cycles, every arc inside a node used once, every
    rank's link to another node used once each way, and the AllGather properties of Sec. 3.2.2."""
    rings = sch.multinode_rings(m, u)
    n = m * u
    assert len(rings) == m and all(len(r) == n for r in rings)
    assert sch.is_multinode_scheme(rings, m, u)
    arcs = [a for ring in rings for a in arcs_of(ring)]
    assert sum(1 for a, b in arcs if a // m == b // m) == u * m * (m - 1)
    assert sum(1 for a, b in arcs if a // m != b // m) == 2 * m * u // 2   # one per rank: all NICs busy
    held = sch.simulate_allgather(rings)                             # asserts zero-copy at every hop
    for rank in range(n):
        table = sch.arrival_table(rings, rank)
        assert table == [held[s][rank] for s in range(n)]
        assert table[0] == [rank] * m
        for i in range(m):                                           # accessibility
            assert sorted(table[s][i] for s in range(n)) == list(range(n))


def test_multinode_8x2_matches_the_figures_of_the_paper():
    """(8-K_8-8)^2: 8 rings over 16 ranks; 2*8 = 16 links between the nodes, i.e. 800 GB/s of a node's
    NICs shared by 8 outgoing rings = 50 GB/s per direction each, against 64 GB/s inside a node."""
    rings = sch.multinode_rings(8, 2)
    arcs = [a for ring in rings for a in arcs_of(ring)]
    cross = [(a, b) for a, b in arcs if a // 8 != b // 8]
    assert len(rings) == 8 and len(cross) == 16
    assert sorted(a for a, _ in cross) == list(range(16))            # every rank starts or ends a path once
    intra0 = sum(1 for a, b in arcs if a < 8 and b < 8)
    assert intra0 == 56 and round(7200 / (intra0 * 2)) == 64
    assert 800 / (len(cross)) == 50
    assert abs(1 - 50 / 64.3) < 0.28 + 1e-9                          # "only a 28 % difference"


@pytest.mark.parametrize("m,u", [(8, 2), (8, 3), (4, 4)])
def test_multinode_induction_step(m, u):
    """Sec. 3.1.3: from u nodes to u+1 by cutting the links last node -> node 0 and routing them
    through the new node."""
    small, big = sch.multinode_rings(m, u), sch.multinode_rings(m, u + 1)
    for i in range(m):
        a = set(arcs_of(small[i]))
        b = set(arcs_of(big[i]))
        removed, added = a - b, b - a
        assert len(removed) == 1 and len(added) == m + 1             # one link cut, m-1 new inside the node, 2 across
        (x, y), = removed
        assert x // m == u - 1 and y // m == 0
        new_node = [v for v in big[i] if v // m == u]
        assert sorted(new_node) == list(range(u * m, (u + 1) * m))
        assert (x, new_node[0]) in added and (new_node[-1], y) in added
        assert big[i][: m * u] == small[i]


def test_multinode_domain_and_planted_mistakes():
    for m, u in [(3, 2), (8, 1), (0, 2), (7, 3)]:
        with pytest.raises(ValueError):
            sch.multinode_rings(m, u)
    rings = sch.multinode_rings(8, 2)
    assert not sch.is_multinode_scheme(sch.hamilton_rings(16)[:8], 8, 2)    # K_16 rings cross nodes freely
    swapped = [list(r) for r in rings]
    swapped[0][0], swapped[0][1] = swapped[0][1], swapped[0][0]             # repeats an arc of another ring
    assert not sch.is_multinode_scheme(swapped, 8, 2)
    same_path = [list(rings[0]) for _ in range(8)]
    assert not sch.is_multinode_scheme(same_path, 8, 2)


@pytest.mark.parametrize("m,u,S", [(8, 2, 16 * 2 * 8 * 3), (4, 2, 8 * 2 * 4 * 5 + 16), (8, 3, 48 * 7)])
@pytest.mark.parametrize("mode", [sch.FULL, sch.ZIGZAG_CAUSAL])
def test_multinode_subchunks_tile_the_sequence_once(m, u, S, mode):
    n = m * u
    if S % (2 * n):
        S = S // (2 * n) * (2 * n)
    seen = []
    for src in range(n):
        for ring in range(m):
            for a, b in sch.subchunk_ranges(n, S, mode, ring, src, n_rings=m):
                seen.extend(range(a, b))
    assert sorted(seen) == list(range(S))
    for src in range(n):                                             # the pieces of a rank are its own chunk
        own = sorted(t for ring in range(m) for a, b in sch.subchunk_ranges(n, S, mode, ring, src, n_rings=m)
                     for t in range(a, b))
        assert own == sorted(sch.local_positions(n, src, S, mode))


# ---------------------------------------------------------------- Sec. 3.2.3 placements
CASES = [(4, 24), (4, 1024), (8, 112), (8, 131072), (16, 524288), (8, 1048576), (12, 264)]


@pytest.mark.parametrize("n,S", CASES)
@pytest.mark.parametrize("mode", [sch.FULL, sch.ZIGZAG_CAUSAL])
def test_subchunks_tile_the_sequence_once(n, S, mode):
    cover = [0] * (S + 1)
    for src in range(n):
        for ring in range(n - 1):
            rs = sch.subchunk_ranges(n, S, mode, ring, src)
            assert len(rs) == (1 if mode == sch.FULL else 2)
            for a, b in rs:
                assert 0 <= a <= b <= S
                cover[a] += 1
                cover[b] -= 1
            if mode == sch.ZIGZAG_CAUSAL:
                assert rs[0][1] - rs[0][0] == rs[1][1] - rs[1][0]    # mirrored halves match
                assert rs[0][0] + rs[1][1] == S and rs[0][1] + rs[1][0] == S
    run = 0
    for t in range(S):
        run += cover[t]
        assert run == 1


@pytest.mark.parametrize("n,S", CASES)
def test_subchunks_of_a_rank_are_its_eq3_or_eq4_chunk(n, S):
    for src in range(n):
        full = sorted(t for ring in range(n - 1) for a, b in sch.subchunk_ranges(n, S, sch.FULL, ring, src)
                      for t in range(a, b)) if S <= 2048 else None
        if full is not None:
            assert full == list(range(src * S // n, (src + 1) * S // n))                  # eq. (3)
            zz = sorted(t for ring in range(n - 1)
                        for a, b in sch.subchunk_ranges(n, S, sch.ZIGZAG_CAUSAL, ring, src) for t in range(a, b))
            H = S // (2 * n)
            assert zz == list(range(src * H, (src + 1) * H)) + \
                list(range((2 * n - src - 1) * H, (2 * n - src) * H))                     # eq. (4)
            assert sorted(sch.local_positions(n, src, S, sch.ZIGZAG_CAUSAL)) == zz


def test_subchunk_sizes_of_the_five_workloads():
    def sizes(n, S, mode):
        return sorted({b - a for ring in range(n - 1) for a, b in sch.subchunk_ranges(n, S, mode, ring, 0)})
    assert sizes(4, 1024, sch.FULL) == [85, 86]
    assert sizes(8, 131072, sch.ZIGZAG_CAUSAL) == [1170, 1171]
    assert sizes(8, 262144, sch.FULL) == [4681, 4682]
    assert sizes(16, 524288, sch.ZIGZAG_CAUSAL) == [1092, 1093]
    assert sizes(8, 1048576, sch.ZIGZAG_CAUSAL) == [9362, 9363]


@pytest.mark.parametrize("n,S", [(8, 112), (8, 131072), (16, 524288)])
def test_load_balance_argument(n, S):
    """Sec. 3.2.3: for src < r every local query lies after piece [0] and before piece [1]; for
    src > r the first half of the queries lies before both pieces and the second half after both."""
    H = S // (2 * n)
    for r in range(n):
        pos = sch.local_positions(n, r, S, sch.ZIGZAG_CAUSAL)
        lo_min, lo_max, hi_min, hi_max = pos[0], pos[H - 1], pos[H], pos[-1]
        for src in range(n):
            if src == r:
                continue
            for ring in range(n - 1):
                (a0, b0), (a1, b1) = sch.subchunk_ranges(n, S, sch.ZIGZAG_CAUSAL, ring, src)
                if src < r:
                    assert b0 - 1 < lo_min and hi_max < a1
                else:
                    assert lo_max < a0 and lo_max < a1 and b0 - 1 < hi_min and b1 - 1 < hi_min


# ---------------------------------------------------------------- frozen canonical lists
def test_golden_pins(golden_dir):
    with open(os.path.join(golden_dir, "schedule_pins.json")) as f:
        pins = json.load(f)
    for n, rings in pins["rings"].items():
        assert sch.hamilton_rings(int(n)) == rings
        assert sch.out_mapping(rings) == pins["out_mapping"][n]
        assert sch.in_mapping(rings) == pins["in_mapping"][n]
    for n, h in pins["sha256"].items():
        rings = sch.hamilton_rings(int(n))
        assert hashlib.sha256(",".join(str(x) for r in rings for x in r).encode()).hexdigest() == h
    for key, table in pins["arrival"].items():
        n, rank = map(int, key.split("/"))
        assert sch.arrival_table(sch.hamilton_rings(n), rank) == table
    # a few rows spelled out, so that the file itself is anchored
    assert pins["rings"]["8"][0] == [0, 1, 5, 2, 4, 3, 6, 7]
    assert pins["rings"]["8"][6] == [6, 0, 5, 3, 4, 1, 2, 7]
    assert pins["arrival"]["8/3"][1] == [4, 0, 2, 6, 7, 1, 5]
    assert pins["arrival"]["4/0"] == [[0, 0, 0], [3, 2, 1], [2, 3, 3], [1, 1, 2]]
    assert pins["out_mapping"]["8"][0] == [-1, 0, 4, 1, 5, 6, 3, 2]
