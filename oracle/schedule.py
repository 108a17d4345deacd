"""Oracle: TASP schedules as plain integer lists (test infrastructure).

What is written here
--------------------
* ``hamilton_rings(n)``      -- the K_n-decomposition of Sec. 3.1.2, Algorithm 1: the complete
                               directed graph on n ranks split into n-1 directed Hamiltonian cycles
                               ("orthogonal ring datapaths", Sec. 3.1.1, eq. (2)).
* ``multinode_rings(m, u)``  -- the (m-K_m-m)^u-decomposition of Sec. 3.1.3: u nodes of m ranks, each K_m
                               cut into m Hamiltonian paths that are chained through the nodes.
* ``routing_table``          -- Algorithm 2 (in / out mapping).
* ``simulate_allgather``     -- the Multi-Ring AllGather of Sec. 3.2.2 / Fig. 4 played hop by hop.
* ``arrival_table``          -- the same thing in closed form for one rank.
* ``subchunk_ranges``        -- the chunk placements of Sec. 3.2.3: eq. (3) (contiguous), eq. (4)
                               (zig-zag halves) and eq. (5), (6) (zig-zag TASP sub-chunks).
* validators                 -- brute-force checks of the definitions (Hamiltonian, arc-disjoint,
                               accessibility, zero-copy), independent of how the rings were built.

Readings taken where the paper leaves a gap (each is pinned by tests/test_oracle_schedule.py):
  R1  Algorithm 1 names GetPath and GenCycles without bodies.  GetPath(m) is read as the m cyclic
      translates of the zig-zag sequence 0,1,m-1,2,m-2,... on Z_m (the row-complete Latin square the
      multi-node paragraph of Sec. 3.1.3 refers to); GenCycles puts the one new vertex in front of a path.
  R2  Data moves list-forward along a ring; out_mapping is Algorithm 2 with d=+1, in_mapping d=-1.
  R3  Sub-chunk index i travels on ring i (t[i,j] of Fig. 4).
  R4  Step 0 is the local sub-chunks; the sub-chunk seen at step s started s hops upstream.
  R5  Sub-chunk bounds use floors: piece i of a length-len block is [i*len//m, (i+1)*len//m).
  R6  Eq. (5), (6) are read with the index (n-1)*j+i (piece i of half-chunk j) and its mirror
      image; the printed index 2nj+i does not tile the sequence.
  R8  Sec. 3.1.3 gives the multi-node scheme in words only.  It is read as: the paths of a node are
      GetPath(m) (the same row-complete Latin square, m even) on that node's ranks c*m .. c*m+m-1;
      ring i is path i of node 0, then path i of node 1, ... and closes from the last node back to
      node 0 (the induction of Sec. 3.1.3 inserts node u between node u-1 and node 0).  There are m
      rings, so a chunk is cut in m sub-chunks instead of n-1.
  R7  n=4 admits no decomposition (Algorithm 1 requires n>=8); three Hamiltonian rings with the
      least possible arc overlap are used instead, the lexicographically smallest such triple.
"""
from itertools import combinations, permutations

FULL = 0           # bi-directional attention, contiguous placement, eq. (3)
ZIGZAG_CAUSAL = 1  # causal attention, zig-zag placement, eq. (4)-(6)


# ----------------------------------------------------------------------------------------------
# Sec. 3.1.2, Algorithm 1
# ----------------------------------------------------------------------------------------------
def zigzag_sequence(m):
    """0, 1, m-1, 2, m-2, ..., m/2: consecutive differences are all distinct mod m (m even)."""
    z = [0]
    for t in range(1, m):
        z.append((t + 1) // 2 if t % 2 == 1 else m - t // 2)
    return z


def get_path(m):
    """GetPath(m) of Algorithm 1 (reading R1): m Hamiltonian paths on Z_m."""
    z = zigzag_sequence(m)
    return [[(i + zt) % m for zt in z] for i in range(m)]


def hub_cycles(m):
    """GenCycles of Algorithm 1 (reading R1): the m paths of GetPath(m), each closed through one extra
    vertex m ("hub").  Returned as successor maps {vertex: next vertex}; together they use every arc
    of the complete directed graph on the m+1 vertices once."""
    cycles = []
    for path in get_path(m):
        nxt = {a: b for a, b in zip(path, path[1:])}
        nxt[m] = path[0]
        nxt[path[-1]] = m
        cycles.append(nxt)
    return cycles


def diverted_arc_head(n, i):
    """Which arc of hub cycle i is taken out and led through rank n-1 instead: the head of that arc,
    given as the number of hops from the hub along the cycle.  The four special cycles and the common
    distance are the shift table of Algorithm 1 (k = n/4 - 1); they are the paper's data."""
    k = n // 4 - 1
    special = {0: 1, k + 1: 4 * k + 2, 2 * k + 2: 3, 3 * k + 2: 4 * k}
    return special.get(i, 2 * k)


def _listed_from(nxt, start):
    ring, v = [], start
    while True:
        ring.append(v)
        v = nxt[v]
        if v == start:
            return ring


def hamilton_rings(n):
    """K_n-decomposition: n-1 rings, each a list of the n ranks; ring[j] sends to ring[(j+1)%n].

    Built on successor maps.  The n-2 hub cycles on ranks 0..n-2 (hub = rank n-2) are each opened at
    one arc a -> b, which becomes a -> n-1 -> b.  The arcs taken out are chosen (by the shift table)
    so that they chain into a single path from the hub through all ranks 0..n-2; that path, closed
    through rank n-1, is the last ring.  Every ring is listed starting at the rank that follows rank
    n-1, so rank n-1 stands last.
    """
    if n == 4:
        return _least_overlap_rings_k4()
    if n < 8 or n % 4 != 0:
        raise ValueError("Algorithm 1 is defined for n >= 8 with n % 4 == 0 (and the n = 4 stand-in)")
    hub, new = n - 2, n - 1
    rings, taken_out = [], {}
    for i, nxt in enumerate(hub_cycles(n - 2)):
        head = hub
        for _ in range(diverted_arc_head(n, i)):
            head = nxt[head]
        tail = next(a for a, b in nxt.items() if b == head)
        assert tail not in taken_out
        taken_out[tail] = head
        nxt = dict(nxt)
        nxt[tail], nxt[new] = new, head
        rings.append(_listed_from(nxt, head))
    # the arcs taken out leave exactly one rank of 0..n-2 without a successor: it sends to rank n-1
    loose = [v for v in range(n - 1) if v not in taken_out]
    assert len(loose) == 1 and hub not in taken_out.values()
    last = dict(taken_out)
    last[loose[0]], last[new] = new, hub
    rings.append(_listed_from(last, hub))
    return rings


def _least_overlap_rings_k4():
    """Reading R7: K_4 has 6 directed Hamiltonian cycles and no 3 of them are arc-disjoint."""
    cycles = [[0] + list(p) for p in permutations([1, 2, 3])]
    best = None
    for triple in combinations(cycles, 3):
        load = {}
        for ring in triple:
            for j in range(4):
                a = (ring[j], ring[(j + 1) % 4])
                load[a] = load.get(a, 0) + 1
        key = (max(load.values()), sum(c - 1 for c in load.values()), [list(r) for r in triple])
        if best is None or key < best:
            best = key
    return best[2]


# ----------------------------------------------------------------------------------------------
# Sec. 3.1.3: (m-K_m-m)^u-decomposition
# ----------------------------------------------------------------------------------------------
def multinode_rings(m, u):
    """m rings over the m*u ranks of u nodes (reading R8).  Inside a node a ring follows one of the
    m Hamiltonian paths of K_m; the last rank of the path sends to the first rank of the same path
    in the next node, so every rank uses its link to another node once for sending and once for
    receiving."""
    if m < 2 or m % 2 or u < 2:
        raise ValueError("m even and >= 2, u >= 2")
    paths = get_path(m)
    return [[c * m + v for c in range(u) for v in paths[i]] for i in range(m)]


# ----------------------------------------------------------------------------------------------
# Algorithm 2
# ----------------------------------------------------------------------------------------------
def ring_of_arc(rings):
    """{(sender, receiver): ring id} over every arc of every ring.  When an arc lies on two rings
    (possible only for the n=4 stand-in, reading R7) the lower ring id is kept."""
    owner = {}
    for i, ring in enumerate(rings):
        for a, b in zip(ring, ring[1:] + ring[:1]):
            owner.setdefault((a, b), i)
    return owner


def routing_table(rings, d):
    """Algorithm 2 as a lookup: table[u][v] = the ring on which v follows u (d=+1: u sends to v) or
    precedes u (d=-1: u receives from v); -1 where the two are not neighbours on any ring."""
    n = len(rings[0])
    owner = ring_of_arc(rings)
    if d == +1:
        return [[owner.get((u, v), -1) for v in range(n)] for u in range(n)]
    return [[owner.get((v, u), -1) for v in range(n)] for u in range(n)]


def out_mapping(looping):
    return routing_table(looping, +1)


def in_mapping(looping):
    return routing_table(looping, -1)


# ----------------------------------------------------------------------------------------------
# Sec. 3.2.2 / Fig. 4: Multi-Ring AllGather
# ----------------------------------------------------------------------------------------------
def simulate_allgather(looping):
    """Play the primitive: held[s][rank][i] = source rank of the sub-chunk that `rank` holds on
    ring i at step s.  Also checks, at every hop, that no buffer slot receives two sub-chunks."""
    n = len(looping[0])
    m = len(looping)
    cur = [[rank for _ in range(m)] for rank in range(n)]     # t[i, j] starts at rank j
    held = [cur]
    for _ in range(n - 1):
        nxt = [[None] * m for _ in range(n)]
        for i, ring in enumerate(looping):
            for j in range(n):
                u, v = ring[j], ring[(j + 1) % n]
                assert nxt[v][i] is None, "two sub-chunks landed in one buffer slot"
                nxt[v][i] = cur[u][i]
        cur = nxt
        held.append(cur)
    return held


def arrival_table(looping, rank):
    """arrival[s][i] = source rank of the sub-chunk seen on ring i at step s (readings R3, R4)."""
    n = len(looping[0])
    table = []
    for s in range(n):
        row = []
        for ring in looping:
            pos = ring.index(rank)
            row.append(ring[(pos - s) % n])
        table.append(row)
    return table


# ----------------------------------------------------------------------------------------------
# Sec. 3.2.3: chunk placement
# ----------------------------------------------------------------------------------------------
def piece(i, length, m):
    """Reading R5."""
    return (i * length) // m, ((i + 1) * length) // m


def subchunk_ranges(n, S, mask_mode, ring, src, n_rings=None):
    """Global token ranges [start, end) of sub-chunk t[ring, src]; one range for FULL (eq. (3) cut
    in n-1 pieces), two for ZIGZAG_CAUSAL (eq. (5) and its mirror image eq. (6)).  With a ring table
    of another size (reading R8) a chunk is cut in n_rings pieces."""
    m = n - 1 if n_rings is None else n_rings
    if mask_mode == FULL:
        if S % n:
            raise ValueError("S must be a multiple of n")
        L = S // n
        a, b = piece(ring, L, m)
        return [(src * L + a, src * L + b)]
    if S % (2 * n):
        raise ValueError("S must be a multiple of 2n")
    H = S // (2 * n)
    a, b = piece(ring, H, m)
    return [(src * H + a, src * H + b), (S - src * H - b, S - src * H - a)]


def local_positions(n, rank, S, mask_mode):
    """Global position of every local query row (eq. (3) or eq. (4))."""
    if mask_mode == FULL:
        L = S // n
        return list(range(rank * L, (rank + 1) * L))
    H = S // (2 * n)
    return list(range(rank * H, (rank + 1) * H)) + list(range(S - (rank + 1) * H, S - rank * H))


# ----------------------------------------------------------------------------------------------
# Brute-force validators (they know nothing about how the rings were made)
# ----------------------------------------------------------------------------------------------
def is_hamiltonian_cycle(ring, n):
    return len(ring) == n and sorted(ring) == list(range(n))


def arc_loads(looping):
    n = len(looping[0])
    load = {}
    for ring in looping:
        for j in range(n):
            a = (ring[j], ring[(j + 1) % n])
            load[a] = load.get(a, 0) + 1
    return load


def is_path_decomposition(paths):
    """m Hamiltonian paths on m vertices in which every ordered pair of distinct vertices is adjacent
    exactly once (all arcs of K_m), and every vertex stands once in every position."""
    m = len(paths)
    if not all(sorted(p) == list(range(m)) for p in paths):
        return False
    arcs = [(p[j], p[j + 1]) for p in paths for j in range(m - 1)]
    if len(set(arcs)) != m * (m - 1):
        return False
    return all(sorted(p[j] for p in paths) == list(range(m)) for j in range(m))


def is_multinode_scheme(looping, m, u):
    """What Sec. 3.1.3 asks of the (m-K_m-m)^u scheme, checked from the rings alone: m Hamiltonian
    cycles on m*u ranks; inside every node each of the m(m-1) arcs is used exactly once; every rank
    sends to another node exactly once and receives from another node exactly once; a ring leaves a
    node only for the next one."""
    n = m * u
    if len(looping) != m or not all(is_hamiltonian_cycle(r, n) for r in looping):
        return False
    load = arc_loads(looping)
    if max(load.values()) != 1:
        return False
    intra = [(a, b) for (a, b) in load if a // m == b // m]
    inter = [(a, b) for (a, b) in load if a // m != b // m]
    if len(intra) != u * m * (m - 1) or len(inter) != n:
        return False
    if sorted(a for a, _ in inter) != list(range(n)) or sorted(b for _, b in inter) != list(range(n)):
        return False
    return all(b // m == (a // m + 1) % u for a, b in inter)


def is_decomposition(looping):
    """n-1 Hamiltonian cycles that use each of the n(n-1) arcs of K_n exactly once."""
    n = len(looping[0])
    if len(looping) != n - 1 or not all(is_hamiltonian_cycle(r, n) for r in looping):
        return False
    load = arc_loads(looping)
    return len(load) == n * (n - 1) and max(load.values()) == 1 and all(u != v for u, v in load)


def count_disjoint_triples_k4():
    """How many triples of directed Hamiltonian cycles of K_4 are arc-disjoint (the answer is 0)."""
    cycles = [[0] + list(p) for p in permutations([1, 2, 3])]
    return sum(1 for t in combinations(cycles, 3) if max(arc_loads(list(t)).values()) == 1)
