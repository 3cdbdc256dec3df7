"""Pins for the oracle's Algorithm 1 (multi-hop sampling into DENSE) and repr_map (CPU only)."""
import os

import numpy as np
import pytest

import oracle
from conftest import random_small_graph, transpose_np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def deltas(d):
    off = d.node_id_offsets
    return [d.node_ids[off[j]:off[j + 1]] for j in range(len(off) - 1)]


def check_dense_invariants(d, g, targets, fanouts, direction=0):
    """Structure every valid DENSE must have, whatever the random numbers were."""
    k = len(fanouts)
    off = d.node_id_offsets
    assert len(off) == k + 2 and off[0] == 0 and off[-1] == len(d.node_ids)
    assert np.all(np.diff(off) >= 0)
    ds = deltas(d)
    assert np.array_equal(ds[k], np.asarray(targets, dtype=np.int32))        # Delta_k = targets, caller order
    assert len(np.unique(d.node_ids)) == len(d.node_ids)                     # Deltas disjoint, no duplicates
    for j in range(k):
        assert np.all(np.diff(ds[j]) > 0)                                    # ascending inside a new Delta
    n_with = len(d.node_ids) - off[1]
    assert len(d.nbr_offsets) == n_with + 1
    assert d.nbr_offsets[0] == 0 and d.nbr_offsets[-1] == len(d.nbrs)
    assert np.array_equal(d.node_ids[d.repr_map], d.nbrs)                    # definition of repr_map
    counts = np.diff(d.nbr_offsets)
    pos = {int(v): r for r, v in enumerate(d.node_ids)}
    new_nodes = [set() for _ in range(k + 1)]
    for q in range(n_with):
        p = off[1] + q
        v = int(d.node_ids[p])
        j = int(np.searchsorted(off, p, side="right") - 1)                   # owner Delta
        hop = k - j
        f = fanouts[hop]
        seg = d.nbrs[d.nbr_offsets[q]:d.nbr_offsets[q + 1]]
        adj_out = g.col_out[g.rowptr_out[v]:g.rowptr_out[v + 1]]
        if direction == 0:
            assert counts[q] == min(len(adj_out), f)
            assert set(seg.tolist()) <= set(adj_out.tolist())
            assert len(set(seg.tolist())) == len(seg)
        elif direction == 2:
            adj_in = g.col_in[g.rowptr_in[v]:g.rowptr_in[v + 1]]
            c_out = min(len(adj_out), f)
            assert counts[q] == c_out + min(len(adj_in), f)
            assert set(seg[:c_out].tolist()) <= set(adj_out.tolist())
            assert set(seg[c_out:].tolist()) <= set(adj_in.tolist())
        for u in seg:
            # a neighbour of a Delta_j node lives in Delta_{j-1} or later
            assert pos[int(u)] >= off[j - 1]
            new_nodes[j - 1].add(int(u))
    # Delta_{j-1} is exactly the set of neighbours of Delta_j not seen before
    seen = set(int(t) for t in targets)
    for j in range(k, 0, -1):
        fresh = new_nodes[j - 1] - seen
        assert fresh == set(ds[j - 1].tolist())
        seen |= fresh


def test_fig2_worked_example():
    """Section 4.1 / Figure 2 text: targets {A,B}, A's sampled neighbours {C,D};
    Delta_2={A,B}, Delta_1={C,D}, Delta_0={E}; layer-1 outputs are {C,D,A,B}."""
    facts = {}
    with open(os.path.join(GOLDEN, "fig2_worked_example.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                key, val = line.split(":")
                facts[key.strip()] = val.split()
    ids = {"A": 0, "B": 1, "C": 2, "D": 3, "E": 4}
    adj = {"A": ["C", "D"], "B": ["C"], "C": ["A", "E"], "D": ["E"], "E": []}
    assert adj["A"] == facts["sampled_neighbours_of_A"]
    rowptr, col = [0], []
    for name in "ABCDE":
        col += sorted(ids[x] for x in adj[name])
        rowptr.append(len(col))
    g = oracle.Graph(5, np.array(rowptr), np.array(col))
    targets = [ids[x] for x in facts["targets"]]
    d = oracle.dense_sample(g, targets, fanouts=[4, 4], seed=0)
    ds = deltas(d)
    assert ds[2].tolist() == [ids[x] for x in facts["delta_2"]]
    assert ds[1].tolist() == [ids[x] for x in facts["delta_1"]]
    assert ds[0].tolist() == [ids[x] for x in facts["delta_0"]]
    assert d.node_ids.tolist() == [ids[x] for x in "ECDAB"]
    assert d.node_id_offsets.tolist() == [0, 1, 3, 5]
    assert d.node_ids[d.node_id_offsets[1]:].tolist() == [ids[x] for x in facts["layer1_output_rows"]]
    # neighbours stored sequentially per node, in node_ids order: C, D, A, B
    assert d.nbrs.tolist() == [0, 4, 4, 2, 3, 2]
    assert d.nbr_offsets.tolist() == [0, 2, 3, 5, 6]
    assert d.repr_map.tolist() == [3, 0, 0, 1, 2, 1]
    # Step 2 after layer 1: E and the neighbours of {C, D} are dropped
    v2 = oracle.dense_layer_view(d, 2)
    assert v2.node_ids.tolist() == [ids[x] for x in "CDAB"]
    assert v2.nbrs.tolist() == [2, 3, 2]
    assert v2.nbr_offsets.tolist() == [0, 2, 3]
    assert v2.node_id_offsets.tolist() == [0, 2, 4]
    assert v2.node_ids[v2.repr_map].tolist() == v2.nbrs.tolist()


def bfs_levels(rowptr, col, targets, k):
    """Brute force: nodes at distance exactly h from the target set, h = 0..k."""
    seen = set(int(t) for t in targets)
    levels = [list(int(t) for t in targets)]
    for _ in range(k):
        nxt = set()
        for v in levels[-1]:
            nxt |= set(int(u) for u in col[rowptr[v]:rowptr[v + 1]])
        nxt -= seen
        seen |= nxt
        levels.append(sorted(nxt))
    return levels


@pytest.mark.parametrize("n,avg_deg,k", [(12, 1.5, 2), (40, 2.0, 3), (64, 3.0, 2), (64, 1.2, 4)])
def test_exhaustive_fanout_gives_bfs_levels(n, avg_deg, k):
    """With fanout >= max degree nothing is random: Delta_{k-h} must be the nodes at BFS
    distance exactly h, and every node's segment must be its whole adjacency list."""
    rng = np.random.default_rng(n * 100 + k)
    for trial in range(20):
        rowptr, col = random_small_graph(rng, n, avg_deg)
        g = oracle.Graph(n, rowptr, col)
        targets = rng.choice(n, size=min(n, 1 + trial % 4), replace=False).astype(np.int32)
        fan = [n] * k
        d = oracle.dense_sample(g, targets, fan, seed=trial)
        levels = bfs_levels(rowptr, col, targets, k)
        ds = deltas(d)
        for h in range(k + 1):
            assert ds[k - h].tolist() == levels[h]
        for q in range(len(d.nbr_offsets) - 1):
            v = int(d.node_ids[d.node_id_offsets[1] + q])
            assert d.nbrs[d.nbr_offsets[q]:d.nbr_offsets[q + 1]].tolist() == col[rowptr[v]:rowptr[v + 1]].tolist()
        check_dense_invariants(d, g, targets, fan)


def reference_levels_from_onehop(g, targets, fanouts, seed, direction):
    """The plain definition: level h+1 = sorted(new nodes among the one-hop samples of level h)."""
    seen = set(int(t) for t in targets)
    levels = [[int(t) for t in targets]]
    samples = {}
    for h, f in enumerate(fanouts):
        nxt = set()
        for v in levels[h]:
            samples[v] = oracle.onehop(g, v, f, seed, h, direction).tolist()
            nxt |= set(samples[v])
        nxt -= seen
        seen |= nxt
        levels.append(sorted(nxt))
    return levels, samples


@pytest.mark.parametrize("direction", [0, 2])
def test_stacking_matches_set_definition_on_rmat(rmat16k, direction):
    rp, col = rmat16k["out"]
    rpi, coli = rmat16k["in"]
    g = oracle.Graph(len(rp) - 1, rp, col, rpi, coli)
    rng = np.random.default_rng(5)
    targets = rng.choice(g.num_nodes, size=64, replace=False).astype(np.int32)
    fan = [4, 3, 2]
    d = oracle.dense_sample(g, targets, fan, seed=77, direction=direction)
    levels, samples = reference_levels_from_onehop(g, targets, fan, 77, direction)
    ds = deltas(d)
    k = len(fan)
    for h in range(k + 1):
        assert ds[k - h].tolist() == levels[h]
    for q in range(len(d.nbr_offsets) - 1):
        v = int(d.node_ids[d.node_id_offsets[1] + q])
        assert d.nbrs[d.nbr_offsets[q]:d.nbr_offsets[q + 1]].tolist() == samples[v]
    check_dense_invariants(d, g, targets, fan, direction)


def test_invariants_on_rmat_config0(rmat16k):
    rp, col = rmat16k["out"]
    g = oracle.Graph(len(rp) - 1, rp, col)
    from workloads import target_batch
    targets = target_batch(g.num_nodes, 256, 0)
    d = oracle.dense_sample(g, targets, [10, 5], seed=0)
    check_dense_invariants(d, g, targets, [10, 5])
    # same inputs -> same bytes; another seed -> another sample
    d2 = oracle.dense_sample(g, targets, [10, 5], seed=0)
    assert np.array_equal(d.nbrs, d2.nbrs) and np.array_equal(d.node_ids, d2.node_ids)
    d3 = oracle.dense_sample(g, targets, [10, 5], seed=1)
    assert not np.array_equal(d.nbrs[:200], d3.nbrs[:200]) or len(d.nbrs) != len(d3.nbrs)


def test_fanout_of_a_node_is_that_of_the_first_hop_that_needed_it():
    """Section 4.1: with sample reuse a node keeps the fanout of the first hop that required
    its neighbours.  Node 1 is first needed at hop 1 (fanout 2) although it would also be
    reached at hop 2 (fanout 1); the target is needed at hop 0 (fanout 3)."""
    #   0 -> 1,2 ; 1 -> 5,6,7 ; 2 -> 1 ; others -> nothing
    adj = {0: [1, 2], 1: [5, 6, 7], 2: [1]}
    rowptr, col = [0], []
    for v in range(8):
        col += adj.get(v, [])
        rowptr.append(len(col))
    g = oracle.Graph(8, np.array(rowptr), np.array(col))
    d = oracle.dense_sample(g, [0], [3, 2, 1], seed=4)
    counts = np.diff(d.nbr_offsets)
    owners = d.node_ids[d.node_id_offsets[1]:]
    by_node = {int(v): int(c) for v, c in zip(owners, counts)}
    assert by_node[0] == 2                            # fewer than f neighbours: all returned
    for v in by_node:
        assert owners.tolist().count(v) == 1          # sampled only once
    assert 1 in d.node_ids[d.node_id_offsets[2]:d.node_id_offsets[3]]   # first needed at hop 1
    assert by_node[1] == 2                            # hop 1's fanout, not hop 2's
    assert by_node[2] == 1


def test_bad_arguments_are_rejected(rmat16k):
    rp, col = rmat16k["out"]
    g = oracle.Graph(len(rp) - 1, rp, col)
    with pytest.raises(ValueError):
        oracle.dense_sample(g, [1, 2, 1], [3], seed=0)         # duplicate target
    with pytest.raises(ValueError):
        oracle.dense_sample(g, [g.num_nodes], [3], seed=0)     # id out of range
    with pytest.raises(ValueError):
        oracle.dense_sample(g, [1], [0], seed=0)               # fanout < 1
    with pytest.raises(ValueError):
        oracle.dense_sample(g, [1], [], seed=0)                # k < 1


def test_degenerate_batches(rmat16k):
    rp, col = rmat16k["out"]
    g = oracle.Graph(len(rp) - 1, rp, col)
    deg = np.diff(rp)
    d = oracle.dense_sample(g, [], [3, 2], seed=0)             # empty batch
    assert d.node_id_offsets.tolist() == [0, 0, 0, 0] and len(d.nbrs) == 0 and d.nbr_offsets.tolist() == [0]
    iso = np.nonzero(deg == 0)[0][:3].astype(np.int32)         # targets without neighbours
    d = oracle.dense_sample(g, iso, [3, 2], seed=0)
    assert d.node_ids.tolist() == iso.tolist() and d.node_id_offsets.tolist() == [0, 0, 0, 3]
    assert d.nbr_offsets.tolist() == [0, 0, 0, 0]


def test_gather_is_row_selection():
    rng = np.random.default_rng(0)
    table = rng.standard_normal((50, 7)).astype(np.float32)
    ids = rng.integers(0, 50, 33).astype(np.int32)
    assert np.array_equal(oracle.dense_gather(table, ids), table[ids])
    t16 = rng.integers(0, 2**16, size=(50, 6)).astype(np.uint16)   # 2-byte rows (bf16 bit patterns)
    assert np.array_equal(oracle.dense_gather(t16, ids), t16[ids])


def test_edge_front_end_targets_and_maps(rmat16k):
    """Targets of a link-prediction batch are the distinct endpoints and negatives; the returned
    indices point back at them, and the sample is the node-target sample of that list."""
    rp, col = rmat16k["out"]
    rpi, coli = rmat16k["in"]
    g = oracle.Graph(len(rp) - 1, rp, col, rpi, coli)
    rng = np.random.default_rng(8)
    e = rng.integers(0, len(col), 300)
    src = np.searchsorted(rp, e, side="right").astype(np.int32) - 1       # real edges of the graph
    dst = col[e]
    neg = rng.integers(0, g.num_nodes, 100).astype(np.int32)
    neg[:5] = src[:5]                                                    # negatives may coincide with endpoints
    d, ls, ld, ln = oracle.dense_sample_edges(g, src, dst, neg, [4], seed=2, direction=2)
    targets = d.node_ids[d.node_id_offsets[1]:]
    assert np.all(np.diff(targets) > 0)
    assert set(targets.tolist()) == set(src.tolist()) | set(dst.tolist()) | set(neg.tolist())
    assert np.array_equal(targets[ls], src) and np.array_equal(targets[ld], dst) and np.array_equal(targets[ln], neg)
    d2 = oracle.dense_sample(g, targets, [4], seed=2, direction=2)
    assert np.array_equal(d.nbrs, d2.nbrs) and np.array_equal(d.node_ids, d2.node_ids)
    check_dense_invariants(d, g, targets, [4], direction=2)


def test_embedding_sgd_touches_only_sampled_rows():
    rng = np.random.default_rng(0)
    table = rng.standard_normal((40, 6)).astype(np.float32)
    ids = np.array([7, 3, 31], dtype=np.int32)
    grad = rng.standard_normal((3, 6)).astype(np.float32)
    out = oracle.embedding_sgd(table, ids, grad, 0.25)
    untouched = np.setdiff1d(np.arange(40), ids)
    assert np.array_equal(out[untouched], table[untouched])
    np.testing.assert_allclose(out[ids], table[ids].astype(np.float64) - 0.25 * grad.astype(np.float64), rtol=0, atol=1e-6)
    assert np.array_equal(oracle.embedding_sgd(table, ids, np.zeros_like(grad), 0.25), table)


def test_openmp_build_gives_the_same_arrays(rmat16k):
    """The same source built with -fopenmp (the per-node sampling loop on all cores) must return identical arrays."""
    import os
    rp, col = rmat16k["out"]
    rpi, coli = rmat16k["in"]
    g = oracle.Graph(16384, rp, col, rpi, coli)
    rng = np.random.default_rng(8)
    os.environ.setdefault("OMP_NUM_THREADS", "4")
    for direction, fanouts in ((0, [10, 5]), (2, [6, 3]), (1, [4, 4, 4])):
        targets = rng.choice(16384, size=300, replace=False).astype(np.int32)
        a = oracle.dense_sample(g, targets, fanouts, seed=31, direction=direction)
        oracle.use_openmp(True)
        try:
            b = oracle.dense_sample(g, targets, fanouts, seed=31, direction=direction)
        finally:
            oracle.use_openmp(False)
        for name in ("node_id_offsets", "node_ids", "nbr_offsets", "nbrs", "repr_map"):
            assert np.array_equal(getattr(a, name), getattr(b, name)), name
