"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host only): the worked example of Section 4.1
(Figure 2's text), R-MAT multi-hop samples in every direction, and the degenerate inputs, run in a subprocess built with
-fsanitize=address,undefined; any finding aborts the run.  The sanitized build's arrays must equal the plain build's."""
import os
import struct
import subprocess

import numpy as np
import pytest

import oracle
from conftest import cached_rmat

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.fixture(scope="module")
def sanitized(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-Wall", "-Wextra", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", os.path.join(HERE, "native", "oracle_sanitize_main.c"),
           os.path.join(ROOT, "oracle", "dense_oracle.c"), "-o", exe]
    subprocess.check_call(cmd)
    return exe


def run_sanitized(exe, tmp_path, g, targets, fanouts, seed, direction):
    targets = np.ascontiguousarray(targets, dtype=np.int32)
    fan = np.ascontiguousarray(fanouts, dtype=np.int32)
    has_in = g.rowptr_in is not None
    inp, outp = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(inp, "wb") as f:
        f.write(struct.pack("<7q", g.num_nodes, len(g.col_out), len(g.col_in) if has_in else -1, len(targets), len(fan),
                            direction, seed))
        f.write(g.rowptr_out.tobytes())
        f.write(g.col_out.tobytes())
        if has_in:
            f.write(g.rowptr_in.tobytes())
            f.write(g.col_in.tobytes())
        f.write(targets.tobytes())
        f.write(fan.tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([exe, inp, outp], env=env, capture_output=True, text=True, timeout=300)
    assert p.returncode == 0, "sanitizer run failed (rc %d):\n%s" % (p.returncode, p.stderr[-4000:])
    raw = open(outp, "rb").read()
    rc, n, e = struct.unpack_from("<3q", raw, 0)
    if rc != 0:
        return rc, None
    pos = 24
    k = len(fan)

    def take(dtype, count):
        nonlocal pos
        a = np.frombuffer(raw, dtype=dtype, count=count, offset=pos)
        pos += a.nbytes
        return a

    node_id_offsets = take(np.int64, k + 2)
    node_ids = take(np.int32, n)
    nbr_offsets = take(np.int64, n - int(node_id_offsets[1]) + 1)
    nbrs = take(np.int32, e)
    repr_map = take(np.int32, e)
    h0 = take(np.int32, 3 * n).reshape(n, 3)
    assert pos == len(raw)
    return 0, dict(node_id_offsets=node_id_offsets, node_ids=node_ids, nbr_offsets=nbr_offsets, nbrs=nbrs,
                   repr_map=repr_map, h0=h0)


def assert_same(res, d):
    for name in ("node_id_offsets", "node_ids", "nbr_offsets", "nbrs", "repr_map"):
        assert np.array_equal(res[name].astype(np.int64), np.asarray(getattr(d, name), dtype=np.int64)), name
    ids = res["node_ids"].astype(np.int64)
    assert np.array_equal(res["h0"], np.stack([ids, 2 * ids, 3 * ids], axis=1))


def test_worked_example_of_section_4_1_under_sanitizers(sanitized, tmp_path):
    # A=0 B=1 C=2 D=3 E=4; A -> C, D; B -> A; C -> E; D -> A (a graph consistent with the text around Figure 2)
    rowptr = np.array([0, 2, 3, 4, 5, 5], dtype=np.int64)
    col = np.array([2, 3, 0, 4, 0], dtype=np.int32)
    g = oracle.Graph(5, rowptr, col)
    rc, res = run_sanitized(sanitized, tmp_path, g, [0, 1], [4, 4], seed=1, direction=0)
    assert rc == 0
    assert res["node_ids"].tolist() == [4, 2, 3, 0, 1]                  # E | C D | A B
    assert res["node_id_offsets"].tolist() == [0, 1, 3, 5]
    assert_same(res, oracle.dense_sample(g, [0, 1], [4, 4], seed=1))


@pytest.mark.parametrize("direction,fanouts,n_targets", [(0, [10, 5], 256), (1, [3, 3, 3], 64), (2, [20], 300), (0, [1, 1, 1, 1], 7),
                                                         (2, [64, 2], 5)])
def test_rmat_samples_under_sanitizers(sanitized, tmp_path, direction, fanouts, n_targets):
    ent = cached_rmat(16384, 262144, 1, with_in=True)
    g = oracle.Graph(16384, ent["out"][0], ent["out"][1], ent["in"][0], ent["in"][1])
    rng = np.random.default_rng(n_targets)
    targets = rng.choice(16384, size=n_targets, replace=False).astype(np.int32)
    rc, res = run_sanitized(sanitized, tmp_path, g, targets, fanouts, seed=123456789012345, direction=direction)
    assert rc == 0
    assert_same(res, oracle.dense_sample(g, targets, fanouts, seed=123456789012345, direction=direction))


def test_degenerate_inputs_under_sanitizers(sanitized, tmp_path):
    ent = cached_rmat(16384, 262144, 1, with_in=True)
    g = oracle.Graph(16384, ent["out"][0], ent["out"][1])
    deg = np.diff(ent["out"][0])
    iso = np.nonzero(deg == 0)[0][:5].astype(np.int32)
    rc, res = run_sanitized(sanitized, tmp_path, g, iso, [4, 2], seed=0, direction=0)       # no neighbour anywhere
    assert rc == 0 and len(res["nbrs"]) == 0
    assert_same(res, oracle.dense_sample(g, iso, [4, 2], seed=0))
    rc, res = run_sanitized(sanitized, tmp_path, g, np.zeros(0, dtype=np.int32), [3], seed=0, direction=0)   # empty batch
    assert rc == 0 and len(res["node_ids"]) == 0
    hub = np.array([int(np.argmax(deg))], dtype=np.int32)
    rc, res = run_sanitized(sanitized, tmp_path, g, hub, [64, 64], seed=9, direction=0)      # the largest fanout
    assert rc == 0
    assert_same(res, oracle.dense_sample(g, hub, [64, 64], seed=9))
    # invalid inputs are refused, not read out of bounds: duplicate target, id out of range
    assert run_sanitized(sanitized, tmp_path, g, [5, 5], [2], seed=0, direction=0)[0] == -1
    assert run_sanitized(sanitized, tmp_path, g, [16384], [2], seed=0, direction=0)[0] == -1
    assert run_sanitized(sanitized, tmp_path, g, [-1], [2], seed=0, direction=0)[0] == -1
