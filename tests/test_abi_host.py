"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes workspaces, and turns bad arguments into error codes."""
import ctypes
import os

import pytest

import paper_2202_02365_amd as dn


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dn.library_path()):
        from paper_2202_02365_amd.build import build
        build(verbose=False)
    return dn.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = dn.declared_symbols()
    assert {"dense_sample", "dense_gather", "sage_forward", "sage_backward"} <= set(names)
    assert len(names) >= 17
    for name in names:
        assert hasattr(lib, name), name


def _ws(lib, V, B, fanouts, direction=0):
    fan = (ctypes.c_int32 * len(fanouts))(*fanouts)
    n = ctypes.c_size_t()
    rc = lib.dn_batch_workspace_size(V, B, len(fanouts), fan, direction, ctypes.byref(n))
    return rc, n.value


def test_workspace_size_scales_with_capacity(lib):
    rc, small = _ws(lib, 16384, 256, [10, 5])
    assert rc == 0 and small > 0 and small % 256 == 0
    rc, big = _ws(lib, 1 << 20, 1000, [15, 10, 5])
    assert rc == 0 and big > small
    rc, both = _ws(lib, 1 << 20, 1000, [15, 10, 5], direction=2)
    assert rc == 0 and both > big
    # config with 111M nodes: the id->position table dominates (4 bytes per node) and it fits easily
    rc, huge = _ws(lib, 111_000_000, 1000, [15, 10, 5])
    assert rc == 0 and 4 * 111_000_000 < huge < 2 * 1024**3


@pytest.mark.parametrize("V,B,fan,direction", [(0, 10, [5], 0), (100, 0, [5], 0), (100, 10, [], 0),
                                               (100, 10, [0], 0), (100, 10, [65], 0), (100, 10, [5], 3),
                                               (100, 10, [2] * 7, 0), (1 << 31, 10, [5], 0)])
def test_bad_batch_arguments_return_einval(lib, V, B, fan, direction):
    rc, _ = _ws(lib, V, B, fan if fan else [1] * 0, direction)
    assert rc == -1
    assert len(lib.dn_last_error()) > 0


def test_null_pointers_are_rejected(lib):
    h = ctypes.c_void_p()
    assert lib.dn_graph_create(ctypes.byref(h), 100, None, None, None, None) == -1
    assert lib.dn_graph_create(None, 100, None, None, None, None) == -1
    assert lib.dense_sample(None, None, None, 0, 0, None) == -1
    assert lib.dense_gather(None, None, 0, 4, 4, None, None) == -1
    assert lib.sage_forward(None, None, None, None, None) == -1
    assert lib.sage_backward(None, None, None, None, None, None, None, None) == -1
    assert lib.dn_batch_counts(None, None, None) == -1
    n = ctypes.c_size_t()
    assert lib.dn_model_workspace_size(None, 2, None, 0, ctypes.byref(n)) == -1
    lib.dn_graph_destroy(None)
    lib.dn_batch_destroy(None)
    lib.dn_model_destroy(None)


def test_no_cpu_fallback_exists():
    """The product package must not import the oracle."""
    import paper_2202_02365_amd.binding as b
    src = open(b.__file__).read() + open(os.path.join(os.path.dirname(b.__file__), "__init__.py")).read()
    assert "oracle" not in src


def _dec_ws(lib, max_edges, chunk, num_neg, dim, max_rows, num_rel):
    n = ctypes.c_size_t()
    rc = lib.dn_decoder_workspace_size(max_edges, chunk, num_neg, dim, max_rows, num_rel, ctypes.byref(n))
    return rc, n.value


def test_decoder_workspace_size_and_bad_arguments(lib):
    rc, small = _dec_ws(lib, 1000, 100, 50, 32, 5000, 7)
    assert rc == 0 and small > 0 and small % 256 == 0
    # the link-prediction workload's shape: dominated by scores (fp32) and probabilities (two bf16 terms) per pair
    rc, full = _dec_ws(lib, 50_000, 1000, 1000, 100, 150_000, 1000)
    pairs_padded = 2 * 50 * 1024 * 1024
    assert rc == 0 and 8 * pairs_padded < full < 16 * pairs_padded
    for bad in [(0, 100, 50, 32, 5000, 7), (1000, 0, 50, 32, 5000, 7), (1000, 100, 0, 32, 5000, 7),
                (1000, 100, 50, 0, 5000, 7), (1000, 100, 50, 2000, 5000, 7), (1000, 100, 50, 32, 0, 7),
                (1000, 100, 50, 32, 5000, 0), (1 << 25, 100, 50, 32, 5000, 7)]:
        assert _dec_ws(lib, *bad)[0] == -1, bad
    assert lib.dn_decoder_workspace_size(1000, 100, 50, 32, 5000, 7, None) == -1
    h = ctypes.c_void_p()
    assert lib.dn_decoder_create(ctypes.byref(h), 1000, 100, 50, 32, 5000, 7, None, 0, None) == -1      # no workspace
    assert lib.dn_decoder_create(ctypes.byref(h), 1000, 100, 50, 32, 5000, 7, ctypes.c_void_p(8), 1 << 30, None) == -1  # misaligned


def test_new_entry_points_reject_null_and_bad_arguments(lib):
    assert lib.distmult_forward(None, None, 0, 0, None, 0, None, None, None, 0, None, None, None, None) == -1
    assert lib.distmult_backward(None, None, 0, None, 0, None) == -1
    assert lib.dn_decoder_scores(None, 0, None, None, None, None) == -1
    assert lib.dn_decoder_status(None, None, None) == -1
    assert lib.sage_forward_table(None, None, None, 0, None, None) == -1
    assert lib.dn_model_set_aggregation(None, 0) == -1
    assert lib.dn_embedding_adagrad(None, None, None, 4, 4, None, 0.1, 1e-8, None) == -1
    # the loss head validates sizes before it touches the device
    assert lib.dn_softmax_xent(None, 4, None, 3, 4, 1.0, None, None, 4, None) == -1          # null with n > 0
    assert lib.dn_softmax_xent(None, 4, None, -1, 4, 1.0, None, None, 4, None) == -1
    assert lib.dn_softmax_xent(None, 4, None, 0, 0, 1.0, None, None, 4, None) == -1          # no classes
    assert lib.dn_softmax_xent(None, 2, None, 0, 4, 1.0, None, None, 4, None) == -1          # row stride below width
    assert lib.dn_softmax_xent(None, 4, None, 0, 4, 1.0, None, None, 4, None) == 0           # empty batch: nothing to do
