"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares, builds the
temporal CSR correctly on the host and reports errors instead of aborting.  No GPU is touched."""
import os
import re

import numpy as np
import pytest

import synth
from oracle import tgnn_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def tgnn():
    from paper_2307_07649_amd import tgnn as t
    return t


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "tgnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tgnn_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(tgnn):
    import ctypes
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2307_07649_amd", "libtgnn.so"))
    names = declared_symbols()
    assert len(names) >= 15 and "tgnn_train_step" in names and "tgnn_sample_recent" in names
    for n in names:
        assert hasattr(lib, n), f"libtgnn.so does not export {n}"
    assert set(tgnn.EXPORTS) == set(names)          # the binding covers exactly the declared ABI


def test_binding_structs_match_header_layout(tgnn):
    import ctypes as C
    assert C.sizeof(tgnn.tgnn_config) == 13 * 4
    assert C.sizeof(tgnn.tgnn_graph) == 6 * 8
    assert C.sizeof(tgnn.tgnn_state) == 6 * 8
    assert C.sizeof(tgnn.tgnn_params) == 19 * 8
    assert C.sizeof(tgnn.tgnn_batch) == 5 * 8 + 8
    assert tgnn.PARAM_NAMES == O.PARAM_NAMES == synth.graphs.PARAM_ORDER


@pytest.mark.parametrize("ties", [False, True])
def test_tcsr_matches_oracle_adjacency(tgnn, ties):
    rng = np.random.default_rng(3)
    n, E = 200, 5000
    src = rng.integers(0, n, E); dst = rng.integers(0, n, E)            # self loops allowed
    ts = np.sort(rng.integers(0, 300, E).astype(np.float64)) if ties else np.sort(rng.uniform(0, 1e6, E))
    indptr, nbr, eid, tso = tgnn.build_tcsr(src, dst, ts, n)
    a = O.build_adjacency(src, dst, ts, n)
    assert np.array_equal(indptr, a[0]) and np.array_equal(nbr, a[1]) and np.array_equal(eid, a[2])
    assert np.array_equal(tso, a[3])


def test_tcsr_on_c0_and_c1(tgnn):
    for name in ("C0", "C1"):
        g = synth.gen_graph(name, with_efeat=False)
        n = synth.CONFIGS[name]["n_nodes"]
        c = tgnn.build_tcsr(g["src"], g["dst"], g["ts"], n)
        a = O.build_adjacency(g["src"], g["dst"], g["ts"], n)
        for x, y in zip(c, a):
            assert np.array_equal(x, y)


def test_tcsr_errors(tgnn):
    with pytest.raises(tgnn.TgnnError) as e:
        tgnn.build_tcsr(np.array([0, 1]), np.array([1, 5]), np.array([1.0, 2.0]), 3)
    assert e.value.code == -4
    with pytest.raises(tgnn.TgnnError) as e:
        tgnn.build_tcsr(np.array([0, 1]), np.array([1, 2]), np.array([2.0, 1.0]), 3)
    assert e.value.code == -5
    with pytest.raises(tgnn.TgnnError) as e:
        tgnn.build_tcsr(np.array([0, 1]), np.array([1, 2]), np.array([2.0, np.nan]), 3)
    assert e.value.code == -5
    ip, nb, ei, ts = tgnn.build_tcsr(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(0), 4)
    assert ip.tolist() == [0] * 5 and len(nb) == 0


def test_create_rejects_bad_configs_without_a_device(tgnn):
    # validation happens before any HIP call, so these fail the same way with or without a GPU
    bad = [dict(d_mem=10, n_heads=3), dict(k=33), dict(n_heads=9, d_mem=18), dict(d_mem=0), dict(d_edge=-1),
           dict(dt_source=2), dict(n_nodes=0), dict(max_batch=0), dict(d_mem=512)]
    base = dict(n_nodes=10, d_mem=8, d_time=4, d_edge=2, d_static=0, n_heads=2, k=3, max_batch=4)
    for b in bad:
        cfg = dict(base); cfg.update(b)
        with pytest.raises(tgnn.TgnnError) as e:
            tgnn.Context(**cfg)
        assert e.value.code in (-1, -4, -6), (b, e.value)
        assert len(str(e.value)) > 20


def test_generators_are_seeded_and_shaped_like_the_configs():
    g1 = synth.gen_graph("C1"); g2 = synth.gen_graph("C1")
    assert all(np.array_equal(g1[k], g2[k]) for k in g1)
    assert g1["efeat"].shape == (157474, 172) and g1["efeat"].dtype == np.float32
    assert g1["src"].max() < 8227 and g1["dst"].min() >= 8227 and g1["dst"].max() < 9227
    assert np.all(np.diff(g1["ts"]) >= 0) and g1["ts"][-1] <= 2.7e6
    g0 = synth.gen_graph("C0")
    d = np.diff(g0["ts"])
    assert g0["ts"][0] == 0 and d.min() >= 1 and d.max() <= 5 and np.all(g0["src"] != g0["dst"])
    neg = synth.gen_negatives("C2", 1000)
    assert neg.min() >= 10000 and neg.max() < 10984
    st = synth.gen_static("C2")
    assert st.shape == (10984, 100) and abs(float(st.std()) - 0.1) < 0.01
    assert synth.gen_static("C1") is None
    g4 = synth.gen_graph("C4", n_events=50_000)
    assert np.all(g4["src"] != g4["dst"]) and abs(g4["ts"][-1] - 1.4e5) < 1e-6 and g4["efeat"].shape[1] == 186


def test_create_rejects_bad_head_and_negative_set_counts(tgnn):
    """n_classes and max_neg_sets are validated before anything touches a device."""
    import ctypes as C
    for field, bad in (("n_classes", -1), ("n_classes", 257), ("max_neg_sets", 65), ("max_neg_sets", -1)):
        kw = dict(n_nodes=10, d_mem=8, d_time=4, d_edge=2, d_static=0, n_heads=2, k=3, max_batch=4, n_replicas=1,
                  dt_source=0, flags=0, max_neg_sets=1, n_classes=0)
        kw[field] = bad
        cfg = tgnn.tgnn_config(*[kw[n] for n, _ in tgnn.tgnn_config._fields_])
        h = C.c_void_p()
        rc = tgnn._lib.tgnn_create(C.byref(cfg), C.byref(h))
        assert rc == -4 and not h.value, (field, bad, rc)          # TGNN_E_OUT_OF_RANGE
        assert field in tgnn._lib.tgnn_last_error().decode()
