"""The seeded input generator: shapes, layout and determinism of the five
benchmark configurations (host logic only)."""
import numpy as np

from paper_2502_00425_amd import workloads as wl


def test_config_shapes_and_spans():
    c0 = wl.workload(0)
    assert (c0.T, c0.n_vis, c0.had_block) == (64, 48, 512) and c0.vis_spans == ((8, 48),)
    c1 = wl.workload(1)
    assert (c1.T, c1.n_vis) == (1280, 1024) and c1.vis_spans == ((16, 1024),)
    assert c1.projections["gate_up"] == (3584, 37888) and c1.projections["down"] == (18944, 3584)
    c2 = wl.workload(2)
    assert (c2.T, c2.n_vis) == (4096, 3584) and c2.vis_spans == ((256, 3584),)
    for t in (1, 4, 16):
        c3 = wl.workload(3, t)
        assert c3.T == t and c3.n_vis == 0 and len(c3.projections) == 7
    c4 = wl.workload(4)
    assert c4.T == 16384 and c4.n_vis == 4 * 3072 and c4.had_block == 128
    assert len(c4.vis_spans) == 4
    end = 0
    for s, l in c4.vis_spans:
        assert s > end and l == 3072
        end = s + l
    assert end < 16384
    for w in (c0, c1, c2, c4):
        for K, N in w.projections.values():
            assert K % w.had_block == 0 and K % 2 == 0


def test_inputs_are_deterministic_and_distributed_as_stated():
    w = wl.workload(0)
    a = wl.make_linear_inputs(w, "lin")
    b = wl.make_linear_inputs(w, "lin")
    for k in ("x", "w_packed", "w_scale", "calib_vis", "calib_txt"):
        assert (a[k] == b[k]).all()
    x = a["x"].astype(np.float64)
    assert a["x"].dtype == np.float16 and a["x"].shape == (64, 512)
    assert a["w_packed"].dtype == np.uint8 and a["w_packed"].shape == (512, 256)
    assert a["w_scale"].dtype == np.float16
    assert 0.005 <= float(a["w_scale"].min()) and float(a["w_scale"].max()) <= 0.02
    txt = np.r_[x[:8], x[56:]]
    vis = x[8:56]
    assert 0.9 < txt.std() < 1.1
    plain = np.delete(vis, list(wl.OUTLIER_CHANNELS), axis=1)
    assert 18 < plain.std() < 22
    assert 700 < vis[:, list(wl.OUTLIER_CHANNELS)].std() < 1300
    assert a["calib_vis"].shape == (256, 512) and a["calib_txt"].shape == (256, 512)
    assert np.isfinite(x).all()


def test_distinct_projections_get_distinct_streams():
    w = wl.workload(3, 4)
    k = wl.make_linear_inputs(w, "k", want_calib=False)
    v = wl.make_linear_inputs(w, "v", want_calib=False)
    assert k["w_packed"].shape == v["w_packed"].shape
    assert (k["w_packed"] != v["w_packed"]).any()
