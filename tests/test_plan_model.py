"""Host-side checks of the planner's cost model (no GPU): the C++ formula equals the Python one the
constants were fitted with, and the committed constants still pick near-best candidates on the
committed timings."""
import math

import numpy as np
import pytest

import paper_2512_02551_amd as hg
from paper_2512_02551_amd import plan_model as pm


@pytest.fixture(scope="module")
def rows():
    return pm.load_rows([pm.DATA])


def test_constants_file_names_every_parameter():
    g = pm.read_inc()
    assert list(g) == pm.NAMES
    assert all(math.isfinite(v) and v > 0 for v in g.values())


def test_cpp_prediction_equals_python_prediction(rows):
    g = pm.read_inc()
    checked = 0
    for r in rows[::15]:
        for s, _ in r["cands"][::5]:
            d = pm.features(r["shape"], pm.parse_spec(s))
            py = float(pm.predict_us(g, {k: np.float64(v) for k, v in d.items()}))
            cc = hg.predict_us(*r["shape"], "mfma," + s)
            assert cc == pytest.approx(py, rel=1e-9), (r["shape"], s)
            checked += 1
    assert checked > 1000


def test_prediction_tracks_measurement(rows):
    g = pm.read_inc()
    D, ts, _ = pm.table(rows)
    err = np.log(pm.predict_us(g, D) / ts)
    assert np.sqrt((err ** 2).mean()) < 0.13          # about 11 % rms over 130 000 (shape, configuration) pairs
    assert abs(err.mean()) < 0.03


def test_regret_of_the_models_pick(rows):
    reg = pm.regret(pm.read_inc(), rows)
    assert math.exp(np.log(reg).mean()) < 1.06
    assert np.quantile(reg, 0.9) < 1.15


def test_monotone_in_problem_size():
    spec = "mfma,bm=128,bn=128,bk=64,wm=2,wn=2,st=3,pf=3,sk=1,gm=8"
    t = [hg.predict_us(n, n, n, spec) for n in (512, 1024, 2048, 4096, 8192)]
    assert all(a < b for a, b in zip(t, t[1:]))
    # eight times the work costs at least four times the time once the chip is full
    assert t[4] / t[3] > 4


def test_predict_us_rejects_what_the_model_does_not_cover():
    with pytest.raises(hg.HgemmError):
        hg.predict_us(256, 256, 256, "generic")
    with pytest.raises(hg.HgemmError):
        hg.predict_us(256, 256, 256, "mfma,bm=128,bn=128,bk=64,wm=2,wn=2,st=3,pf=3,sk=1,gm=8,sm=1")
    with pytest.raises(hg.HgemmError):
        hg.predict_us(0, 256, 256, "mfma,bm=128,bn=128,bk=64,wm=2,wn=2,st=3,pf=3,sk=1,gm=8")
    with pytest.raises(hg.HgemmError):
        hg.predict_us(256, 256, 256, "mfma,bm=96,bn=128,bk=64,wm=2,wn=2,st=3,pf=3,sk=1,gm=8")


def test_model_prefers_split_k_for_skinny_long_k_and_big_tiles_for_big_squares():
    def pick(M, N, K):
        cands = [s for s in hg.candidates(M, N, K) if "sm=1" not in s and "tb=1" not in s and "ps=1" not in s and "gm=8" in s]
        return min(cands, key=lambda s: hg.predict_us(M, N, K, s))

    s = pm.parse_spec(pick(16, 4096, 8192))
    assert s["sk"] > 1 and s["bm"] == 32
    s = pm.parse_spec(pick(8192, 8192, 8192))
    assert s["bm"] == 256 and s["bn"] == 256 and s["sk"] == 1
    s = pm.parse_spec(pick(96, 96, 96))
    assert s["bm"] <= 64 and s["bn"] <= 64 and s["sk"] == 1
