"""Host-side tests of the learned cost-model tooling (gradient-boosted trees, feature layout, generated tables)."""
import os
import re

import numpy as np

from paper_2306_15155_amd.costmodel import train

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_gbt_fits_a_piecewise_smooth_function():
    rng = np.random.default_rng(0)
    X = rng.uniform(0.0, 10.0, size=(600, 3))
    y = np.where(X[:, 0] > 5.0, 2.0, -1.0) + 0.3 * X[:, 1] + np.sin(X[:, 2])
    m = train.Gbt().fit(X[:500], y[:500])
    assert np.median(np.abs(m.predict(X[:500]) - y[:500])) < 0.05
    assert np.median(np.abs(m.predict(X[500:]) - y[500:])) < 0.25          # generalises to unseen points
    assert abs(m.predict(np.array([[7.0, 5.0, 1.0]]))[0] - m.predict(np.array([[3.0, 5.0, 1.0]]))[0] - 3.0) < 0.5  # found the step


def test_feature_vectors_have_the_layout_the_library_uses():
    f = train.spmm_features(1000, 2000, 50_000, 400, 3_000_000, 64, "scaled")
    assert len(f) == 8 + len(train.FLAVOURS) == 12
    assert f[:3] == [np.log2(1000), np.log2(2000), np.log2(50_000)]
    assert abs(f[3] - np.log2(50.0)) < 1e-12 and abs(f[5] - 6.0) < 1e-12
    assert abs(f[6] - np.log2(400 / 50.0)) < 1e-12 and abs(f[7] - np.log2(3_000_000 / 1000 / 2500.0)) < 1e-12
    assert f[8:] == [0.0, 0.0, 1.0, 0.0]
    assert train.gemm_features(8, 16, 32) == [3.0, 4.0, 5.0]
    assert train.spmm_work(1024, 4) == 12.0 and train.gemm_work(2, 4, 8) == 6.0
    # the same constants on the library side
    src = open(os.path.join(ROOT, "paper_2306_15155_amd", "csrc", "api.hip")).read()
    assert "double x[12]" in src and "x[8 + flavour] = 1.0;  // pattern, weighted, scaled, softmax" in src


def test_emitted_tables_round_trip(tmp_path):
    rng = np.random.default_rng(1)
    X = rng.uniform(0.0, 4.0, size=(200, 2))
    y = X[:, 0] * 2.0 - X[:, 1]
    m = train.Gbt().fit(X, y)
    out = tmp_path / "model.inc"
    train.emit({"Toy": m}, str(out))
    text = out.read_text()
    nodes = [tuple(float(v) for v in re.findall(r"-?\d+\.?\d*(?:e-?\d+)?", line.replace("(float)", "")))
             for line in text.splitlines() if line.startswith("    {")]
    roots = [int(v) for v in re.search(r"kToyRoots\[\] = \{([^}]*)\}", text).group(1).split(",")]
    base = float(re.search(r"kToyBase = \(float\)(\S+);", text).group(1))
    assert len(nodes) == len(m.nodes) and roots == m.roots

    def predict(x):  # the traversal the library performs
        s = base
        for r in roots:
            k = r
            while nodes[k][0] >= 0:
                k = int(nodes[k][1]) if x[int(nodes[k][0])] <= np.float32(nodes[k][3]) else int(nodes[k][2])
            s += nodes[k][4]
        return s

    for x in X[:20]:
        assert abs(predict(x) - m.predict(x[None, :])[0]) < 1e-4


def test_committed_tables_exist_and_name_both_models():
    text = open(os.path.join(ROOT, "paper_2306_15155_amd", "csrc", "learned_model.inc")).read()
    for name in ("kSpmmNodes", "kSpmmRoots", "kSpmmBase", "kGemmNodes", "kGemmRoots", "kGemmBase"):
        assert name in text
    assert text.count("kSpmmRoots[] = {") == 1 and len(re.search(r"kSpmmRoots\[\] = \{([^}]*)\}", text).group(1).split(",")) == train.N_TREES
