"""The selector compiled into the library must be the model selector_train.py wrote: walk the JSON
copy of the trees in Python and compare with da_spmm_select on random feature vectors."""
import json
import os

import numpy as np
import pytest

from paper_2202_08556_amd import selector_train as st

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(not os.path.exists(st.MODEL_JSON), reason="no trained model yet")
def test_compiled_selector_matches_json_model():
    from paper_2202_08556_amd import binding as da
    model = json.load(open(st.MODEL_JSON))
    rng = np.random.Generator(np.random.PCG64(5))
    for _ in range(3000):
        rows = int(2 ** rng.uniform(2, 21))
        mean = float(2 ** rng.uniform(0, 8))
        cv = float(rng.uniform(0, 20))
        f = dict(rows=rows, nnz=int(rows * mean), row_nnz_mean=mean, row_nnz_std=cv * mean,
                 row_nnz_max=mean * float(2 ** rng.uniform(0, 10)), N=int(2 ** rng.integers(0, 10)))
        assert da.da_spmm_select(f) == st.walk(model, st.feature_vector(f))


def test_normalized_performance_metric_matches_oracle_definition():
    from oracle import reference as orc
    rng = np.random.Generator(np.random.PCG64(6))
    T = rng.uniform(1.0, 100.0, size=(40, 8))
    ch = rng.integers(0, 8, size=40)
    assert st.normalized_performance(T, ch) == pytest.approx(orc.normalized_performance(T, ch), rel=1e-12)
    assert st.normalized_performance(T, T.argmin(axis=1)) == pytest.approx(1.0)
