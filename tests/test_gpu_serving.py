"""Serving sweep at toy size on the GPU: every policy produces the token streams of the solo
full-width run, and a row's result does not depend on what shares its launch."""
import numpy as np
import pytest
import torch

from paper_2603_15042_amd import harness as H, serving, vte

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("chunk", [16, 32, 64])
def test_row_result_is_independent_of_batch_neighbours_and_position(chunk):
    srv = serving.Server(layers=2, small=True, chunk=chunk)
    try:
        rng = np.random.RandomState(3)
        toks = rng.randint(0, srv.shp.V, size=40)
        srv.reference_next(toks)                     # rows grouped 16 at a time in sorted order
        first = dict(srv.next_of)
        srv.next_of.clear()
        for t in toks[::-1]:                         # one row at a time, position 0, neighbours all token 0
            srv.reference_next([t])
        assert srv.next_of == first
    finally:
        srv.close()


@pytest.mark.parametrize("chunk", [16, 32, 64])
def test_serving_policies_reproduce_solo_tokens(chunk):
    out = serving.sweep([60.0], 1.0, layers=2, small=True, modes=("fixed", "tput", "tpot"), chunk=chunk)
    res = out["rates"]["60.0"]
    for mode in ("solo", "fixed", "tput", "tpot"):
        r = res[mode]
        assert r["tokens"] > 0 and r["transitions_checked"] == r["tokens"]
        assert r["token_mismatches_vs_solo_full_width"] == 0, mode
    assert res["tpot"]["tpot_first"][0]["standing_width"] is not None
    assert res["fixed"]["gemm_per_s"] > 0 and res["tput"]["gemm_per_s"] > 0
