"""The ratio / budget sweep (Sec. 5.4, Tab. 2 settings) on a reduced shape: counts follow the paper's
"3 -> r" notation and the chunk-level attention map is a distribution that agrees with the oracle."""
import numpy as np
import pytest
import torch

import oracle
import wk_synth as ws
from paper_2605_22718_amd import sweep
from wkt import dev

pytestmark = pytest.mark.gpu


def test_sweep_settings_follow_the_paper_counts_and_masses_match_oracle():
    cfg = ws.get_config(1).with_(H=2, T=64, native_frames=6)
    seen = {}
    for r in sweep.SETTINGS:
        row = sweep.run_setting(cfg, r, 10, dev())
        seen[r] = row
        assert row["stored_tokens"] == round(r * cfg.T)                 # 3 -> r keeps r frame-equivalents
        assert row["retrieved_chunks"] == int(9 / r)                    # what fits in the 9-frame region
        assert row["N_kv"] == cfg.n_native + row["retrieved_chunks"] * row["stored_tokens"]
        assert row["N_kv"] <= cfg.n_native + 9 * cfg.T
        m = np.array([row["mass_native"]] + row["mass_per_retrieved_chunk"])
        assert abs(m.sum() - 1.0) < 1e-9 and (m > 0).all()
    # the three inter-chunk rows of Tab. 2 are among the settings: 3->3, 6->3 and 9->3 chunks in one budget
    assert [seen[r]["retrieved_chunks"] for r in (3.0, 1.5, 1.0)] == [3, 6, 9]
    assert seen[3.0]["N_kv"] == seen[1.5]["N_kv"] == seen[1.0]["N_kv"]
    # the attention map of one setting against the oracle (joint softmax over native rows + retrieved chunks)
    row = seen[1.5]
    P = (1.5 - 1.0) / (cfg.F - 1)
    Q = ws.make_queries(cfg)
    Kn, _ = ws.make_native(cfg)
    parts = [Kn]
    for c in row["retrieved_ids"]:
        K, V, _ = ws.make_chunk(cfg, c)
        _, oK, _, _ = oracle.compress(K, V, None, cfg.T, cfg.F, P, oracle.RATIO_NONANCHOR)
        parts.append(oK)
    _, _, o_mass = oracle.score_chunks_query(Q, parts, 1)
    got = np.array([row["mass_native"]] + row["mass_per_retrieved_chunk"])
    np.testing.assert_allclose(got, o_mass, rtol=1e-2)
    poses, cur = ws.make_poses(10, cfg.seed)
    o_ids, _, _ = oracle.score_chunks(poses, cur, row["retrieved_chunks"])
    assert row["retrieved_ids"] == [int(i) for i in o_ids]
