"""Host-side checks of the synthetic search inputs (CPU only)."""
import numpy as np

import oracle
from paper_2302_08141_amd.workloads import graphs, specs as sp, synthetic as syn

INF = oracle.INF


def test_streams_are_seeded_and_in_range():
    a = syn.random_chain_problem(5, 6, 9, 1000, 5000)
    b = syn.random_chain_problem(5, 6, 9, 1000, 5000)
    c = syn.random_chain_problem(6, 6, 9, 1000, 5000)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and not np.array_equal(a[1], c[1])
    assert 0 <= a[0].min() and a[0].max() < 1000 and 0 <= a[1].min() and a[1].max() < 5000
    assert all(a[1][i, k, k] == 0 for i in range(5) for k in range(9))
    seg = syn.segment_costs(0, 4096)
    assert seg.min() >= 1 and seg.max() < 100000 and len(np.unique(seg)) > 3000
    cb, Rb = syn.random_chain_batch([3], 4, 5, 10, 10, Kp=16)
    assert cb.shape == (1, 4, 16) and np.all(cb[0, :, 5:] == INF) and np.all(Rb[0, :, 5:, :] == INF)


def test_gpt_like_chain_shape_and_feasibility():
    g = graphs.gpt_chain()
    assert g["N"] == 24 * 10 + 2 and g["Kp"] == 64 and g["dims"].shape == (241, 4)
    assert tuple(g["dims"][0]) == (8, 2048, 4096, 1) and [8, 2048, 12288, 1] in g["dims"].tolist()
    c = g["c"]
    finite = c < INF
    assert finite.any(axis=1).all() and c[finite].max() < (1 << 36) and c[finite].min() >= 0
    # a finite node cost implies valid specs on both sides
    for i in (0, 1, 2, 3, 4, 8, 241):
        for j in np.nonzero(finite[i])[0]:
            assert g["out_spec"][i, j] != sp.EMPTY and g["in_spec"][i, j] != sp.EMPTY
    # sharding over both axes of the 8x8 mesh divides compute by 64
    qkv = g["names"].index("qkv")
    rr = 0                                    # (replicate, replicate)
    both = 2 * 8 + 4                          # (split batch on axis 0, split seq on axis 1)
    assert abs(c[qkv, rr] / c[qkv, both] - 64) < 1
    R = oracle.build_reshard(g["m"], g["bw_bytes_per_us"], g["alpha_ns"], g["K"][:12], g["out_spec"][:12],
                             g["in_spec"][:12], g["dims"][:11], g["elem_bytes"][:11])
    arg, _, total, last = oracle.chain(np.ascontiguousarray(c[None, :12]), R[None])
    assert total[0] < INF and R[R < INF].max() < (1 << 36)


def test_moe_shaped_chain_shape():
    g = graphs.moe_chain()
    assert g["N"] == 96 * 85 + 32 == 8192 and g["Kp"] == 256 and g["m"] == (32, 32)
    assert [32, 64, 32, 12288] in g["dims"].tolist()          # dispatched tokens [G, E, C, H]
    finite = g["c"] < INF
    assert finite.any(axis=1).all() and g["c"][finite].max() < (1 << 36)
    assert (g["out_spec"] != sp.EMPTY).sum(axis=1).min() == 256
