"""gad_subgraph_variance_static (the variance call that allocates nothing) against gad_subgraph_variance.

Both run the same kernels; only the reduction buffer differs (a fixed device array inside the library instead of
memory of the graph), so the results must agree bit for bit -- inside the 1e-4 bar of the float32 path by a wide
margin.  Two calls in a row share the array; the second has a smaller input, so words the first call wrote and the
second does not overwrite are still there when it runs.
"""
import numpy as np
import pytest
import torch

from paper_2110_02987_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gad():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2110_02987_amd import gad as g
    g.lib()
    return g


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def build(gad, name):
    gr = wl.make_graph(wl.CONFIGS[name])
    return gad.build_subgraph(dev(gr["src"]), dev(gr["dst"]), gr["n_global"], dev(gr["local_ids"]), dev(gr["halo_ids"]))


def both(gad, g, V, beta, with_per_node):
    res = []
    for fn in (gad.subgraph_variance_static, gad.subgraph_variance):
        out3 = torch.full((3,), -1.0, dtype=torch.float64, device="cuda")
        per = torch.full((g.n,), -1.0, device="cuda") if with_per_node else None
        fn(g, V, beta, out3, per)
        torch.cuda.synchronize()
        res.append((out3.cpu().numpy(), None if per is None else per.cpu().numpy()))
    return res


def test_static_variance_two_calls_second_smaller(gad):
    print("static variance: products_small F=300, then tiny F=17", flush=True)
    big, small = build(gad, "products_small"), build(gad, "tiny")
    cases = [(big, wl.make_features(big.n, 300, sub=1) * 1.7 + 0.3, 1.0),
             (small, wl.make_features(small.n, 17, sub=2) - 0.2, 0.1)]
    for g, V, beta in cases:
        (a3, ap), (b3, bp) = both(gad, g, dev(V), beta, True)
        assert np.all(np.isfinite(a3)) and a3[0] > 0 and a3[2] > 0
        assert np.abs(a3 - b3).max() <= 1e-4 * np.abs(b3).max() and np.array_equal(a3, b3)
        assert np.array_equal(ap, bp)
    # and once more on the large input: what the small call left in the array does not leak into it
    g, V, beta = cases[0]
    (a3, _), (b3, _) = both(gad, g, dev(V), beta, False)
    assert np.array_equal(a3, b3)


def test_static_variance_bf16_and_limits(gad):
    print("static variance: bf16 vectors, size limits", flush=True)
    g = build(gad, "tiny")
    V = torch.randn(g.n, 64, device="cuda").to(torch.bfloat16)
    (a3, ap), (b3, bp) = both(gad, g, V, 1.0, True)
    assert np.array_equal(a3, b3) and np.array_equal(ap, bp)
    out3 = torch.zeros(3, dtype=torch.float64, device="cuda")
    wide = torch.zeros(g.n, 1025, device="cuda")
    with pytest.raises(gad.GadError) as e:                       # one past the widest vector the array holds
        gad.subgraph_variance_static(g, wide, 1.0, out3)
    assert e.value.status == -2
    gad.subgraph_variance_static(g, wide[:, :1024].contiguous(), 1.0, out3)     # the limit itself is accepted
    torch.cuda.synchronize()
    assert out3[2].item() == 0.0
    for beta in (0.0, float("nan")):
        with pytest.raises(gad.GadError):
            gad.subgraph_variance_static(g, V, beta, out3)
