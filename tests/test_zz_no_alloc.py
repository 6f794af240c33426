"""som_neighborhood_update_static (the update for callers that cannot allocate) against som_neighborhood_update.

Both run the same kernels, one on a workspace grown on demand, the other on the library's fixed per-GPU array, so
the weights must agree bit for bit; the oracle bounds both.  Two calls in a row share the fixed array: the second
one is smaller and must not see what the first one left behind.
"""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu


def _case(seed, shape, D, kind):
    rng = np.random.default_rng(seed)
    K = shape[0] * shape[1]
    W = rng.normal(size=(K, D)).astype(np.float32)
    n = rng.integers(0, 60, size=K).astype(np.int64)
    n[rng.random(K) < 0.35] = 0
    S = rng.normal(size=(K, D)) * n[:, None]
    G = oracle.graph_distances(kind, lattice=shape).astype(np.float32)
    return W, S, n, G


def test_static_update_matches_the_allocating_update_on_two_calls_in_a_row():
    from paper_2604_26555_amd import Som, SomError, SOM_EINVAL
    som = Som(0)
    try:
        calls = [((32, 32), 50, "hex", 3.0, "threshold"),      # 1024 x 51 cells: most of the array
                 ((10, 10), 8, "rect", 0.6, "threshold"),      # a smaller call right after it
                 ((16, 16), 63, "hex", 0.3, "shift"),          # widest rows, shifted exponents (uses the shift cells)
                 ((5, 6), 4, "rect", 0.05, "threshold")]
        for it, (shape, D, kind, sigma, guard) in enumerate(calls):
            W, S, n, G = _case(100 + it, shape, D, kind)
            K = len(W)
            Sd, nd, Gd = torch.from_numpy(S).cuda(), torch.from_numpy(n).cuda(), torch.from_numpy(G).cuda()
            print(f"static update call {it}: K={K} D={D} sigma={sigma} safeguard={guard}", flush=True)
            som.som_set_safeguard(guard)
            Wa, Wb = torch.from_numpy(W).cuda(), torch.from_numpy(W).cuda()
            ga = torch.full((1,), -1, dtype=torch.int32, device="cuda")
            gb = torch.full((1,), -2, dtype=torch.int32, device="cuda")
            som.som_neighborhood_update_static(Sd, nd, Gd, sigma, Wa, n_guarded=ga)
            som.som_neighborhood_update(Sd, nd, Gd, sigma, Wb, n_guarded=gb)
            som.som_sync()
            assert torch.equal(Wa, Wb) and int(ga.item()) == int(gb.item())
            if guard == "threshold":
                W_or, guarded, den = oracle.neighborhood_update(S, n, G.astype(np.float64), sigma, W)
                keep = ~((den > oracle.DEFAULT_EPS_H / 4) & (den < oracle.DEFAULT_EPS_H * 4))
                assert abs(int(ga.item()) - int(guarded.sum())) <= int((~keep).sum())
            else:
                W_or, unchanged = oracle.neighborhood_update_shifted(S, n, G.astype(np.float64), sigma, W)
                keep = np.ones(K, dtype=bool)
                assert int(ga.item()) == int(unchanged.sum())
            scale = np.maximum(np.abs(W_or).max(axis=1, keepdims=True), 1e-30)
            err = np.abs(Wa.cpu().numpy() - W_or) / scale
            assert (err[keep] <= 1e-4).all(), f"max relative weight error {err[keep].max():.2e}"
        som.som_set_safeguard("threshold")
        # beyond the fixed array: a clear error, nothing touched
        W, S, n, G = _case(7, (36, 36), 63, "rect")                      # 1296 x 64 = 82944 cells
        Wd = torch.from_numpy(W).cuda()
        with pytest.raises(SomError) as e:
            som.som_neighborhood_update_static(torch.from_numpy(S).cuda(), torch.from_numpy(n).cuda(), torch.from_numpy(G).cuda(), 1.0, Wd)
        assert e.value.code == SOM_EINVAL and "65536" in str(e.value)
        W, S, n, G = _case(8, (4, 4), 64, "rect")                        # D + 1 > 64
        with pytest.raises(SomError):
            som.som_neighborhood_update_static(torch.from_numpy(S).cuda(), torch.from_numpy(n).cuda(), torch.from_numpy(G).cuda(), 1.0,
                                               torch.from_numpy(W).cuda())
        assert torch.equal(Wd.cpu(), torch.from_numpy(W if False else _case(7, (36, 36), 63, "rect")[0]))
    finally:
        som.close()
