"""GPU parity of the merge entry points (Sec. 2.2 operator) against the oracle."""
import numpy as np
import pytest

from oracle import attention as A
from gpu_util import LSE_TOL

pytestmark = pytest.mark.gpu


def states(rng, n_rows, n_states, D=128, empty_frac=0.2):
    o = rng.standard_normal((n_rows, n_states, D)).astype(np.float32)
    lse = (rng.standard_normal((n_rows, n_states)) * 4).astype(np.float32)
    mask = rng.random((n_rows, n_states)) < empty_frac
    lse[mask] = -np.inf
    o[mask] = np.nan                     # whatever rides on an empty state must not leak
    if n_rows > 1:
        lse[1, :] = -np.inf; o[1] = 0    # a row with only empty states
    return o, lse


@pytest.mark.parametrize("n_rows,n_states", [(1, 1), (7, 2), (300, 5), (33, 70), (5, 200), (4, 0)])
def test_merge_states(n_rows, n_states):
    import torch
    import paper_2501_01005_amd as fi
    rng = np.random.default_rng(n_rows * 1000 + n_states)
    o, lse = states(rng, n_rows, n_states)
    print(f"[case] merge_states {n_rows}x{n_states}", flush=True)
    o_ref, lse_ref = A.merge_states(np.nan_to_num(o.astype(np.float64), nan=0.0), lse.astype(np.float64))
    d_o = torch.from_numpy(o).cuda(); d_l = torch.from_numpy(lse).cuda()
    out_o = torch.full((n_rows, 128), float("nan"), device="cuda"); out_l = torch.full((n_rows,), float("nan"), device="cuda")
    fi.fi_merge_states(d_o, d_l, n_rows, n_states, 128, out_o, out_l, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    go = out_o.double().cpu().numpy(); gl = out_l.double().cpu().numpy()
    assert np.array_equal(np.isneginf(gl), np.isneginf(lse_ref))
    fin = np.isfinite(lse_ref)
    assert np.abs(go - o_ref).max() <= 1e-5 and (not fin.any() or np.abs(gl[fin] - lse_ref[fin]).max() <= 1e-5)


def test_merge_state_pair_and_in_place():
    import torch
    import paper_2501_01005_amd as fi
    rng = np.random.default_rng(9)
    n = 2048 + 3
    oa, la = states(rng, n, 1); ob, lb = states(rng, n, 1)
    oa, ob, la, lb = oa[:, 0], ob[:, 0], la[:, 0], lb[:, 0]
    o_ref, l_ref = A.merge_pair(np.nan_to_num(oa.astype(np.float64)), la.astype(np.float64),
                                np.nan_to_num(ob.astype(np.float64)), lb.astype(np.float64))
    t = [torch.from_numpy(x).cuda() for x in (oa, la, ob, lb)]
    out_o = torch.empty((n, 128), device="cuda"); out_l = torch.empty((n,), device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    fi.fi_merge_state_pair(t[0], t[1], t[2], t[3], n, 128, out_o, out_l, s)
    fi.fi_merge_state_pair(t[0], t[1], t[2], t[3], n, 128, t[0], t[1], s)       # in place on a
    torch.cuda.synchronize()
    for go, gl in ((out_o, out_l), (t[0], t[1])):
        go = go.double().cpu().numpy(); gl = gl.double().cpu().numpy()
        assert np.array_equal(np.isneginf(gl), np.isneginf(l_ref))
        fin = np.isfinite(l_ref)
        assert np.abs(go - o_ref).max() <= 1e-5 and np.abs(gl[fin] - l_ref[fin]).max() <= 1e-5
