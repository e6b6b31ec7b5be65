"""The entry point that allocates nothing (mukv_prefill_attend_static, for callers that cannot call
hipMalloc): its fixed per-GPU scratch must give what mukv_prefill_attend gives with a caller's
workspace -- bit for bit, since both run the same kernels -- and what the oracle gives, on two
calls in a row, the second one smaller, so that what the first call left in the scratch is there
when the second runs."""
import numpy as np
import pytest
import torch

from paper_2605_22269_amd import binding as mk
from paper_2605_22269_amd import synth
from mukv_testlib import Pair, np_view, out_err, to_f64

pytestmark = pytest.mark.gpu

W = synth.WORKLOADS


def _inputs(w, n_q, n_old, B, seed):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(B, n_q, w.n_q_heads, w.head_dim, generator=g).to(w.torch_dtype)
    offs = np.arange(B + 1, dtype=np.int32) * (n_old + n_q)
    kl = torch.randn(int(offs[-1]), w.n_kv_heads, w.head_dim, generator=g).to(w.torch_dtype)
    vl = torch.randn(int(offs[-1]), w.n_kv_heads, w.head_dim, generator=g).to(w.torch_dtype)
    return q, kl, vl, offs


def _both_ways(p, layer, n_q, n_old, frame_idx, seed):
    """One prefill through the workspace call and through the static-scratch call, both through the C ABI;
    returns the static call's (out, signal) after checking them against the other call and the oracle."""
    w = p.w
    B = len(frame_idx)
    q, kl, vl, offs = _inputs(w, n_q, n_old, B, seed)
    qd, kd, vd, od = q.cuda(), kl.cuda(), vl.cuda(), torch.from_numpy(offs).cuda()
    fi = torch.tensor(frame_idx, dtype=torch.int32, device="cuda")
    out_ws, sig_ws = p.gpu.prefill_attend(layer, qd, fi, kd, vd, od, True)
    torch.cuda.synchronize()
    out_st = torch.full_like(qd, 7.0)
    sig_st = torch.full((B, n_q), -3.0, dtype=torch.float32, device="cuda")
    free_before = torch.cuda.mem_get_info()[0]
    p.gpu.prefill_attend_static(layer, qd, fi, kd, vd, od, True, out_st, sig_st)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before            # no device memory taken or given back
    np.testing.assert_array_equal(np_view(out_st.cpu()), np_view(out_ws.cpu()))
    np.testing.assert_array_equal(sig_st.cpu().numpy(), sig_ws.cpu().numpy())
    got, got_sig = to_f64(np_view(out_st.cpu())), sig_st.cpu().numpy().astype(np.float64)
    tol = 2e-2 if w.dtype == "bf16" else 1e-5
    for b in range(B):
        kb, vb = np_view(kl[offs[b]:offs[b + 1]]), np_view(vl[offs[b]:offs[b + 1]])
        want, want_sig = p.orc.prefill_attend(layer, np_view(q[b]), frame_idx[b], kb, vb, True)
        assert out_err(got[b], want) <= tol
        assert np.abs(got_sig[b] - want_sig).max() <= 1e-6
    return out_st, sig_st


@pytest.mark.parametrize("name,kw", [("7b", {"n_layers": 2}), ("tiny", {"n_layers": 2})])
def test_static_scratch_prefill_twice_in_a_row(name, kw):
    # 7b: the matrix-core prefill (records of split tiles, log-sum-exps and column sums in the scratch);
    # tiny: the fp32 path (split records, log-sum-exps, column sums of its own kernels)
    w = W[name].scaled(n_frames=12, n_questions=2, **kw)
    p = Pair(w, seed=4400, chunk=4)
    p.ingest()
    P = w.tokens_per_frame
    _both_ways(p, 1, P + 3, 5, [[7, 2, 9], [0, 11, 4]], seed=4401)         # two questions, ragged tile
    _both_ways(p, 0, P // 2, 0, [[3, 8, 1]], seed=4402)                     # smaller: one question, half a frame
    _both_ways(p, 1, P, 2, [[10, -1, 6]], seed=4403)                        # and one frame, a padded list
    p.close()


def test_static_scratch_refuses_what_does_not_fit():
    w = W["7b"].scaled(n_frames=4, n_layers=1, n_questions=8)
    p = Pair(w, seed=4410, chunk=4)
    p.ingest()
    n_q, B = 2048, 8
    need = mk.mukv_prefill_workspace_size(p.gpu.h, n_q, 2, B)
    assert need > mk.MUKV_STATIC_SCRATCH_BYTES
    q, kl, vl, offs = _inputs(w, n_q, 0, B, 4411)
    qd = q.cuda()
    out, sig = torch.empty_like(qd), torch.empty(B, n_q, dtype=torch.float32, device="cuda")
    fi = torch.zeros(B, 2, dtype=torch.int32, device="cuda")
    with pytest.raises(mk.MuKVError) as e:
        p.gpu.prefill_attend_static(0, qd, fi, kl.cuda(), vl.cuda(), torch.from_numpy(offs).cuda(), True, out, sig)
    assert e.value.status == mk.MUKV_ERR_CAPACITY
    p.close()
