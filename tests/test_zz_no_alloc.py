"""The entry point that allocates nothing (ssd_dense_decode_attn_static: partial results of the row splits in a
fixed scratch array inside the library) against the entry point it is a variant of (ssd_dense_decode_attn with a
caller's workspace): same kernels, so the same bits.  Two calls in a row share the scratch, the second smaller."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_18716_amd as ssd
from harness import check_outputs

FAKE = 1 << 24


def _inputs(B, H, d, dtype, n_cap, seed):
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator().manual_seed(seed)
    q = torch.randn((B, H, d), generator=g).to(tdt)
    K = torch.randn((B, H, n_cap, d), generator=g).to(tdt)
    V = torch.randn((B, H, n_cap, d), generator=g).to(tdt)
    return q, K, V, tdt


def _both(B, H, d, dtype, n_cap, n, seed, vis_start, w):
    """One call through each entry point on the same inputs; returns (static, workspace) results and the host inputs."""
    q, K, V, tdt = _inputs(B, H, d, dtype, n_cap, seed)
    qd, Kd, Vd = q.cuda(), K.cuda(), V.cuda()
    res = []
    for static in (True, False):
        out = torch.full((B, H, d), 7.0, dtype=tdt, device="cuda")
        far = torch.full((B, H), -7.0, device="cuda")
        tot = torch.full((B, H), -7.0, device="cuda")
        if static:
            ssd.ssd_dense_decode_attn_static(qd, Kd, Vd, out, B, H, d, dtype, n_cap, n, 0.0, far, tot, 1, vis_start, w)
        else:
            ws = torch.empty(ssd.ssd_dense_workspace_bytes(B, H, d, n), dtype=torch.uint8, device="cuda")
            ssd.ssd_dense_decode_attn(qd, Kd, Vd, out, B, H, d, dtype, n_cap, n, 0.0, far, tot, 1, vis_start, w, ws)
        torch.cuda.synchronize()
        res.append((out.float().cpu().numpy(), far.cpu().numpy(), tot.cpu().numpy()))
    return res[0], res[1], (q, K, V)


@pytest.mark.gpu
def test_static_scratch_entry_point_equals_the_workspace_entry_point_on_two_calls_in_a_row():
    # first call: 256 units in 5 row splits (2.7 MB of the scratch in use); second call: a smaller input, 24 units
    # in 2 splits, which finds the first call's partial results still in the scratch; third: one split, no scratch
    shapes = [(8, 32, 128, "bf16", 700, 640, 64, 32), (4, 6, 64, "f32", 300, 257, 9, 32), (2, 3, 128, "bf16", 70, 67, 0, 16)]
    for i, (B, H, d, dtype, n_cap, n, vis_start, w) in enumerate(shapes):
        (o_s, f_s, t_s), (o_w, f_w, t_w), (q, K, V) = _both(B, H, d, dtype, n_cap, n, 100 + i, vis_start, w)
        assert np.array_equal(o_s, o_w), ("outputs differ", i, float(np.abs(o_s - o_w).max()))
        assert np.array_equal(f_s, f_w) and np.array_equal(t_s, t_w), ("masses differ", i)
        # and both are the attention the oracle defines (a few units suffice: the two are bit-equal)
        for b, h in [(0, 0), (B - 1, H - 1)]:
            ref, _, p64 = oracle.dense_attend(q[b, h].float().numpy(), K[b, h].float().numpy(), V[b, h].float().numpy(), n, 1.0 / np.sqrt(d))
            check_outputs(o_s[b, h], ref, dtype, "static dense unit (%d,%d) of call %d" % (b, h, i))
            f_ref, t_ref = oracle.far_tot(p64, vis_start, n - vis_start, w)
            assert abs(f_s[b, h] - f_ref) < 2e-5 + 1e-4 * f_ref and abs(t_s[b, h] - t_ref) < 2e-5 + 1e-4 * t_ref


def test_static_scratch_entry_point_refuses_what_does_not_fit_before_any_launch():
    # 8000 units in 2 row splits would leave 8.45 MB of partial results: more than the 8 MiB scratch
    lib = ssd.lib
    rc = lib.ssd_dense_decode_attn_static(FAKE, FAKE, FAKE, FAKE, 250, 32, 128, ssd.SSD_BF16, 256, 256, 0.0, None, None, 1, 0, 32, None)
    assert rc == ssd.SSD_ERR_INVALID_ARG
    assert "static scratch" in ssd.ssd_last_error() and str(ssd.SSD_DENSE_STATIC_SCRATCH_BYTES) in ssd.ssd_last_error()
    # the ordinary argument checks come first
    assert lib.ssd_dense_decode_attn_static(None, FAKE, FAKE, FAKE, 2, 2, 128, ssd.SSD_BF16, 256, 256, 0.0, None, None, 1, 0, 32, None) == ssd.SSD_ERR_INVALID_ARG
    assert lib.ssd_dense_decode_attn_static(FAKE, FAKE, FAKE, FAKE, 2, 2, 96, ssd.SSD_BF16, 256, 256, 0.0, None, None, 1, 0, 32, None) == ssd.SSD_ERR_INVALID_ARG
