"""sik_decode_step_static (the decode step on the library's built-in scratch buffer, for callers that cannot
allocate) against sik_decode_step with a caller workspace: same kernels, so the output bits and the index sets
must be identical; two calls in a row, the second on a smaller input, which finds the first call's leftovers in
the shared buffer."""
import numpy as np
import pytest
import torch

import sik_workloads as W
from helpers import dev
from test_gpu_parity import GpuState, cfg_small, sync

pytestmark = pytest.mark.gpu

import paper_2603_14224_amd as sik  # noqa: E402


def both_ways(oracle, cfg, capacity, seq_len, append, step):
    """One decode step through each entry point from identical states; returns nothing, asserts equality."""
    res = []
    for static in (False, True):
        st = GpuState(cfg, oracle, capacity=capacity, seq_len=seq_len, offset_std=0.5, out_dtype=torch.float32)
        B, Hq, k = cfg.batch, cfg.n_q_heads, min(cfg.top_k, capacity)
        q, kn, vn = W.make_step_inputs(cfg, step)
        dkn, dvn = (dev(kn, cfg.dtype), dev(vn, cfg.dtype)) if append else (None, None)
        out = torch.full((B, Hq, 128), 7.0, device="cuda")
        idx = torch.full((B, Hq, k), -5, dtype=torch.int32, device="cuda")
        if static:
            sik.sik_decode_step_static(st.layout, dev(q, cfg.dtype), dkn, dvn, st.dK, st.dV, st.dsl, st.dmu, st.dcb,
                                       st.dcodes, k, 0.0, out, idx)
        else:
            sik.sik_decode_step(st.layout, dev(q, cfg.dtype), dkn, dvn, st.dK, st.dV, st.dsl, st.dmu, st.dcb,
                                st.dcodes, k, 0.0, out, idx, st.ws)
        sync()
        res.append((out.cpu().numpy(), np.sort(idx.cpu().numpy(), -1), st.dsl.cpu().numpy(),
                    st.dcodes.cpu().numpy(), st.dK.view(torch.int16).cpu().numpy()))
    for a, b in zip(*res):
        assert np.array_equal(a, b)
    assert np.all(np.isfinite(res[0][0])) and (res[0][1][..., -1] >= 0).any()


def test_static_scratch_entry_point_matches_workspace_entry_point(oracle):
    # a 20000-token layer with append, then a smaller ragged batch that reuses the buffer the first call left
    both_ways(oracle, cfg_small("C2", context=20000, top_k=600), 20008, None, True, 0)
    both_ways(oracle, cfg_small("C2", batch=3, n_kv_heads=2, n_q_heads=8, context=3000, top_k=64), 3004,
              [3000, 17, 1500], True, 1)
    # and a third, without append, selecting everything
    both_ways(oracle, cfg_small("C2", n_kv_heads=1, n_q_heads=4, context=900, top_k=1024), 1100, None, False, 2)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    big = sik.make_layout(32, 8, 32, 128, 16384, torch.bfloat16)          # needs 286 MB of scratch
    assert sik.sik_workspace_bytes(big, 512) > sik.SIK_STATIC_SCRATCH_BYTES
    t = torch.zeros(16, device="cuda")
    with pytest.raises(sik.SikError) as e:
        sik.sik_decode_step_static(big, t, None, None, t, t, t, t, t, t, 512, 0.0, t, None)
    assert e.value.status == -9 and "built-in" in str(e.value)
    fits = sik.make_layout(1, 8, 32, 128, 131072 + 64, torch.bfloat16)    # the 128K workload fits
    assert 0 < sik.sik_workspace_bytes(fits, 2048) <= sik.SIK_STATIC_SCRATCH_BYTES
