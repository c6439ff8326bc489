"""The allocation-free form of the isolated cache update + attention entry point (for callers that cannot
allocate: graph capture, serving loops): same kernels, scratch in the library's static device array.
Checked against the workspace-taking entry point (bit for bit: same kernels, same plan) and against the
oracle, on two calls in a row, the second on a smaller input, on shapes whose keys are sliced over
workgroups so that the scratch array is really used."""
import numpy as np
import pytest
import torch

import dkv_inputs as D
from dkv_inputs.configs import BF16
from oracle.attn_update import attn_update as oracle_attn_update
from gpu_parity import check_close, tolerances

pytestmark = pytest.mark.gpu


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(device="cuda", dtype=torch.bfloat16)


def _both_entries(shape, counts, seed):
    import paper_2505_15781_amd as P
    c = D.attn_update_case(shape, None, seed, ragged=counts)
    rows, max_rows = int(c["active_off"][-1]), max(counts)
    nb = P.attn_update_workspace_bytes(shape.batch, shape.n_q_heads, shape.n_kv_heads, shape.seq_len,
                                       shape.head_dim, BF16, max_rows)
    assert 0 < nb <= P.binding.STATIC_SCRATCH_BYTES, "the case must use scratch memory, within the static limit"
    q, kn, vn = _dev(c["q"]), _dev(c["k_new"]), _dev(c["v_new"])
    idx, off = torch.from_numpy(c["active_idx"]).cuda(), torch.from_numpy(c["active_off"]).cuda()
    outs, caches = [], []
    for static in (False, True):
        kc, vc = _dev(c["k_cache"]), _dev(c["v_cache"])
        out = torch.zeros((rows, shape.n_q_heads, shape.head_dim), dtype=torch.bfloat16, device="cuda")
        if static:
            P.attn_update_static(kc, vc, q, kn, vn, idx, off, out, rows, max_rows, BF16)
        else:
            ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
            P.attn_update(kc, vc, q, kn, vn, idx, off, out, rows, max_rows, BF16, ws)
        torch.cuda.synchronize()
        outs.append(out.float().cpu().numpy())
        caches.append((kc.float().cpu().numpy(), vc.float().cpu().numpy()))
    rk, rv = c["k_cache"].astype(np.float64), c["v_cache"].astype(np.float64)
    ref = oracle_attn_update(rk, rv, c["q"], c["k_new"], c["v_new"], c["active_idx"], c["active_off"])
    assert np.array_equal(outs[0], outs[1]), "static-scratch entry differs from the workspace entry"
    assert np.array_equal(caches[1][0].astype(np.float64), rk) and np.array_equal(caches[1][1].astype(np.float64), rv)
    check_close(outs[1], ref, tolerances(BF16), f"static-scratch attention {counts}")


def test_static_scratch_entry_matches_the_workspace_entry_on_two_calls_in_a_row():
    big = D.AttnUpdateShape(batch=2, n_q_heads=4, n_kv_heads=2, seq_len=2085, head_dim=128, dtype=BF16)
    _both_entries(big, [21, 40], 61)
    small = D.AttnUpdateShape(batch=1, n_q_heads=4, n_kv_heads=2, seq_len=1031, head_dim=128, dtype=BF16)
    _both_entries(small, [3], 62)          # fewer rows, fewer keys, fewer slices: old records stay in the array


def test_static_scratch_entry_rejects_what_does_not_fit():
    import paper_2505_15781_amd as P
    # 2 heads, 100 rows over 60000 keys: keys sliced 12 ways, 5.5 MB of partial records, above the 4 MiB of the static array
    B, Hq, Hkv, L, dh, rows = 1, 2, 2, 60000, 128, 100
    nb = P.attn_update_workspace_bytes(B, Hq, Hkv, L, dh, BF16, rows)
    if nb <= P.binding.STATIC_SCRATCH_BYTES:
        pytest.skip("the planner does not slice this shape")
    kc = torch.zeros((B, Hkv, L, dh), dtype=torch.bfloat16, device="cuda")
    q = torch.zeros((rows, Hq, dh), dtype=torch.bfloat16, device="cuda")
    kn = torch.zeros((rows, Hkv, dh), dtype=torch.bfloat16, device="cuda")
    idx = torch.arange(rows, dtype=torch.int32, device="cuda")
    off = torch.tensor([0, rows], dtype=torch.int32, device="cuda")
    with pytest.raises(P.DkvError) as e:
        P.attn_update_static(kc, kc.clone(), q, kn, kn, idx, off, q.clone(), rows, rows, BF16)
    assert e.value.code == -4 and "static scratch" in str(e.value)
