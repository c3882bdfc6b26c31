"""laser_verify_head_static (the entry point for callers that cannot allocate device memory) against
laser_verify_head, through the C ABI: accepted lengths and emitted tokens must be identical (both run the same
kernels; only the place of the partial statistics differs) on two calls in a row, the second with a smaller input
(the static array then still holds the first call's records beyond the rows in use)."""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


def test_static_head_matches_the_allocating_head_on_two_calls_in_a_row():
    import paper_2408_05676_amd as laser
    V, d = 32000, 1024
    sh = synth.ModelShape("h", 0, d, 8, 1024, V)
    wlm = torch.tensor(synth.gen_weight(sh, "wlm"), device="cuda").to(torch.bfloat16)
    model = laser.Model(0, d, 8, 1024, V, {"wlm": wlm}, 16, 16, 0)
    r = np.random.default_rng(7)
    for B, K, k, p, mode in ((2, 7, 2, 0.001, 0), (3, 2, 3, 0.0005, 1)):          # 16 rows, then 9
        h = torch.tensor(r.standard_normal((B, K + 1, d)).astype(np.float32) * 4, device="cuda").to(torch.float16)
        ref_logits = (h.float().reshape(-1, d) @ wlm.float().T).reshape(B, K + 1, V)
        order = torch.argsort(-ref_logits, dim=-1, stable=True)
        drafts = torch.empty((B, K), dtype=torch.int32, device="cuda")
        for b in range(B):
            for j in range(K):
                drafts[b, j] = order[b, j, (b + j) % 3]                          # ranks 0..2
        dl = torch.tensor([K - (b % 2) for b in range(B)], dtype=torch.int32, device="cuda")
        acc0, out0, _ = laser.verify_head(model, h, drafts, dl, k, p, mode)
        acc1 = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        out1 = torch.full((B, K + 1), -7, dtype=torch.int32, device="cuda")
        laser.verify_head_static(model, h, drafts, dl, k, p, mode, out=(acc1, out1))
        torch.cuda.synchronize()
        assert acc1.cpu().tolist() == acc0.cpu().tolist(), (B, K)
        assert out1.cpu().tolist() == out0.cpu().tolist(), (B, K)
        assert max(acc0.cpu().tolist()) > 0                                       # something was accepted
    # sizes beyond the static array are refused with a clear error, nothing is launched
    B, K = 3, 7                                                                   # 24 rows
    h = torch.zeros((B, K + 1, d), dtype=torch.float16, device="cuda")
    big = laser.Model(0, d, 8, 1024, V, {"wlm": wlm}, 32, 16, 0)
    with pytest.raises(laser.LaserError, match="rows exceed"):
        laser.verify_head_static(big, h, torch.zeros((B, K), dtype=torch.int32, device="cuda"),
                                 torch.zeros(B, dtype=torch.int32, device="cuda"), 1, 0.0, 0,
                                 out=(torch.zeros(B, dtype=torch.int32, device="cuda"),
                                      torch.zeros((B, K + 1), dtype=torch.int32, device="cuda")))
    model.close(); big.close()
