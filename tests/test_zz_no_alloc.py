"""The head call that allocates nothing (its scratch is a fixed array inside the library image)
against the ordinary head call with a caller-supplied workspace: same kernels, so the tokens and
logits must be identical bit for bit - on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2507_22424_amd import binding as sv

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,H,V", [("bf16", 4096, 32000), ("f32", 256, 512)])
def test_head_without_allocation_matches_the_workspace_form(dtype, H, V):
    nh, d = (H // 128, 128) if dtype == "bf16" else (4, 64)
    cfg = sv.model_cfg(dtype, H, nh, d, 3 * H if dtype == "f32" else 11008, V, 1e-5, 10000.0)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    gen = torch.Generator().manual_seed(7)
    g = (1.0 + 0.1 * torch.randn(H, generator=gen)).to(tdt).cuda()
    w = (0.02 * torch.randn(V, H, generator=gen)).to(tdt).cuda()
    lo, hi = V - 256, V
    for n_rows in (60, 26):                       # the second call is smaller than the first
        x = torch.randn(n_rows, H, generator=gen, dtype=torch.float32).cuda()
        ws = torch.empty(sv.sv_workspace_bytes(cfg, 1, n_rows, hi - lo), dtype=torch.uint8, device="cuda")
        sv.sv_workspace_init(cfg, 1, n_rows, hi - lo, ws)
        tok_a = torch.zeros(n_rows, dtype=torch.int32, device="cuda")
        tok_b = torch.full((n_rows,), -1, dtype=torch.int32, device="cuda")
        log_a = torch.zeros(n_rows, hi - lo, dtype=torch.float32, device="cuda")
        log_b = torch.full((n_rows, hi - lo), float("nan"), dtype=torch.float32, device="cuda")
        sv.sv_action_head_argmax(cfg, g, w, x, n_rows, lo, hi, tok_a, log_a, ws)
        sv.sv_action_head_argmax_noalloc(cfg, g, w, x, n_rows, lo, hi, tok_b, log_b)
        torch.cuda.synchronize()
        assert np.array_equal(tok_a.cpu().numpy(), tok_b.cpu().numpy())
        assert np.array_equal(log_a.cpu().numpy(), log_b.cpu().numpy())
        assert (tok_b.cpu().numpy() >= lo).all()


def test_head_without_allocation_rejects_what_its_scratch_cannot_hold():
    cfg = sv.model_cfg("bf16", 4096, 32, 128, 11008, 32000, 1e-5, 10000.0)
    one = torch.zeros(1, dtype=torch.uint8, device="cuda")
    import ctypes as C
    lib = sv.lib()
    p = C.c_void_p(one.data_ptr())
    assert lib.sv_action_head_argmax_noalloc(C.byref(cfg), p, p, p, 65, 31744, 32000, p, None, None) == sv.SV_ERR_WORKSPACE
    assert lib.sv_action_head_argmax_noalloc(C.byref(cfg), p, p, p, 60, 0, 32000, p, None, None) == sv.SV_ERR_WORKSPACE
    assert lib.sv_action_head_argmax_noalloc(C.byref(cfg), p, p, None, 60, 31744, 32000, p, None, None) == sv.SV_ERR_NULL
