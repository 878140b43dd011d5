"""spmoe_moe_layer_resident_static (the entry point that allocates nothing: its intermediates live in a fixed
device array) against spmoe_moe_verify_layer with every expert resident: same kernels, same summation order, so
the outputs must be bit-identical; and both within the parity bar of the CPU oracle."""
import numpy as np
import pytest

import spmoe_inputs as si
from parity_util import REL_L2_BF16, REL_L2_F32, check_elements, ELEM_C_BF16, ELEM_C_F32, oracle_layer

pytestmark = pytest.mark.gpu


def _case(wl, T_max):
    import torch
    from paper_2510_10302_amd import workload as W
    L = W.Loaded(wl, W.make_config(wl, max_tokens=T_max))
    gate = torch.from_numpy(wl.gate[0].view(np.int16) if wl.dtype == "bf16" else wl.gate[0]).cuda()
    cfg = L.cfg
    blobs = []
    import paper_2510_10302_amd as sp
    for e in range(wl.E):
        blobs.append(torch.from_numpy(sp.pack_expert(cfg, *wl.expert(0, e))).cuda())
    for s in range(wl.n_shared):
        blobs.append(torch.from_numpy(sp.pack_expert(cfg, *wl.shared[0][s])).cuda())
    return L, gate, blobs


@pytest.mark.parametrize("d,f,E,k,shared,dtype,T_first,T_second", [
    (512, 1408, 16, 2, 1, "bf16", 32, 5),      # second call smaller: the array still holds the first call's data
    (4096, 14336, 8, 2, 0, "bf16", 8, 3),      # benchmark configuration 2's layer
    (256, 416, 8, 2, 2, "f32", 11, 4),         # fp32-weight kernels
])
def test_static_scratch_entry_point_matches_the_context_one(d, f, E, k, shared, dtype, T_first, T_second, oracle32):
    import torch
    import paper_2510_10302_amd as sp
    from paper_2510_10302_amd import workload as W
    wl = W.Workload(d=d, f=f, E=E, k=k, shared=shared, dtype=dtype, layers=1, seed=77, gate_std=0.05, std=0.05)
    L, gate, blobs = _case(wl, max(T_first, T_second))
    tol, c = (REL_L2_BF16, ELEM_C_BF16) if dtype == "bf16" else (REL_L2_F32, ELEM_C_F32)
    for call, T in enumerate((T_first, T_second, T_first)):
        x = si.hidden(77, T, d, iteration=call)
        dx = torch.from_numpy(x).cuda()
        want = torch.full((T, d), float("nan"), device="cuda")
        L.ctx.moe_verify_layer(0, dx, want)
        L.ctx.sync()
        got = torch.full((T, d), float("nan"), device="cuda")
        sp.moe_layer_resident_static(L.cfg, gate, blobs, dx, got)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int32), want.view(torch.int32)), (call, T)
        ref = oracle_layer(oracle32, wl, 0, x)
        check_elements(got.cpu().numpy(), ref["out"], range(T), c, tol)
    L.close()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import torch
    import paper_2510_10302_amd as sp
    # A = 32 * (8 + 8) = 512 assignments of f = 16384 bf16 values alone are 16 MiB: more than the array holds
    cfg = sp.Config(n_layers=1, d_model=1024, d_ff=16384, n_experts=8, top_k=8, n_shared=8, max_tokens=32)
    x = torch.zeros((32, 1024), device="cuda")
    out = torch.zeros((32, 1024), device="cuda")
    gate = torch.zeros((8, 1024), dtype=torch.int16, device="cuda")
    blob = torch.zeros(16, dtype=torch.uint8, device="cuda")     # never read: the call must fail before any launch
    with pytest.raises(sp.SpmoeError) as e:
        sp.moe_layer_resident_static(cfg, gate, [blob] * 16, x, out)
    assert e.value.status_name == "SPMOE_ERANGE"
    sp.moe_layer_resident_static(cfg, gate, [blob] * 16, x[:0], out[:0])      # an empty batch is a no-op
    cfg33 = sp.Config(n_layers=1, d_model=1024, d_ff=64, n_experts=8, top_k=2, n_shared=0, max_tokens=4)
    with pytest.raises(sp.SpmoeError) as e:
        sp.moe_layer_resident_static(cfg33, gate, [blob] * 8, x[:5], out[:5])    # T > max_tokens
    assert e.value.status_name == "SPMOE_ERANGE"
    torch.cuda.synchronize()
