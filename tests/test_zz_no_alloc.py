"""The preconditioning entry point that allocates nothing (its intermediate lives in a buffer inside the
library image) against the ordinary entry point with a caller workspace: same kernels, same inputs, so the
outputs must agree bit for bit.  Two calls in a row, the second on a smaller layer (the buffer keeps the first
call's contents), then an over-sized layer, which must be rejected before any launch."""
import numpy as np
import pytest
import torch

import paper_2206_15143_amd as kf

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(desc, seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    dA, dG = kf.kfac_dim_A(desc), kf.kfac_dim_G(desc)
    def sym(n):
        m = torch.randn((n, n), generator=g, device=DEV)
        return ((m + m.T) * 0.5).contiguous()
    return sym(dA), sym(dG), torch.randn((dG, dA), generator=g, device=DEV)


def test_static_scratch_preconditioning_matches_the_workspace_entry_point():
    big = kf.LayerDesc.conv2d(64, 160, 3, 1, 1)        # d_A 577, d_G 160: wave-unit GEMM path
    small = kf.LayerDesc.linear(64, 32)                # d_A 65, d_G 32: small-tile path
    for k, desc in enumerate((big, small)):
        A_inv, G_inv, grad = _case(desc, 77 + k)
        ref = torch.full_like(grad, float("nan"))
        ws = torch.empty(kf.kfac_workspace_bytes(desc, 8, 8, 8), dtype=torch.uint8, device=DEV)
        kf.kfac_precondition(desc, A_inv, G_inv, grad, ref, ws)
        out = torch.full_like(grad, float("nan"))
        kf.kfac_precondition_static(desc, A_inv, G_inv, grad, out)
        torch.cuda.synchronize()
        assert torch.isfinite(ref).all()
        assert torch.equal(out, ref), f"call {k}: static-scratch result differs from the workspace result"
        # and against the definition, P = G_inv grad A_inv, in fp64 on the host
        want = G_inv.double().cpu().numpy() @ grad.double().cpu().numpy() @ A_inv.double().cpu().numpy()
        err = np.linalg.norm(out.double().cpu().numpy() - want) / np.linalg.norm(want)
        assert err < 1e-5, err


def test_static_scratch_rejects_a_layer_beyond_its_buffer():
    desc = kf.LayerDesc.linear(4096, 4096)             # 4097 * 4096 * 4 bytes = 64 MiB > 32 MiB
    assert kf.kfac_dim_A(desc) * kf.kfac_dim_G(desc) * 4 > kf.KFAC_STATIC_SCRATCH_BYTES
    x = torch.zeros(16, device=DEV)                    # never read: the size check comes first
    with pytest.raises(kf.KfacError) as e:
        kf.kfac_precondition_static(desc, x, x, x, x)
    assert e.value.status == 8
