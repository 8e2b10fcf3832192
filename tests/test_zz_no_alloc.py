"""zipvl_decode_attn_static (the entry point that allocates nothing) against zipvl_decode_attn, through
the C ABI: two calls in a row on the library's one scratch array, the second with a smaller input (the size
limit is checked without a GPU in test_host_abi.py).  Collected last on purpose (file name): a failure here must not hide the other GPU tests."""
import sys

import numpy as np
import pytest
import torch

import paper_2410_08584_amd as z
from oracle import zipvl_oracle as oz

DEV = "cuda:0"


def _case(B, Hq, Hkv, cap, d, lens, seed):
    units = B * Hkv
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    Kc = torch.randn((units, cap, d), generator=g, device=DEV).to(torch.bfloat16)
    Vc = torch.randn((units, cap, d), generator=g, device=DEV).to(torch.bfloat16)
    q = (2 * torch.randn((B * Hq, d), generator=g, device=DEV)).to(torch.bfloat16)
    ln = torch.tensor(lens, dtype=torch.int32, device=DEV)
    return q, Kc, Vc, ln


@pytest.mark.gpu
def test_decode_attn_static_matches_decode_attn_on_two_calls_in_a_row():
    scale = 1.0 / np.sqrt(128.0)
    worst = 0.0
    # first call: many splits per unit and long rows; second call: fewer units, shorter rows, other group size
    for (B, Hq, Hkv, cap, lens, seed) in ((2, 8, 2, 6000, [5999, 1, 3000, 257], 1), (1, 3, 3, 700, [700, 0, 65], 2)):
        print(f"decode_attn_static B={B} Hq={Hq} Hkv={Hkv} cap={cap}", flush=True); sys.stdout.flush()
        q, Kc, Vc, ln = _case(B, Hq, Hkv, cap, 128, lens, seed)
        o_ref = z.zipvl_decode_attn(q, Kc, Vc, ln, scale, B=B, Hq=Hq, Hkv=Hkv)
        o = torch.full((B * Hq, 128), 7.0, dtype=torch.bfloat16, device=DEV)
        z.zipvl_decode_attn_static(q, Kc, Vc, ln, scale, B=B, Hq=Hq, Hkv=Hkv, o=o)
        torch.cuda.synchronize()
        assert torch.equal(o, o_ref), "same kernels, same split: the outputs must be identical"
        # and both meet the oracle (Eq. (5)) within the attention tolerance
        G = Hq // Hkv
        oh = o.float().cpu().numpy().astype(np.float64)
        for bh in range(B * Hq):
            b, h = divmod(bh, Hq)
            u = b * Hkv + h // G
            if lens[u] == 0:
                assert not oh[bh].any()
                continue
            ref = oz.decode_attention(q[bh].float().cpu().numpy(), Kc[u].float().cpu().numpy(), Vc[u].float().cpu().numpy(), lens[u], scale)
            worst = max(worst, np.abs(oh[bh] - ref).max())
    assert worst <= 2e-2, worst
