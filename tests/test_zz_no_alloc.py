"""The selection entry point that allocates nothing (its workspace is a fixed
array inside the library) against mosaic_bsa_select, through the C ABI: two
calls in a row on one stream, the second with a smaller input, each compared
bit for bit with the result of the entry point that takes a caller workspace;
and the rejection of a problem that does not fit the fixed array."""
import numpy as np
import pytest
import torch

from inputs.fields import round_to_bf16
from tests.helpers import rand_qkv, shape_ns

pytestmark = pytest.mark.gpu


def test_static_selection_equals_the_workspace_form_on_two_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2604_16429_amd as M
    from paper_2604_16429_amd import binding
    from tests import gpu_util as G

    shapes = [shape_ns(2, 4, 120, 240, 8, 8, 64, 16, "bf16"),     # m = 450, 8 slices
              shape_ns(1, 2, 32, 64, 8, 8, 64, 4, "bf16")]        # smaller: m = 32, 2 slices
    inputs, expect = [], []
    for t, cfg in enumerate(shapes):
        q, k, _ = (round_to_bf16(x) for x in rand_qkv(cfg, 4100 + t))
        q_d, k_d = G.to_dev(q, cfg), G.to_dev(k, cfg)
        inputs.append((cfg, q_d, k_d))
        expect.append(G.select_dev(cfg, q_d, k_d))               # caller workspace
    torch.cuda.synchronize()
    got = []
    for cfg, q_d, k_d in inputs:                                  # back to back, nothing between
        prm = G.params_of(cfg)
        assert M.mosaic_bsa_workspace_bytes(prm, binding.OP_SELECT) <= 32 << 20
        idx = torch.full((cfg.batch, cfg.heads, cfg.n_blocks, cfg.n_select), -1,
                         dtype=torch.int32, device="cuda")
        M.mosaic_bsa_select_static(prm, q_d, k_d, idx)
        got.append(idx)
    torch.cuda.synchronize()
    for a, b in zip(got, expect):
        assert torch.equal(a, b)
    # once more in the other order: the array keeps the last call's contents
    cfg, q_d, k_d = inputs[0]
    idx = torch.full_like(expect[0], -1)
    M.mosaic_bsa_select_static(G.params_of(cfg), q_d, k_d, idx)
    torch.cuda.synchronize()
    assert torch.equal(idx, expect[0])


def test_static_selection_rejects_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2604_16429_amd as M
    from paper_2604_16429_amd import binding
    from tests import gpu_util as G
    cfg = shape_ns(24, 16, 120, 240, 8, 8, 64, 16, "bf16")       # 132 MB of selection workspace
    prm = G.params_of(cfg)
    assert M.mosaic_bsa_workspace_bytes(prm, binding.OP_SELECT) > 32 << 20
    fake = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select_static(prm, fake, fake, fake)
    assert e.value.code == -6                                    # MOSAIC_BSA_ERR_WORKSPACE
