"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before launching
anything."""
import ctypes
import os
import re

import pytest

import paper_2604_16429_amd as M
from paper_2604_16429_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def good(**kw):
    base = dict(batch=1, heads=2, grid_h=32, grid_w=64, block_h=8, block_w=8,
                head_dim=32, n_select=4, dtype=binding.F32)
    base.update(kw)
    return M.Params(**base)


def test_library_exports_every_declared_symbol():
    lib = M.load_library()
    header = open(os.path.join(ROOT, "include", "mosaic_bsa.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(mosaic_bsa_[a-z_]+)\s*\(", header))
    assert {"mosaic_bsa_select", "mosaic_bsa_fwd", "mosaic_bsa_bwd",
            "mosaic_bsa_workspace_bytes", "mosaic_bsa_strerror",
            "mosaic_bsa_fwd_three_branch",
            "mosaic_bsa_three_branch_workspace_bytes"} <= names
    for name in names:
        assert hasattr(lib, name), name
    # the Python binding carries the same names
    for name in names:
        assert callable(getattr(M, name)), name


def test_struct_layout_matches_header():
    assert ctypes.sizeof(binding._CParams) == 44


def test_workspace_bytes():
    p = good()
    m = 32
    per = (1 * 2 * m * 32 * 4 + 255) // 256 * 256
    # pooled q, pooled k, and the ranking's interleaved copy of pooled k
    assert M.mosaic_bsa_workspace_bytes(p, binding.OP_SELECT) == 3 * per
    assert M.mosaic_bsa_workspace_bytes(p, binding.OP_FWD) == 0
    # delta and lse * log2(e), fp32 [B, heads, N] each
    # delta + lse in base 2 (fp32 per token) + one bit per (slice, key block, query block)
    assert M.mosaic_bsa_workspace_bytes(p, binding.OP_BWD) == 2 * (1 * 2 * 2048 * 4) + 2 * 32 * 4
    assert M.mosaic_bsa_workspace_bytes(good(head_dim=48), binding.OP_SELECT) == 0


@pytest.mark.parametrize("kw,code", [
    (dict(batch=0), -2), (dict(grid_h=30), -2), (dict(grid_w=60), -2),
    (dict(block_h=0), -2), (dict(block_h=32, block_w=64), -2),   # b > 1024
    (dict(n_select=-1), -3), (dict(n_select=32), -3),
    (dict(head_dim=48), -4), (dict(dtype=7), -5),
    (dict(kv_heads=3), -2), (dict(kv_heads=4), -2), (dict(kv_heads=-1), -2),   # heads = 2
])
def test_bad_params_are_rejected_before_any_launch(kw, code):
    p = good(**kw)
    fake = 0x1000      # never dereferenced: validation fails first
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select(p, fake, fake, fake, fake, stream=0, workspace_bytes=1 << 30)
    assert e.value.code == code
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_fwd(p, fake, fake, fake, fake, fake, None, None, stream=0)
    assert e.value.code == code
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_bwd(p, *([fake] * 10), fake, stream=0, workspace_bytes=1 << 40)
    assert e.value.code == code


def test_null_alignment_and_workspace_errors():
    p = good()
    fake = 0x1000
    ws = M.mosaic_bsa_workspace_bytes(p, binding.OP_SELECT)
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select(p, None, fake, fake, fake, stream=0, workspace_bytes=ws)
    assert e.value.code == -1
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select(p, fake, fake, None, fake, stream=0, workspace_bytes=ws)
    assert e.value.code == -1
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select(p, fake + 4, fake, fake, fake, stream=0, workspace_bytes=ws)
    assert e.value.code == -7
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select(p, fake, fake, fake, fake, stream=0, workspace_bytes=ws - 1)
    assert e.value.code == -6
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select(p, fake, fake, fake, None, stream=0, workspace_bytes=0)
    assert e.value.code == -6
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_fwd(p, fake, fake, None, fake, fake, None, None, stream=0)
    assert e.value.code == -1
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_fwd(p, fake, fake, fake + 8, fake, fake, None, None, stream=0)
    assert e.value.code == -7
    wb = M.mosaic_bsa_workspace_bytes(p, binding.OP_BWD)
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_bwd(p, *([fake] * 5), None, *([fake] * 4), fake, stream=0, workspace_bytes=wb)
    assert e.value.code == -1
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_bwd(p, *([fake] * 10), fake, stream=0, workspace_bytes=wb - 1)
    assert e.value.code == -6
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_bwd(p, *([fake] * 9), fake + 2, fake, stream=0, workspace_bytes=wb)
    assert e.value.code == -7


def test_more_blocks_than_the_ranking_holds_are_rejected_on_the_host():
    """The scores of one query block must fit a workgroup's LDS (36,864 words):
    m = 36,864 is accepted (a missing workspace is what is reported), the next
    larger grid of 1 x 1 tiles is a shape error, before anything is launched."""
    fake = 0x1000
    ok = good(heads=1, grid_h=192, grid_w=192, block_h=1, block_w=1, n_select=3)
    assert M.mosaic_bsa_workspace_bytes(ok, binding.OP_SELECT) > 0
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select(ok, fake, fake, fake, fake, stream=0, workspace_bytes=0)
    assert e.value.code == -6
    big = good(heads=1, grid_h=193, grid_w=192, block_h=1, block_w=1, n_select=3)
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select(big, fake, fake, fake, fake, stream=0, workspace_bytes=1 << 40)
    assert e.value.code == -2
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select_static(big, fake, fake, fake, stream=0)
    assert e.value.code == -2


def test_strerror_covers_all_codes():
    texts = {M.mosaic_bsa_strerror(c) for c in range(0, -10, -1)}
    assert len(texts) == 10 and "unknown error code" not in texts
    assert M.mosaic_bsa_strerror(-99) == "unknown error code"


def test_three_branch_arguments_are_checked_on_the_host():
    p = good(n_select=32)        # n = m is allowed here: the own block is a candidate
    fake = 0x1000
    m, N, D = 32, 2048, 32

    def part(nbytes):
        return (nbytes + 255) // 256 * 256
    expect = (5 * part(2 * m * D * 4) + part(2 * m * 3 * 4) + 2 * part(2 * N * D * 4)
              + 2 * part(2 * N * 4))            # the two branches' log-sum-exps
    assert M.mosaic_bsa_three_branch_workspace_bytes(p, 2, 2) == expect
    assert M.mosaic_bsa_three_branch_workspace_bytes(p, 3, 2) == 0      # 4 x 8 tiles
    assert M.mosaic_bsa_three_branch_workspace_bytes(good(n_select=0), 1, 1) == 0
    args = [fake] * 7
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_fwd_three_branch(good(n_select=33), 1, 1, *args, stream=0,
                                      workspace_bytes=1 << 30)
    assert e.value.code == -3
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_fwd_three_branch(p, 2, 3, *args, stream=0, workspace_bytes=1 << 30)
    assert e.value.code == -2
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_fwd_three_branch(p, 2, 2, fake, fake, fake, None, fake, fake, fake,
                                      stream=0, workspace_bytes=1 << 30)
    assert e.value.code == -1
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_fwd_three_branch(p, 2, 2, *args, stream=0, workspace_bytes=expect - 1)
    assert e.value.code == -6


def test_three_branch_backward_arguments_are_checked_on_the_host():
    p = good(n_select=4)
    fake = 0x1000
    nbytes = M.mosaic_bsa_three_branch_bwd_workspace_bytes(p, 2, 2)
    assert nbytes > 0 and nbytes % 256 == 0
    assert M.mosaic_bsa_three_branch_bwd_workspace_bytes(p, 3, 2) == 0
    assert M.mosaic_bsa_three_branch_bwd_workspace_bytes(good(n_select=0), 2, 2) == 0
    args = [fake] * 11
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_bwd_three_branch(p, 2, 2, *args, fake, stream=0, workspace_bytes=nbytes - 1)
    assert e.value.code == -6
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_bwd_three_branch(p, 2, 5, *args, fake, stream=0, workspace_bytes=nbytes)
    assert e.value.code == -2
    bad = list(args)
    bad[6] = None                       # the forward's workspace
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_bwd_three_branch(p, 2, 2, *bad, fake, stream=0, workspace_bytes=nbytes)
    assert e.value.code == -1
    bad = list(args)
    bad[7] = fake + 8                   # dq misaligned
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_bwd_three_branch(p, 2, 2, *bad, fake, stream=0, workspace_bytes=nbytes)
    assert e.value.code == -7


def test_probe_arguments_are_checked_on_the_host():
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_probe_mfma(None, 4, 10, stream=0)
    assert e.value.code == -1
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_probe_mfma(0x1000, 0, 10, stream=0)
    assert e.value.code == -2


def test_selection_checker_arguments_are_checked_on_the_host():
    p = good()
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_check_selection(p, 0x1000, False, None, stream=0)
    assert e.value.code == -1
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_check_selection(good(n_select=32), 0x1000, False, 0x1000, stream=0)
    assert e.value.code == -3                           # n = m only with the own block allowed


def test_static_selection_checks_arguments_and_size_on_the_host():
    """The entry point without a workspace argument: argument errors and a
    problem that needs more than the library's fixed array are reported before
    any GPU call is made."""
    fake = 4096
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select_static(good(), None, fake, fake, stream=0)
    assert e.value.code == -1
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select_static(good(), fake + 4, fake, fake, stream=0)
    assert e.value.code == -7
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select_static(good(head_dim=48), fake, fake, fake, stream=0)
    assert e.value.code == -4
    big = good(batch=24, heads=16, grid_h=120, grid_w=240, head_dim=64, n_select=16,
               dtype=binding.BF16)
    assert M.mosaic_bsa_workspace_bytes(big, binding.OP_SELECT) > 32 << 20
    with pytest.raises(M.BsaError) as e:
        M.mosaic_bsa_select_static(big, fake, fake, fake, stream=0)
    assert e.value.code == -6
