"""bmx_binary_fc_static, the fully connected entry point that allocates nothing (its packed
activations live in an array inside the library's device code), against bmx_binary_fc with a
caller-provided workspace: same integers, same floats, on two calls in a row, the second with a
smaller input, so that what the first call left in the shared array is there to be misread."""
import numpy as np
import pytest
import torch

from paper_1705_09864_amd import binding as B

pytestmark = pytest.mark.gpu


def _layer(seed, batch, fin, fout):
    g = torch.Generator(device="cuda").manual_seed(seed)
    x = torch.randn((batch, fin), generator=g, device="cuda", dtype=torch.float32)
    w = torch.rand((fout, fin), generator=g, device="cuda", dtype=torch.float32) * 2 - 1
    return x, B.binarize_pack(w, 1), B.alpha_mean_abs(w)


def test_static_scratch_fc_matches_workspace_fc():
    # the first call fills far more of the array than the second reads; the second has a K tail
    # inside a word and rows that end inside a padded chunk
    # (very small layers take a one-launch kernel that packs into LDS and never touches the array:
    # first with that kernel switched off, so that every call goes through the array, then as is)
    for small_off in (1, 0):
        assert B.lib().bmx_tune_set(15, small_off) == 0
        try:
            for seed, (batch, fin, fout) in enumerate([(200, 5000, 300), (37, 1000, 70), (256, 9216, 512), (3, 65, 5)]):
                x, Wp, alpha = _layer(100 + seed, batch, fin, fout)
                want_f = B.binary_fc(x, Wp, alpha=alpha)
                want_i = B.binary_fc(x, Wp, integer_out=True)
                got_f = torch.full((batch, fout), float("nan"), dtype=torch.float32, device="cuda")
                got_i = torch.full((batch, fout), -7, dtype=torch.int32, device="cuda")
                B.binary_fc_static(x, Wp, alpha=alpha, out=got_f)
                if small_off:
                    assert "fc_small" not in B.last_kernel()
                B.binary_fc_static(x, Wp, integer_out=True, out=got_i)
                torch.cuda.synchronize()
                assert torch.equal(got_i, want_i), (batch, fin, fout)
                assert torch.equal(got_f, want_f), (batch, fin, fout)          # one fp32 multiply of equal integers
        finally:
            B.lib().bmx_tune_set(15, 0)


def test_static_scratch_limit_and_errors():
    L = B.lib()
    P = 0x7F0000001000
    # 4 MiB of packed activations: 4096 rows of 8192 features fit exactly, one more row does not
    assert B.workspace_bytes(B.OP_BINARY_FC, (4096, 8192, 8)) == 4 << 20
    assert L.bmx_binary_fc_static(P, 8192, P, 128, None, 4097, 8192, 8, None, P, 8, None) == -6
    assert L.bmx_binary_fc_static(None, 8192, P, 128, None, 4, 8192, 8, None, P, 8, None) == -1
    assert L.bmx_binary_fc_static(P, 8192, P, 128, None, 0, 8192, 8, None, P, 8, None) == 0
