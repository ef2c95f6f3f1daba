"""The allocation-free decode entry point against the workspace-taking one it is a variant of.

morph_linear_w4a16_noalloc runs the same kernel with its hand-over arrays in the library's own
device array; its output must equal morph_linear_w4a16's bit for bit (the bar for this path: the
same numbers added in the same order), and the latter is held to the oracle elsewhere.  Two calls in
a row, the second on a smaller problem, share the array: the second must not be disturbed by what the
first left there.
"""
import numpy as np
import pytest
import torch

from paper_2506_02006_amd import binding as B
from paper_2506_02006_amd import synth

pytestmark = pytest.mark.gpu


def _record(seed, K, N):
    W = synth.weights(seed, K, N)
    return B.quantize_layer(torch.from_numpy(W).cuda())


def _pair(M, K, N, rec, seed):
    """(no-alloc output, workspace output) as uint16 arrays."""
    x = torch.from_numpy(synth.activations(seed, M, K)).cuda()
    y_ws = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    y_na = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    ws = B.new_workspace(B.workspace_bytes(B.KIND_W4A16, M, K, N))
    B.linear_w4a16(x, rec[0], rec[1], rec[2], ws, out=y_ws)
    B.linear_w4a16_noalloc(x, rec[0], rec[1], rec[2], out=y_na)
    torch.cuda.synchronize()
    return y_na.cpu().numpy().view(np.uint16), y_ws.cpu().numpy().view(np.uint16)


def test_noalloc_equals_workspace_call_twice_in_a_row():
    B.lib()
    assert B.lib().morph_noalloc_scratch_bytes() <= 8 << 20
    big = _record(11, 4096, 4096)          # 16 column tiles, K split 16 ways: the hand-over is used
    small = _record(12, 1024, 1288)        # ragged last tile, fewer splits
    # first call: the large problem; second call, right behind it: the smaller one
    for M, (K, N, rec) in ((16, (4096, 4096, big)), (3, (1024, 1288, small))):
        y_na, y_ws = _pair(M, K, N, rec, seed=20 + M)
        assert np.array_equal(y_na, y_ws), f"M={M} K={K} N={N}: {(y_na != y_ws).sum()} of {y_na.size} outputs differ"
        assert not np.isnan(y_na.view(np.float16)).any()
    # and again in the other order, M = 1 (the one-row kernel variant)
    for M, (K, N, rec) in ((1, (1024, 1288, small)), (1, (4096, 4096, big))):
        y_na, y_ws = _pair(M, K, N, rec, seed=30 + M)
        assert np.array_equal(y_na, y_ws)


def test_noalloc_against_oracle(oracle):
    K, N, M = 2048, 2056, 5
    W = synth.weights(13, K, N)
    qw, sc, qz = oracle.quantize_w4(W)
    x = synth.activations(14, M, K)
    rec = (torch.from_numpy(qw.view(np.int32)).cuda(), torch.from_numpy(sc).cuda(), torch.from_numpy(qz.view(np.int32)).cuda())
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    B.linear_w4a16_noalloc(torch.from_numpy(x).cuda(), *rec, out=y)
    err = oracle.error_metric(y.cpu().numpy(), oracle.linear_w4a16(x, qw, sc, qz))["err"]
    assert err <= 5e-3, err


def test_noalloc_rejects_what_it_cannot_hold():
    rec = _record(15, 256, 512)
    x = torch.zeros((17, 256), dtype=torch.float16, device="cuda")
    y = torch.empty((17, 512), dtype=torch.float16, device="cuda")
    with pytest.raises(B.MorphError) as e:
        B.linear_w4a16_noalloc(x, rec[0], rec[1], rec[2], out=y)
    assert e.value.status == 5            # MORPH_ERR_UNSUPPORTED: more than 16 rows
