"""tt_fc_forward_static (the execute call whose scratch is part of the library, for callers that cannot allocate)
against tt_fc_forward with a caller's workspace: same bits, on two calls in a row of which the second is smaller, with
forms that leave partial sums and converted operands in the scratch; and against the oracle."""
import numpy as np
import pytest
import torch

import paper_1805_04170_amd as tt
from oracle import layers as ly
from oracle import tiling as tl
from synthetic import bf16_bits_to_f64, normal_f32, to_bf16_bits

import gpu_util
import test_gpu_fc
from gpu_util import alloc_shards, shards_to_dev, shards_to_np

pytestmark = pytest.mark.gpu

# (batch, n_in, n_out, k, tX, tW, tY, forms): the first is the larger; both cut the reduction dimension, so the
# scratch holds fp32 partial sums (and, where stored and aligned block shapes differ, converted operands)
CASES = [
    (128, 1024, 768, 3, "RCr", "CRC", "CrR", "313"),
    (64, 256, 192, 2, "CC", "RR", "rC", "33"),
]


def _run_both(case, seed, relu):
    b, ni, no, k, tX, tW, tY, f = case
    lay = tt.layer("fc", "relu" if relu else "none", ni, no)
    X = to_bf16_bits(normal_f32(seed, 0, (b, ni), 1.0))
    W = to_bf16_bits(normal_f32(seed, 1, (ni, no), 0.05))
    Xs, Ws = shards_to_dev(X, tX, True), shards_to_dev(W, tW, True)
    need = tt.tt_fc_workspace_bytes(lay, b, k, "bf16", tt.TT_OP_FWD, tX, tW, tY, forms_a=f)
    assert 0 < need <= tt.TT_STATIC_SCRATCH_BYTES
    ws = test_gpu_fc.workspace(need)
    ref = alloc_shards(b, no, tY, torch.bfloat16, fill=float("nan"))
    tt.tt_fc_forward(lay, b, k, "bf16", tX, tW, tY, f, Xs, Ws, ref, ws)
    got = alloc_shards(b, no, tY, torch.bfloat16, fill=float("nan"))
    tt.tt_fc_forward_static(lay, b, k, "bf16", tX, tW, tY, f, Xs, Ws, got)
    torch.cuda.synchronize()
    for g, r in zip(got, ref):
        assert torch.equal(g.view(torch.int16), r.view(torch.int16)), case
    Xf, Wf = bf16_bits_to_f64(X), bf16_bits_to_f64(W)
    want = ly.fc_forward(Xf, Wf, relu)
    have = bf16_bits_to_f64(tl.untile(shards_to_np(got), tY, b, no))
    assert np.all(np.abs(have - want) <= 1e-2 * ly.abs_product(Xf, Wf)), case      # the bf16 contraction bound


def test_static_scratch_forward_twice_second_smaller():
    _run_both(CASES[0], 301, True)
    _run_both(CASES[1], 302, False)
    _run_both(CASES[0], 303, False)      # and the large one again, over what the small one left


def test_static_scratch_refuses_what_does_not_fit():
    # 16 partial sums of 2048 x 4096 fp32 (512 MiB) cannot come from the library's array
    b, ni, no, k = 2048, 4096, 4096, 4
    lay = tt.layer("fc", "none", ni, no)
    need = tt.tt_fc_workspace_bytes(lay, b, k, "bf16", tt.TT_OP_FWD, "CCCC", "RRRR", "RRRR", forms_a="3333")
    assert need > tt.TT_STATIC_SCRATCH_BYTES
    dummy = torch.zeros(16, dtype=torch.bfloat16, device=gpu_util.DEV)
    with pytest.raises(tt.TilingError) as e:
        tt.tt_fc_forward_static(lay, b, k, "bf16", "CCCC", "RRRR", "RRRR", "3333", [dummy] * 16, [dummy] * 16, [dummy] * 16)
    assert e.value.status == 6      # TT_EWORKSPACE, before anything is launched
