"""The allocation-free entry point, through the C ABI, against the entry point it is a variant of.

ff_predict_static keeps the predictor's scratch in a fixed array inside the library instead of the
caller's workspace.  Two calls in a row, the second on a smaller input (the array keeps the first
call's bytes): lists and scores must equal ff_predict's bit for bit, and the oracle's lists."""
import numpy as np
import pytest
import torch

from oracle import ff_oracle as O
from paper_2602_00397_amd import binding as B
from paper_2602_00397_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(shp, n_tokens, with_q):
    lt = W.make_layer(shp, with_q_pred=with_q)
    x_bits = W.make_hidden(shp, n_tokens=n_tokens)
    x = B.to_device_bf16(x_bits, DEV)
    dev, pred, _, _ = B.make_structs(lt, DEV)
    shape = B.Shape(shp.d_model, shp.d_ffn, n_tokens, shp.block, shp.r_pred, shp.r_comp)
    return lt, x_bits, x, dev, pred, shape


def test_static_scratch_predict_equals_predict_twice_in_a_row():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    ref_ctx = B.Context(0)
    ctx = B.Context(0)            # never given a workspace: the entry point under test must not need one
    try:
        # first the Llama-3.1-8B layer (8 MiB of the array, softmax pooling so that every piece of
        # scratch is in use), then the tiny layer with unequal K and a ragged last block
        calls = ((W.CONFIGS["c2"], 8192, None, True), (W.CONFIGS["c0"], 230, [688, 345, 101, 1], False))
        for shp, T, ks, with_q in calls:
            lt, x_bits, x, dev, pred, shape = _inputs(shp, T, with_q)
            nB = -(-T // shp.block)
            ks = ks or [O.k_from_sparsity(shp.d_ffn, 0.5)] * nB
            k_stride = max(ks) + 8
            ref_ctx.ensure_workspace(shape, max(ks))
            out = {}
            for name, fn in (("workspace", ref_ctx.predict), ("static", ctx.predict_static)):
                idx = torch.full((nB, k_stride), -7, dtype=torch.int32, device=DEV)
                sc = torch.full((nB, shp.d_ffn), float("nan"), dtype=torch.float64, device=DEV)
                fn(shape, x, pred, ks, k_stride, idx, sc)
                torch.cuda.synchronize()
                out[name] = (idx, sc)
            assert torch.equal(out["static"][0], out["workspace"][0]), f"{shp.name}: lists differ from ff_predict's"
            assert torch.equal(out["static"][1].view(torch.int64), out["workspace"][1].view(torch.int64)), f"{shp.name}: scores differ"
            # without the optional scores output the scores live in the array as well
            idx2 = torch.full((nB, k_stride), -7, dtype=torch.int32, device=DEV)
            ctx.predict_static(shape, x, pred, ks, k_stride, idx2, None)
            assert torch.equal(idx2, out["workspace"][0])
            f = W.bf16_to_f32
            q = f(lt.q_pred) if lt.q_pred is not None else None
            ref = O.fastforward_layer(f(x_bits), None, None, None, f(lt.w1), f(lt.w2), shp.block, ks, q_pred=q, compute_ffn=False)
            got = idx2.cpu().numpy()
            for b in range(nB):
                np.testing.assert_array_equal(got[b, :ks[b]], ref.indices[b], err_msg=f"{shp.name} block {b}")
                assert (got[b, ks[b]:] == -1).all()
        # a shape beyond the array is refused on the host (the Llama-3.1-8B layer with 512 blocks)
        big = B.Shape(4096, 14336, 512 * 128, 128, 128, 64)
        with pytest.raises(B.FFError) as e:
            ctx.predict_static(big, x, pred, [7168] * 512, 7168, idx2, None)
        assert e.value.status == 5
    finally:
        torch.cuda.synchronize()
        ctx.close()
        ref_ctx.close()
