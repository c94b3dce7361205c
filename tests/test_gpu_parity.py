"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.

Bars (from the benchmark definition): selected indices bit-exact; FFN outputs
rel-RMS error <= 1e-2 and max-abs error <= 5e-2 (bf16 inputs, fp32 accumulate,
H rounded to bf16 once)."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import ff_oracle as O
from paper_2602_00397_amd import binding as B
from paper_2602_00397_amd import workloads as W

pytestmark = pytest.mark.gpu

REL_RMS_BAR = 1e-2
MAX_ABS_BAR = 5e-2
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = B.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def _f32(bits):
    return W.bf16_to_f32(bits)


def _errs(y_gpu: torch.Tensor, y_ref: np.ndarray):
    got = y_gpu.float().cpu().numpy().astype(np.float64)
    mask = ~np.isnan(y_ref).any(axis=1)
    d = got[mask] - y_ref[mask]
    rel_rms = float(np.sqrt((d * d).mean()) / np.sqrt((y_ref[mask] ** 2).mean()))
    return rel_rms, float(np.abs(d).max())


def _check_y(y_gpu, y_ref, what=""):
    """Both bars exactly as the benchmark states them, on the fp32 output (the accumulators as they
    are).  Rows of y_ref that hold NaN were not computed by the oracle and are skipped."""
    assert y_gpu.dtype == torch.float32, "the stated bars are held against the fp32 output"
    rel, mx = _errs(y_gpu, y_ref)
    print(f"[parity] {what}: rel_rms={rel:.3e} max_abs={mx:.3e}", flush=True)
    assert rel <= REL_RMS_BAR and mx <= MAX_ABS_BAR, (what, rel, mx)


def _check_bf16_storage(y_bf16, y_f32, y_ref=None, what=""):
    """The bf16 output of a call is the fp32 output of the same call (same tiles, same accumulators)
    stored with one round-to-nearest-even: bit for bit, every element, so storage needs no tolerance
    of its own.  Its raw distance to the oracle is printed for the record, not gated."""
    assert y_bf16.dtype == torch.bfloat16 and y_f32.dtype == torch.float32
    same = torch.equal(y_bf16.view(torch.int16), y_f32.to(torch.bfloat16).view(torch.int16))
    if y_ref is not None:
        rel, mx = _errs(y_bf16, y_ref)
        print(f"[parity] {what}: bf16 storage of the fp32 output, raw rel_rms={rel:.3e} max_abs={mx:.3e}", flush=True)
    assert same, f"{what}: bf16 output is not the round-to-nearest-even of the fp32 output"


def _check_both(c, ctx, idx, ks, y_ref, what, **kw):
    """fp32 output against the oracle at the stated bars, bf16 output bit-equal to its rounding."""
    y32 = c.gpu_sparse(ctx, idx, ks, out_f32=True, **kw)
    _check_y(y32, y_ref, what + " f32")
    _check_bf16_storage(c.gpu_sparse(ctx, idx, ks, out_f32=False, **kw), y32, y_ref, what)
    return y32


class Case:
    """A layer's inputs on the host (exact float32 values) and on the GPU."""

    def __init__(self, shp: W.Shape, n_tokens=None, with_q=False, seed=W.MASTER_SEED, layer=0):
        self.shp = shp
        T = shp.n_tokens if n_tokens is None else n_tokens
        self.T = T
        self.lt = W.make_layer(shp, layer=layer, seed=seed, with_q_pred=with_q)
        self.x_bits = W.make_hidden(shp, seed=seed, n_tokens=T)
        self.x = B.to_device_bf16(self.x_bits, DEV)
        self.dev, self.pred, self.w, self.comp = B.make_structs(self.lt, DEV)
        self.shape = B.Shape(shp.d_model, shp.d_ffn, T, shp.block, shp.r_pred, shp.r_comp)
        self.n_blocks = -(-T // shp.block)

    def host(self, name):
        return _f32(getattr(self.lt, name))

    def oracle_layer(self, ks, comp=True, blocks=None, compute_ffn=True, indices_override=None, act="silu"):
        q = _f32(self.lt.q_pred) if self.lt.q_pred is not None else None
        return O.fastforward_layer(
            _f32(self.x_bits), self.host("w_gate"), self.host("w_up"), self.host("w_down").T,
            self.host("w1"), self.host("w2"), self.shp.block, ks, q_pred=q,
            wc1=self.host("wc1").T if comp else None, wc2=self.host("wc2") if comp else None,
            comp_act=act, blocks=blocks, compute_ffn=compute_ffn, indices_override=indices_override)

    def gpu_predict(self, ctx, ks, k_stride=None, scores=False):
        k_stride = k_stride or max(ks)
        ctx.ensure_workspace(self.shape, max(ks))
        idx = torch.full((self.n_blocks, k_stride), -7, dtype=torch.int32, device=DEV)
        sc = torch.empty((self.n_blocks, self.shp.d_ffn), dtype=torch.float64, device=DEV) if scores else None
        ctx.predict(self.shape, self.x, self.pred, ks, k_stride, idx, sc)
        return idx, sc

    def gpu_sparse(self, ctx, idx, ks, comp=True, out_f32=False, act="silu"):
        ctx.ensure_workspace(self.shape, max(ks))
        y = torch.empty((self.T, self.shp.d_model), dtype=torch.float32 if out_f32 else torch.bfloat16, device=DEV)
        c = None
        if comp:
            c = B.Compensator(self.comp.wc1, self.comp.wc2, B.ACT[act])
        ctx.sparse_ffn(self.shape, self.x, self.w, c, idx, ks, idx.shape[1], y, B.OUT_F32 if out_f32 else B.OUT_BF16)
        return y


def _assert_indices(idx_gpu: torch.Tensor, ref_indices, ks):
    got = idx_gpu.cpu().numpy()
    for b, ref in enumerate(ref_indices):
        np.testing.assert_array_equal(got[b, :ks[b]], ref, err_msg=f"block {b}")
        assert (got[b, ks[b]:] == -1).all(), f"block {b}: tail not -1"


# ------------------------------------------------------------------ c0: everything, exhaustively

@pytest.fixture(scope="module")
def c0():
    return Case(W.CONFIGS["c0"])


def test_c0_predict_indices_and_scores(ctx, c0):
    k = O.k_from_sparsity(c0.shp.d_ffn, 0.5)
    ks = [k] * c0.n_blocks
    ref = c0.oracle_layer(ks, compute_ffn=False)
    idx, sc = c0.gpu_predict(ctx, ks, k_stride=k + 24, scores=True)
    _assert_indices(idx, ref.indices, ks)
    ref_s = np.stack([O.predictor_scores(_f32(c0.x_bits)[b * 64:(b + 1) * 64], None, c0.host("w1"), c0.host("w2"))
                      for b in range(c0.n_blocks)])
    np.testing.assert_allclose(sc.cpu().numpy(), ref_s, rtol=1e-12, atol=1e-14)
    assert min(ref.margins) > 1e-9 * max(ref.score_absmax)


@pytest.mark.parametrize("sparsity", [0.0, 0.25, 0.5, 0.75])
def test_c0_sparse_ffn_sweep(ctx, c0, sparsity):
    k = O.k_from_sparsity(c0.shp.d_ffn, sparsity)
    ks = [k] * c0.n_blocks
    ref = c0.oracle_layer(ks)
    idx, _ = c0.gpu_predict(ctx, ks)
    _assert_indices(idx, ref.indices, ks)
    _check_both(c0, ctx, idx, ks, ref.y, f"c0 s={sparsity}")


def test_c0_without_compensator_and_other_activations(ctx, c0):
    k = 344
    ks = [k] * c0.n_blocks
    idx, _ = c0.gpu_predict(ctx, ks)
    _check_y(c0.gpu_sparse(ctx, idx, ks, comp=False, out_f32=True), c0.oracle_layer(ks, comp=False).y, "c0 no comp")
    for act in ("relu", "identity"):
        _check_y(c0.gpu_sparse(ctx, idx, ks, act=act, out_f32=True), c0.oracle_layer(ks, act=act).y, f"c0 comp {act}")


def test_c0_dense_and_sparsity_zero(ctx, c0):
    ref = O.dense_ffn(_f32(c0.x_bits), c0.host("w_gate"), c0.host("w_up"), c0.host("w_down").T)
    ctx.ensure_workspace(c0.shape, c0.shp.d_ffn)
    y = torch.empty((c0.T, c0.shp.d_model), dtype=torch.float32, device=DEV)
    ctx.dense_ffn(c0.shape, c0.x, c0.w, y, B.OUT_F32)
    _check_y(y, ref, "c0 dense")
    # sparsity 0 without compensator is the dense FFN
    ks = [c0.shp.d_ffn] * c0.n_blocks
    idx, _ = c0.gpu_predict(ctx, ks)
    np.testing.assert_array_equal(idx.cpu().numpy(), np.tile(np.arange(c0.shp.d_ffn, dtype=np.int32), (c0.n_blocks, 1)))
    ys = c0.gpu_sparse(ctx, idx, ks, comp=False, out_f32=True)
    _check_y(ys, ref, "c0 sparse K=d_ffn")
    # same products, same accumulation order per tile row -> the two GPU paths agree tightly
    assert (ys - y).abs().max().item() <= 2e-3


def test_c0_every_gemm_variant(ctx, c0):
    k = 344
    ks = [k] * c0.n_blocks
    ref = c0.oracle_layer(ks)
    idx, _ = c0.gpu_predict(ctx, ks)
    def variants(option):
        v = 0
        while True:
            try:
                ctx.set_option(option, v)
            except B.FFError:
                return
            yield v
            v += 1

    try:
        n1 = n2 = 0
        for v in variants("gemm1_variant"):
            _check_y(c0.gpu_sparse(ctx, idx, ks, out_f32=True), ref.y, f"c0 gemm1 variant {v}")
            n1 += 1
        ctx.set_option("gemm1_variant", -1)
        for v in variants("gemm2_variant"):
            _check_y(c0.gpu_sparse(ctx, idx, ks, out_f32=True), ref.y, f"c0 gemm2 variant {v}")
            n2 += 1
        assert n1 >= 2 and n2 >= 2
    finally:
        ctx.set_option("gemm1_variant", -1)
        ctx.set_option("gemm2_variant", -1)


def test_gemm2_column_split(ctx):
    """The last output-column tiles of the down GEMM may run as a second launch of smaller tiles
    (the launcher does so when the last round of workgroups would be mostly empty).  Forced on and
    off on a d_model that is no multiple of the tile width: the same sums up to fp32 rounding order,
    sparse and dense, and within the bars against the oracle."""
    shp = W.Shape("g2split", 1280, 1024, 300, 128, 8, 16)
    c = Case(shp)
    ks = [512, 300, 1024]
    ref = c.oracle_layer(ks)
    idx, _ = c.gpu_predict(ctx, ks, k_stride=1024)
    ref_d = O.dense_ffn(_f32(c.x_bits), c.host("w_gate"), c.host("w_up"), c.host("w_down").T)
    try:
        for variant in (0, 2):          # 128 x 512 and 256 x 256 tiles
            ctx.set_option("gemm2_variant", variant)
            ys, yd = {}, {}
            for split in (0, 1):
                ctx.set_option("gemm2_split", split)
                ys[split] = c.gpu_sparse(ctx, idx, ks, out_f32=True)
                _check_y(ys[split], ref.y, f"gemm2 variant {variant} split {split}")
                ctx.ensure_workspace(c.shape, shp.d_ffn)
                yd[split] = torch.empty((c.T, shp.d_model), dtype=torch.float32, device=DEV)
                ctx.dense_ffn(c.shape, c.x, c.w, yd[split], B.OUT_F32)
                _check_y(yd[split], ref_d, f"dense, gemm2 variant {variant} split {split}")
            # the second launch's tile adds its two k-groups' sums at the end: fp32 rounding order only
            assert (ys[0] - ys[1]).abs().max().item() <= 1e-4 and (yd[0] - yd[1]).abs().max().item() <= 1e-4
    finally:
        ctx.set_option("gemm2_variant", -1)
        ctx.set_option("gemm2_split", -1)


def test_gemm2_streamed_list(ctx):
    """Lists too long for the eight-wavefront down-GEMM tile's LDS table (more than about 8000 ids)
    stream through a small ring of list entries instead.  Long lists, a very short one in between
    (fewer k-steps than the ring preloads), with and without the compensator, against the oracle
    and against the default tile."""
    shp = W.Shape("g2stream", 512, 9216, 300, 128, 8, 16)
    c = Case(shp)
    for ks, comp in (([9000, 50, 9216], True), ([8300, 8300, 8300], False)):
        ref = c.oracle_layer(ks, comp=comp)
        idx, _ = c.gpu_predict(ctx, ks, k_stride=9216)
        try:
            y_def = c.gpu_sparse(ctx, idx, ks, comp=comp, out_f32=True)
            ctx.set_option("gemm2_variant", 4)
            y_str = c.gpu_sparse(ctx, idx, ks, comp=comp, out_f32=True)
        finally:
            ctx.set_option("gemm2_variant", -1)
        _check_y(y_def, ref.y, f"default tile ks={ks}")
        _check_y(y_str, ref.y, f"streamed list ks={ks}")
        assert (y_def - y_str).abs().max().item() <= 1e-4


def test_gemm2_scalar_loads_of_the_list(ctx):
    """The down GEMM's fallback source of row ids: scalar loads of the list in the k-loop, taken when
    the ids do not fit 16 bits (d_ffn + r_comp > 65536) or no LDS is left for a table.  Forced on lists
    the table takes as well (must agree with it and with the oracle, on the two main tile shapes), and
    reached the natural way on a layer of 65536 neurons plus compensator units."""
    shp = W.Shape("g2scalar", 256, 4096, 300, 128, 8, 16)
    c = Case(shp)
    try:
        for ks, comp in (([2048, 37, 4096], True), ([1000, 1000, 1000], False)):
            ref = c.oracle_layer(ks, comp=comp)
            idx, _ = c.gpu_predict(ctx, ks, k_stride=4096)
            for variant in (0, 1, 4):
                ctx.set_option("gemm2_variant", variant)
                ys = {}
                for mode in (1, 2):
                    ctx.set_option("gemm2_row_mode", mode)
                    ys[mode] = c.gpu_sparse(ctx, idx, ks, comp=comp, out_f32=True)
                    _check_y(ys[mode], ref.y, f"gemm2 variant {variant} row ids mode {mode} ks={ks}")
                assert torch.equal(ys[1], ys[2]), "same tiles, same rows, same order: the sums must be the same bits"
        # a tile that has no streamed-list kernel refuses mode 3 instead of running something else
        ctx.set_option("gemm2_variant", 0)
        ctx.set_option("gemm2_row_mode", 3)
        with pytest.raises(B.FFError):
            c.gpu_sparse(ctx, idx, ks, comp=False, out_f32=True)
    finally:
        ctx.set_option("gemm2_variant", -1)
        ctx.set_option("gemm2_row_mode", -1)
    wide = Case(W.Shape("g2wide", 128, 65536, 200, 128, 8, 16))
    ks = [3000, 65536]
    ref = wide.oracle_layer(ks)
    idx, _ = wide.gpu_predict(ctx, ks, k_stride=65536)
    _assert_indices(idx, ref.indices, ks)
    _check_both(wide, ctx, idx, ks, ref.y, "d_ffn 65536 + 16 compensator units (ids beyond 16 bits)")


def test_nothing_is_written_outside_the_buffers(ctx):
    """Guard zones in front of and behind every buffer the library writes (index lists, scores, the
    output, the workspace) keep their pattern: equal K with a pitch above K, unequal K with a ragged
    last block, both output types."""
    G = 1024                                            # guard bytes on either side (keeps 256-byte alignment)

    def guarded(nbytes, fill):
        raw = torch.full((nbytes + 2 * G,), fill, dtype=torch.uint8, device=DEV)
        return raw, raw[G:G + nbytes]

    def intact(raw, nbytes, fill, what):
        assert (raw[:G] == fill).all() and (raw[G + nbytes:] == fill).all(), f"{what}: bytes outside the buffer were written"

    for n_tokens, ks, k_stride in ((256, [344] * 4, 344 + 8), (230, [688, 345, 101, 688], 688)):
        c = Case(W.CONFIGS["c0"], n_tokens=n_tokens)
        nB, dm, df = c.n_blocks, c.shp.d_model, c.shp.d_ffn
        need = B.workspace_bytes(c.shape, max(ks))
        ws_raw, ws = guarded(need, 0x5A)
        keep = ctx._ws
        ctx.set_workspace(ws)
        try:
            idx_raw, idx_b = guarded(nB * k_stride * 4, 0xA5)
            sc_raw, sc_b = guarded(nB * df * 8, 0xA5)
            idx = idx_b.view(torch.int32).view(nB, k_stride)
            sc = sc_b.view(torch.float64).view(nB, df)
            ctx.predict(c.shape, c.x, c.pred, ks, k_stride, idx, sc)
            ref = c.oracle_layer(ks)
            _assert_indices(idx, ref.indices, ks)
            for f32 in (True, False):
                y_raw, y_b = guarded(n_tokens * dm * (4 if f32 else 2), 0xA5)
                y = y_b.view(torch.float32 if f32 else torch.bfloat16).view(n_tokens, dm)
                ctx.sparse_ffn(c.shape, c.x, c.w, c.comp, idx, ks, k_stride, y, B.OUT_F32 if f32 else B.OUT_BF16)
                torch.cuda.synchronize()
                if f32:
                    _check_y(y, ref.y, f"guarded buffers, T={n_tokens}")
                intact(y_raw, y_b.numel(), 0xA5, "y")
            intact(idx_raw, idx_b.numel(), 0xA5, "indices")
            intact(sc_raw, sc_b.numel(), 0xA5, "scores")
            intact(ws_raw, need, 0x5A, "workspace")
        finally:
            ctx.set_workspace(keep)


@pytest.mark.parametrize("block", [64, 32, 16])
def test_short_blocks_run_on_merged_lists(ctx, block):
    """Blocks shorter than the 128-token tile: the library may run the union of the lists of the
    128 / block neighbouring blocks over all their tokens, with the activations of the (block, neuron)
    pairs nobody selected written as zero.  Forced on and off: both within the bars against the oracle,
    and the same sums up to fp32 rounding order; long and short lists, unequal K, a ragged last block and a
    last group with fewer blocks than the others, with and without the compensator."""
    shp = W.Shape(f"merge{block}", 256, 2048, 300, block, 8, 16)
    c = Case(shp)
    nB = c.n_blocks
    g = np.random.Generator(np.random.Philox(key=[64, block]))
    try:
        for ks, comp in (([1800] * nB, True), ([int(v) for v in g.integers(1, 2049, size=nB)], True),
                         ([300] * nB, False), ([2048] * (nB - 1) + [5], True)):
            ref = c.oracle_layer(ks, comp=comp)
            idx, _ = c.gpu_predict(ctx, ks, k_stride=2048)
            _assert_indices(idx, ref.indices, ks)
            ys = {}
            for merge in (0, 1, -1):
                ctx.set_option("merge_blocks", merge)
                ys[merge] = _check_both(c, ctx, idx, ks, ref.y, f"block {block} ks[0]={ks[0]} comp={comp} merge_blocks={merge}", comp=comp)
            assert (ys[0] - ys[1]).abs().max().item() <= 2e-3
    finally:
        ctx.set_option("merge_blocks", -1)


def test_sizes_at_the_documented_limits(ctx):
    """The largest values the header allows: 4096 compensator units (far more than selected neurons), the
    most blocks a call takes (16384 one-token blocks), and 4096-token blocks with softmax pooling plus a
    short last block.  Small widths keep the oracle fast; lists exact, outputs within the bars."""
    # (a) r_comp = 4096 next to K = 40 of 256 neurons
    c = Case(W.Shape("lim_rc", 128, 256, 200, 64, 8, 4096))
    ks = [40, 256, 1, 100]
    ref = c.oracle_layer(ks)
    idx, _ = c.gpu_predict(ctx, ks, k_stride=256)
    _assert_indices(idx, ref.indices, ks)
    _check_both(c, ctx, idx, ks, ref.y, "r_comp 4096")
    # (b) 16384 blocks of one token
    c = Case(W.Shape("lim_nb", 128, 64, 16384, 1, 8, 8))
    ks = [24] * 16384
    ref = c.oracle_layer(ks, blocks=list(range(0, 16384, 257)) + [16383])
    idx, _ = c.gpu_predict(ctx, ks)
    _assert_indices(idx, ref.indices, ks)
    _check_both(c, ctx, idx, ks, ref.y, "16384 one-token blocks (sampled)")
    # (c) blocks of 4096 tokens, softmax pooling, last block of 100 tokens
    c = Case(W.Shape("lim_blk", 256, 512, 4196, 4096, 16, 8), with_q=True)
    ks = [200, 333]
    ref = c.oracle_layer(ks)
    idx, _ = c.gpu_predict(ctx, ks, k_stride=336)
    _assert_indices(idx, ref.indices, ks)
    _check_both(c, ctx, idx, ks, ref.y, "4096-token blocks, softmax pooling")
    # (d) a wide model (d_model 8320: 65 k-steps of 128, 16.25 column tiles of 512), blocks of 128 and a short last one
    c = Case(W.Shape("lim_dm", 8320, 512, 300, 128, 16, 8))
    ks = [256, 512, 77]
    ref = c.oracle_layer(ks)
    idx, _ = c.gpu_predict(ctx, ks, k_stride=512)
    _assert_indices(idx, ref.indices, ks)
    _check_both(c, ctx, idx, ks, ref.y, "d_model 8320")
    c = Case(W.Shape("lim_blk", 256, 512, 4196, 4096, 16, 8), with_q=True)
    with pytest.raises(B.FFError) as e:          # one token more per block is refused with softmax pooling
        big = B.Shape(256, 512, 4196, 4097, 16, 8)
        ctx.predict(big, c.x, c.pred, [200, 333], 336, idx, None)
    assert e.value.status == 2


def test_gemm1_remainder_split(ctx, c0):
    """The positions beyond the last full N tile of the gate/up GEMM may run as a second
    launch with small tiles; forced on and off, uniform and per-block K, with and without
    the compensator, results stay within the bars (and agree with each other)."""
    try:
        for ks, comp in (([344] * c0.n_blocks, True), ([300] * c0.n_blocks, False),
                         ([c0.shp.d_ffn, 345, 101, 129][:c0.n_blocks] + [200] * max(0, c0.n_blocks - 4), True)):
            ref = c0.oracle_layer(ks, comp=comp)
            idx, _ = c0.gpu_predict(ctx, ks, k_stride=c0.shp.d_ffn)
            ys = {}
            for split in (0, 1, -1):
                ctx.set_option("gemm1_split", split)
                ys[split] = c0.gpu_sparse(ctx, idx, ks, comp=comp, out_f32=True)
                _check_y(ys[split], ref.y, f"c0 gemm1_split {split} ks[1]={ks[1]} comp={comp}")
            assert (ys[0] - ys[1]).abs().max().item() <= 2e-3
    finally:
        ctx.set_option("gemm1_split", -1)


def test_static_expert_one_list_for_all_tokens(ctx):
    """Static-expert mode (Sec. 5 ablation "first-block static"): the first block's selection
    serves the whole prompt.  It needs no entry point of its own: ff_sparse_ffn with
    block = n_tokens and that one list (the GEMMs then use their largest token tiles)."""
    c = Case(W.CONFIGS["c1"], n_tokens=640)                    # 5 blocks of 128
    k = 2048
    idx_blocks, _ = c.gpu_predict(ctx, [k] * c.n_blocks)
    first = idx_blocks[:1].contiguous()                        # [1][k]
    static_shape = B.Shape(c.shp.d_model, c.shp.d_ffn, c.T, c.T, c.shp.r_pred, c.shp.r_comp)
    ctx.ensure_workspace(static_shape, k)
    y = torch.empty((c.T, c.shp.d_model), dtype=torch.float32, device=DEV)
    comp = B.Compensator(c.comp.wc1, c.comp.wc2, B.ACT["silu"])
    ctx.sparse_ffn(static_shape, c.x, c.w, comp, first, [k], k, y, B.OUT_F32)
    lst = first[0].cpu().numpy()
    ref = c.oracle_layer([k] * c.n_blocks, indices_override=[lst] * c.n_blocks)
    np.testing.assert_array_equal(ref.indices[0], c.oracle_layer([k] * c.n_blocks, compute_ffn=False).indices[0])
    _check_y(y, ref.y, "static expert, one list, block = T")


def test_single_token_blocks(ctx):
    """Blocks of one token (the generation-time regime): pooling is the identity, every token
    has its own list; and one short block holding the whole (tiny) prompt."""
    shp = W.CONFIGS["c0"]
    for T, blk in ((5, 1), (3, 3)):
        c = Case(dataclasses.replace(shp, block=blk, n_tokens=T), n_tokens=T)
        ks = [200] * c.n_blocks
        ref = c.oracle_layer(ks)
        idx, _ = c.gpu_predict(ctx, ks)
        _assert_indices(idx, ref.indices, ks)
        _check_y(c.gpu_sparse(ctx, idx, ks, out_f32=True), ref.y, f"T={T} block={blk}")


def test_first_and_last_block_dense(ctx):
    """Sec. 3.4: the first and the last block keep every neuron, the others K.  The library
    schedules such a few longer lists ahead of the rest; results must not depend on that.
    Also a block shorter than the common K, and more long blocks than the scheduler singles out."""
    c = Case(W.CONFIGS["c1"], n_tokens=12 * 128)
    D, k = c.shp.d_ffn, 4096
    for ks in ([D] + [k] * 10 + [D],
               [D, k, k, 1000, k, k, k, 5000, k, k, k, D],
               [D if b % 2 == 0 else k for b in range(12)]):
        ref = c.oracle_layer(ks, blocks=[0, 3, 7, 11])
        idx, _ = c.gpu_predict(ctx, ks, k_stride=D)
        _assert_indices(idx, ref.indices, ks)
        for split in (-1, 0):
            ctx.set_option("gemm1_split", split)
            try:
                _check_y(c.gpu_sparse(ctx, idx, ks, out_f32=True), ref.y, f"first/last dense ks[1]={ks[1]} ks[3]={ks[3]} split={split}")
            finally:
                ctx.set_option("gemm1_split", -1)


def test_long_lists_cut_along_k(ctx):
    """A few lists much longer than the rest (Sec. 3.4) are cut along the list in the down GEMM: a tile like
    everybody else's plus short pieces, fp32 partial sums added in piece order by one more launch.  Forced
    off, into 1, 3 and 16 short pieces and left to the launcher; two long lists of different length, the
    last one on a block of 37 tokens, d_model no multiple of the tile width.  Every setting against the
    oracle (fp32 at the stated bars, bf16 bit-equal to its rounding); rows of the other blocks must not
    change at all, rows of the long ones only by fp32 rounding order; and the stack's residual write of
    those rows is bf16(h + bf16(y)) of the same sums."""
    shp = W.Shape("ksplit", 640, 3072, 5 * 128 + 37, 128, 8, 16)
    c = Case(shp)
    ks = [3072, 704, 704, 100, 704, 2900]
    ref = c.oracle_layer(ks)
    idx, _ = c.gpu_predict(ctx, ks, k_stride=3072)
    _assert_indices(idx, ref.indices, ks)
    long_rows = np.r_[0:128, 5 * 128:c.T]
    other_rows = np.r_[128:5 * 128]
    try:
        ys = {}
        for ksplit in (0, 1, 3, 16, -1):
            ctx.set_option("gemm2_ksplit", ksplit)
            ys[ksplit] = _check_both(c, ctx, idx, ks, ref.y, f"long lists cut into {ksplit} pieces")
            assert torch.equal(ys[ksplit][other_rows], ys[0][other_rows]), ksplit
            assert (ys[ksplit][long_rows] - ys[0][long_rows]).abs().max().item() <= 1e-4, ksplit
            if ksplit != 0:
                assert not torch.equal(ys[ksplit][long_rows], ys[0][long_rows]), "the cut was not taken"
            # residual write of a one-layer stack on the same lists
            h = c.x.clone()
            idx1 = torch.empty((1, c.n_blocks, 3072), dtype=torch.int32, device=DEV)
            x1 = torch.empty((1, c.T, shp.d_model), dtype=torch.bfloat16, device=DEV)
            ctx.ffn_stack(c.shape, h, [c.pred], [c.w], [c.comp], np.array([ks], dtype=np.int32), 3072, 1e-6, idx1, x1)
            y32 = torch.empty((c.T, shp.d_model), dtype=torch.float32, device=DEV)
            ctx.sparse_ffn(c.shape, x1[0], c.w, c.comp, idx1[0], ks, 3072, y32, B.OUT_F32)
            expect = (c.x.float() + y32.to(torch.bfloat16).float()).to(torch.bfloat16)
            assert torch.equal(h.view(torch.int16), expect.view(torch.int16)), f"residual write, ksplit={ksplit}"
        # the pieces' row ids from each of the kernel's sources: scalar loads, and the streamed list of the
        # eight-wavefront tile
        ctx.set_option("gemm2_ksplit", 5)
        for variant, row_mode in ((-1, 2), (4, 3)):
            ctx.set_option("gemm2_variant", variant)
            ctx.set_option("gemm2_row_mode", row_mode)
            y = c.gpu_sparse(ctx, idx, ks, out_f32=True)
            _check_y(y, ref.y, f"long lists cut, tile {variant}, row ids from source {row_mode}")
            assert (y - ys[0]).abs().max().item() <= 1e-4
    finally:
        ctx.set_option("gemm2_ksplit", -1)
        ctx.set_option("gemm2_variant", -1)
        ctx.set_option("gemm2_row_mode", -1)


@pytest.mark.parametrize("n_tokens,block", [(256, 64), (6, 4)])
def test_calls_can_be_captured_in_a_hip_graph(n_tokens, block):
    """predict + sparse_ffn with one K for all blocks enqueue kernels only (no copies, no
    synchronisation, no allocation), so a caller may capture them in a HIP graph.  The graph is
    replayed several times on changing inputs, with eager work in between, and every replay is
    compared with the eager result for the same input.  Six tokens take the few-token kernels."""
    c0 = Case(dataclasses.replace(W.CONFIGS["c0"], n_tokens=n_tokens, block=block), n_tokens=n_tokens)
    stream = torch.cuda.Stream()
    ctx = B.Context(0, stream)
    try:
        k = 344
        ks = [k] * c0.n_blocks
        ctx.ensure_workspace(c0.shape, k)
        x = c0.x.clone()
        idx = torch.empty((c0.n_blocks, k), dtype=torch.int32, device=DEV)
        y = torch.empty((c0.T, c0.shp.d_model), dtype=torch.float32, device=DEV)
        comp = B.Compensator(c0.comp.wc1, c0.comp.wc2, B.ACT["silu"])

        def step():
            ctx.predict(c0.shape, x, c0.pred, ks, k, idx, None)
            ctx.sparse_ffn(c0.shape, x, c0.w, comp, idx, ks, k, y, B.OUT_F32)

        with torch.cuda.stream(stream):
            step()                                   # first-use set-up happens outside the capture
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step()
        gen = torch.Generator(device=DEV)
        gen.manual_seed(5)
        for rep in range(4):
            x_new = (torch.randn(x.shape, device=DEV, generator=gen) * 1.5).to(torch.bfloat16)
            x.copy_(x_new)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            y_graph, idx_graph = y.clone(), idx.clone()
            y.zero_(); idx.zero_()
            with torch.cuda.stream(stream):
                step()
            stream.synchronize()
            assert torch.equal(idx_graph, idx), f"replay {rep}: indices differ from the eager call"
            assert torch.equal(y_graph, y), f"replay {rep}: outputs differ from the eager call"
        assert not torch.equal(y_graph, torch.zeros_like(y_graph))
        # K that differs between blocks is staged through a host buffer at call time: under capture the
        # call is refused (a replay would read whatever the buffer holds by then) and nothing is enqueued
        if c0.n_blocks > 1:
            ks_ragged = [k] * (c0.n_blocks - 1) + [k - 1]
            g2 = torch.cuda.CUDAGraph()
            seen = []
            with torch.cuda.graph(g2, stream=stream):
                try:
                    ctx.predict(c0.shape, x, c0.pred, ks_ragged, k, idx, None)
                except B.FFError as e:
                    seen.append(e.status)
            assert seen == [1], seen
        # the validate option reads a result back and waits for it: refused under capture as well
        ctx.set_option("validate", 1)
        g3 = torch.cuda.CUDAGraph()
        seen = []
        with torch.cuda.graph(g3, stream=stream):
            try:
                ctx.sparse_ffn(c0.shape, x, c0.w, comp, idx, ks, k, y, B.OUT_F32)
            except B.FFError as e:
                seen.append(e.status)
        ctx.set_option("validate", 0)
        assert seen == [1], seen
    finally:
        torch.cuda.synchronize()
        ctx.close()


def test_the_stack_can_be_captured_in_a_hip_graph():
    """ff_ffn_stack with one K per layer (different between layers) enqueues kernels only: three layers of
    the c0 shape captured once, replayed on changing hidden states with eager work in between, every replay
    bit-equal to the eager call on the same input (hidden state and all layers' lists)."""
    shp = W.CONFIGS["c0"]
    L = 3
    cases = [Case(shp, layer=l) for l in range(L)]
    nB = cases[0].n_blocks
    ks = np.array([[k] * nB for k in (344, 516, 172)], dtype=np.int32)
    stream = torch.cuda.Stream()
    ctx = B.Context(0, stream)
    try:
        ctx.ensure_workspace(cases[0].shape, 516)
        h = cases[0].x.clone()
        idx = torch.empty((L, nB, 516), dtype=torch.int32, device=DEV)
        args = (cases[0].shape, h, [c.pred for c in cases], [c.w for c in cases], [c.comp for c in cases], ks, 516, 1e-6, idx, None)
        with torch.cuda.stream(stream):
            ctx.ffn_stack(*args)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            ctx.ffn_stack(*args)
        gen = torch.Generator(device=DEV)
        gen.manual_seed(11)
        for rep in range(3):
            h0 = (torch.randn(h.shape, device=DEV, generator=gen) * 1.5).to(torch.bfloat16)
            h.copy_(h0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            h_graph, idx_graph = h.clone(), idx.clone()
            h.copy_(h0); idx.zero_()
            with torch.cuda.stream(stream):
                ctx.ffn_stack(*args)
            stream.synchronize()
            assert torch.equal(idx_graph, idx), f"replay {rep}: lists differ from the eager call"
            assert torch.equal(h_graph.view(torch.int16), h.view(torch.int16)), f"replay {rep}: hidden state differs"
            assert not torch.equal(h_graph.view(torch.int16), h0.view(torch.int16))
    finally:
        torch.cuda.synchronize()
        ctx.close()


def test_random_shapes_blocks_and_list_lengths(ctx):
    """Seeded sweep over small shapes: block sizes that are no multiple of any tile, ragged last
    blocks, d_ffn no multiple of 64, with and without compensator, one K for all blocks, a few
    longer lists among equal ones, and arbitrary per-block K; indices exact, outputs within the bars."""
    g = np.random.Generator(np.random.Philox(key=[97, 3]))
    for case in range(24):
        dm = int(g.choice([128, 256, 384]))
        df = 8 * int(g.integers(25, 150))
        blk = int(g.choice([1, 7, 32, 64, 100, 128, 200, 256, 300]))
        T = int(g.integers(1, 6 * min(blk, 96) + 2))
        r = int(g.choice([8, 32]))
        rc = int(g.choice([0, 8, 16, 64]))
        shp = W.Shape(f"rnd{case}", dm, df, T, blk, r, max(rc, 8))
        c = Case(shp, n_tokens=T, seed=1000 + case)
        nB = c.n_blocks
        mode = case % 3
        if mode == 0:
            ks = [int(g.integers(1, df + 1))] * nB
        elif mode == 1:
            ks = [int(g.integers(1, df // 2 + 1))] * nB
            for b in g.choice(nB, size=min(nB, int(g.integers(1, 3))), replace=False):
                ks[int(b)] = int(g.integers(df // 2, df + 1))
        else:
            ks = [int(v) for v in g.integers(1, df + 1, size=nB)]
        comp = rc > 0
        ref = c.oracle_layer(ks, comp=comp)
        assert min(ref.margins) > 1e-9 * max(ref.score_absmax)
        idx, _ = c.gpu_predict(ctx, ks, k_stride=max(ks) + int(g.integers(0, 9)))
        _assert_indices(idx, ref.indices, ks)
        _check_both(c, ctx, idx, ks, ref.y,
                    f"rnd {case}: dm {dm} dffn {df} T {T} block {blk} r {r} rc {rc if comp else 0} mode {mode}", comp=comp)


def test_few_token_calls_take_the_gemv_path(ctx):
    """Calls with at most 8 tokens (generation time) run gather-GEMV kernels instead of the MFMA
    tiles.  Both ways against the oracle and against each other: one list for all tokens, a list per
    token, ragged blocks, unequal K, with and without the compensator, both output types, a d_model
    that is no multiple of the 512-element lane stride."""
    g = np.random.Generator(np.random.Philox(key=[8, 8]))
    cases = [(W.CONFIGS["c1"], 1, 1), (W.CONFIGS["c1"], 8, 8), (W.CONFIGS["c1"], 8, 1), (W.CONFIGS["c1"], 7, 3),
             (W.Shape("gv384", 384, 1016, 5, 2, 8, 16), 5, 2), (W.Shape("gv384", 384, 1016, 5, 1, 8, 16), 5, 1),
             (W.CONFIGS["c0"], 6, 4)]
    try:
        for shp, T, blk in cases:
            c = Case(dataclasses.replace(shp, n_tokens=T, block=blk), n_tokens=T, seed=4242 + T)
            nB = c.n_blocks
            for mode in ("uniform", "ragged"):
                ks = [shp.d_ffn // 2] * nB if mode == "uniform" else [int(v) for v in g.integers(1, shp.d_ffn + 1, size=nB)]
                for comp in (True, False):
                    ref = c.oracle_layer(ks, comp=comp)
                    idx, _ = c.gpu_predict(ctx, ks)
                    _assert_indices(idx, ref.indices, ks)
                    out = {}
                    for small in (1, 0):
                        ctx.set_option("small_path", small)
                        out[small, True] = _check_both(c, ctx, idx, ks, ref.y,
                                                       f"{shp.name} T={T} block={blk} {mode} comp={comp} small_path={small}", comp=comp)
                    assert (out[1, True] - out[0, True]).abs().max().item() <= 2e-3
                    # several lists in a few-token call may be merged into one (read once for all tokens, H zero
                    # where a token did not select the neuron): forced off and on
                    if nB > 1:
                        ctx.set_option("small_path", 1)
                        for merge in (0, 1):
                            ctx.set_option("merge_blocks", merge)
                            ym = _check_both(c, ctx, idx, ks, ref.y, f"{shp.name} T={T} block={blk} {mode} comp={comp} merge_blocks={merge}", comp=comp)
                            assert (ym - out[1, True]).abs().max().item() <= 2e-3
                        ctx.set_option("merge_blocks", -1)
            # the dense FFN of the same few tokens (no list: position p is row p)
            ref_d = O.dense_ffn(_f32(c.x_bits), c.host("w_gate"), c.host("w_up"), c.host("w_down").T)
            ctx.ensure_workspace(c.shape, shp.d_ffn)
            for small in (1, 0):
                ctx.set_option("small_path", small)
                y = torch.empty((T, shp.d_model), dtype=torch.float32, device=DEV)
                ctx.dense_ffn(c.shape, c.x, c.w, y, B.OUT_F32)
                _check_y(y, ref_d, f"{shp.name} T={T} dense small_path={small}")
    finally:
        ctx.set_option("small_path", 1)
        ctx.set_option("merge_blocks", -1)


def test_c0_ragged_tail_and_per_block_k(ctx):
    # 230 tokens in blocks of 64 -> 64, 64, 64, 38; first and last block dense, odd K elsewhere
    c = Case(W.CONFIGS["c0"], n_tokens=230)
    ks = [c.shp.d_ffn, 345, 101, c.shp.d_ffn]
    ref = c.oracle_layer(ks)
    idx, _ = c.gpu_predict(ctx, ks, k_stride=c.shp.d_ffn)
    _assert_indices(idx, ref.indices, ks)
    _check_both(c, ctx, idx, ks, ref.y, "c0 ragged per-block K")
    # canaries: rows past n_tokens of an oversized output must stay untouched
    big = torch.full((256, c.shp.d_model), 7.0, dtype=torch.bfloat16, device=DEV)
    ctx.sparse_ffn(c.shape, c.x, c.w, c.comp, idx, ks, idx.shape[1], big, B.OUT_BF16)
    assert (big[230:] == 7.0).all()
    # The library keeps the per-block K it copied to the device last and reuses that copy for equal values:
    # other values of the same length in between, then the first ones again, must each give their own lists.
    ks2 = [200, 345, c.shp.d_ffn, 7]
    for cur in (ks, ks2, ks, ks, ks2):
        r = c.oracle_layer(cur, compute_ffn=False)
        i2, _ = c.gpu_predict(ctx, cur, k_stride=c.shp.d_ffn)
        _assert_indices(i2, r.indices, cur)
    _check_y(c.gpu_sparse(ctx, idx, ks, out_f32=True), ref.y, "c0 ragged per-block K, after other K in between")


def test_c0_softmax_pooling(ctx):
    c = Case(W.CONFIGS["c0"], with_q=True)
    ks = [344] * c.n_blocks
    ref = c.oracle_layer(ks, compute_ffn=False)
    idx, _ = c.gpu_predict(ctx, ks)
    _assert_indices(idx, ref.indices, ks)
    # q_pred = 0 selects what mean pooling selects
    c.dev["q_pred"].zero_()
    idx0, _ = c.gpu_predict(ctx, ks)
    c2 = Case(W.CONFIGS["c0"])
    idxm, _ = c2.gpu_predict(ctx, ks)
    assert torch.equal(idx0, idxm)


@pytest.mark.parametrize("r", [1, 12, 40, 320, 1024])
def test_predictor_ranks_and_widths(ctx, r):
    """The predictor kernels over the ranks they treat differently (a multiple of 8 or not; 8, 64 or 128
    outputs per 16-byte column group; more than 256 outputs) and over widths that are no multiple of the
    512-channel slices, with mean and softmax pooling, a ragged last block and unequal K: scores to 1e-12
    of the oracle's, lists bit-exact, and the diagnostic calls ff_copy / ff_mfma_peak beside them."""
    for dm, df, T, blk in ((128, 1000, 150, 64), (640, 2048, 200, 128), (1152, 1280, 70, 16)):
        for with_q in (False, True):
            shp = W.Shape(f"pred{r}", dm, df, T, blk, r, 8)
            c = Case(shp, with_q=with_q, seed=77 + r)
            nB = c.n_blocks
            ks = [max(1, (df * (b + 1)) // (nB + 1)) for b in range(nB)]
            ref = c.oracle_layer(ks, compute_ffn=False)
            idx, sc = c.gpu_predict(ctx, ks, k_stride=max(ks) + 3, scores=True)
            q = _f32(c.lt.q_pred) if with_q else None
            x = _f32(c.x_bits)
            ref_s = np.stack([O.predictor_scores(x[b * blk:min(T, (b + 1) * blk)], q, c.host("w1"), c.host("w2")) for b in range(nB)])
            np.testing.assert_allclose(sc.cpu().numpy(), ref_s, rtol=1e-12, atol=1e-13 * np.abs(ref_s).max())
            # (with one hidden unit a score is one product h * w2[j]: equal bf16 weights, or h = 0 after ReLU, give
            #  exact ties, the same on both sides, and the lower index wins; otherwise ties must not decide)
            assert r == 1 or min(ref.margins) > 1e-9 * max(ref.score_absmax)
            _assert_indices(idx, ref.indices, ks)


def test_diagnostic_calls(ctx):
    a = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    b = torch.zeros_like(a)
    ctx.copy(b, a)
    assert torch.equal(a, b)
    flops = ctx.mfma_peak(100, False)
    assert flops == 1024 * 8 * 100 * 8 * 2.0 * 32 * 32 * 16
    assert ctx.mfma_peak(10, True) == flops / 10
    torch.cuda.synchronize()
    with pytest.raises(B.FFError):
        ctx.mfma_peak(0)


def test_exact_ties_on_gpu(ctx):
    # integer-valued inputs: all predictor sums are exact, so ties are exact on both sides
    dm, df, T, r = 128, 640, 128, 8
    ic = W.integer_valued_case(dm, df, T, r)
    w2 = ic["w2"].copy()
    w2[:, df // 2:] = w2[:, :df // 2]                 # duplicated columns -> pairs of equal scores
    x, w1 = _f32(ic["x"]), _f32(ic["w1"])
    shape = B.Shape(dm, df, T, 64, r, 0)
    xd, w1d, w2d = (B.to_device_bf16(a, DEV) for a in (ic["x"], ic["w1"], w2))
    pred = B.Predictor(None, w1d.data_ptr(), w2d.data_ptr())
    ctx.ensure_workspace(shape, df)
    for k in (1, 7, 320, 321, 500, 640):
        idx = torch.empty((2, k), dtype=torch.int32, device=DEV)
        ctx.predict(shape, xd, pred, [k, k], k, idx, None)
        for b in range(2):
            s = O.predictor_scores(x[b * 64:(b + 1) * 64], None, w1, _f32(w2))
            np.testing.assert_array_equal(idx[b].cpu().numpy(), O.select_topk(s, k))
    # ReLU kills every hidden unit: all scores 0 -> the first K indices
    xp = W.f32_to_bf16_bits(np.abs(x) + 1.0)
    w1n = W.f32_to_bf16_bits(-np.abs(w1) - 1.0)
    xpd, w1nd = B.to_device_bf16(xp, DEV), B.to_device_bf16(w1n, DEV)
    idx = torch.empty((2, 5), dtype=torch.int32, device=DEV)
    ctx.predict(shape, xpd, B.Predictor(None, w1nd.data_ptr(), w2d.data_ptr()), [5, 5], 5, idx, None)
    assert idx.cpu().tolist() == [[0, 1, 2, 3, 4]] * 2


@pytest.mark.parametrize("df", [2048, 20480, 28672, 40960, 147456])
def test_heavy_ties_at_the_threshold(ctx, df):
    # 1500 scores are exactly equal and the K-th largest lies among them: the bucket holding the
    # threshold overflows the ranking step and the radix path decides.  The sizes take the five
    # top-K kernels: keys in 16, 24 or 32 registers per thread; beyond 32768 neurons the general kernel,
    # with a class byte per key in LDS for the compaction and, at 147456, without it.
    dm, T, r = 128, 64, 8
    ic = W.integer_valued_case(dm, df, T, r, seed=11)
    w2 = ic["w2"].copy()
    w2[:, 300:1800] = w2[:, 300:301]
    x, w1 = _f32(ic["x"]), _f32(ic["w1"])
    s = O.predictor_scores(x, None, w1, _f32(w2))
    assert (s[300:1800] == s[300]).all()
    shape = B.Shape(dm, df, T, 64, r, 0)
    xd, w1d, w2d = (B.to_device_bf16(a, DEV) for a in (ic["x"], ic["w1"], w2))
    pred = B.Predictor(None, w1d.data_ptr(), w2d.data_ptr())
    ctx.ensure_workspace(shape, df)
    n_above = int((s > s[300]).sum())
    for k in sorted({1, max(1, n_above), n_above + 1, n_above + 700, n_above + 1500, min(df, n_above + 1501), df}):
        idx = torch.empty((1, k), dtype=torch.int32, device=DEV)
        ctx.predict(shape, xd, pred, [k], k, idx, None)
        np.testing.assert_array_equal(idx[0].cpu().numpy(), O.select_topk(s, k), err_msg=f"k={k}")
    # the same sizes without the planted ties (bucket + ranking path), two blocks, a pitch above K
    s2 = [O.predictor_scores(x[b * 32:(b + 1) * 32], None, w1, _f32(ic["w2"])) for b in range(2)]
    shape2 = B.Shape(dm, df, T, 32, r, 0)
    w2o = B.to_device_bf16(ic["w2"], DEV)
    ks = [df // 2, df // 3 + 1]
    idx = torch.empty((2, df // 2 + 5), dtype=torch.int32, device=DEV)
    ctx.predict(shape2, xd, B.Predictor(None, w1d.data_ptr(), w2o.data_ptr()), ks, idx.shape[1], idx, None)
    _assert_indices(idx, [O.select_topk(s2[b], ks[b]) for b in range(2)], ks)


@pytest.mark.parametrize("df", [2048, 40960])
def test_scores_that_are_not_finite_still_give_a_valid_list(ctx, df):
    """Scores are expected to be finite.  If they are not (an infinity among the hidden states makes
    every score of its block NaN or infinite), the list written is still exactly K distinct, ascending,
    in-range indices with a -1 tail, and nothing is written past the row; the other block is unaffected.
    2048 neurons take the register kernel, 40960 the general one."""
    dm, T, r = 128, 128, 8
    ic = W.integer_valued_case(dm, df, T, r, seed=3)
    x_bits = ic["x"].copy()
    x_bits[5, 7] = 0x7F80                                 # +inf in block 0
    x_bits[9, 3] = 0xFF80                                 # -inf in block 0: pooled value NaN
    shape = B.Shape(dm, df, T, 64, r, 0)
    xd, w1d, w2d = (B.to_device_bf16(a, DEV) for a in (x_bits, ic["w1"], ic["w2"]))
    pred = B.Predictor(None, w1d.data_ptr(), w2d.data_ptr())
    ctx.ensure_workspace(shape, df)
    s1 = O.predictor_scores(_f32(ic["x"])[64:], None, _f32(ic["w1"]), _f32(ic["w2"]))
    for k in (1, df // 3, df - 1):
        stride = k + 8
        raw = torch.full((2 * stride + 64,), -7, dtype=torch.int32, device=DEV)
        idx = raw[:2 * stride].view(2, stride)
        ctx.predict(shape, xd, pred, [k, k], stride, idx, None)
        got = idx.cpu().numpy()
        row = got[0, :k]
        assert (row >= 0).all() and (row < df).all() and (np.diff(row) > 0).all(), f"k={k}: block 0's list is not valid"
        assert (got[:, k:] == -1).all()
        np.testing.assert_array_equal(got[1, :k], O.select_topk(s1, k))
        assert (raw[2 * stride:] == -7).all()


def test_run_to_run_determinism(ctx, c0):
    ks = [344] * c0.n_blocks
    idx, _ = c0.gpu_predict(ctx, ks)
    y1 = c0.gpu_sparse(ctx, idx, ks)
    idx2, _ = c0.gpu_predict(ctx, ks)
    y2 = c0.gpu_sparse(ctx, idx2, ks)
    assert torch.equal(idx, idx2) and torch.equal(y1.view(torch.int16), y2.view(torch.int16))


def test_any_ascending_index_list_is_accepted(ctx, c0):
    g = np.random.Generator(np.random.Philox(key=[3, 3]))
    ks = [200, 13, 344, 1]
    lists = [np.sort(g.choice(c0.shp.d_ffn, size=k, replace=False)).astype(np.int32) for k in ks]
    idx = torch.full((4, 344), -1, dtype=torch.int32, device=DEV)
    for b, l in enumerate(lists):
        idx[b, :len(l)] = torch.from_numpy(l).to(DEV)
    ref = c0.oracle_layer(ks, indices_override=lists)
    _check_y(c0.gpu_sparse(ctx, idx, ks, out_f32=True), ref.y, "c0 arbitrary lists")


# ------------------------------------------------------------------ error paths (host-side checks)

def test_argument_errors_do_not_launch(ctx, c0):
    ks = [344] * c0.n_blocks
    idx, _ = c0.gpu_predict(ctx, ks)
    y = torch.empty((c0.T, c0.shp.d_model), dtype=torch.bfloat16, device=DEV)

    def status(fn):
        with pytest.raises(B.FFError) as e:
            fn()
        return e.value.status

    bad = B.Shape(200, 688, 256, 64, 32, 16)
    assert status(lambda: ctx.sparse_ffn(bad, c0.x, c0.w, c0.comp, idx, ks, 344, y)) == 2
    assert status(lambda: ctx.sparse_ffn(c0.shape, c0.x, c0.w, c0.comp, idx, [344, 344, 0, 344], 344, y)) == 1
    assert status(lambda: ctx.sparse_ffn(c0.shape, c0.x, c0.w, c0.comp, idx, ks, 100, y)) == 1
    assert status(lambda: ctx.sparse_ffn(c0.shape, c0.x, c0.w, c0.comp, idx, ks, 344, y, 5)) == 1
    assert status(lambda: ctx.sparse_ffn(c0.shape, c0.x, B.FfnWeights(None, c0.w.w_up, c0.w.w_down), None, idx, ks, 344, y)) == 1
    mis = B.FfnWeights(c0.w.w_gate + 2, c0.w.w_up, c0.w.w_down)
    assert status(lambda: ctx.sparse_ffn(c0.shape, c0.x, mis, None, idx, ks, 344, y)) == 3
    small = torch.empty(1024, dtype=torch.uint8, device=DEV)
    keep = ctx._ws
    ctx.set_workspace(small)
    assert status(lambda: ctx.sparse_ffn(c0.shape, c0.x, c0.w, c0.comp, idx, ks, 344, y)) == 5
    ctx.set_workspace(keep)
    # validate mode: a descending pair is reported, nothing is computed
    ctx.set_option("validate", 1)
    try:
        ctx.sparse_ffn(c0.shape, c0.x, c0.w, c0.comp, idx, ks, 344, y)          # good list passes
        badidx = idx.clone()
        badidx[2, 10] = badidx[2, 9]
        assert status(lambda: ctx.sparse_ffn(c0.shape, c0.x, c0.w, c0.comp, badidx, ks, 344, y)) == 4
    finally:
        ctx.set_option("validate", 0)


# ------------------------------------------------------------------ stack glue

@pytest.mark.parametrize("dm", [384, 4608, 8320])   # row in 8 or 16 registers per lane, or read twice
def test_rmsnorm_and_residual(ctx, dm):
    g = np.random.Generator(np.random.Philox(key=[8, 8]))
    h_bits = W.f32_to_bf16_bits((g.standard_normal((300, dm)) * 3).astype(np.float32))
    y_bits = W.f32_to_bf16_bits(g.standard_normal((300, dm)).astype(np.float32))
    h, y = B.to_device_bf16(h_bits, DEV), B.to_device_bf16(y_bits, DEV)
    x = torch.empty_like(h)
    ctx.rmsnorm(h, 1e-6, x)
    ref = O.bf16_round(O.rmsnorm_rows(_f32(h_bits), 1e-6))
    got = x.float().cpu().numpy().astype(np.float64)
    # float64 statistics on both sides: equal except where a value sits on a bf16 rounding tie
    assert (got != ref).mean() < 1e-3
    np.testing.assert_allclose(got, ref, rtol=2 ** -7)
    ctx.residual_add(h, y)
    ref_h = O.bf16_round(_f32(h_bits).astype(np.float64) + _f32(y_bits))
    np.testing.assert_array_equal(h.float().cpu().numpy().astype(np.float64), ref_h)


@pytest.mark.parametrize("n_tokens,block", [(256, 64), (6, 4)])
def test_small_stack_layerwise(ctx, n_tokens, block):
    # three layers of the c0 shape; each layer checked from the GPU's own layer input.  The six-token
    # case runs the few-token kernels, which add to the residual stream themselves.
    shp = dataclasses.replace(W.CONFIGS["c0"], n_tokens=n_tokens, block=block)
    L = 3
    cases = [Case(shp, n_tokens=n_tokens, layer=l) for l in range(L)]
    k = [344, 516, 172]
    ks = np.array([[k[l]] * cases[0].n_blocks for l in range(L)], dtype=np.int32)
    h0_bits = cases[0].x_bits
    h = B.to_device_bf16(h0_bits, DEV).clone()
    nB = cases[0].n_blocks
    idx = torch.empty((L, nB, 516), dtype=torch.int32, device=DEV)
    xd = torch.empty((L, shp.n_tokens, shp.d_model), dtype=torch.bfloat16, device=DEV)
    ctx.ensure_workspace(cases[0].shape, 516)
    ctx.ffn_stack(cases[0].shape, h, [c.pred for c in cases], [c.w for c in cases], [c.comp for c in cases],
                  ks, 516, 1e-6, idx, xd)
    h_prev = _f32(h0_bits).astype(np.float64)
    for l, c in enumerate(cases):
        x_gpu = xd[l].float().cpu().numpy().astype(np.float64)
        x_ref = O.bf16_round(O.rmsnorm_rows(h_prev, 1e-6))
        if l == 0:
            assert (x_gpu != x_ref).mean() < 1e-3
        else:   # h_prev is the oracle's own running state from here on: close, not equal
            np.testing.assert_allclose(x_gpu, x_ref, atol=0.05, rtol=0.02)
        # teacher forcing: the oracle computes layer l from the GPU's own layer input
        res = O.fastforward_layer(x_gpu, c.host("w_gate"), c.host("w_up"), c.host("w_down").T, c.host("w1"),
                                  c.host("w2"), shp.block, ks[l], wc1=c.host("wc1").T, wc2=c.host("wc2"))
        _assert_indices(idx[l], res.indices, list(ks[l]))
        h_prev = O.bf16_round(h_prev + res.y)
    got_h = h.float().cpu().numpy().astype(np.float64)
    d = got_h - h_prev
    assert np.sqrt((d * d).mean()) / np.sqrt((h_prev ** 2).mean()) < 1e-2
    # Every layer's write, element by element, with the merged lists of short blocks forced off and on (the
    # stack decides per layer by itself; 64-token blocks qualify): h_out = bf16(h_in + bf16(y)) of the fp32
    # output of ff_sparse_ffn on the same layer input and lists under the same setting.
    try:
        for merge in (0, 1):
            ctx.set_option("merge_blocks", merge)
            hm = B.to_device_bf16(h0_bits, DEV).clone()
            for l, c in enumerate(cases):
                h_in = hm.clone()
                idx1 = torch.empty((1, nB, 516), dtype=torch.int32, device=DEV)
                x1 = torch.empty((1, shp.n_tokens, shp.d_model), dtype=torch.bfloat16, device=DEV)
                ctx.ffn_stack(cases[0].shape, hm, [c.pred], [c.w], [c.comp], ks[l:l + 1], 516, 1e-6, idx1, x1)
                y32 = torch.empty((shp.n_tokens, shp.d_model), dtype=torch.float32, device=DEV)
                ctx.sparse_ffn(cases[0].shape, x1[0], c.w, c.comp, idx1[0], list(ks[l]), 516, y32, B.OUT_F32)
                expect = (h_in.float() + y32.to(torch.bfloat16).float()).to(torch.bfloat16)
                assert torch.equal(hm.view(torch.int16), expect.view(torch.int16)), f"merge_blocks={merge} layer {l}"
            dm_ = hm.float().cpu().numpy().astype(np.float64) - h_prev
            assert np.sqrt((dm_ * dm_).mean()) / np.sqrt((h_prev ** 2).mean()) < 1e-2
    finally:
        ctx.set_option("merge_blocks", -1)


# ------------------------------------------------------------------ the boundary without PyTorch

def test_plain_c_caller_outside_pytorch(tmp_path, c0):
    """csrc/ff_c_example.c (plain C, HIP runtime, libfastforward; built beforehand by build()) runs
    predict + sparse_ffn on the c0 inputs in a process of its own; its lists and outputs are held
    against the oracle like the binding's."""
    import os
    import subprocess
    pkg = os.path.dirname(os.path.abspath(B.__file__))
    exe = os.path.join(pkg, "_build", "ff_c_example")
    if not os.path.exists(exe):
        pytest.skip("ff_c_example not built (python -c 'import __graft_entry__ as g; g.build()')")
    shp, lt, k = c0.shp, c0.lt, 344
    inp, out = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(inp, "wb") as f:
        np.array([shp.d_model, shp.d_ffn, c0.T, shp.block, shp.r_pred, shp.r_comp, k], dtype=np.int32).tofile(f)
        for a in (c0.x_bits, lt.w_gate, lt.w_up, lt.w_down, lt.w1, lt.w2, lt.wc1, lt.wc2):
            np.ascontiguousarray(a, dtype=np.uint16).tofile(f)
    r = subprocess.run([exe, str(inp), str(out)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert r.returncode == 0, r.stdout
    nB = c0.n_blocks
    idx = np.fromfile(out, dtype=np.int32, count=nB * k).reshape(nB, k)
    y = np.fromfile(out, dtype=np.float32, offset=nB * k * 4).reshape(c0.T, shp.d_model)
    ks = [k] * nB
    ref = c0.oracle_layer(ks)
    for b in range(nB):
        np.testing.assert_array_equal(idx[b], ref.indices[b], err_msg=f"block {b}")
    _check_y(torch.from_numpy(y), ref.y, "plain C caller")


# ------------------------------------------------------------------ c1 whole, c2 sampled

def test_c1_full_layer(ctx):
    c = Case(W.CONFIGS["c1"])
    k = O.k_from_sparsity(c.shp.d_ffn, 0.5)
    ks = [k] * c.n_blocks
    ref = c.oracle_layer(ks)
    idx, _ = c.gpu_predict(ctx, ks)
    _assert_indices(idx, ref.indices, ks)
    _check_both(c, ctx, idx, ks, ref.y, "c1")


def test_c2_indices_all_blocks_outputs_sampled(ctx):
    c = Case(W.CONFIGS["c2"])
    k = O.k_from_sparsity(c.shp.d_ffn, 0.5)
    ks = [k] * c.n_blocks
    sample = [0, 17, 40, c.n_blocks - 1]
    ref = c.oracle_layer(ks, blocks=sample)
    idx, _ = c.gpu_predict(ctx, ks)
    _assert_indices(idx, ref.indices, ks)
    assert min(ref.margins) > 1e-9 * max(ref.score_absmax)
    _check_both(c, ctx, idx, ks, ref.y, "c2 (4 blocks sampled)")
    # dense at the same shape (Eq. 10): one whole block of tokens and rows spread over the prompt,
    # fp32 output at the stated bars; the bf16 output is its rounding, every element
    ctx.ensure_workspace(c.shape, c.shp.d_ffn)
    y32 = torch.empty((c.T, c.shp.d_model), dtype=torch.float32, device=DEV)
    ctx.dense_ffn(c.shape, c.x, c.w, y32, B.OUT_F32)
    rows = np.concatenate([np.arange(23 * 128, 24 * 128), [0, 1, 127, 128, 4095, 8191]])
    yd = O.dense_ffn(_f32(c.x_bits)[rows], c.host("w_gate"), c.host("w_up"), c.host("w_down").T)
    _check_y(y32[torch.from_numpy(rows).to(DEV)], yd, "c2 dense (block 23 whole + 6 rows)")
    y16 = torch.empty((c.T, c.shp.d_model), dtype=torch.bfloat16, device=DEV)
    ctx.dense_ffn(c.shape, c.x, c.w, y16, B.OUT_BF16)
    _check_bf16_storage(y16, y32, None, "c2 dense")


def test_c2_softmax_pooling_indices_all_blocks(ctx):
    # Eq. 12 with a query vector at the benchmark's size: every block's list, bit for bit
    c = Case(W.CONFIGS["c2"], with_q=True)
    k = O.k_from_sparsity(c.shp.d_ffn, 0.5)
    ks = [k] * c.n_blocks
    ref = c.oracle_layer(ks, compute_ffn=False)
    idx, _ = c.gpu_predict(ctx, ks)
    _assert_indices(idx, ref.indices, ks)
    assert min(ref.margins) > 1e-9 * max(ref.score_absmax)


# ------------------------------------------------------------------ c3: sparsity sweep, two block sizes

@pytest.mark.parametrize("block", W.C3_BLOCKS)
def test_c3_sweep_indices_all_blocks_outputs_sampled(ctx, block):
    base = W.CONFIGS["c3"]
    shp = W.Shape(base.name, base.d_model, base.d_ffn, base.n_tokens, block, base.r_pred, base.r_comp)
    c = Case(shp)
    g = np.random.Generator(np.random.Philox(key=[31, block]))
    dense_macs = 3 * shp.n_tokens * shp.d_model * shp.d_ffn
    for sparsity in W.C3_SPARSITIES:
        k = O.k_from_sparsity(shp.d_ffn, sparsity)
        assert k == B.k_from_sparsity(shp.d_ffn, sparsity)
        ks = [k] * c.n_blocks
        sample = sorted({0, c.n_blocks - 1, int(g.integers(1, c.n_blocks - 1))})
        ref = c.oracle_layer(ks, blocks=sample)
        idx, _ = c.gpu_predict(ctx, ks)
        _assert_indices(idx, ref.indices, ks)
        assert min(ref.margins) > 1e-9 * max(ref.score_absmax)
        _check_both(c, ctx, idx, ks, ref.y, f"c3 block {block} s={sparsity}")
        # FLOPs of the sampled blocks scale with 1 - sparsity
        tok = sum(min(shp.n_tokens, (b + 1) * block) - b * block for b in sample)
        assert ref.macs_ffn * shp.n_tokens == dense_macs * tok * k // shp.d_ffn


# ------------------------------------------------------------------ c4: 28-layer stack, layer-wise teacher forced

def test_c4_stack_indices_all_layers_outputs_sampled(ctx):
    shp = W.CONFIGS["c4"]
    L = shp.n_layers
    T, dm, nB = shp.n_tokens, shp.d_model, shp.n_blocks
    spars = W.layer_sparsities(L)
    assert abs(spars.mean() - 0.5) < 1e-12
    k_layer = [O.k_from_sparsity(shp.d_ffn, s) for s in spars]
    ks = np.array([[k] * nB for k in k_layer], dtype=np.int32)
    k_stride = int(max(k_layer))
    shape = B.Shape(dm, shp.d_ffn, T, shp.block, shp.r_pred, shp.r_comp)
    sampled_layers = [0, 13, L - 1]
    host = {}
    dev, preds, ws, comps = [], [], [], []
    for l in range(L):
        lt = W.make_layer(shp, layer=l)
        d, pr, w, cp = B.make_structs(lt, DEV)
        dev.append(d); preds.append(pr); ws.append(w); comps.append(cp)
        host[l] = {"w1": _f32(lt.w1), "w2": _f32(lt.w2)}
        if l in sampled_layers:
            host[l].update({n: _f32(getattr(lt, n)) for n in ("w_gate", "w_up", "w_down", "wc1", "wc2")})
        del lt
        print(f"[c4] layer {l} weights on the device", flush=True)
    h0_bits = W.make_hidden(shp)
    h = B.to_device_bf16(h0_bits, DEV).clone()
    idx = torch.empty((L, nB, k_stride), dtype=torch.int32, device=DEV)
    xd = torch.empty((L, T, dm), dtype=torch.bfloat16, device=DEV)
    ctx.ensure_workspace(shape, k_stride)
    ctx.ffn_stack(shape, h, preds, ws, comps, ks, k_stride, 1e-6, idx, xd)
    torch.cuda.synchronize()
    print("[c4] stack done", flush=True)
    g = np.random.Generator(np.random.Philox(key=[41, 41]))
    # x of layer 0 is the RMSNorm of the input prompt
    x0 = xd[0].float().cpu().numpy().astype(np.float64)
    ref_x0 = O.bf16_round(O.rmsnorm_rows(_f32(h0_bits), 1e-6))
    assert (x0 != ref_x0).mean() < 1e-3
    np.testing.assert_allclose(x0, ref_x0, rtol=2 ** -7, atol=1e-30)
    min_margin = np.inf
    for l in range(L):
        x_gpu = xd[l].float().cpu().numpy().astype(np.float64)       # teacher forcing: the GPU's own layer input
        kl = list(ks[l])
        blocks = sorted({0, nB - 1, int(g.integers(1, nB - 1))}) if l in sampled_layers else []
        hw = host[l]
        if l in sampled_layers:
            res = O.fastforward_layer(x_gpu, hw["w_gate"], hw["w_up"], hw["w_down"].T, hw["w1"], hw["w2"], shp.block,
                                      kl, wc1=hw["wc1"].T, wc2=hw["wc2"], blocks=blocks)
        else:
            res = O.fastforward_layer(x_gpu, None, None, None, hw["w1"], hw["w2"], shp.block, kl, compute_ffn=False)
        _assert_indices(idx[l], res.indices, kl)
        min_margin = min(min_margin, min(m / a for m, a in zip(res.margins, res.score_absmax)))
        if l in sampled_layers:
            # y of the layer = h_next - h is not kept; recompute it on the GPU from the dumped x and indices
            y = torch.empty((T, dm), dtype=torch.float32, device=DEV)
            ctx.sparse_ffn(shape, xd[l], ws[l], comps[l], idx[l], kl, k_stride, y, B.OUT_F32)
            _check_y(y, res.y, f"c4 layer {l} (blocks {blocks}) f32")
            # What the stack itself writes, every element: its first l layers followed by layer l alone
            # give the same lists and the same layer input as the full pass, and the carried state is
            # bf16(h + bf16(y)) of the fp32 output of the same kernels on that input (the residual add
            # sits in the down GEMM's epilogue: same accumulators, two roundings).
            h_l = B.to_device_bf16(h0_bits, DEV).clone()
            if l > 0:
                ctx.ffn_stack(shape, h_l, preds[:l], ws[:l], comps[:l], ks[:l], k_stride, 1e-6, None, None)
            h_in = h_l.clone()
            idx1 = torch.empty((1, nB, k_stride), dtype=torch.int32, device=DEV)
            x1 = torch.empty((1, T, dm), dtype=torch.bfloat16, device=DEV)
            ctx.ffn_stack(shape, h_l, preds[l:l + 1], ws[l:l + 1], comps[l:l + 1], ks[l:l + 1], k_stride, 1e-6, idx1, x1)
            assert torch.equal(idx1[0], idx[l]) and torch.equal(x1[0].view(torch.int16), xd[l].view(torch.int16))
            expect = (h_in.float() + y.to(torch.bfloat16).float()).to(torch.bfloat16)
            assert torch.equal(h_l.view(torch.int16), expect.view(torch.int16)), f"layer {l}: carried state is not bf16(h + bf16(y))"
            if l == L - 1:
                assert torch.equal(h_l.view(torch.int16), h.view(torch.int16)), "the full pass ends elsewhere than its layers one by one"
            del h_l, h_in, idx1, x1, expect
        print(f"[c4] layer {l} checked", flush=True)
    # Layers after the first see the GPU's own carried state, so their margins are no fixed property of the
    # workload: with 3584 blocks a relative margin below 1e-9 ("numerically tied") turns up now and then
    # (chance of a few per cent).  The lists above are bit-equal all the same; what must hold is that the
    # smallest margin stays far above the rounding of the fp64 sums (about 1e-13 relative).
    print(f"[c4] smallest relative selection margin over all layers and blocks: {min_margin:.3e}", flush=True)
    assert min_margin > 1e-12
    assert torch.isfinite(h.float()).all()
