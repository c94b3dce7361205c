"""Pins for the CPU oracle: each check compares an oracle function with
something that is not the oracle - a closed form worked out by hand, a brute
force scalar loop on a tiny input, a library routine (torch fp64 / scipy) on a
special case, or an invariant the paper's equations imply.  CPU only."""
import itertools
import math

import numpy as np
import pytest
import torch

from oracle import ff_oracle as O
from paper_2602_00397_amd import workloads as W


def _rand(shape, seed, std=1.0):
    g = np.random.Generator(np.random.Philox(key=[seed, 1234]))
    return g.standard_normal(shape) * std


def _tiny(seed=0, T=12, dm=6, df=10, r=4, rc=3):
    return dict(
        x=_rand((T, dm), seed + 1), wg=_rand((df, dm), seed + 2, 0.5),
        wu=_rand((df, dm), seed + 3, 0.5), wd=_rand((dm, df), seed + 4, 0.5),
        w1=_rand((dm, r), seed + 5), w2=_rand((r, df), seed + 6),
        wc1=_rand((dm, rc), seed + 7, 0.5), wc2=_rand((rc, dm), seed + 8, 0.5))


# ---------------------------------------------------------------- K and SiLU

def test_k_from_sparsity_values():
    # 50% / 25% / 75% of the benchmark widths; exact products, no rounding doubt
    assert O.k_from_sparsity(688, 0.5) == 344
    assert O.k_from_sparsity(8192, 0.5) == 4096
    assert O.k_from_sparsity(14336, 0.5) == 7168
    assert O.k_from_sparsity(14336, 0.25) == 10752
    assert O.k_from_sparsity(14336, 0.75) == 3584
    assert O.k_from_sparsity(18944, 0.5) == 9472
    assert O.k_from_sparsity(688, 0.25) == 516 and O.k_from_sparsity(688, 0.75) == 172
    assert O.k_from_sparsity(14336, 0.0) == 14336
    assert O.k_from_sparsity(10, 1.0) == 1          # at least one neuron
    assert O.k_from_sparsity(7, 0.5) == 4           # 3.5 rounds half up


def test_silu_closed_forms_and_scipy():
    from scipy.special import expit
    assert O.silu(np.array([0.0]))[0] == 0.0
    # silu(ln 3) = ln3 / (1 + 1/3) = 0.75 ln 3 ; silu(-ln 3) = -ln3 / 4
    assert O.silu(np.array([math.log(3)]))[0] == pytest.approx(0.75 * math.log(3), rel=1e-15)
    assert O.silu(np.array([-math.log(3)]))[0] == pytest.approx(-0.25 * math.log(3), rel=1e-15)
    v = np.linspace(-30, 30, 601)
    np.testing.assert_allclose(O.silu(v), v * expit(v), rtol=1e-14, atol=1e-300)
    # far tails: silu(v) -> v and -> 0 without overflow warnings turning to nan
    assert O.silu(np.array([800.0]))[0] == 800.0
    assert O.silu(np.array([-800.0]))[0] == 0.0


# ---------------------------------------------------------------- pooling, Eq. 12

def test_pool_mean_is_q_zero_and_single_token():
    x = _rand((7, 5), 11)
    a_mean = O.pool_block(x, None)
    np.testing.assert_allclose(a_mean, x.mean(axis=0), rtol=1e-15)
    a_q0 = O.pool_block(x, np.zeros(5))
    np.testing.assert_allclose(a_q0, a_mean, rtol=1e-15, atol=1e-16)
    # N_block = 1: the softmax over one token is 1, a = x
    np.testing.assert_array_equal(O.pool_block(x[:1], _rand((5,), 3)), x[0])


def test_pool_softmax_hand_example():
    # d_model = 4 so sqrt(d_model) = 2.  q = (2 ln 3, 0, 0, 0); tokens x0 =
    # (1,10,0,0), x1 = (0,20,0,0): z = (ln 3, 0), softmax = (3/4, 1/4),
    # a = (3/4, 7.5 + 5, 0, 0).
    q = np.array([2 * math.log(3), 0, 0, 0])
    x = np.array([[1.0, 10, 0, 0], [0.0, 20, 0, 0]])
    np.testing.assert_allclose(O.pool_block(x, q), [0.75, 12.5, 0, 0], rtol=1e-15)


def test_pool_against_torch_softmax():
    x = _rand((9, 16), 21)
    q = _rand((16,), 22)
    xt, qt = torch.tensor(x), torch.tensor(q)
    ref = torch.softmax((qt @ xt.T) / math.sqrt(16), dim=0) @ xt
    np.testing.assert_allclose(O.pool_block(x, q), ref.numpy(), rtol=1e-13)


# ---------------------------------------------------------------- scores, Eq. 13

def test_scores_hand_example_and_relu():
    # one token so a = x = (1, -2); W1 = [[1, 1], [1, -1]] -> a W1 = (-1, 3),
    # ReLU -> (0, 3); W2 = [[5, 6, 7], [1, -1, 2]] -> s = (3, -3, 6).
    x = np.array([[1.0, -2.0]])
    w1 = np.array([[1.0, 1.0], [1.0, -1.0]])
    w2 = np.array([[5.0, 6.0, 7.0], [1.0, -1.0, 2.0]])
    np.testing.assert_array_equal(O.predictor_scores(x, None, w1, w2), [3.0, -3.0, 6.0])


def test_scores_against_torch():
    t = _tiny(31)
    xt = torch.tensor(t["x"][:5])
    ref = torch.relu(xt.mean(0) @ torch.tensor(t["w1"])) @ torch.tensor(t["w2"])
    np.testing.assert_allclose(O.predictor_scores(t["x"][:5], None, t["w1"], t["w2"]),
                               ref.numpy(), rtol=1e-13)


# ---------------------------------------------------------------- top-K, Eq. 14

def _brute_topk(s, k):
    order = sorted(range(len(s)), key=lambda j: (-s[j], j))
    return sorted(order[:k])


def test_topk_brute_force_with_ties():
    g = np.random.Generator(np.random.Philox(key=[5, 5]))
    for trial in range(200):
        n = int(g.integers(1, 40))
        s = g.integers(-3, 4, size=n).astype(np.float64)     # many ties
        k = int(g.integers(1, n + 1))
        got = O.select_topk(s, k)
        assert got.dtype == np.int32
        assert got.tolist() == _brute_topk(s.tolist(), k)
        # threshold characterisation of "among the top-K"
        theta = np.sort(s)[::-1][k - 1]
        sel = np.zeros(n, bool); sel[got] = True
        assert (s[sel] >= theta).all() and (s[~sel] <= theta).all()
        assert (s > theta).sum() <= k <= (s >= theta).sum()
        tied = np.flatnonzero(s == theta)
        n_tied_taken = k - int((s > theta).sum())
        assert sel[tied].tolist() == [True] * n_tied_taken + [False] * (len(tied) - n_tied_taken)


def test_topk_all_equal_and_signed_zero():
    assert O.select_topk(np.zeros(9), 4).tolist() == [0, 1, 2, 3]
    s = np.array([-0.0, 0.0, -0.0, 0.0, 1.0])
    assert O.select_topk(s, 3).tolist() == [0, 1, 4]         # zeros tie regardless of sign
    assert O.select_topk(np.arange(6.0), 6).tolist() == [0, 1, 2, 3, 4, 5]


def test_topk_against_torch_on_tie_free_data():
    s = _rand((500,), 77)
    for k in (1, 17, 250, 499, 500):
        ref = torch.topk(torch.tensor(s), k).indices.sort().values.numpy()
        np.testing.assert_array_equal(O.select_topk(s, k), ref)


def test_exact_tie_cases_integer_inputs():
    # integer-valued inputs: every predictor sum is exact, ties are real ties
    c = W.integer_valued_case(d_model=16, d_ffn=40, n_tokens=64, r=8)
    x, w1, w2 = (W.bf16_to_f32(c[n]) for n in ("x", "w1", "w2"))
    # duplicated W2 columns -> equal scores -> the lower duplicate ranks first
    w2d = w2.copy(); w2d[:, 20:] = w2d[:, :20]
    s = O.predictor_scores(x, None, w1, w2d)
    np.testing.assert_array_equal(s[:20], s[20:])
    for k in (1, 7, 20, 21, 33):
        assert O.select_topk(s, k).tolist() == _brute_topk(s.tolist(), k)
    # ReLU kills every hidden unit -> all scores 0 -> first K indices
    xpos = np.abs(x) + 1.0
    w1neg = -np.abs(w1) - 1.0
    s0 = O.predictor_scores(xpos, None, w1neg, w2)
    assert (s0 == 0).all()
    assert O.select_topk(s0, 5).tolist() == [0, 1, 2, 3, 4]


def test_selection_margin():
    s = np.array([5.0, 1.0, 3.0, 2.5])
    assert O.selection_margin(s, 2) == 0.5
    assert O.selection_margin(s, 4) == float("inf")
    assert O.selection_margin(np.zeros(4), 2) == 0.0


# ---------------------------------------------------------------- FFN, Eq. 10 / 15-18

def _scalar_loop_sparse_ffn(x, wg, wu, wd, idx):
    """Eq. 18 spelled as scalar loops (math module only)."""
    T, dm = len(x), len(x[0])
    y = [[0.0] * dm for _ in range(T)]
    for t in range(T):
        for j in idx:
            g = sum(x[t][c] * wg[j][c] for c in range(dm))
            u = sum(x[t][c] * wu[j][c] for c in range(dm))
            h = g / (1.0 + math.exp(-g)) * u
            for c in range(dm):
                y[t][c] += h * wd[c][j]
    return np.array(y)


def test_sparse_ffn_against_scalar_loops():
    t = _tiny(41)
    idx = [1, 4, 5, 9]
    ref = _scalar_loop_sparse_ffn(t["x"].tolist(), t["wg"].tolist(), t["wu"].tolist(),
                                  t["wd"].tolist(), idx)
    np.testing.assert_allclose(O.sparse_ffn_block(t["x"], t["wg"], t["wu"], t["wd"], idx),
                               ref, rtol=1e-12, atol=1e-14)


def test_single_neuron_closed_form():
    # one neuron j: y_t = silu(x_t.wg_j) * (x_t.wu_j) * wd[:, j].  x = (1, 2),
    # wg_j = (ln3, 0) -> g = ln 3, silu = 0.75 ln 3; wu_j = (0, 2) -> u = 4;
    # wd[:, j] = (1, -1) -> y = (3 ln 3, -3 ln 3).  Other neurons hold junk.
    wg = np.array([[9.0, 9.0], [math.log(3), 0.0]])
    wu = np.array([[9.0, 9.0], [0.0, 2.0]])
    wd = np.array([[7.0, 1.0], [7.0, -1.0]])
    y = O.sparse_ffn_block(np.array([[1.0, 2.0]]), wg, wu, wd, [1])
    np.testing.assert_allclose(y, [[3 * math.log(3), -3 * math.log(3)]], rtol=1e-15)


def test_gate_zero_gives_zero_and_large_gate_is_linear():
    t = _tiny(43)
    y0 = O.sparse_ffn_block(t["x"], np.zeros_like(t["wg"]), t["wu"], t["wd"], [0, 3, 7])
    assert (y0 == 0).all()
    # gate pre-activation = +100 for every token: silu(100) = 100 to 1e-42
    x = np.abs(t["x"]) + 0.1
    wg = np.zeros_like(t["wg"]); wg[:, 0] = 100.0 / 1.0
    xs = x.copy(); xs[:, 0] = 1.0
    idx = [2, 6]
    y = O.sparse_ffn_block(xs, wg, t["wu"], t["wd"], idx)
    lin = (100.0 * (xs @ t["wu"][idx].T)) @ t["wd"][:, idx].T
    np.testing.assert_allclose(y, lin, rtol=1e-13)


def test_all_neurons_selected_is_dense_ffn():
    # Eq. 18 with M = 1 is Eq. 10
    t = _tiny(45, T=16)
    df = t["wg"].shape[0]
    ys = O.sparse_ffn_block(t["x"], t["wg"], t["wu"], t["wd"], np.arange(df))
    yd = O.dense_ffn(t["x"], t["wg"], t["wu"], t["wd"])
    np.testing.assert_allclose(ys, yd, rtol=1e-14, atol=1e-15)
    # and the dense form against torch's own silu / matmul, in the X W orientation of Eq. 10
    X = torch.tensor(t["x"])
    ref = (torch.nn.functional.silu(X @ torch.tensor(t["wg"]).T) * (X @ torch.tensor(t["wu"]).T)) \
        @ torch.tensor(t["wd"]).T
    np.testing.assert_allclose(yd, ref.numpy(), rtol=1e-13, atol=1e-14)


def test_sparse_equals_dense_with_unselected_neurons_zeroed():
    # dropping a neuron == zeroing its down column: ties Eq. 15-17's gather to Eq. 10
    t = _tiny(47)
    idx = np.array([0, 2, 3, 8])
    wd0 = np.zeros_like(t["wd"]); wd0[:, idx] = t["wd"][:, idx]
    np.testing.assert_allclose(O.sparse_ffn_block(t["x"], t["wg"], t["wu"], t["wd"], idx),
                               O.dense_ffn(t["x"], t["wg"], t["wu"], wd0), rtol=1e-13, atol=1e-15)


def test_neuron_permutation_invariance():
    t = _tiny(49, T=8)
    df = t["wg"].shape[0]
    perm = np.random.Generator(np.random.Philox(key=[1, 2])).permutation(df)
    k = 4
    r0 = O.fastforward_layer(t["x"], t["wg"], t["wu"], t["wd"], t["w1"], t["w2"], 4, [k, k])
    r1 = O.fastforward_layer(t["x"], t["wg"][perm], t["wu"][perm], t["wd"][:, perm],
                             t["w1"], t["w2"][:, perm], 4, [k, k])
    for b in range(2):
        assert sorted(perm[r1.indices[b]].tolist()) == r0.indices[b].tolist()
    np.testing.assert_allclose(r1.y, r0.y, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- compensator, Eq. 20-21

def test_compensator_hand_example_and_sum():
    # x = (1, 1); Wc1 = [[ln3], [0]] -> pre = ln 3 -> silu = 0.75 ln 3;
    # Wc2 = [[2, -4]] -> Y_comp = (1.5 ln 3, -3 ln 3)
    yc = O.compensator_block(np.array([[1.0, 1.0]]), np.array([[math.log(3)], [0.0]]),
                             np.array([[2.0, -4.0]]))
    np.testing.assert_allclose(yc, [[1.5 * math.log(3), -3 * math.log(3)]], rtol=1e-15)
    t = _tiny(51)
    k = [3, 3, 3]
    plain = O.fastforward_layer(t["x"], t["wg"], t["wu"], t["wd"], t["w1"], t["w2"], 4, k)
    comp = O.fastforward_layer(t["x"], t["wg"], t["wu"], t["wd"], t["w1"], t["w2"], 4, k,
                               wc1=t["wc1"], wc2=t["wc2"])
    X = torch.tensor(t["x"])
    ref = torch.nn.functional.silu(X @ torch.tensor(t["wc1"])) @ torch.tensor(t["wc2"])
    np.testing.assert_allclose(comp.y - plain.y, ref.numpy(), rtol=1e-10, atol=1e-13)
    for name, fn in (("relu", lambda v: np.maximum(v, 0)), ("identity", lambda v: v)):
        np.testing.assert_allclose(O.compensator_block(t["x"], t["wc1"], t["wc2"], name),
                                   fn(t["x"] @ t["wc1"]) @ t["wc2"], rtol=1e-13)


# ---------------------------------------------------------------- whole layer

def test_layer_blocking_independence_and_mac_counts():
    t = _tiny(53, T=14, df=12)          # blocks of 4 -> 4, 4, 4, 2 (short tail)
    ks = [6, 6, 6, 6]
    r0 = O.fastforward_layer(t["x"], t["wg"], t["wu"], t["wd"], t["w1"], t["w2"], 4, ks,
                             wc1=t["wc1"], wc2=t["wc2"])
    assert [len(i) for i in r0.indices] == ks and not np.isnan(r0.y).any()
    # block 1 must not change when every other block's tokens change
    x2 = t["x"].copy(); x2[:4] += 1.0; x2[8:] -= 2.0
    r1 = O.fastforward_layer(x2, t["wg"], t["wu"], t["wd"], t["w1"], t["w2"], 4, ks,
                             wc1=t["wc1"], wc2=t["wc2"])
    np.testing.assert_array_equal(r0.indices[1], r1.indices[1])
    np.testing.assert_array_equal(r0.y[4:8], r1.y[4:8])
    assert not np.array_equal(r0.y[:4], r1.y[:4])
    # each block equals the one-block computation on its own tokens
    for b, (a, e) in enumerate(O.block_ranges(14, 4)):
        s = O.predictor_scores(t["x"][a:e], None, t["w1"], t["w2"])
        np.testing.assert_array_equal(O.select_topk(s, 6), r0.indices[b])
    # MACs: 3 T d_model K for the FFN, 2 T d_model r' for the compensator
    T, dm = t["x"].shape
    assert r0.macs_ffn == 3 * T * dm * 6
    assert r0.macs_comp == 2 * T * dm * t["wc1"].shape[1]


def test_ffn_macs_scale_with_one_minus_sparsity():
    shp = W.CONFIGS["c0"]
    dm, df = 32, shp.d_ffn            # narrow d_model keeps this fast; d_ffn = 688 as in c0
    x = _rand((128, dm), 61); wg = _rand((df, dm), 62); wu = _rand((df, dm), 63)
    wd = _rand((dm, df), 64); w1 = _rand((dm, 8), 65); w2 = _rand((8, df), 66)
    dense_macs = 3 * 128 * dm * df
    for s in (0.0, 0.25, 0.5, 0.75):
        k = O.k_from_sparsity(df, s)
        r = O.fastforward_layer(x, wg, wu, wd, w1, w2, 64, [k, k])
        assert r.macs_ffn * 4 == dense_macs * round(4 * (1 - s))
        if s == 0.0:
            np.testing.assert_allclose(r.y, O.dense_ffn(x, wg, wu, wd), rtol=1e-12, atol=1e-13)


def test_layer_on_c0_against_torch_pipeline():
    # the whole tiny benchmark config against torch fp64 library calls
    shp = W.CONFIGS["c0"]
    lt = W.make_layer(shp)
    x = W.bf16_to_f32(W.make_hidden(shp))
    f = {n: W.bf16_to_f32(getattr(lt, n)) for n in ("w_gate", "w_up", "w_down", "w1", "w2", "wc1", "wc2")}
    k = O.k_from_sparsity(shp.d_ffn, shp.sparsity)
    res = O.fastforward_layer(x, f["w_gate"], f["w_up"], f["w_down"].T, f["w1"], f["w2"], shp.block,
                              [k] * shp.n_blocks, wc1=f["wc1"].T, wc2=f["wc2"])
    assert min(res.margins) > 0          # tie-free, so torch.topk is a valid reference
    X = torch.tensor(x, dtype=torch.float64)
    tw = {n: torch.tensor(v, dtype=torch.float64) for n, v in f.items()}
    for b in range(shp.n_blocks):
        Xb = X[b * shp.block:(b + 1) * shp.block]
        s = torch.relu(Xb.mean(0) @ tw["w1"]) @ tw["w2"]
        idx = torch.topk(s, k).indices.sort().values
        np.testing.assert_array_equal(res.indices[b], idx.numpy())
        h = torch.nn.functional.silu(Xb @ tw["w_gate"][idx].T) * (Xb @ tw["w_up"][idx].T)
        y = h @ tw["w_down"][idx] + torch.nn.functional.silu(Xb @ tw["wc1"].T) @ tw["wc2"]
        np.testing.assert_allclose(res.y[b * shp.block:(b + 1) * shp.block], y.numpy(),
                                   rtol=1e-9, atol=1e-12)


# ---------------------------------------------------------------- stack glue

def test_bf16_round_rne():
    one = 1.0
    cases = {one: one, one + 2 ** -8: one, one + 3 * 2 ** -8: one + 2 ** -6,
             one + 2 ** -8 + 2 ** -20: one + 2 ** -7, -(one + 3 * 2 ** -8): -(one + 2 ** -6),
             0.0: 0.0, 3.0e38: float(np.float32(2.0 ** 127 * 1.765625))}
    for v, want in cases.items():
        assert O.bf16_round(np.array([v]))[0] == want
    v = _rand((4096,), 71).astype(np.float32)
    ref = torch.tensor(v).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.bf16_round(v), ref)


def test_rmsnorm_against_torch():
    h = _rand((5, 32), 73) * 3
    ref = torch.nn.functional.rms_norm(torch.tensor(h), (32,), eps=1e-6).numpy()
    np.testing.assert_allclose(O.rmsnorm_rows(h, 1e-6), ref, rtol=1e-13)
    # constant row c: mean square c^2 -> x = c / sqrt(c^2 + eps)
    np.testing.assert_allclose(O.rmsnorm_rows(np.full((1, 8), 2.0), 0.0), np.ones((1, 8)), rtol=1e-15)


def test_stack_layer_composition():
    t = _tiny(75, T=8)
    lw = dict(w_gate=t["wg"], w_up=t["wu"], w_down=t["wd"], w1=t["w1"], w2=t["w2"],
              wc1=t["wc1"], wc2=t["wc2"])
    h = O.bf16_round(t["x"])
    x, res, h1 = O.stack_layer(h, lw, 4, [5, 5], 1e-6)
    ref_x = torch.nn.functional.rms_norm(torch.tensor(h), (6,), eps=1e-6).to(torch.bfloat16).double().numpy()
    np.testing.assert_array_equal(x, ref_x)
    y = O.fastforward_layer(ref_x, block=4, k_per_block=[5, 5], **lw).y
    np.testing.assert_array_equal(h1, torch.tensor(h + y).to(torch.bfloat16).double().numpy())


# ---------------------------------------------------------------- Alg. 1

def test_alg1_hand_worked_examples():
    # scores (1,2,1), B = 0.5, L = 3: T = 1.5, S = 4
    #   b1 = min(1, 1/4 * 1.5) = 0.375      T = 1.125, S = 3
    #   b2 = min(1, 2/3 * 1.125) = 0.75     T = 0.375, S = 1
    #   b3 = min(1, 1/1 * 0.375) = 0.375
    np.testing.assert_allclose(O.layerwise_budgets([1, 2, 1], 0.5), [0.375, 0.75, 0.375], rtol=1e-15)
    # scores (6,1,1): first share 6/8 * 1.5 = 1.125 is capped at 1, the rest
    # (0.5) is split over what is left: 0.25, 0.25
    np.testing.assert_allclose(O.layerwise_budgets([6, 1, 1], 0.5), [1.0, 0.25, 0.25], rtol=1e-15)


def test_alg1_invariants():
    np.testing.assert_allclose(O.layerwise_budgets([3.0] * 7, 0.4), [0.4] * 7, rtol=1e-14)
    g = np.random.Generator(np.random.Philox(key=[9, 9]))
    for _ in range(50):
        L = int(g.integers(2, 33))
        s = g.random(L) + 0.05
        B = float(g.uniform(0.2, 0.8))
        b = O.layerwise_budgets(s, B)
        assert (b <= 1.0).all() and (b > 0).all()
        # the last layer takes all that is left unless the cap stops it
        if b[-1] < 1.0:
            assert b.sum() == pytest.approx(B * L, rel=1e-12)
        else:
            assert b.sum() <= B * L + 1e-12
        if (s / s.sum() * B * L <= 1).all():                  # no cap hit: plain proportional split
            np.testing.assert_allclose(b, s / s.sum() * B * L, rtol=1e-12)


# ---------------------------------------------------------------- synthetic inputs

def test_workload_generator_is_deterministic_and_bf16():
    shp = W.CONFIGS["c0"]
    a, b = W.make_hidden(shp), W.make_hidden(shp)
    np.testing.assert_array_equal(a, b)
    assert a.dtype == np.uint16 and a.shape == (256, 256)
    np.testing.assert_array_equal(W.make_hidden(shp, n_tokens=64), a[:64])
    lt = W.make_layer(shp)
    w = W.bf16_to_f32(lt.w_gate)
    assert lt.w_gate.shape == (688, 256) and lt.w_down.shape == (688, 256)
    assert abs(w.std() - 0.02) < 1e-3 and abs(W.bf16_to_f32(lt.w1).std() - 0.05) < 3e-3
    v = _rand((1000,), 5).astype(np.float32)
    np.testing.assert_array_equal(W.f32_to_bf16_bits(v).view(np.int16),
                                  torch.tensor(v).to(torch.bfloat16).view(torch.int16).numpy())
    s = W.layer_sparsities(28)
    assert s.mean() == pytest.approx(0.5, abs=1e-12) and s.min() >= 0.25 and s.max() <= 0.75


def test_c0_digest_fixture_is_current():
    """tests/golden/c0_oracle_digest.json (written by tests/golden/make_c0_fixture.py from the
    oracle alone) still describes what the oracle and the input generator produce: a change of
    either must come with a regenerated, reviewed fixture."""
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_c0_fixture", os.path.join(here, "make_c0_fixture.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.digest()
    with open(os.path.join(here, "c0_oracle_digest.json")) as fh:
        stored = json.load(fh)
    assert now["indices_sha256"] == stored["indices_sha256"]
    assert (now["k"], now["macs_ffn"], now["macs_comp"], now["macs_predictor"]) == \
           (stored["k"], stored["macs_ffn"], stored["macs_comp"], stored["macs_predictor"])
    for key in ("y_sum", "y_l2", "y_absmax"):
        assert abs(now[key] - stored[key]) <= 1e-10 * abs(stored[key])
    for (t, c, v), (t2, c2, v2) in zip(now["y_samples"], stored["y_samples"]):
        assert (t, c) == (t2, c2) and abs(v - v2) <= 1e-10 * max(abs(v2), 1e-3)
    for m, m2 in zip(now["margins"], stored["margins"]):
        assert abs(m - m2) <= 1e-6 * abs(m2)
