"""Pins for the fp64 oracle's model, gradients and optimizer: finite
differences, an autograd re-derivation through library primitives, closed
forms, invariants and degenerate cases.  Each would fail on a dropped term, a
wrong sign or index, or a transposed operand somewhere in oracle/model.py."""
import math

import numpy as np
import pytest
import torch

from oracle import model as om
from paper_2202_01306_amd import synth
from tests.helpers import f64, max_rel_err, oracle_spec, tiny_cfg


def _setup(cfg, seed=0, mlm=False):
    spec = oracle_spec(cfg)
    params = f64(synth.gen_params(cfg, seed, bench_init=False))
    # larger weights than the benchmark recipe so that attention is not uniform
    for k in params:
        if params[k].ndim == 2:
            params[k] = params[k] * 10.0
    ids = synth.gen_tokens(cfg, seed)
    tg = synth.mlm_targets(ids, 0.3, seed) if mlm else synth.decoder_targets(ids)
    return spec, params, ids, tg


@pytest.mark.parametrize("causal,mlm", [(1, False), (0, True), (1, True)])
def test_gradients_match_central_finite_differences(causal, mlm):
    cfg = tiny_cfg(causal=causal)
    spec, params, ids, tg = _setup(cfg, seed=3, mlm=mlm)
    _, grads = om.iteration_microbatch_major(spec, params, ids, tg)
    rng = np.random.default_rng(0)
    h = 1e-5
    for name, w in params.items():
        gmax = max(np.abs(grads[name]).max(), 1e-12)
        flat = w.reshape(-1)
        picks = rng.choice(flat.size, size=min(6, flat.size), replace=False)
        if name == "wte":  # make sure rows that are actually used get probed
            used = np.unique(ids)[:3]
            picks = np.concatenate([picks, used * w.shape[1] + 1])
        for i in picks:
            old = flat[i]
            flat[i] = old + h
            lp = om.forward_loss(spec, params, ids, tg)
            flat[i] = old - h
            lm = om.forward_loss(spec, params, ids, tg)
            flat[i] = old
            fd = (lp - lm) / (2 * h)
            an = grads[name].reshape(-1)[i]
            assert abs(fd - an) <= 2e-7 * gmax + 1e-10, (name, i, fd, an)


def _torch_loss(cfg, params_t, ids, tg):
    """The same model through torch library primitives (F.layer_norm, F.linear,
    F.gelu(tanh), softmax, F.cross_entropy) -- gradients come from autograd."""
    import torch.nn.functional as F
    d, H, s = cfg["d_model"], cfg["n_heads"], cfg["seq_len"]
    dh = d // H
    n_tgt = int((tg >= 0).sum())
    total = 0.0
    for mb in range(ids.shape[0]):
        idt = torch.from_numpy(ids[mb].astype(np.int64))
        b = idt.shape[0]
        x = params_t["wte"][idt] + params_t["wpe"][None, :s]
        for l in range(1, cfg["n_blocks"] + 1):
            p = f"h{l}."
            a = F.layer_norm(x, (d,), params_t[p + "ln1_g"], params_t[p + "ln1_b"], synth.LN_EPS)
            qkv = F.linear(a, params_t[p + "wqkv"], params_t[p + "bqkv"])
            q, k, v = qkv.split(d, dim=-1)
            q = q.view(b, s, H, dh).transpose(1, 2)
            k = k.view(b, s, H, dh).transpose(1, 2)
            v = v.view(b, s, H, dh).transpose(1, 2)
            att = q @ k.transpose(-1, -2) / math.sqrt(dh)
            if cfg["causal"]:
                mask = torch.ones(s, s, dtype=torch.bool).tril()
                att = att.masked_fill(~mask, float("-inf"))
            o = (torch.softmax(att, dim=-1) @ v).transpose(1, 2).reshape(b, s, d)
            x = x + F.linear(o, params_t[p + "wo"], params_t[p + "bo"])
            hh = F.layer_norm(x, (d,), params_t[p + "ln2_g"], params_t[p + "ln2_b"], synth.LN_EPS)
            u = F.linear(hh, params_t[p + "w1"], params_t[p + "b1"])
            x = x + F.linear(F.gelu(u, approximate="tanh"), params_t[p + "w2"], params_t[p + "b2"])
        z = F.layer_norm(x, (d,), params_t["lnf_g"], params_t["lnf_b"], synth.LN_EPS)
        logits = F.linear(z, params_t["wh"])
        tt = torch.from_numpy(tg[mb].astype(np.int64)).reshape(-1)
        total = total + F.cross_entropy(logits.reshape(-1, cfg["vocab"]), tt,
                                        ignore_index=-1, reduction="sum") / n_tgt
    return total


@pytest.mark.parametrize("causal", [1, 0])
def test_loss_and_all_gradients_match_torch_autograd(causal):
    cfg = tiny_cfg(causal=causal, n_blocks=2, d_model=24, n_heads=3, d_ffn=40, seq_len=10, vocab=37,
                   M=3, b=2)
    spec, params, ids, tg = _setup(cfg, seed=5, mlm=not causal)
    loss, grads = om.iteration_microbatch_major(spec, params, ids, tg)
    pt = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in params.items()}
    lt = _torch_loss(cfg, pt, ids, tg)
    lt.backward()
    assert abs(loss - lt.item()) <= 1e-12 * abs(lt.item())
    for name in params:
        assert max_rel_err(grads[name], pt[name].grad.numpy()) < 1e-11, name


def test_microbatch_split_does_not_change_gradients():
    cfg = tiny_cfg(M=4, b=2)
    spec, params, ids, tg = _setup(cfg, seed=1)
    l1, g1 = om.iteration_microbatch_major(spec, params, ids, tg)
    ids2 = ids.reshape(1, 8, cfg["seq_len"])
    tg2 = tg.reshape(1, 8, cfg["seq_len"])
    l2, g2 = om.iteration_microbatch_major(spec, params, ids2, tg2)
    assert abs(l1 - l2) < 1e-13 * abs(l1)
    for name in g1:
        assert max_rel_err(g1[name], g2[name]) < 1e-12, name


@pytest.mark.parametrize("cfgname", ["tiny"])
def test_loss_at_benchmark_init_is_log_vocab(cfgname):
    cfg = dict(synth.CONFIGS[cfgname])
    spec = oracle_spec(cfg)
    params = f64(synth.gen_params(cfg, 0, bench_init=True))
    ids = synth.gen_tokens(cfg, 0, M=1)
    tg = synth.decoder_targets(ids)
    loss = om.forward_loss(spec, params, ids, tg)
    assert abs(loss - math.log(cfg["vocab"])) < 0.01 * math.log(cfg["vocab"])   # ln 512 = 6.238


def test_layernorm_closed_forms():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 12)) * 3 + 1.5
    eps = 1e-5
    y, cache = om.layernorm_fwd(x, np.ones(12), np.zeros(12), eps)
    assert np.abs(y.mean(axis=1)).max() < 1e-14
    var = x.var(axis=1)                       # numpy's biased variance
    np.testing.assert_allclose(y.var(axis=1), var / (var + eps), rtol=1e-12)
    # shift invariance and a library cross-check
    y2, _ = om.layernorm_fwd(x + 100.0, np.ones(12), np.zeros(12), eps)
    np.testing.assert_allclose(y2, y, atol=1e-10)
    g = rng.standard_normal(12)
    bta = rng.standard_normal(12)
    yt = torch.nn.functional.layer_norm(torch.tensor(x), (12,), torch.tensor(g), torch.tensor(bta), eps)
    np.testing.assert_allclose(om.layernorm_fwd(x, g, bta, eps)[0], yt.numpy(), rtol=1e-12, atol=1e-13)
    dy = rng.standard_normal((7, 12))
    dx, dg, db = om.layernorm_bwd(dy, om.layernorm_fwd(x, g, bta, eps)[1], g)
    np.testing.assert_allclose(db, dy.sum(axis=0), rtol=1e-13)
    # with eps = 0, dx is orthogonal to the all-ones vector and to xhat
    # (the Jacobian of normalisation projects both directions out)
    _, c0 = om.layernorm_fwd(x, g, bta, 0.0)
    dx0, _, _ = om.layernorm_bwd(dy, c0, g)
    assert np.abs(dx0.sum(axis=1)).max() < 1e-12
    assert np.abs((dx0 * c0[0]).sum(axis=1)).max() < 1e-12
    assert np.abs(dx.sum(axis=1)).max() < 1e-12


def test_gelu_values_and_derivative():
    assert om.gelu_fwd(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(om.gelu_fwd(np.array([10.0, -10.0])), [10.0, 0.0], atol=1e-12)
    # published value of tanh-GELU at 1: 0.841192
    assert abs(om.gelu_fwd(np.array([1.0]))[0] - 0.8411919906) < 1e-9
    u = np.linspace(-4, 4, 41)
    h = 1e-6
    fd = (om.gelu_fwd(u + h) - om.gelu_fwd(u - h)) / (2 * h)
    np.testing.assert_allclose(om.gelu_bwd(np.ones_like(u), u), fd, atol=1e-8)
    ut = torch.tensor(u)
    np.testing.assert_allclose(om.gelu_fwd(u),
                               torch.nn.functional.gelu(ut, approximate="tanh").numpy(), atol=1e-14)


def test_attention_invariants():
    cfg = tiny_cfg(d_model=16, n_heads=2, seq_len=8)
    rng = np.random.default_rng(2)
    b, s, d = 2, 8, 16
    qkv = rng.standard_normal((b * s, 3 * d))
    for causal in (True, False):
        spec = oracle_spec(dict(cfg, causal=int(causal)))
        out, (q, k, v, P) = om.attention_fwd(qkv, spec, b)
        np.testing.assert_allclose(P.sum(axis=-1), 1.0, rtol=1e-13)
        if causal:
            assert np.all(np.triu(P, k=1) == 0.0)
            # position 0 sees only itself: output == its own value vector
            np.testing.assert_allclose(out[0], qkv[0, 2 * d:], rtol=1e-13)
            np.testing.assert_allclose(out[s], qkv[s, 2 * d:], rtol=1e-13)
            # changing FUTURE tokens leaves earlier outputs unchanged
            qkv2 = qkv.copy()
            qkv2[5:8] = rng.standard_normal((3, 3 * d))
            out2, _ = om.attention_fwd(qkv2, spec, b)
            np.testing.assert_array_equal(out2[:5], out[:5])
            assert np.abs(out2[5:8] - out[5:8]).max() > 1e-3
        else:
            # permuting the positions of a sequence permutes the outputs
            perm = rng.permutation(s)
            qkv2 = qkv.copy()
            qkv2[:s] = qkv[:s][perm]
            out2, _ = om.attention_fwd(qkv2, spec, b)
            np.testing.assert_allclose(out2[:s], out[:s][perm], rtol=1e-12, atol=1e-14)
    # sequences do not mix
    spec = oracle_spec(cfg)
    qkv2 = qkv.copy()
    qkv2[s:] = 0.0
    np.testing.assert_array_equal(om.attention_fwd(qkv2, spec, b)[0][:s],
                                  om.attention_fwd(qkv, spec, b)[0][:s])


def test_attention_head_layout_matches_library_sdpa():
    """Which columns belong to which head and to q/k/v: checked against
    torch's scaled_dot_product_attention on explicitly sliced heads."""
    cfg = tiny_cfg(d_model=24, n_heads=3, seq_len=6)
    spec = oracle_spec(cfg)
    rng = np.random.default_rng(4)
    b, s, d, H, dh = 2, 6, 24, 3, 8
    qkv = rng.standard_normal((b * s, 3 * d))
    out, _ = om.attention_fwd(qkv, spec, b)
    t = torch.tensor(qkv).view(b, s, 3 * d)
    for hd in range(H):
        q = t[:, :, 0 * d + hd * dh: 0 * d + (hd + 1) * dh]
        k = t[:, :, 1 * d + hd * dh: 1 * d + (hd + 1) * dh]
        v = t[:, :, 2 * d + hd * dh: 2 * d + (hd + 1) * dh]
        o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
        np.testing.assert_allclose(out.reshape(b, s, d)[:, :, hd * dh:(hd + 1) * dh], o.numpy(),
                                   rtol=1e-12, atol=1e-14)


def test_sequence_length_one_collapses_attention_to_value_projection():
    """s = 1: softmax over one key is 1, so the block is an MLP in v; the
    q and k rows of Wqkv and bqkv get exactly zero gradient."""
    cfg = tiny_cfg(n_blocks=1, d_model=8, n_heads=1, d_ffn=16, seq_len=1, vocab=11, M=1, b=5, causal=0)
    spec = oracle_spec(cfg)
    params = f64(synth.gen_params(cfg, 0, bench_init=False))
    ids = synth.gen_tokens(cfg, 0)
    tg = ids.copy()
    _, grads = om.iteration_microbatch_major(spec, params, ids, tg)
    d = 8
    assert np.all(grads["h1.wqkv"][:2 * d] == 0.0)
    assert np.all(grads["h1.bqkv"][:2 * d] == 0.0)
    assert np.abs(grads["h1.wqkv"][2 * d:]).max() > 0


def test_dlogits_rows_sum_to_zero_and_nontarget_rows_vanish():
    cfg = tiny_cfg()
    spec, params, ids, tg = _setup(cfg, seed=2, mlm=True)
    n_tgt = om.count_targets(tg)
    x = None
    for layer in range(spec.n_layers):
        x, c = om.layer_fwd(layer, x, params, spec, ids[0], tg[0], n_tgt)
    lnf, z, logits, lse, tgt, _ = c
    # re-derive dlogits through the public backward: dz = dlogits @ wh with wh = I
    p2 = dict(params)
    V, d = cfg["vocab"], cfg["d_model"]
    # direct check on the internal formula through linear_bwd identity
    dl = np.zeros_like(logits)
    rows = np.nonzero(tgt >= 0)[0]
    dl[rows] = np.exp(logits[rows] - lse[rows, None])
    assert np.abs(dl[rows].sum(axis=1) - 1.0).max() < 1e-12     # softmax rows sum to 1
    dx, g = om.head_bwd(c, params, spec)
    # rows without a target contribute nothing to dwh: remove them and recompute
    keep = tgt >= 0
    assert keep.sum() < keep.size
    c2 = (lnf, z, logits, lse, np.where(keep, tgt, -1), n_tgt)
    np.testing.assert_array_equal(om.head_bwd(c2, params, spec)[1]["wh"], g["wh"])
    # gradient of the loss w.r.t. a constant shift of all logits is zero:
    # dwh summed over the vocabulary axis is zero
    assert np.abs(g["wh"].sum(axis=0)).max() < 1e-15 * V + 1e-14


def test_linear_backward_identities():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((9, 5))
    W = rng.standard_normal((4, 5))
    dy = rng.standard_normal((9, 4))
    dx, dW, db = om.linear_bwd(dy, x, W)
    np.testing.assert_allclose(db, dy.sum(axis=0))
    # <dy, x W^T> = <dx, x> = <dW, W>
    ip = (dy * om.linear_fwd(x, W)).sum()
    assert abs(ip - (dx * x).sum()) < 1e-12 * abs(ip)
    assert abs(ip - (dW * W).sum()) < 1e-12 * abs(ip)
    assert dW.shape == W.shape and dx.shape == x.shape


def test_adam_first_step_closed_form():
    rng = np.random.default_rng(0)
    w = rng.standard_normal(100)
    g = rng.standard_normal(100) * 10.0 ** rng.integers(-6, 2, 100)
    hp = om.AdamHP(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, step=1)
    w2, m2, v2 = om.adam_update(w, g, np.zeros(100), np.zeros(100), hp)
    np.testing.assert_allclose(w2 - w, -hp.lr * g / (np.abs(g) + hp.eps), rtol=1e-9)
    np.testing.assert_allclose(m2, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v2, 0.001 * g * g, rtol=1e-9)


def test_adam_matches_torch_optimizer_over_several_steps():
    rng = np.random.default_rng(1)
    w0 = rng.standard_normal(64)
    gs = [rng.standard_normal(64) * 0.1 for _ in range(5)]
    wt = torch.tensor(w0, requires_grad=True)
    opt = torch.optim.Adam([wt], lr=3e-4, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.0)
    w, m, v = w0.copy(), np.zeros(64), np.zeros(64)
    for k, g in enumerate(gs, start=1):
        wt.grad = torch.tensor(g)
        opt.step()
        w, m, v = om.adam_update(w, g, m, v, om.AdamHP(3e-4, 0.9, 0.95, 1e-8, k))
        np.testing.assert_allclose(w, wt.detach().numpy(), rtol=1e-12, atol=1e-15)
