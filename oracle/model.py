"""The transformer stack, its gradients and Adam in plain numpy float64.

TEST INFRASTRUCTURE: the reference the GPU path is compared against.  Nothing
here is blocked, fused or reordered; every function is the textbook definition
of the operation so that it can be checked by eye.

The paper (Section 3, "Training in Harmony") consumes an ordinary sequential
model, decomposes it into R layers and a minibatch into microbatches, and
promises synchronous-SGD semantics: whatever the schedule, one iteration yields
the gradients of the whole minibatch and one optimizer step.  The paper does
not print model equations (it trains BERT and GPT-2 variants taken from model
zoos, Section 5.1), so the model is a reading, stated in full here:

  layer 0        token + learned position embedding
  layers 1..L    pre-LayerNorm transformer block (attention, then MLP), each
                 half added onto the residual stream; biases on all four
                 linear maps; tanh-form GELU; no dropout
  layer L+1      final LayerNorm, bias-free LM head (own matrix), masked
                 softmax cross-entropy summed over target positions and
                 divided by the number of targets in the WHOLE minibatch

Linear maps store W as [out, in]:  y = x @ W.T + bias.
`causal=True` masks keys j > i (decoder); False attends everywhere (encoder).

Microbatch data: ids[M, b, s] int, targets[M, b, s] int with -1 = no target.
Activations of one microbatch are [T, d] with T = b*s, row t = (sequence t // s,
position t % s).
"""
from __future__ import annotations

from collections import OrderedDict
from dataclasses import dataclass

import numpy as np

F64 = np.float64


@dataclass(frozen=True)
class Spec:
    n_blocks: int
    d_model: int
    n_heads: int
    d_ffn: int
    seq_len: int
    vocab: int
    causal: bool = True
    ln_eps: float = 1e-5

    @property
    def n_layers(self) -> int:
        """R: embedding + blocks + (final norm, head, loss)."""
        return self.n_blocks + 2

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads


BLOCK_TENSORS = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
                 "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


def layer_param_shapes(spec: Spec, layer: int) -> "OrderedDict[str, tuple]":
    """Names and shapes of the parameters of one layer, in storage order."""
    d, f, s, V = spec.d_model, spec.d_ffn, spec.seq_len, spec.vocab
    out: "OrderedDict[str, tuple]" = OrderedDict()
    if layer == 0:
        out["wte"] = (V, d)
        out["wpe"] = (s, d)
    elif layer <= spec.n_blocks:
        p = f"h{layer}."
        out[p + "ln1_g"] = (d,)
        out[p + "ln1_b"] = (d,)
        out[p + "wqkv"] = (3 * d, d)
        out[p + "bqkv"] = (3 * d,)
        out[p + "wo"] = (d, d)
        out[p + "bo"] = (d,)
        out[p + "ln2_g"] = (d,)
        out[p + "ln2_b"] = (d,)
        out[p + "w1"] = (f, d)
        out[p + "b1"] = (f,)
        out[p + "w2"] = (d, f)
        out[p + "b2"] = (d,)
    elif layer == spec.n_blocks + 1:
        out["lnf_g"] = (d,)
        out["lnf_b"] = (d,)
        out["wh"] = (V, d)
    else:
        raise ValueError(f"layer {layer} outside 0..{spec.n_blocks + 1}")
    return out


def param_shapes(spec: Spec) -> "OrderedDict[str, tuple]":
    out: "OrderedDict[str, tuple]" = OrderedDict()
    for layer in range(spec.n_layers):
        out.update(layer_param_shapes(spec, layer))
    return out


def layer_param_count(spec: Spec, layer: int) -> int:
    return sum(int(np.prod(s)) for s in layer_param_shapes(spec, layer).values())


# --------------------------------------------------------------------------
# elementary operations, forward and backward
# --------------------------------------------------------------------------

def layernorm_fwd(x, gamma, beta, eps):
    """Row-wise LayerNorm: mean and BIASED variance over the feature axis."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return gamma * xhat + beta, (xhat, rstd)


def layernorm_bwd(dy, cache, gamma):
    xhat, rstd = cache
    dgamma = (dy * xhat).sum(axis=0)
    dbeta = dy.sum(axis=0)
    dxhat = dy * gamma
    dx = (dxhat - dxhat.mean(axis=-1, keepdims=True)
          - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True)) * rstd
    return dx, dgamma, dbeta


GELU_C = np.sqrt(2.0 / np.pi)
GELU_A = 0.044715


def gelu_fwd(u):
    """tanh-form GELU."""
    return 0.5 * u * (1.0 + np.tanh(GELU_C * (u + GELU_A * u ** 3)))


def gelu_bwd(dg, u):
    th = np.tanh(GELU_C * (u + GELU_A * u ** 3))
    dth = (1.0 - th ** 2) * GELU_C * (1.0 + 3.0 * GELU_A * u ** 2)
    return dg * (0.5 * (1.0 + th) + 0.5 * u * dth)


def linear_fwd(x, W, bias=None):
    y = x @ W.T
    if bias is not None:
        y = y + bias
    return y


def linear_bwd(dy, x, W, has_bias=True):
    dx = dy @ W
    dW = dy.T @ x
    db = dy.sum(axis=0) if has_bias else None
    return dx, dW, db


def attention_fwd(qkv, spec: Spec, b: int):
    """Multi-head softmax attention on one microbatch.

    qkv is [T, 3d]: columns [0,d) = q, [d,2d) = k, [2d,3d) = v; head h owns
    columns h*d_h .. (h+1)*d_h-1 of each third.
    """
    s, H, dh, d = spec.seq_len, spec.n_heads, spec.d_head, spec.d_model
    q = qkv[:, 0 * d:1 * d].reshape(b, s, H, dh).transpose(0, 2, 1, 3)
    k = qkv[:, 1 * d:2 * d].reshape(b, s, H, dh).transpose(0, 2, 1, 3)
    v = qkv[:, 2 * d:3 * d].reshape(b, s, H, dh).transpose(0, 2, 1, 3)
    S = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(F64(dh))          # [b,H,s,s]
    if spec.causal:
        future = np.triu(np.ones((s, s), dtype=bool), k=1)          # j > i
        S = np.where(future, -np.inf, S)
    S = S - S.max(axis=-1, keepdims=True)
    P = np.exp(S)
    P = P / P.sum(axis=-1, keepdims=True)
    o = P @ v                                                        # [b,H,s,dh]
    out = o.transpose(0, 2, 1, 3).reshape(b * s, d)
    return out, (q, k, v, P)


def attention_bwd(dout, cache, spec: Spec, b: int):
    s, H, dh, d = spec.seq_len, spec.n_heads, spec.d_head, spec.d_model
    q, k, v, P = cache
    do = dout.reshape(b, s, H, dh).transpose(0, 2, 1, 3)
    dv = P.transpose(0, 1, 3, 2) @ do
    dP = do @ v.transpose(0, 1, 3, 2)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    scale = 1.0 / np.sqrt(F64(dh))
    dq = (dS @ k) * scale
    dk = (dS.transpose(0, 1, 3, 2) @ q) * scale
    dqkv = np.empty((b * s, 3 * d), dtype=F64)
    dqkv[:, 0 * d:1 * d] = dq.transpose(0, 2, 1, 3).reshape(b * s, d)
    dqkv[:, 1 * d:2 * d] = dk.transpose(0, 2, 1, 3).reshape(b * s, d)
    dqkv[:, 2 * d:3 * d] = dv.transpose(0, 2, 1, 3).reshape(b * s, d)
    return dqkv


# --------------------------------------------------------------------------
# the R layers; each callable alone (the paper's Decomposer output, Section 4.1)
# --------------------------------------------------------------------------

def embed_fwd(ids_mb, params, spec: Spec):
    """ids_mb [b, s] -> x [T, d]."""
    b, s = ids_mb.shape
    x = params["wte"][ids_mb.reshape(-1)] + np.tile(params["wpe"][:s], (b, 1))
    return x, (ids_mb,)


def embed_bwd(dx, cache, params, spec: Spec):
    (ids_mb,) = cache
    b, s = ids_mb.shape
    dwte = np.zeros_like(params["wte"])
    np.add.at(dwte, ids_mb.reshape(-1), dx)
    dwpe = np.zeros_like(params["wpe"])
    dwpe[:s] = dx.reshape(b, s, -1).sum(axis=0)
    return None, {"wte": dwte, "wpe": dwpe}


def block_fwd(x, params, spec: Spec, layer: int, b: int):
    p = f"h{layer}."
    a, ln1 = layernorm_fwd(x, params[p + "ln1_g"], params[p + "ln1_b"], spec.ln_eps)
    qkv = linear_fwd(a, params[p + "wqkv"], params[p + "bqkv"])
    o, att = attention_fwd(qkv, spec, b)
    x_mid = x + linear_fwd(o, params[p + "wo"], params[p + "bo"])
    h, ln2 = layernorm_fwd(x_mid, params[p + "ln2_g"], params[p + "ln2_b"], spec.ln_eps)
    u = linear_fwd(h, params[p + "w1"], params[p + "b1"])
    g = gelu_fwd(u)
    y = x_mid + linear_fwd(g, params[p + "w2"], params[p + "b2"])
    return y, (ln1, a, att, o, ln2, h, u, g)


def block_bwd(dy, cache, params, spec: Spec, layer: int, b: int):
    p = f"h{layer}."
    ln1, a, att, o, ln2, h, u, g = cache
    grads = {}
    # MLP half: y = x_mid + W2 gelu(W1 LN2(x_mid))
    dg, grads[p + "w2"], grads[p + "b2"] = linear_bwd(dy, g, params[p + "w2"])
    du = gelu_bwd(dg, u)
    dh, grads[p + "w1"], grads[p + "b1"] = linear_bwd(du, h, params[p + "w1"])
    dx_ln2, grads[p + "ln2_g"], grads[p + "ln2_b"] = layernorm_bwd(dh, ln2, params[p + "ln2_g"])
    dx_mid = dy + dx_ln2
    # attention half: x_mid = x + Wo attn(Wqkv LN1(x))
    do, grads[p + "wo"], grads[p + "bo"] = linear_bwd(dx_mid, o, params[p + "wo"])
    dqkv = attention_bwd(do, att, spec, b)
    da, grads[p + "wqkv"], grads[p + "bqkv"] = linear_bwd(dqkv, a, params[p + "wqkv"])
    dx_ln1, grads[p + "ln1_g"], grads[p + "ln1_b"] = layernorm_bwd(da, ln1, params[p + "ln1_g"])
    return dx_mid + dx_ln1, grads


def head_fwd(x, params, spec: Spec, targets_mb, n_tgt: int):
    """Final norm, LM head and loss.  Returns this microbatch's share of the loss:
    (sum over its target positions of -log softmax[target]) / n_tgt."""
    z, lnf = layernorm_fwd(x, params["lnf_g"], params["lnf_b"], spec.ln_eps)
    logits = linear_fwd(z, params["wh"])
    tgt = targets_mb.reshape(-1)
    mx = logits.max(axis=-1, keepdims=True)
    lse = mx[:, 0] + np.log(np.exp(logits - mx).sum(axis=-1))
    rows = np.nonzero(tgt >= 0)[0]
    loss = (lse[rows] - logits[rows, tgt[rows]]).sum() / n_tgt
    return loss, (lnf, z, logits, lse, tgt, n_tgt)


def head_bwd(cache, params, spec: Spec):
    lnf, z, logits, lse, tgt, n_tgt = cache
    rows = np.nonzero(tgt >= 0)[0]
    dlogits = np.zeros_like(logits)
    dlogits[rows] = np.exp(logits[rows] - lse[rows, None])
    dlogits[rows, tgt[rows]] -= 1.0
    dlogits /= n_tgt
    dz, dwh, _ = linear_bwd(dlogits, z, params["wh"], has_bias=False)
    dx, dg, db = layernorm_bwd(dz, lnf, params["lnf_g"])
    return dx, {"wh": dwh, "lnf_g": dg, "lnf_b": db}


def layer_fwd(layer: int, x, params, spec: Spec, ids_mb, targets_mb, n_tgt: int):
    """Run one of the R layers.  For the last layer the returned 'activation'
    is the scalar loss share."""
    b = ids_mb.shape[0]
    if layer == 0:
        return embed_fwd(ids_mb, params, spec)
    if layer <= spec.n_blocks:
        return block_fwd(x, params, spec, layer, b)
    return head_fwd(x, params, spec, targets_mb, n_tgt)


def layer_bwd(layer: int, dy, cache, params, spec: Spec, b: int):
    if layer == 0:
        return embed_bwd(dy, cache, params, spec)
    if layer <= spec.n_blocks:
        return block_bwd(dy, cache, params, spec, layer, b)
    return head_bwd(cache, params, spec)


def count_targets(targets) -> int:
    return int((np.asarray(targets) >= 0).sum())


def accumulate(total: dict, part: dict) -> None:
    """total[name] += part[name]; microbatches arrive in ascending order."""
    for name, g in part.items():
        if name in total:
            total[name] = total[name] + g
        else:
            total[name] = g.copy()


# --------------------------------------------------------------------------
# the definition: microbatch-major, nothing swapped, nothing recomputed
# --------------------------------------------------------------------------

def forward_loss(spec: Spec, params, ids, targets) -> float:
    """Loss of the whole minibatch (used by the finite-difference pins)."""
    n_tgt = count_targets(targets)
    total = 0.0
    for mb in range(ids.shape[0]):
        x = None
        for layer in range(spec.n_layers):
            x, _ = layer_fwd(layer, x, params, spec, ids[mb], targets[mb], n_tgt)
        total += x
    return float(total)


def iteration_microbatch_major(spec: Spec, params, ids, targets):
    """For each microbatch in turn: every layer forward, the loss, every layer
    backward; gradients summed over microbatches in ascending order.
    Returns (loss, grads)."""
    n_tgt = count_targets(targets)
    grads: dict = {}
    loss = 0.0
    for mb in range(ids.shape[0]):
        b = ids[mb].shape[0]
        caches = []
        x = None
        for layer in range(spec.n_layers):
            x, c = layer_fwd(layer, x, params, spec, ids[mb], targets[mb], n_tgt)
            caches.append(c)
        loss += x
        dy = None
        for layer in reversed(range(spec.n_layers)):
            dy, g = layer_bwd(layer, dy, caches[layer], params, spec, b)
            accumulate(grads, g)
    return float(loss), grads


# --------------------------------------------------------------------------
# Adam
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class AdamHP:
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    step: int = 1          # 1-based


def adam_update(w, g, m, v, hp: AdamHP):
    """One Adam step with bias correction, no weight decay.  Returns (w, m, v)."""
    m = hp.beta1 * m + (1.0 - hp.beta1) * g
    v = hp.beta2 * v + (1.0 - hp.beta2) * g * g
    mhat = m / (1.0 - hp.beta1 ** hp.step)
    vhat = v / (1.0 - hp.beta2 ** hp.step)
    w = w - hp.lr * mhat / (np.sqrt(vhat) + hp.eps)
    return w, m, v


def adam_all(params, grads, m, v, hp: AdamHP):
    new_w, new_m, new_v = {}, {}, {}
    for name in params:
        new_w[name], new_m[name], new_v[name] = adam_update(
            params[name], grads[name], m[name], v[name], hp)
    return new_w, new_m, new_v


def training_iteration(spec: Spec, params, ids, targets, m, v, hp: AdamHP):
    """The whole reference iteration: gradients of the minibatch, then Adam.
    Returns dict(loss, grads, weights, m, v)."""
    loss, grads = iteration_microbatch_major(spec, params, ids, targets)
    w2, m2, v2 = adam_all(params, grads, m, v, hp)
    return {"loss": loss, "grads": grads, "weights": w2, "m": m2, "v": v2}
