"""fp64 CPU oracle for layered gradient accumulation over a GPT layer stack.

THIS IS TEST INFRASTRUCTURE.  It exists to check the HIP path; nothing in the
product (the package, its C library) may import or call it.  Only tests, the
smoke entry and the benchmark's cpu_baseline leg use it.  It shares no code
with the HIP path.

What is computed, and where the paper defines it:

* A stack of identical transformer layers, each a multi-head attention module
  followed by a two-layer feed-forward network of width d_I = n_I * d_m
  (paper section 5, "Model").  Table B.1's closed form 12 x^5 + 13 x^3 for the
  X_[x] family (d_m = x^2, d_l = x) fixes the exact per-layer inventory at
  12 d_m^2 + 13 d_m: every one of the four linear maps carries a bias and both
  layer norms carry gain and bias.  The build's workload is the decoder
  (causal) pre-LN variant the paper says its results carry over to; the
  paper's own encoder differs in that every position attends to the whole
  sequence (`StackShape.causal = False`).
* Gradient accumulation: the batch is cut into n_mu micro-batches that are
  processed one after the other between two weight updates (section 2.5), the
  gradients being summed.  This file's main driver, `step_microbatch_major`,
  is exactly that plain definition: no checkpointing, no recompute, no fusion.
* Layered gradient accumulation (section 3) processes every micro-batch for
  one layer before going to the next layer, with layers delimited by the
  activation checkpoints.  It is a reordering only, so its result has the
  plain definition above; `step_layered` walks the paper's order (layer-major
  forward keeping only boundary activations, layer-major backward that
  recomputes inside the layer, Adam for a layer as soon as its gradient is
  complete, appendix C.3) and exists to show the two orders agree.
* Adam with fp32-equivalent state (sections 2.5, 5; appendix C.3).  The paper
  only names the optimizer; the variant is Kingma & Ba's with bias correction,
  no weight decay, eps added to the root of the corrected second moment.
* Gradient scaling for half precision (section 2.2 only says that gradients
  are scaled dynamically against under- and overflow): the output gradient
  arrives multiplied by a loss scale, Adam divides by it, an update whose
  gradient holds an infinity or NaN is left out, and `LossScaler` halves the
  scale after such a step and doubles it after a run of clean ones.  In fp64
  the scaling itself changes nothing (exactly nothing for powers of two),
  which is the pin.

Readings taken where the paper is silent (GELU in its tanh form, LayerNorm
with biased variance and eps inside the root, softmax scale 1/sqrt(d_h), sum
loss so micro-batch gradients add without a 1/n factor) are listed in the
design notes at the repository root.

Everything is float64 numpy.  `@` (BLAS matmul) is the only library primitive.
End-to-end numeric values of a forward/backward are not printed anywhere in the
paper; this oracle is pinned instead by finite differences, the accumulation
and ordering invariants, textbook special cases, an autograd cross-check built
from library routines, and hand-worked Adam values (tests/test_oracle_*.py).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64

# Canonical per-layer parameter order (flat fp32 vector handed across the C ABI).
PARAM_ORDER = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2",
)


@dataclass(frozen=True)
class StackShape:
    """Shape of the stack in the paper's notation (section 2.4 / section 5)."""
    d_l: int          # layers
    d_m: int          # width
    d_a: int          # heads
    d_I: int          # feed-forward width
    d_s: int          # sequence length
    b_mu: int         # sequences per micro-batch
    n_mu: int         # micro-batches per step
    ln_eps: float = 1e-5
    causal: bool = True   # decoder: position i attends to j <= i; False: the encoder of section 5, no mask

    @property
    def d_h(self) -> int:
        return self.d_m // self.d_a


def param_shapes(d_m: int, d_I: int) -> Dict[str, Tuple[int, ...]]:
    """Tensor shapes of one layer; matrices are [in, out] so that y = x @ W + b."""
    return {
        "ln1_g": (d_m,), "ln1_b": (d_m,),
        "w_qkv": (d_m, 3 * d_m), "b_qkv": (3 * d_m,),
        "w_o": (d_m, d_m), "b_o": (d_m,),
        "ln2_g": (d_m,), "ln2_b": (d_m,),
        "w_1": (d_m, d_I), "b_1": (d_I,),
        "w_2": (d_I, d_m), "b_2": (d_m,),
    }


def params_per_layer(d_m: int, d_I: int) -> int:
    """p_l.  With d_I = 4 d_m this is 12 d_m^2 + 13 d_m (Table B.1, X_[x] row)."""
    return sum(int(np.prod(s)) for s in param_shapes(d_m, d_I).values())


def unflatten_layer(flat: np.ndarray, d_m: int, d_I: int) -> Dict[str, np.ndarray]:
    """Split one layer's flat vector (canonical order, row-major) into fp64 tensors."""
    out, off = {}, 0
    shapes = param_shapes(d_m, d_I)
    for name in PARAM_ORDER:
        n = int(np.prod(shapes[name]))
        out[name] = np.asarray(flat[off:off + n], dtype=F64).reshape(shapes[name]).copy()
        off += n
    if off != flat.size:
        raise ValueError(f"flat layer vector has {flat.size} entries, expected {off}")
    return out


def flatten_layer(p: Dict[str, np.ndarray]) -> np.ndarray:
    return np.concatenate([np.asarray(p[name], dtype=F64).ravel() for name in PARAM_ORDER])


# --------------------------------------------------------------------------
# Elementary pieces
# --------------------------------------------------------------------------

_GELU_C = math.sqrt(2.0 / math.pi)
_GELU_A = 0.044715


def gelu(u: np.ndarray) -> np.ndarray:
    """GELU, tanh form: 0.5 u (1 + tanh(sqrt(2/pi) (u + 0.044715 u^3)))."""
    return 0.5 * u * (1.0 + np.tanh(_GELU_C * (u + _GELU_A * u ** 3)))


def gelu_grad(u: np.ndarray) -> np.ndarray:
    """d gelu / d u of the tanh form."""
    z = _GELU_C * (u + _GELU_A * u ** 3)
    th = np.tanh(z)
    dz = _GELU_C * (1.0 + 3.0 * _GELU_A * u ** 2)
    return 0.5 * (1.0 + th) + 0.5 * u * (1.0 - th ** 2) * dz


def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray, eps: float):
    """LayerNorm over the last axis: biased variance, eps inside the root."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * g + b, xhat, rstd


def layer_norm_backward(dy: np.ndarray, xhat: np.ndarray, rstd: np.ndarray, g: np.ndarray):
    """Gradients of LayerNorm w.r.t. input, gain and bias."""
    lead = tuple(range(dy.ndim - 1))
    dg = (dy * xhat).sum(axis=lead)
    db = dy.sum(axis=lead)
    dxhat = dy * g
    dx = rstd * (dxhat
                 - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, dg, db


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, causal: bool):
    """Softmax attention per sequence and head; position i attends to j <= i (causal,
    the decoder) or to every position of its sequence (the encoder of section 5).

    q, k, v: [b, heads, s, d_h].  Scores are scaled by 1/sqrt(d_h).
    Returns the output [b, heads, s, d_h] and the probabilities.
    """
    s, d_h = q.shape[-2], q.shape[-1]
    scores = (q @ np.swapaxes(k, -1, -2)) / math.sqrt(d_h)
    if causal:
        future = np.triu(np.ones((s, s), dtype=bool), k=1)
        scores = np.where(future, -np.inf, scores)
    scores = scores - scores.max(axis=-1, keepdims=True)
    e = np.exp(scores)
    prob = e / e.sum(axis=-1, keepdims=True)
    return prob @ v, prob


def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray):
    return attention(q, k, v, True)


def causal_attention_backward(dout, q, k, v, prob):
    """Backward of `attention` given its probabilities: masked positions have probability 0,
    so the same formula serves both variants."""
    d_h = q.shape[-1]
    dv = np.swapaxes(prob, -1, -2) @ dout
    dprob = dout @ np.swapaxes(v, -1, -2)
    dscores = prob * (dprob - (dprob * prob).sum(axis=-1, keepdims=True))
    dscores = dscores / math.sqrt(d_h)
    dq = dscores @ k
    dk = np.swapaxes(dscores, -1, -2) @ q
    return dq, dk, dv


def _split_heads(t: np.ndarray, d_a: int) -> np.ndarray:
    b, s, d = t.shape
    return t.reshape(b, s, d_a, d // d_a).transpose(0, 2, 1, 3)


def _merge_heads(t: np.ndarray) -> np.ndarray:
    b, h, s, dh = t.shape
    return t.transpose(0, 2, 1, 3).reshape(b, s, h * dh)


# --------------------------------------------------------------------------
# One layer (section 5 "Model": attention module, then feed-forward module;
# pre-LN residual form, causal)
# --------------------------------------------------------------------------

def layer_forward(x: np.ndarray, p: Dict[str, np.ndarray], d_a: int, eps: float, causal: bool = True):
    """x: [b, s, d_m] -> (y, cache of every intermediate)."""
    d = x.shape[-1]
    h, xhat1, rstd1 = layer_norm(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = h @ p["w_qkv"] + p["b_qkv"]
    q = _split_heads(qkv[..., 0:d], d_a)
    k = _split_heads(qkv[..., d:2 * d], d_a)
    v = _split_heads(qkv[..., 2 * d:3 * d], d_a)
    att, prob = attention(q, k, v, causal)
    a = _merge_heads(att)
    x1 = x + a @ p["w_o"] + p["b_o"]
    h2, xhat2, rstd2 = layer_norm(x1, p["ln2_g"], p["ln2_b"], eps)
    u = h2 @ p["w_1"] + p["b_1"]
    gl = gelu(u)
    y = x1 + gl @ p["w_2"] + p["b_2"]
    cache = dict(x=x, h=h, xhat1=xhat1, rstd1=rstd1, q=q, k=k, v=v, prob=prob, a=a,
                 x1=x1, h2=h2, xhat2=xhat2, rstd2=rstd2, u=u, gl=gl)
    return y, cache


def layer_backward(dy: np.ndarray, cache: Dict[str, np.ndarray], p: Dict[str, np.ndarray], d_a: int):
    """dy: [b, s, d_m] -> (dx, gradient of every parameter tensor, summed over b and s)."""
    d = dy.shape[-1]
    two = lambda t: t.reshape(-1, t.shape[-1])
    g: Dict[str, np.ndarray] = {}

    # y = x1 + gl @ W2 + b2
    g["w_2"] = two(cache["gl"]).T @ two(dy)
    g["b_2"] = two(dy).sum(axis=0)
    dgl = dy @ p["w_2"].T
    du = dgl * gelu_grad(cache["u"])
    # u = h2 @ W1 + b1
    g["w_1"] = two(cache["h2"]).T @ two(du)
    g["b_1"] = two(du).sum(axis=0)
    dh2 = du @ p["w_1"].T
    dx1_ln, g["ln2_g"], g["ln2_b"] = layer_norm_backward(dh2, cache["xhat2"], cache["rstd2"], p["ln2_g"])
    dx1 = dy + dx1_ln
    # x1 = x + a @ Wo + bo
    g["w_o"] = two(cache["a"]).T @ two(dx1)
    g["b_o"] = two(dx1).sum(axis=0)
    da = dx1 @ p["w_o"].T
    dq, dk, dv = causal_attention_backward(_split_heads(da, d_a), cache["q"], cache["k"], cache["v"], cache["prob"])
    dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=-1)
    # qkv = h @ Wqkv + bqkv
    g["w_qkv"] = two(cache["h"]).T @ two(dqkv)
    g["b_qkv"] = two(dqkv).sum(axis=0)
    dh = dqkv @ p["w_qkv"].T
    dx_ln, g["ln1_g"], g["ln1_b"] = layer_norm_backward(dh, cache["xhat1"], cache["rstd1"], p["ln1_g"])
    dx = dx1 + dx_ln
    return dx, g


# --------------------------------------------------------------------------
# Adam (the optimizer the paper assumes, section 5 "Training")
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class AdamHyper:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    step: int = 1     # t >= 1, the number of the update being applied
    # Gradient scaling for half precision (section 2.2): g arrives multiplied by loss_scale and is divided by it
    # before use; with skip_nonfinite an update whose gradient holds an infinity or a NaN is not applied at all.
    loss_scale: float = 1.0
    skip_nonfinite: bool = False


def adam_skips(g, hp: AdamHyper) -> bool:
    """Whether the update with gradient g is left out (overflowed gradient, section 2.2)."""
    return bool(hp.skip_nonfinite and not np.all(np.isfinite(g)))


def adam_update(w, m, v, g, hp: AdamHyper):
    """One Adam update; returns new (w, m, v).  No weight decay."""
    if adam_skips(g, hp):
        return np.array(w, dtype=F64), np.array(m, dtype=F64), np.array(v, dtype=F64)
    g = np.asarray(g, dtype=F64) / hp.loss_scale
    m_new = hp.beta1 * m + (1.0 - hp.beta1) * g
    v_new = hp.beta2 * v + (1.0 - hp.beta2) * g * g
    m_hat = m_new / (1.0 - hp.beta1 ** hp.step)
    v_hat = v_new / (1.0 - hp.beta2 ** hp.step)
    w_new = w - hp.lr * m_hat / (np.sqrt(v_hat) + hp.eps)
    return w_new, m_new, v_new


@dataclass
class LossScaler:
    """Dynamic loss scale (section 2.2 says the gradients are scaled dynamically; the rule is the customary one of
    mixed precision training: halve at once after an overflow, double after a run of clean steps)."""
    scale: float = 65536.0
    growth: float = 2.0
    backoff: float = 0.5
    min_scale: float = 1.0
    max_scale: float = 2.0 ** 24
    growth_interval: int = 2000
    good_steps: int = 0


def loss_scaler_update(s: LossScaler, overflowed: bool) -> None:
    if overflowed:
        s.scale = max(s.scale * s.backoff, s.min_scale)
        s.good_steps = 0
        return
    s.good_steps += 1
    if s.good_steps >= s.growth_interval:
        s.scale = min(s.scale * s.growth, s.max_scale)
        s.good_steps = 0


# --------------------------------------------------------------------------
# Training step drivers
# --------------------------------------------------------------------------

@dataclass
class StepResult:
    boundaries: np.ndarray            # [d_l + 1, n_mu, b_mu, d_s, d_m]; [0] is the input, [d_l] the output
    grads: List[np.ndarray]           # per layer, flat canonical order, summed over micro-batches
    dx: np.ndarray                    # [n_mu, b_mu, d_s, d_m], gradient w.r.t. the input
    new_params: Optional[List[np.ndarray]] = None
    new_m: Optional[List[np.ndarray]] = None
    new_v: Optional[List[np.ndarray]] = None
    loss: float = 0.0
    skipped: Optional[List[bool]] = None   # per layer: update left out (AdamHyper.skip_nonfinite)


def _as_layers(flat_params: Sequence[np.ndarray], shape: StackShape):
    if len(flat_params) != shape.d_l:
        raise ValueError("one flat parameter vector per layer expected")
    return [unflatten_layer(np.asarray(f, dtype=F64), shape.d_m, shape.d_I) for f in flat_params]


def _apply_adam(flat_params, grads, hp, m0, v0):
    new_w, new_m, new_v = [], [], []
    for l, g in enumerate(grads):
        w = np.asarray(flat_params[l], dtype=F64)
        m = np.zeros_like(w) if m0 is None else np.asarray(m0[l], dtype=F64)
        v = np.zeros_like(w) if v0 is None else np.asarray(v0[l], dtype=F64)
        a, b, c = adam_update(w, m, v, g, hp)
        new_w.append(a); new_m.append(b); new_v.append(c)
    return new_w, new_m, new_v


def step_microbatch_major(x, G, flat_params, shape: StackShape, adam: Optional[AdamHyper] = None,
                          m0=None, v0=None) -> StepResult:
    """Standard gradient accumulation (section 2.5): for each micro-batch, the whole
    stack forward then backward; weight gradients summed; one Adam update at the end.

    x, G: [n_mu, b_mu, d_s, d_m].  The loss is sum(y * G), so dL/dy = G.
    """
    x = np.asarray(x, dtype=F64); G = np.asarray(G, dtype=F64)
    layers = _as_layers(flat_params, shape)
    L = shape.d_l
    bounds = np.empty((L + 1,) + x.shape, dtype=F64)
    grads = [np.zeros(params_per_layer(shape.d_m, shape.d_I), dtype=F64) for _ in range(L)]
    dx = np.empty_like(x)
    loss = 0.0
    for mu in range(shape.n_mu):
        act = x[mu]
        bounds[0, mu] = act
        caches = []
        for l in range(L):
            act, cache = layer_forward(act, layers[l], shape.d_a, shape.ln_eps, shape.causal)
            caches.append(cache)
            bounds[l + 1, mu] = act
        loss += float((act * G[mu]).sum())
        d = G[mu]
        for l in reversed(range(L)):
            d, g = layer_backward(d, caches[l], layers[l], shape.d_a)
            grads[l] += flatten_layer(g)
        dx[mu] = d
    res = StepResult(boundaries=bounds, grads=grads, dx=dx, loss=loss)
    if adam is not None:
        res.new_params, res.new_m, res.new_v = _apply_adam(flat_params, grads, adam, m0, v0)
        res.skipped = [adam_skips(g, adam) for g in grads]
    return res


def step_layered(x, G, flat_params, shape: StackShape, adam: Optional[AdamHyper] = None,
                 m0=None, v0=None) -> StepResult:
    """Layered gradient accumulation (section 3) in the paper's order.

    Forward: layer by layer, every micro-batch through layer l before layer l+1,
    keeping only the layer-boundary activations (the checkpoints).  Backward: from
    the last layer down, every micro-batch through layer l (intermediates recomputed
    from the checkpoint), gradients of layer l summed over micro-batches, then Adam
    for layer l at once (appendix C.3), before layer l-1 is touched.
    """
    x = np.asarray(x, dtype=F64); G = np.asarray(G, dtype=F64)
    layers = _as_layers(flat_params, shape)
    L = shape.d_l
    bounds = np.empty((L + 1,) + x.shape, dtype=F64)
    bounds[0] = x
    for l in range(L):
        for mu in range(shape.n_mu):
            bounds[l + 1, mu], _ = layer_forward(bounds[l, mu], layers[l], shape.d_a, shape.ln_eps, shape.causal)
    loss = float((bounds[L] * G).sum())
    d = G.copy()
    grads: List[Optional[np.ndarray]] = [None] * L
    new_w: List[Optional[np.ndarray]] = [None] * L
    new_m: List[Optional[np.ndarray]] = [None] * L
    new_v: List[Optional[np.ndarray]] = [None] * L
    for l in reversed(range(L)):
        gl = np.zeros(params_per_layer(shape.d_m, shape.d_I), dtype=F64)
        for mu in range(shape.n_mu):
            _, cache = layer_forward(bounds[l, mu], layers[l], shape.d_a, shape.ln_eps, shape.causal)   # recompute
            d[mu], g = layer_backward(d[mu], cache, layers[l], shape.d_a)
            gl += flatten_layer(g)
        grads[l] = gl
        if adam is not None:
            w = np.asarray(flat_params[l], dtype=F64)
            m = np.zeros_like(w) if m0 is None else np.asarray(m0[l], dtype=F64)
            v = np.zeros_like(w) if v0 is None else np.asarray(v0[l], dtype=F64)
            new_w[l], new_m[l], new_v[l] = adam_update(w, m, v, gl, adam)
    res = StepResult(boundaries=bounds, grads=grads, dx=d, loss=loss)
    if adam is not None:
        res.new_params, res.new_m, res.new_v = new_w, new_m, new_v
        res.skipped = [adam_skips(g, adam) for g in grads]
    return res


def loss_only(x, G, flat_params, shape: StackShape) -> float:
    """sum(stack(x) * G) - the scalar whose derivatives the steps above return."""
    x = np.asarray(x, dtype=F64); G = np.asarray(G, dtype=F64)
    layers = _as_layers(flat_params, shape)
    total = 0.0
    for mu in range(x.shape[0]):
        act = x[mu]
        for l in range(shape.d_l):
            act, _ = layer_forward(act, layers[l], shape.d_a, shape.ln_eps, shape.causal)
        total += float((act * G[mu]).sum())
    return total


# --------------------------------------------------------------------------
# The paper's resource bookkeeping (appendix C.1, C.3), used to pin the
# counters the benchmark prints.
# --------------------------------------------------------------------------

def flops_per_step_paper(b: int, d_s: int, p: int) -> float:
    """Appendix C.1: 2 flop per token per parameter forward; backward (input
    gradient, parameter gradient, recompute) three times that: 8 b d_s p."""
    return 8.0 * b * d_s * p


def memory_model_bytes(p: int, p_l: int, b: int, d_s: int, d_m: int, d_l: int):
    """Appendix C.3: state 12 p, layer buffers 6 p_l, checkpoints 2 b d_s d_m d_l (bytes)."""
    return {"state": 12.0 * p, "buffers": 6.0 * p_l, "checkpoints": 2.0 * b * d_s * d_m * d_l}
