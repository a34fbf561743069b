"""Pins for the fp64 oracle: every check here is against something other than the oracle
itself - values the paper prints, closed forms, invariants, textbook special cases,
brute force, finite differences, and an autograd build from library routines."""
import math
import os

import numpy as np
import pytest

from oracle import lga_oracle as O
import synth_inputs as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


def tiny_shape(d_l=2, d_m=8, d_a=2, d_s=5, b_mu=2, n_mu=3, causal=True):
    return O.StackShape(d_l=d_l, d_m=d_m, d_a=d_a, d_I=4 * d_m, d_s=d_s, b_mu=b_mu, n_mu=n_mu, causal=causal)


def tiny_problem(shape, seed=3, weight_std=0.3, bias_std=0.2):
    w = S.Workload("tiny", shape.d_l, shape.d_m, shape.d_a, shape.d_I, shape.d_s, shape.b_mu, shape.n_mu, "fp32")
    x, G, params = S.make_inputs(w, seed=seed, weight_std=weight_std, bias_std=bias_std)
    return x.astype(np.float64), G.astype(np.float64), [p.astype(np.float64) for p in params]


# ---------------------------------------------------------------- parameter inventory

@pytest.mark.parametrize("row", _read_table("table_b1_parameter_counts.txt"), ids=lambda r: r[0])
def test_parameter_count_matches_table_b1(row):
    _, d_m, d_l, printed, tol = row
    d_m, d_l, printed, tol = int(d_m), int(d_l), float(printed), float(tol)
    p = d_l * O.params_per_layer(d_m, 4 * d_m)
    if tol == 0:
        assert p == int(printed)
    else:
        assert abs(p - printed) / printed <= tol


def test_parameter_count_closed_form_and_layout():
    for x in (2, 3, 8, 32):
        d_m = x * x
        assert x * O.params_per_layer(d_m, 4 * d_m) == 12 * x ** 5 + 13 * x ** 3
    d_m, d_I = 8, 32
    flat = np.arange(O.params_per_layer(d_m, d_I), dtype=np.float64)
    p = O.unflatten_layer(flat, d_m, d_I)
    assert np.array_equal(O.flatten_layer(p), flat)
    # the shared input module lays tensors out at the same offsets
    sl = S.tensor_slices(d_m, d_I)
    for name in O.PARAM_ORDER:
        assert np.array_equal(p[name].ravel(), flat[sl[name]])
    assert tuple(S.PARAM_ORDER) == tuple(O.PARAM_ORDER)


def test_resource_bookkeeping_matches_printed_x160_numbers():
    gold = {r[0]: (float(r[1]), float(r[2])) for r in _read_table("x160_resource_numbers.txt")}
    d_m, d_l, d_s = 25600, 160, 2560
    p_l = O.params_per_layer(d_m, 4 * d_m)
    p = d_l * p_l
    gib = 2.0 ** 30

    def close(key, value):
        ref, tol = gold[key]
        assert abs(value - ref) / ref <= tol, (key, value, ref)

    flop = O.flops_per_step_paper(2420, d_s, p) * 1e5
    close("total_flop_100k_steps", flop)
    close("a100_gpu_days", flop / 312e12 / 86400.0)
    mem = O.memory_model_bytes(p, p_l, 2416, d_s, d_m, d_l)
    close("state_gib", mem["state"] / gib)
    close("buffers_gib", mem["buffers"] / gib)
    close("checkpoints_gib_b2416", mem["checkpoints"] / gib)
    close("state_gib_3d_improved", mem["state"] / 38640 / gib)
    close("buffers_gib_na16", mem["buffers"] / 16 / gib)


# ---------------------------------------------------------------- elementary pieces

def test_gelu_tanh_form_known_values():
    # values of 0.5 u (1 + tanh(sqrt(2/pi)(u + 0.044715 u^3))) worked out separately
    known = {1.0: 0.8411919906082768, -1.0: -0.15880800939172324, 2.0: 1.954597694087775,
             0.5: 0.34571400982514394, -3.0: -0.0036373920817729943, 0.0: 0.0}
    for u, val in known.items():
        assert abs(float(O.gelu(np.array(u))) - val) < 1e-15
    u = np.linspace(-6, 6, 101)
    assert np.allclose(O.gelu(u) - O.gelu(-u), u, atol=1e-14)           # odd part is u/2 + u/2
    assert abs(float(O.gelu(np.array(30.0))) - 30.0) < 1e-12
    # the exact (erf) GELU differs from the tanh form by a few 1e-4 at most: guards against a wrong constant
    from scipy.special import erf
    diff = np.abs(O.gelu(u) - 0.5 * u * (1 + erf(u / math.sqrt(2))))
    assert 1e-5 < diff.max() < 1e-3


def test_gelu_grad_by_central_difference():
    u = np.linspace(-4, 4, 81)
    h = 1e-6
    fd = (O.gelu(u + h) - O.gelu(u - h)) / (2 * h)
    assert np.allclose(O.gelu_grad(u), fd, atol=1e-9)


def test_layer_norm_statistics_and_input_gradient_sum():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 7, 16)) * 3 + 1.5
    g = np.full(16, 2.5); b = np.full(16, -0.75)
    y, xhat, rstd = O.layer_norm(x, g, b, 0.0)
    assert np.allclose(y.mean(-1), -0.75, atol=1e-12)
    assert np.allclose(y.var(-1), 2.5 ** 2, atol=1e-10)
    # with eps: rstd = 1/sqrt(var + eps), biased variance
    _, _, rstd_e = O.layer_norm(x, g, b, 1e-5)
    assert np.allclose(rstd_e[..., 0], 1 / np.sqrt(x.var(-1) + 1e-5), rtol=1e-13)
    dy = rng.standard_normal(x.shape)
    dx, dg, db = O.layer_norm_backward(dy, xhat, rstd, np.ones(16))
    assert np.allclose(dx.sum(-1), 0.0, atol=1e-12)          # shifts of a row do not change its output
    assert np.allclose((dx * xhat).sum(-1), 0.0, atol=1e-12)  # nor do rescalings
    assert np.allclose(db, dy.sum((0, 1)))


def test_attention_single_position_returns_v():
    rng = np.random.default_rng(1)
    q, k, v = (rng.standard_normal((2, 3, 1, 4)) for _ in range(3))
    out, prob = O.causal_attention(q, k, v)
    assert np.allclose(out, v) and np.allclose(prob, 1.0)


def test_attention_equal_scores_give_prefix_mean():
    rng = np.random.default_rng(2)
    s = 6
    v = rng.standard_normal((1, 2, s, 4))
    q = np.zeros((1, 2, s, 4)); k = rng.standard_normal((1, 2, s, 4))
    out, _ = O.causal_attention(q, k, v)
    prefix_mean = np.cumsum(v, axis=2) / np.arange(1, s + 1)[None, None, :, None]
    assert np.allclose(out, prefix_mean, atol=1e-14)


def test_attention_is_causal_and_matches_brute_force():
    rng = np.random.default_rng(3)
    b, h, s, dh = 2, 2, 5, 3
    q, k, v = (rng.standard_normal((b, h, s, dh)) for _ in range(3))
    out, _ = O.causal_attention(q, k, v)
    ref = np.zeros_like(out)
    for bi in range(b):
        for hi in range(h):
            for i in range(s):
                w = [math.exp(sum(q[bi, hi, i, c] * k[bi, hi, j, c] for c in range(dh)) / math.sqrt(dh))
                     for j in range(i + 1)]
                z = sum(w)
                for c in range(dh):
                    ref[bi, hi, i, c] = sum(w[j] * v[bi, hi, j, c] for j in range(i + 1)) / z
    assert np.allclose(out, ref, atol=1e-13)
    k2, v2 = k.copy(), v.copy()
    k2[:, :, 3:] += 5.0; v2[:, :, 3:] -= 7.0                  # change the future of positions 0..2
    out2, _ = O.causal_attention(q, k2, v2)
    assert np.array_equal(out[:, :, :3], out2[:, :, :3])


def test_full_attention_equal_scores_give_sequence_mean_and_brute_force():
    """The encoder variant (section 5): no mask.  Equal scores average V over the whole sequence; random
    scores match the definition written as loops; and every output depends on the last position."""
    rng = np.random.default_rng(4)
    b, h, s, dh = 2, 2, 5, 3
    v = rng.standard_normal((b, h, s, dh))
    out, prob = O.attention(np.zeros((b, h, s, dh)), rng.standard_normal((b, h, s, dh)), v, False)
    assert np.allclose(out, np.broadcast_to(v.mean(axis=2, keepdims=True), v.shape), atol=1e-14)
    assert np.allclose(prob, 1.0 / s)
    q, k = (rng.standard_normal((b, h, s, dh)) for _ in range(2))
    out, _ = O.attention(q, k, v, False)
    ref = np.zeros_like(out)
    for bi in range(b):
        for hi in range(h):
            for i in range(s):
                w = [math.exp(sum(q[bi, hi, i, c] * k[bi, hi, j, c] for c in range(dh)) / math.sqrt(dh)) for j in range(s)]
                z = sum(w)
                for c in range(dh):
                    ref[bi, hi, i, c] = sum(w[j] * v[bi, hi, j, c] for j in range(s)) / z
    assert np.allclose(out, ref, atol=1e-13)
    v2 = v.copy(); v2[:, :, -1] += 1.0
    out2, _ = O.attention(q, k, v2, False)
    assert (np.abs(out2 - out).max(axis=-1) > 1e-6).all()
    # the causal variant keeps its first position blind to it
    c1, _ = O.attention(q, k, v, True); c2, _ = O.attention(q, k, v2, True)
    assert np.array_equal(c1[:, :, :-1], c2[:, :, :-1])


def test_encoder_stack_is_equivariant_under_permutations_of_the_positions():
    """Without a mask nothing in the stack knows the order of the positions (there is no positional input):
    permuting them permutes outputs and input gradients and leaves the summed weight gradients unchanged.
    With the causal mask that symmetry is broken."""
    shape = tiny_shape(d_l=2, d_m=8, d_a=2, d_s=6, b_mu=2, n_mu=2, causal=False)
    x, G, params = tiny_problem(shape)
    perm = np.array([3, 0, 5, 1, 4, 2])
    a = O.step_microbatch_major(x, G, params, shape)
    b = O.step_microbatch_major(x[:, :, perm], G[:, :, perm], params, shape)
    assert np.allclose(a.boundaries[:, :, :, perm], b.boundaries, rtol=1e-12, atol=1e-13)
    assert np.allclose(a.dx[:, :, perm], b.dx, rtol=1e-11, atol=1e-13)
    for l in range(shape.d_l):
        assert np.allclose(a.grads[l], b.grads[l], rtol=1e-10, atol=1e-12)
    causal = tiny_shape(d_l=2, d_m=8, d_a=2, d_s=6, b_mu=2, n_mu=2)
    c = O.step_microbatch_major(x, G, params, causal)
    d = O.step_microbatch_major(x[:, :, perm], G[:, :, perm], params, causal)
    assert not np.allclose(c.boundaries[:, :, :, perm], d.boundaries, rtol=1e-3, atol=1e-3)


def test_sequences_in_a_micro_batch_do_not_mix():
    shape = tiny_shape(d_l=1, n_mu=1)
    x, G, params = tiny_problem(shape)
    r = O.step_microbatch_major(x, G, params, shape)
    x2 = x.copy(); x2[0, 1] += 1.0
    r2 = O.step_microbatch_major(x2, G, params, shape)
    assert np.array_equal(r.boundaries[-1][0, 0], r2.boundaries[-1][0, 0])


# ---------------------------------------------------------------- backward formulas

@pytest.mark.parametrize("causal", [True, False])
def test_gradients_by_central_finite_differences(causal):
    shape = tiny_shape(d_l=2, d_m=8, d_a=2, d_s=5, b_mu=2, n_mu=2, causal=causal)
    x, G, params = tiny_problem(shape)
    res = O.step_microbatch_major(x, G, params, shape)
    assert abs(res.loss - O.loss_only(x, G, params, shape)) < 1e-9
    h = 1e-5
    worst = 0.0
    rng = np.random.default_rng(0)
    sl = S.tensor_slices(shape.d_m, shape.d_I)
    for l in range(shape.d_l):
        for name in O.PARAM_ORDER:           # every tensor: all entries if small, else a random sample
            idx = np.arange(sl[name].start, sl[name].stop)
            if idx.size > 24:
                idx = rng.choice(idx, 24, replace=False)
            for i in idx:
                pp = [p.copy() for p in params]; pm = [p.copy() for p in params]
                pp[l][i] += h; pm[l][i] -= h
                fd = (O.loss_only(x, G, pp, shape) - O.loss_only(x, G, pm, shape)) / (2 * h)
                an = res.grads[l][i]
                worst = max(worst, abs(fd - an) / max(1.0, abs(an)))
    flat_idx = rng.choice(x.size, 40, replace=False)
    for i in flat_idx:
        xp = x.copy().ravel(); xm = x.copy().ravel()
        xp[i] += h; xm[i] -= h
        fd = (O.loss_only(xp.reshape(x.shape), G, params, shape) - O.loss_only(xm.reshape(x.shape), G, params, shape)) / (2 * h)
        an = res.dx.ravel()[i]
        worst = max(worst, abs(fd - an) / max(1.0, abs(an)))
    assert worst < 2e-7, worst


@pytest.mark.parametrize("causal", [True, False])
def test_against_autograd_built_from_library_routines(causal):
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    shape = tiny_shape(d_l=2, d_m=16, d_a=4, d_s=7, b_mu=2, n_mu=2, causal=causal)
    x, G, params = tiny_problem(shape)
    res = O.step_microbatch_major(x, G, params, shape)
    sl = S.tensor_slices(shape.d_m, shape.d_I)
    shp = S.tensor_shapes(shape.d_m, shape.d_I)
    tp = [{n: torch.tensor(p[sl[n]].reshape(shp[n]), dtype=torch.float64, requires_grad=True) for n in O.PARAM_ORDER}
          for p in params]
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    d, H = shape.d_m, shape.d_a
    outs = []
    for mu in range(shape.n_mu):
        a = tx[mu]
        for l in range(shape.d_l):
            P = tp[l]
            h = F.layer_norm(a, (d,), P["ln1_g"], P["ln1_b"], shape.ln_eps)
            qkv = F.linear(h, P["w_qkv"].T, P["b_qkv"])
            q, k, v = (t.reshape(shape.b_mu, shape.d_s, H, d // H).transpose(1, 2) for t in qkv.split(d, dim=-1))
            att = F.scaled_dot_product_attention(q, k, v, is_causal=causal)
            att = att.transpose(1, 2).reshape(shape.b_mu, shape.d_s, d)
            a = a + F.linear(att, P["w_o"].T, P["b_o"])
            h2 = F.layer_norm(a, (d,), P["ln2_g"], P["ln2_b"], shape.ln_eps)
            a = a + F.linear(F.gelu(F.linear(h2, P["w_1"].T, P["b_1"]), approximate="tanh"), P["w_2"].T, P["b_2"])
        outs.append(a)
    y = torch.stack(outs)
    (y * torch.tensor(G)).sum().backward()
    assert np.allclose(res.boundaries[-1], y.detach().numpy(), rtol=1e-11, atol=1e-11)
    assert np.allclose(res.dx, tx.grad.numpy(), rtol=1e-10, atol=1e-11)
    for l in range(shape.d_l):
        for n in O.PARAM_ORDER:
            assert np.allclose(res.grads[l][sl[n]].reshape(shp[n]), tp[l][n].grad.numpy(), rtol=1e-10, atol=1e-11), (l, n)


# ---------------------------------------------------------------- accumulation and ordering invariants

def test_accumulation_over_micro_batches_equals_full_batch_gradient():
    shape = tiny_shape(d_l=2, n_mu=4, b_mu=2)
    x, G, params = tiny_problem(shape)
    acc = O.step_microbatch_major(x, G, params, shape)
    full_shape = O.StackShape(shape.d_l, shape.d_m, shape.d_a, shape.d_I, shape.d_s, shape.b_mu * shape.n_mu, 1)
    merge = lambda t: t.reshape((1, shape.n_mu * shape.b_mu) + t.shape[2:])
    full = O.step_microbatch_major(merge(x), merge(G), params, full_shape)
    for l in range(shape.d_l):
        assert np.allclose(acc.grads[l], full.grads[l], rtol=1e-12, atol=1e-12)
    assert np.allclose(merge(acc.dx), full.dx, rtol=1e-13, atol=1e-13)
    assert np.allclose(merge(acc.boundaries[-1]), full.boundaries[-1], rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("causal", [True, False])
def test_layered_order_equals_micro_batch_major_order_including_early_adam(causal):
    shape = tiny_shape(d_l=3, n_mu=3, causal=causal)
    x, G, params = tiny_problem(shape)
    rng = np.random.default_rng(5)
    m0 = [0.1 * rng.standard_normal(p.size) for p in params]
    v0 = [0.01 * rng.random(p.size) for p in params]
    hp = O.AdamHyper(lr=1e-2, step=4)
    a = O.step_microbatch_major(x, G, params, shape, hp, m0, v0)
    b = O.step_layered(x, G, params, shape, hp, m0, v0)
    assert np.allclose(a.boundaries, b.boundaries, rtol=1e-13, atol=1e-13)
    assert np.allclose(a.dx, b.dx, rtol=1e-12, atol=1e-13)
    assert abs(a.loss - b.loss) < 1e-9
    for l in range(shape.d_l):
        assert np.allclose(a.grads[l], b.grads[l], rtol=1e-12, atol=1e-12)
        assert np.allclose(a.new_params[l], b.new_params[l], rtol=1e-13, atol=1e-13)
        assert np.allclose(a.new_m[l], b.new_m[l], rtol=1e-13, atol=1e-14)
        assert np.allclose(a.new_v[l], b.new_v[l], rtol=1e-13, atol=1e-14)


# ---------------------------------------------------------------- Adam

def test_adam_hand_worked_values():
    # w=0.5 m=0.1 v=0.04 g=-0.2 lr=0.01 b1=0.9 b2=0.99 t=2:
    # m' = 0.09 - 0.02 = 0.07 ; v' = 0.0396 + 0.01*0.04 = 0.04
    # mhat = 0.07/0.19 ; vhat = 0.04/0.0199 ; w' = 0.5 - 0.01*mhat/(sqrt(vhat)+1e-8)
    hp = O.AdamHyper(lr=0.01, beta1=0.9, beta2=0.99, eps=1e-8, step=2)
    w, m, v = O.adam_update(np.array([0.5]), np.array([0.1]), np.array([0.04]), np.array([-0.2]), hp)
    assert abs(m[0] - 0.07) < 1e-16
    assert abs(v[0] - 0.04) < 1e-16
    assert abs(w[0] - 0.4974013907589168) < 1e-15


def test_adam_first_step_is_signed_unit_step_and_zero_gradient_is_a_fixed_point():
    hp = O.AdamHyper()            # lr 1e-3, betas (0.9, 0.999), eps 1e-8, t = 1
    g = np.array([3.0, -0.25, 1e-3, 0.0])
    w0 = np.array([1.0, 2.0, -1.0, 0.7])
    w, m, v = O.adam_update(w0, np.zeros(4), np.zeros(4), g, hp)
    # g / (|g| + eps) up to rounding of the bias corrections
    assert np.allclose(w, w0 - 1e-3 * g / (np.abs(g) + 1e-8), rtol=0, atol=1e-15)
    assert w[3] == w0[3] and m[3] == 0.0 and v[3] == 0.0
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)
    # literal: first entry moves by lr * 3/(3+1e-8)
    assert abs((w0[0] - w[0]) - 1e-3 * (1 - 1e-8 / 3)) < 1e-15


# ---------------------------------------------------------------- gradient scaling (section 2.2)

@pytest.mark.parametrize("order", ["mbmajor", "layered"])
def test_a_power_of_two_loss_scale_changes_nothing_in_fp64(order):
    # Scaling by 2^k is exact in binary floating point (no overflow in fp64 here), and every gradient is linear in
    # the output gradient: the step with (G * S, loss_scale = S) equals the step with (G, no scaling) bit for bit,
    # while the gradients it reports are S times larger.
    shape = tiny_shape(d_l=2, n_mu=2)
    x, G, params = tiny_problem(shape)
    step = O.step_layered if order == "layered" else O.step_microbatch_major
    hp = O.AdamHyper(lr=1e-2, step=3)
    S_ = 1024.0
    a = step(x, G, params, shape, hp)
    b = step(x, G * S_, params, shape, O.AdamHyper(lr=1e-2, step=3, loss_scale=S_, skip_nonfinite=True))
    assert b.skipped == [False] * shape.d_l
    for l in range(shape.d_l):
        assert np.array_equal(b.grads[l], S_ * a.grads[l])
        assert np.array_equal(a.new_params[l], b.new_params[l])
        assert np.array_equal(a.new_m[l], b.new_m[l]) and np.array_equal(a.new_v[l], b.new_v[l])
    # a scale that is not a power of two: equal up to rounding only
    c = step(x, G * 3.0, params, shape, O.AdamHyper(lr=1e-2, step=3, loss_scale=3.0))
    for l in range(shape.d_l):
        solid = np.abs(a.grads[l]) > 1e-9          # the key bias' gradient is rounding noise, its update a coin toss
        assert np.allclose(a.new_params[l][solid], c.new_params[l][solid], rtol=1e-13, atol=1e-15)
        assert np.allclose(a.new_m[l], c.new_m[l], rtol=1e-12, atol=1e-15)


def test_an_update_with_a_non_finite_gradient_is_left_out_as_a_whole_only_when_asked():
    w0, m0, v0 = np.array([0.5, -1.0, 2.0]), np.array([0.1, 0.0, -0.2]), np.array([0.04, 0.01, 0.0])
    for bad in (np.inf, -np.inf, np.nan):
        g = np.array([0.3, bad, -0.1])
        w, m, v = O.adam_update(w0, m0, v0, g, O.AdamHyper(loss_scale=8.0, skip_nonfinite=True))
        assert np.array_equal(w, w0) and np.array_equal(m, m0) and np.array_equal(v, v0)
        assert O.adam_skips(g, O.AdamHyper(skip_nonfinite=True)) and not O.adam_skips(g, O.AdamHyper())
        w, m, v = O.adam_update(w0, m0, v0, g, O.AdamHyper(loss_scale=8.0))
        assert not np.isfinite(m[1]) and np.isfinite(w[0]) and w[0] != w0[0]      # without the test the value spreads
    g = np.array([0.3, 1e300, -0.1])                                             # huge but finite: a normal update
    assert not O.adam_skips(g, O.AdamHyper(skip_nonfinite=True))
    # a step whose output gradient holds an infinity reaches every layer below it: all of them are left out
    shape = tiny_shape(d_l=2, n_mu=2)
    x, G, params = tiny_problem(shape)
    G = G.copy()
    G[1, 0, 2, 1] = np.inf
    with np.errstate(invalid="ignore", over="ignore"):
        r = O.step_layered(x, G, params, shape, O.AdamHyper(skip_nonfinite=True))
    assert r.skipped == [True, True]
    for l in range(shape.d_l):
        assert np.array_equal(r.new_params[l], np.asarray(params[l], dtype=np.float64))
        assert not r.new_m[l].any() and not r.new_v[l].any()


def test_loss_scaler_follows_its_closed_form():
    # n clean steps from scale s0 with growth interval k: s0 * 2^(n // k), capped; an overflow halves it (floored)
    # and restarts the count
    s = O.LossScaler(scale=4.0, growth_interval=3, max_scale=64.0, min_scale=1.0)
    seen = []
    for n in range(1, 16):
        O.loss_scaler_update(s, False)
        seen.append(s.scale)
        assert s.scale == min(4.0 * 2.0 ** (n // 3), 64.0)
    assert seen[-1] == 64.0
    O.loss_scaler_update(s, False)                   # 16th clean step: one past a growth, count is 1
    O.loss_scaler_update(s, True)
    assert s.scale == 32.0 and s.good_steps == 0
    O.loss_scaler_update(s, False); O.loss_scaler_update(s, False)
    assert s.scale == 32.0 and s.good_steps == 2     # the overflow restarted the run of clean steps
    O.loss_scaler_update(s, False)
    assert s.scale == 64.0
    for _ in range(10):
        O.loss_scaler_update(s, True)
    assert s.scale == 1.0                            # floor


def test_key_bias_gradient_vanishes_identically():
    # Softmax does not change when every score of a row moves by the same amount, and adding a
    # constant vector c to every key moves row i's scores by q_i . c: so dL/d(key bias) = 0.
    shape = tiny_shape(d_l=2, d_m=8, d_a=2, d_s=6, b_mu=2, n_mu=2)
    x, G, params = tiny_problem(shape)
    res = O.step_microbatch_major(x, G, params, shape)
    sl = S.tensor_slices(shape.d_m, shape.d_I)
    d = shape.d_m
    for l in range(shape.d_l):
        gb = res.grads[l][sl["b_qkv"]]
        assert np.abs(gb[d:2 * d]).max() < 1e-13 * np.abs(gb[:d]).max()
