"""Pins for the oracle's attention-layer functions (projections around the cached attention).

SubGCache Sec. 3.4 feeds the representative prompt, then each query's question tokens, through the
LLM's layers; the paper never writes the layer down, so the arithmetic is the textbook one:
y = Attention(x Wq^T, x Wk^T, x Wv^T) Wo^T with weights stored "out features x in features".
What is checked against what:
  * brute force       -> pure-Python loops for both projections around the pinned brute-force attention,
                         on shapes where every dimension differs (a transposed weight cannot pass)
  * special case      -> identity weights reduce the layer to the already pinned attention routines
  * closed form       -> zero query weights give uniform attention: y_i = mean of the visible projected
                         values, projected back (written with cumulative sums, no softmax)
  * invariants        -> linear in Wo and in Wv; a permutation of the model dimension applied to x and to
                         the weight columns changes nothing; swapping two query heads together with Wo's
                         column blocks changes nothing inside a KV group and changes the result across
                         groups (the head-major feature order is observable); a hand-made weight with one
                         entry per feature fixes which feature is which head and channel
  * cache             -> the layer's cache is the rotated projected K and the projected V
"""
import numpy as np
import pytest

from oracle import oracle as orc

RNG = np.random.default_rng(20250510)


def _weights(D, Hq, Hkv, d):
    w_qkv = RNG.standard_normal(((Hq + 2 * Hkv) * d, D)) / np.sqrt(D)
    w_o = RNG.standard_normal((D, Hq * d)) / np.sqrt(Hq * d)
    return w_qkv, w_o


def _loops_project(x, w):
    """y[t][f] = sum_i x[t][i] * w[f][i], nested Python loops on lists."""
    xs, ws = x.tolist(), w.tolist()
    return [[sum(xt[i] * wf[i] for i in range(len(xt))) for wf in ws] for xt in xs]


def _split_heads(rows, n_heads, d, first):
    return [[[r[first + h * d + c] for c in range(d)] for h in range(n_heads)] for r in rows]


@pytest.mark.parametrize("P,S,D,Hq,Hkv,d,base", [(3, 2, 5, 2, 1, 4, 10000.0), (4, 3, 7, 4, 2, 2, 500000.0),
                                                   (0, 3, 3, 2, 2, 4, 10000.0), (5, 1, 6, 3, 1, 6, 0.0)])
def test_layer_against_python_loops(P, S, D, Hq, Hkv, d, base):
    w_qkv, w_o = _weights(D, Hq, Hkv, d)
    xp, xs = RNG.standard_normal((P, D)), RNG.standard_normal((S, D))
    # prompt: un-rotated projected K, V by loops
    pp = _loops_project(xp, w_qkv) if P else []
    pk = np.array(_split_heads(pp, Hkv, d, Hq * d)).reshape(P, Hkv, d)
    pv = np.array(_split_heads(pp, Hkv, d, (Hq + Hkv) * d)).reshape(P, Hkv, d)
    sp = _loops_project(xs, w_qkv)
    q = np.array(_split_heads(sp, Hq, d, 0))
    k = np.array(_split_heads(sp, Hkv, d, Hq * d))
    v = np.array(_split_heads(sp, Hkv, d, (Hq + Hkv) * d))
    o, _ = orc.brute_force_suffix(pk, pv, q, k, v, base)
    o_flat = np.array([[o[i][h][c] for h in range(Hq) for c in range(d)] for i in range(S)])
    y_loops = np.array(_loops_project(o_flat, w_o))
    if P:
        ck, cv, _ = orc.attention_layer_prefix(xp, w_qkv, w_o, Hq, Hkv, d, base)
    else:
        ck = cv = np.zeros((0, Hkv, d))
    y = orc.attention_layer_suffix(ck, cv, xs, w_qkv, w_o, Hq, Hkv, d, base)
    assert y.shape == (S, D)
    np.testing.assert_allclose(y, y_loops, rtol=0, atol=1e-12)


def test_prefix_layer_against_python_loops_via_empty_cache():
    """The prompt's own output: causal attention over the prompt = a suffix over an empty cache."""
    P, D, Hq, Hkv, d, base = 6, 5, 4, 2, 4, 10000.0
    w_qkv, w_o = _weights(D, Hq, Hkv, d)
    x = RNG.standard_normal((P, D))
    pr = _loops_project(x, w_qkv)
    q = np.array(_split_heads(pr, Hq, d, 0))
    k = np.array(_split_heads(pr, Hkv, d, Hq * d))
    v = np.array(_split_heads(pr, Hkv, d, (Hq + Hkv) * d))
    e = np.zeros((0, Hkv, d))
    o, _ = orc.brute_force_suffix(e, e, q, k, v, base)
    o_flat = np.array([[o[i][h][c] for h in range(Hq) for c in range(d)] for i in range(P)])
    y_loops = np.array(_loops_project(o_flat, w_o))
    ck, cv, y = orc.attention_layer_prefix(x, w_qkv, w_o, Hq, Hkv, d, base)
    np.testing.assert_allclose(y, y_loops, rtol=0, atol=1e-12)
    # the cache: rotated projected K (independent numpy rotation), projected V untouched
    np.testing.assert_allclose(ck, orc.rope_numpy(k, np.arange(P), base), rtol=0, atol=1e-12)
    np.testing.assert_allclose(cv, v, rtol=0, atol=1e-13)


def test_identity_weights_reduce_to_plain_attention():
    """D = Hq d = Hkv d and Wq = Wk = Wv = Wo = I: q = k = v = x viewed as heads, y = o flattened."""
    H, d, P, S, base = 3, 8, 11, 5, 10000.0
    D = H * d
    eye = np.eye(D)
    w_qkv = np.concatenate([eye, eye, eye])
    xp, xs = RNG.standard_normal((P, D)), RNG.standard_normal((S, D))
    ck, cv, y_p = orc.attention_layer_prefix(xp, w_qkv, eye, H, H, d, base)
    kp = xp.reshape(P, H, d)
    ck2, cv2, o_p, _ = orc.prefix_prefill(kp, kp, kp, base)
    np.testing.assert_allclose(ck, ck2, atol=1e-14)
    np.testing.assert_allclose(y_p, o_p.reshape(P, D), atol=1e-14)
    y_s = orc.attention_layer_suffix(ck, cv, xs, w_qkv, eye, H, H, d, base)
    ks = xs.reshape(S, H, d)
    # concatenation form, dense numpy: rows P.. of causal attention over [prompt; question]
    o_full = orc.full_causal_numpy(np.concatenate([kp, ks]), np.concatenate([kp, ks]), np.concatenate([kp, ks]), base)
    o_full = o_full[0] if isinstance(o_full, tuple) else o_full
    np.testing.assert_allclose(y_s, o_full[P:].reshape(S, D), atol=1e-12)


def test_zero_query_weights_give_running_mean_of_values():
    P, S, D, Hq, Hkv, d, base = 9, 6, 7, 4, 2, 4, 500000.0
    w_qkv, w_o = _weights(D, Hq, Hkv, d)
    w_qkv[: Hq * d] = 0.0
    xp, xs = RNG.standard_normal((P, D)), RNG.standard_normal((S, D))
    ck, cv, y_p = orc.attention_layer_prefix(xp, w_qkv, w_o, Hq, Hkv, d, base)
    y_s = orc.attention_layer_suffix(ck, cv, xs, w_qkv, w_o, Hq, Hkv, d, base)
    w_v = w_qkv[(Hq + Hkv) * d:]
    v_all = np.concatenate([xp, xs]) @ w_v.T                      # [P+S][Hkv d]
    mean = np.cumsum(v_all, axis=0) / np.arange(1, P + S + 1)[:, None]
    g = Hq // Hkv
    o = mean.reshape(P + S, Hkv, d)[:, np.repeat(np.arange(Hkv), g), :].reshape(P + S, Hq * d)
    y = o @ w_o.T
    np.testing.assert_allclose(y_p, y[:P], atol=1e-12)
    np.testing.assert_allclose(y_s, y[P:], atol=1e-12)


def test_linear_in_output_and_value_weights():
    P, S, D, Hq, Hkv, d, base = 7, 4, 6, 4, 2, 4, 10000.0
    w_qkv, w_o = _weights(D, Hq, Hkv, d)
    _, w_o2 = _weights(D, Hq, Hkv, d)
    xp, xs = RNG.standard_normal((P, D)), RNG.standard_normal((S, D))

    def run(wq, wo):
        ck, cv, yp = orc.attention_layer_prefix(xp, wq, wo, Hq, Hkv, d, base)
        return np.concatenate([yp, orc.attention_layer_suffix(ck, cv, xs, wq, wo, Hq, Hkv, d, base)])

    y1, y2 = run(w_qkv, w_o), run(w_qkv, w_o2)
    np.testing.assert_allclose(run(w_qkv, 2.0 * w_o - 3.0 * w_o2), 2.0 * y1 - 3.0 * y2, atol=1e-12)
    w_scaled = w_qkv.copy()
    w_scaled[(Hq + Hkv) * d:] *= -2.5
    np.testing.assert_allclose(run(w_scaled, w_o), -2.5 * y1, atol=1e-12)


def test_model_dimension_permutation_changes_nothing():
    P, S, D, Hq, Hkv, d, base = 5, 4, 9, 2, 1, 8, 10000.0
    w_qkv, w_o = _weights(D, Hq, Hkv, d)
    xp, xs = RNG.standard_normal((P, D)), RNG.standard_normal((S, D))
    perm = RNG.permutation(D)
    ck, cv, yp = orc.attention_layer_prefix(xp, w_qkv, w_o, Hq, Hkv, d, base)
    ys = orc.attention_layer_suffix(ck, cv, xs, w_qkv, w_o, Hq, Hkv, d, base)
    ck2, cv2, yp2 = orc.attention_layer_prefix(xp[:, perm], w_qkv[:, perm], w_o[perm], Hq, Hkv, d, base)
    ys2 = orc.attention_layer_suffix(ck2, cv2, xs[:, perm], w_qkv[:, perm], w_o[perm], Hq, Hkv, d, base)
    np.testing.assert_allclose(ck2, ck, atol=1e-13)
    np.testing.assert_allclose(yp2, yp[:, perm], atol=1e-12)
    np.testing.assert_allclose(ys2, ys[:, perm], atol=1e-12)


def test_query_heads_permute_with_output_column_blocks_inside_a_group_only():
    P, S, D, Hq, Hkv, d, base = 6, 3, 5, 4, 2, 4, 10000.0
    w_qkv, w_o = _weights(D, Hq, Hkv, d)
    xp, xs = RNG.standard_normal((P, D)), RNG.standard_normal((S, D))

    def run(wq, wo):
        ck, cv, yp = orc.attention_layer_prefix(xp, wq, wo, Hq, Hkv, d, base)
        return np.concatenate([yp, orc.attention_layer_suffix(ck, cv, xs, wq, wo, Hq, Hkv, d, base)])

    def swap_heads(a, b):
        wq, wo = w_qkv.copy(), w_o.copy()
        wq[a * d:(a + 1) * d], wq[b * d:(b + 1) * d] = w_qkv[b * d:(b + 1) * d], w_qkv[a * d:(a + 1) * d]
        wo[:, a * d:(a + 1) * d], wo[:, b * d:(b + 1) * d] = w_o[:, b * d:(b + 1) * d], w_o[:, a * d:(a + 1) * d]
        return wq, wo

    y = run(w_qkv, w_o)
    np.testing.assert_allclose(run(*swap_heads(0, 1)), y, atol=1e-12)       # heads 0, 1 share KV head 0
    assert np.abs(run(*swap_heads(1, 2)) - y).max() > 1e-3                   # heads 1, 2 read different KV heads


def test_projection_shapes_and_feature_order():
    D, Hq, Hkv, d, n = 4, 3, 1, 2, 2
    w = np.zeros(((Hq + 2 * Hkv) * d, D))
    for f in range(w.shape[0]):
        w[f, f % D] = f + 1.0          # feature f reads input f % D with weight f + 1
    x = np.array([[1.0, 10.0, 100.0, 1000.0], [2.0, 20.0, 200.0, 2000.0]])
    q, k, v = orc.project_qkv(x, w, Hq, Hkv, d)
    assert q.shape == (n, Hq, d) and k.shape == (n, Hkv, d) and v.shape == (n, Hkv, d)
    assert q[0, 0, 0] == 1.0 and q[0, 0, 1] == 20.0 and q[0, 1, 0] == 300.0 and q[0, 2, 1] == 6 * 10.0
    assert k[1, 0, 0] == 7 * 200.0 and k[1, 0, 1] == 8 * 2000.0
    assert v[0, 0, 0] == 9 * 1.0 and v[1, 0, 1] == 10 * 20.0
    o = np.arange(n * Hq * d, dtype=np.float64).reshape(n, Hq, d)
    wo = np.zeros((3, Hq * d))
    wo[0, 0] = 1.0
    wo[1, 3] = 2.0      # head 1, channel 1
    wo[2, 5] = -1.0     # head 2, channel 1
    y = orc.project_out(o, wo)
    assert y.tolist() == [[0.0, 6.0, -5.0], [6.0, 18.0, -11.0]]
