"""Pins of the oracle's expert-capacity mode and load-balance loss against things other than
itself: brute force in Python written from the definitions, closed forms, invariants and finite
differences.  CPU only."""
import numpy as np
import pytest

from test_oracle_pins import gelu64, rand_layer


def brute_keep(idx, N, capacity):
    """Walk the pairs in flat order; an expert takes its first `capacity` pairs."""
    held = [0] * N
    keep = np.zeros(idx.shape, np.int32)
    for t in range(idx.shape[0]):
        for j in range(idx.shape[1]):
            e = int(idx[t, j])
            if capacity <= 0 or held[e] < capacity:
                keep[t, j] = 1
                held[e] += 1
    return keep


@pytest.mark.parametrize("T,k,N,cap", [(1, 1, 1, 1), (40, 3, 5, 7), (300, 4, 16, 50), (64, 2, 8, 1), (100, 2, 128, 3)])
def test_capacity_permutation_brute_force(oracle, T, k, N, cap):
    rng = np.random.default_rng(21)
    pr = 1.0 / np.arange(1, N + 1) ** 1.1                        # skewed, so that experts overflow
    idx = np.stack([rng.choice(N, size=k, replace=False, p=pr / pr.sum()) for _ in range(T)]).astype(np.int32)
    offsets, slot_of, src_of, keep = oracle.permutation(idx, N, capacity=cap, want_keep=True)
    bk = brute_keep(idx, N, cap)
    assert np.array_equal(keep, bk)
    flat, kf = idx.ravel(), bk.ravel().astype(bool)
    counts = np.bincount(flat[kf], minlength=N)
    assert counts.max() <= cap and np.array_equal(counts, np.minimum(np.bincount(flat, minlength=N), cap))
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    kept = offsets[N]
    assert kept == kf.sum()
    # kept pairs: the stable sort by expert of the kept flat indices; dropped pairs: -1, no slot
    order = np.flatnonzero(kf)
    order = order[np.argsort(flat[order], kind="stable")]
    assert np.array_equal(src_of[:kept], order) and np.all(src_of[kept:] == -1)
    assert np.all(slot_of.ravel()[~kf] == -1)
    assert np.array_equal(slot_of.ravel()[order], np.arange(kept))


def test_capacity_at_least_the_largest_expert_is_dropless(oracle):
    rng = np.random.default_rng(22)
    T, k, N = 90, 3, 7
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    big = int(np.bincount(idx.ravel(), minlength=N).max())
    a = oracle.permutation(idx, N)
    b = oracle.permutation(idx, N, capacity=big, want_keep=True)
    for u, v in zip(a, b[:3]):
        assert np.array_equal(u, v)
    assert b[3].all()
    c = oracle.permutation(idx, N, capacity=big - 1, want_keep=True)
    assert c[3].sum() < T * k


def test_dispatch_combine_skip_dropped_pairs(oracle):
    rng = np.random.default_rng(23)
    T, k, N, w, cap = 50, 2, 4, 8, 9
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    offsets, slot_of, src_of, keep = oracle.permutation(idx, N, capacity=cap, want_keep=True)
    xl = rng.standard_normal((T, w)).astype(np.float32)
    xp = np.full((T * k, w), np.nan, np.float32)
    xp[:] = oracle.dispatch(xl, slot_of)                          # rows past offsets[N] are never written
    kept = offsets[N]
    assert np.array_equal(xp[:kept], xl[src_of[:kept] // k])
    gate = rng.random((T, k))
    y = oracle.combine(np.nan_to_num(xp.astype(np.float64)), slot_of, gate)
    ref = (gate * keep)[:, :, None] * xl.astype(np.float64)[:, None, :]
    assert np.abs(y - ref.sum(1)).max() < 1e-12


def brute_forward_keep(p, keep):
    x = p["x"].astype(np.float64)
    T, d = x.shape
    y = np.zeros((T, d))
    for t in range(T):
        logit = (x[t].astype(np.float32) @ p["w_gate"]).astype(np.float64)
        chosen = sorted(range(len(logit)), key=lambda n: (-logit[n], n))[:p["k"]]
        z = np.exp(logit[chosen] - logit[chosen].max())
        gate = z / z.sum()                                        # over all k picks, dropped or not
        xl = x[t] @ p["w_down"].astype(np.float64)
        acc = np.zeros_like(xl)
        for j, (g, e) in enumerate(zip(gate, chosen)):
            if keep[t, j]:
                acc += g * (gelu64(xl @ p["w1"][e].astype(np.float64)) @ p["w2"][e].astype(np.float64))
        y[t] = acc @ p["w_up"].astype(np.float64)
    return y


def test_forward_with_capacity_brute_force(oracle):
    rng = np.random.default_rng(24)
    T, d, r, N, k, h, cap = 24, 64, 8, 4, 2, 12, 8
    p = rand_layer(rng, T, d, r, N, k, h)
    idx, _, _ = oracle.route(p["x"], p["w_gate"], None, k)
    keep = oracle.permutation(idx, N, capacity=cap, want_keep=True)[3]
    assert 0 < keep.sum() < T * k
    y = oracle.bigmac_forward(p["x"], p["w_gate"], None, p["w_down"], p["w_up"], p["w1"], p["w2"], k, keep=keep)
    yb = brute_forward_keep(p, keep)
    assert np.abs(y - yb).max() < 1e-5 * np.abs(yb).max()
    # a token that lost every pick gets exactly zero
    lost = np.flatnonzero(keep.sum(1) == 0)
    assert np.all(y[lost] == 0.0)
    # and the fine-grained layer with identity projections agrees (r == d)
    everything = oracle.bigmac_forward(p["x"], p["w_gate"], None, p["w_down"], p["w_up"], p["w1"], p["w2"], k,
                                       keep=np.ones_like(keep))
    full = oracle.bigmac_forward(p["x"], p["w_gate"], None, p["w_down"], p["w_up"], p["w1"], p["w2"], k)
    assert np.array_equal(everything, full)


def test_backward_with_capacity_finite_differences(oracle):
    rng = np.random.default_rng(25)
    T, d, r, N, k, h, cap = 12, 64, 8, 4, 2, 12, 4
    p = rand_layer(rng, T, d, r, N, k, h, w_std=0.3)
    dy = rng.standard_normal((T, d)).astype(np.float32)
    idx0, _, _ = oracle.route(p["x"], p["w_gate"], None, k)
    keep = oracle.permutation(idx0, N, capacity=cap, want_keep=True)[3]
    assert 0 < keep.sum() < T * k

    def loss():
        y = oracle.bigmac_forward(p["x"], p["w_gate"], None, p["w_down"], p["w_up"], p["w1"], p["w2"], k, keep=keep)
        return float((y * dy).sum())

    g = oracle.bigmac_backward(p["x"], dy, p["w_gate"], None, p["w_down"], p["w_up"], p["w1"], p["w2"], k, keep=keep)
    names = {"x": "dx", "w_down": "d_w_down", "w_up": "d_w_up", "w_gate": "d_w_gate", "w1": "d_w1", "w2": "d_w2"}
    checked = 0
    for name, gname in names.items():
        flat = p[name].reshape(-1)
        for pos in rng.choice(flat.size, size=12, replace=False):
            old = flat[pos]
            hi, lo = np.float32(old + 2e-3), np.float32(old - 2e-3)
            flat[pos] = hi
            same_hi = np.array_equal(oracle.route(p["x"], p["w_gate"], None, k)[0], idx0)
            lp = loss()
            flat[pos] = lo
            same_lo = np.array_equal(oracle.route(p["x"], p["w_gate"], None, k)[0], idx0)
            lm = loss()
            flat[pos] = old
            if not (same_hi and same_lo):
                continue                                          # the top-k set moved (the keep mask is held fixed with it)
            fd = (lp - lm) / (np.float64(hi) - np.float64(lo))
            an = g[gname].reshape(-1)[pos]
            assert abs(fd - an) <= 5e-4 * max(1.0, abs(an)), (name, pos, fd, an)
            checked += 1
    assert checked > 50
    # experts' gradients come from their kept rows only: an expert whose pairs were all dropped has none
    # (construct: capacity 0 is dropless, so compare a starved expert by masking it out entirely)
    mask = keep * (idx0 != 0)
    g2 = oracle.bigmac_backward(p["x"], dy, p["w_gate"], None, p["w_down"], p["w_up"], p["w1"], p["w2"], k, keep=mask)
    assert not np.any(g2["d_w1"][0]) and not np.any(g2["d_w2"][0])


# ------------------------------------------------------------------ load-balance loss --------

def test_aux_loss_closed_forms(oracle):
    T, N, k, alpha = 16, 4, 2, 0.25
    # uniform softmax and balanced routing: f_e = P_e = 1/N, loss = alpha * N * N / N^2 = alpha
    logits = np.zeros((T, N), np.float32)
    idx = np.array([[(t + j) % N for j in range(k)] for t in range(T)], np.int32)
    loss, f, dl = oracle.aux_loss(logits, idx, alpha)
    assert abs(loss - alpha) < 1e-15 and np.allclose(f, 1.0 / N)
    assert np.abs(dl).max() < 1e-18                               # balanced: f_n equals the mix for every n
    # everything on expert 0, softmax saturated on expert 0: f = P = e_0, loss = alpha * N
    logits = np.full((T, N), -50.0, np.float32)
    logits[:, 0] = 50.0
    idx = np.zeros((T, 1), np.int32)
    loss, f, _ = oracle.aux_loss(logits, idx, alpha)
    assert abs(loss - alpha * N) < 1e-12 and f[0] == 1.0
    # shift invariance of the softmax
    rng = np.random.default_rng(26)
    z = rng.standard_normal((T, N))
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    a = oracle.aux_loss(z, idx, alpha)
    b = oracle.aux_loss(z + rng.standard_normal((T, 1)), idx, alpha)
    assert abs(a[0] - b[0]) < 1e-14 and np.abs(a[2] - b[2]).max() < 1e-15


def test_aux_loss_brute_force_and_finite_differences(oracle):
    rng = np.random.default_rng(27)
    T, N, k, alpha = 9, 6, 3, 0.01
    z = rng.standard_normal((T, N)) * 2.0
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    loss, f, dl = oracle.aux_loss(z, idx, alpha)
    total = 0.0
    for e in range(N):                                            # the definition, one expert at a time
        f_e = sum(1 for t in range(T) for j in range(k) if idx[t, j] == e) / (T * k)
        P_e = sum(np.exp(z[t, e]) / np.exp(z[t]).sum() for t in range(T)) / T
        assert abs(f[e] - f_e) < 1e-15
        total += f_e * P_e
    assert abs(loss - alpha * N * total) < 1e-14
    assert np.abs(dl.sum(axis=1)).max() < 1e-16                   # softmax gradients sum to zero per token
    for _ in range(40):
        t, n = rng.integers(T), rng.integers(N)
        zp, zm = z.copy(), z.copy()
        zp[t, n] += 1e-5
        zm[t, n] -= 1e-5
        fd = (oracle.aux_loss(zp, idx, alpha)[0] - oracle.aux_loss(zm, idx, alpha)[0]) / 2e-5
        assert abs(fd - dl[t, n]) < 1e-9


def test_aux_loss_layer_terms_finite_differences(oracle):
    rng = np.random.default_rng(28)
    T, d, N, k, alpha = 7, 64, 5, 2, 0.05
    x = rng.standard_normal((T, d))
    wg = rng.standard_normal((d, N)) * 0.2
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    dl = oracle.aux_loss(x @ wg, idx, alpha)[2]
    terms = oracle.aux_loss_layer_terms(x, wg, dl)
    for name, arr, gname in (("x", x, "dx"), ("wg", wg, "d_w_gate")):
        for _ in range(20):
            pos = tuple(rng.integers(s) for s in arr.shape)
            old = arr[pos]
            arr[pos] = old + 1e-5
            lp = oracle.aux_loss(x @ wg, idx, alpha)[0]
            arr[pos] = old - 1e-5
            lm = oracle.aux_loss(x @ wg, idx, alpha)[0]
            arr[pos] = old
            assert abs((lp - lm) / 2e-5 - terms[gname][pos]) < 1e-9, (name, pos)
