"""Pins of the oracle's attention-loss analysis (Sec. 3, Eq. 5-7) to things other
than itself: a hand-worked fixture, explicit set sums, the pairwise form of the
gap, closed forms and invariants, and the already pinned decode-attention
routine for the attention scores themselves.  CPU only."""
import os

import numpy as np
import pytest

import oracle


def parse_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = line.split("=", 1)
            out[key.strip()] = [float(v) for v in val.split()]
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def test_hand_worked_example(golden_dir):
    g = parse_golden(os.path.join(golden_dir, "attention_loss_example.txt"))
    n32 = np.array(g["norm2"], dtype=np.float32)
    a = np.array(g["a"])
    assert list(oracle.drop_order(n32)) == [int(v) for v in g["drop_order"]]
    Y, Ym = oracle.alr(a, n32)
    assert np.allclose(Ym, g["Ym"], atol=1e-15)
    assert abs(Y - g["Y"][0]) < 1e-14
    for m in range(1, 6):
        assert abs(oracle.attention_loss(a, n32, m) - g["L"][m - 1]) < 1e-15
        assert abs(oracle.attention_loss_ref(a, m) - g["Lref"][m - 1]) < 1e-15
    assert oracle.attention_loss(a, n32, 0) == 0.0 and oracle.attention_loss_ref(a, 0) == 0.0


def explicit_losses(a, n32, m):
    """Eq. 5 with the dropped set built by rank counting (no sort, no prefix sums)."""
    bits = n32.view(np.uint32)
    T = len(a)
    dropped, lowest = [], []
    for p in range(T):
        later = sum(1 for q in range(T) if bits[q] > bits[p] or (bits[q] == bits[p] and q > p))
        if later < m:                       # fewer than m pairs are discarded before p
            dropped.append(p)
        below = sum(1 for q in range(T) if a[q] < a[p] or (a[q] == a[p] and q < p))
        if below < m:
            lowest.append(p)
    assert len(dropped) == m and len(lowest) == m
    return sum(a[p] for p in dropped), sum(a[p] for p in lowest)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_against_explicit_sets_and_pairwise_form(seed):
    rng = np.random.default_rng(seed)
    T = 37
    n32 = rng.integers(1, 9, T).astype(np.float32)            # many ties
    a = rng.random(T) ** 3
    a[rng.integers(0, T, 5)] = a[0]                            # tied scores too
    a /= a.sum()
    Y, Ym = oracle.alr(a, n32)
    total = 0.0
    for m in range(1, T + 1):
        L, Lref = explicit_losses(a, n32, m)
        assert abs(oracle.attention_loss(a, n32, m) - L) < 1e-14
        assert abs(oracle.attention_loss_ref(a, m) - Lref) < 1e-14
        assert abs(Ym[m - 1] - (L - Lref)) < 1e-14
        total += L - Lref
    assert abs(Y - total) < 1e-12
    # pairwise form: each unordered pair adds max(a_p, a_q) minus the score of the pair member
    # that the norm rule discards later
    bits = n32.view(np.uint32)
    pair = 0.0
    for p in range(T):
        for q in range(p + 1, T):
            q_goes_first = bits[q] > bits[p] or bits[q] == bits[p]          # q > p breaks the tie
            pair += max(a[p], a[q]) - (a[p] if q_goes_first else a[q])
    assert abs(Y - pair) < 1e-12


def test_invariants_and_closed_forms():
    rng = np.random.default_rng(7)
    T = 200
    n32 = (rng.standard_normal(T) ** 2).astype(np.float32)
    a = rng.random(T)
    a /= a.sum()
    Y, Ym = oracle.alr(a, n32)
    assert np.all(Ym >= -1e-15) and abs(Ym[-1]) < 1e-12         # gap is non-negative, zero at m = T
    assert Y >= 0
    # uniform attention: every rule loses m/T
    Yu, Ymu = oracle.alr(np.full(T, 1.0 / T), n32)
    assert abs(Yu) < 1e-12
    assert abs(oracle.attention_loss(np.full(T, 1.0 / T), n32, 50) - 0.25) < 1e-14
    # attention falling exactly as the norm rises: the norm rule IS the ideal rule
    order = oracle.drop_order(n32)
    a_sorted = np.sort(a)
    a_ideal = np.empty(T)
    a_ideal[order] = a_sorted                                   # first dropped gets the lowest score
    assert abs(oracle.alr(a_ideal, n32)[0]) < 1e-12
    # the opposite pairing is the worst case: sum_j a_(j) * (2j - (T-1)) over ascending scores
    a_worst = np.empty(T)
    a_worst[order] = a_sorted[::-1]
    j = np.arange(T)
    assert abs(oracle.alr(a_worst, n32)[0] - np.sum(a_sorted * (2 * j - (T - 1)))) < 1e-10
    # all attention on the pair that is discarded first: L^m = 1 for m >= 1, reference 0 until m = T
    one = np.zeros(T)
    one[order[0]] = 1.0
    assert abs(oracle.alr(one, n32)[0] - (T - 1)) < 1e-12
    # ... and on the pair discarded last: no gap at all
    last = np.zeros(T)
    last[order[-1]] = 1.0
    assert abs(oracle.alr(last, n32)[0]) < 1e-12
    # Y only depends on the norm ORDER: a monotone map of the norms changes nothing
    assert abs(oracle.alr(a, np.sqrt(n32))[0] - Y) < 1e-12


def test_drop_order_is_reverse_of_selection_order():
    rng = np.random.default_rng(3)
    n32 = rng.integers(0, 6, 50).astype(np.float32)
    order = oracle.drop_order(n32)
    assert sorted(order) == list(range(50))
    for k in (1, 7, 25, 50):
        kept = oracle.select(n32[None], k)[0]
        assert sorted(order[50 - k:]) == list(kept)            # the last k to go are the kept ones
        assert sorted(order[:50 - k]) == sorted(set(range(50)) - set(kept))


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_attention_scores_match_decode_attention_with_indicator_values(dt):
    # With V = identity rows (T == D), decode attention returns the scores themselves.
    rng = np.random.default_rng(5)
    B, Hkv, G, D = 2, 2, 3, 64
    T = D
    K = rng.standard_normal((B, Hkv, T, D)).astype(np.float32)
    Q = rng.standard_normal((B, Hkv * G, D)).astype(np.float32)
    V = np.broadcast_to(np.eye(T, dtype=np.float32), (B, Hkv, T, D)).copy()
    if dt == "bf16":
        K, Q, V = f32_to_bf16_bits(K), f32_to_bf16_bits(Q), f32_to_bf16_bits(V)
    a = oracle.attn_probs(Q, K, dt)
    want = oracle.decode_attn(Q, K, V, dt)
    assert a.shape == (B, Hkv * G, T)
    assert np.abs(a - want).max() < 2e-7                       # decode output is rounded to fp32
    assert np.allclose(a.sum(-1), 1.0, atol=1e-12)
    # explicit scale
    a2 = oracle.attn_probs(Q, K, dt, scale=0.05)
    want2 = oracle.decode_attn(Q, K, V, dt, scale=0.05)
    assert np.abs(a2 - want2).max() < 2e-7


def test_attention_scores_closed_forms_and_gqa():
    D, T = 64, 9
    K = np.zeros((1, 2, T, D), dtype=np.float32)
    w = np.array([5, 1, 2, 7, 3, 4, 2, 6, 1], dtype=np.float64)
    for t in range(T):
        K[0, 0, t, t] = 2.0                                     # head 0: logit t = 2 * q_t / 8
        K[0, 1, t, t] = 1.0
    Q = np.zeros((1, 4, D), dtype=np.float32)
    Q[0, 0, :T] = 4.0 * np.log(w)                               # -> softmax weights proportional to w
    Q[0, 2, :T] = 8.0 * np.log(w[::-1])                         # query head 2 reads KV head 1
    a = oracle.attn_probs(Q, K, "f32")
    assert np.allclose(a[0, 0], w / w.sum(), rtol=1e-6)
    assert np.allclose(a[0, 1], 1.0 / T, rtol=1e-12)            # zero query: uniform
    assert np.allclose(a[0, 2], w[::-1] / w.sum(), rtol=1e-6)


def test_alr_heads_wiring():
    rng = np.random.default_rng(9)
    B, Hkv, G, T, D = 2, 2, 2, 33, 64
    K = rng.standard_normal((B, Hkv, T, D)).astype(np.float32)
    Q = rng.standard_normal((B, Hkv * G, D)).astype(np.float32)
    n32, _ = oracle.norms(K, "f32")
    Y, Lm, Lref = oracle.alr_heads(Q, K, n32, "f32", m=10)
    a = oracle.attn_probs(Q, K, "f32")
    for b in range(B):
        for hq in range(Hkv * G):
            L, R = explicit_losses(a[b, hq], n32[b, hq // G], 10)
            assert abs(Lm[b, hq] - L) < 1e-13 and abs(Lref[b, hq] - R) < 1e-13
            assert abs(Y[b, hq] - oracle.alr(a[b, hq], n32[b, hq // G])[0]) < 1e-15
    assert np.all(Lm >= Lref - 1e-15)
