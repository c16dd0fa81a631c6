"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests calls the HIP library.  Every check compares the oracle
with something other than itself: hand values of the Code equation, numpy
one-liners, a dict-of-lists brute-force clustering, a textbook dense attention,
a full argsort, and closed-form special cases.
"""
import os

import numpy as np
import pytest

import sik_workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bits_of(x, dtype):
    return W.to_bits(np.asarray(x, np.float32), dtype)


def f64(bits, dtype):
    return W.from_bits(bits, dtype).astype(np.float64)


def small_cfg(**kw):
    base = dict(batch=2, n_kv_heads=2, n_q_heads=4, head_dim=32, context=200, top_k=17, dtype="bf16",
                sigma="lognormal", outlier_frac=0.05, outlier_scale=8.0, seed=11)
    base.update(kw)
    return W.scaled(W.CONFIGS["C2"], **base)


def dense_attention(q, K, V, scale):
    """Textbook softmax(q K^T * scale) V for one head, fp64."""
    z = (K @ q) * scale
    p = np.exp(z - z.max())
    p /= p.sum()
    return p @ V


# --------------------------------------------------------------------------- widening
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_widen_all_bit_patterns(oracle, dtype):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.widen(bits, dtype)
    with np.errstate(all="ignore"):
        want = f64(bits, dtype)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


# --------------------------------------------------------------------------- Code / pack
def test_code_hand_values_eq3(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "eq3_sign_codes.txt")) if l[0] in "+-"]
    assert len(rows) == 16
    for dtype in ("fp16", "bf16"):
        for g in range(8):  # place the pattern in group g of a D=32 key, all other dims negative
            for *signs, code in rows:
                k = -np.ones((1, 1, 1, 32), np.float32)
                for e, s in enumerate(signs):
                    k[0, 0, 0, 4 * g + e] = 1.5 if s == "+" else -0.25
                c = oracle.encode(bits_of(k, dtype), dtype, np.zeros((1, 1, 32), np.float32), 0, 1)
                byte = int(c[0, 0, 0, g // 2])
                nib = (byte >> 4) if g % 2 == 0 else (byte & 15)
                assert nib == int(code), (dtype, g, signs)
                other = (byte & 15) if g % 2 == 0 else (byte >> 4)
                assert other == 0
                assert int(c.sum()) == byte  # nothing leaked into other bytes


def test_plane_size_matches_overhead_analysis(oracle):
    d, nbytes = [l.split() for l in open(os.path.join(GOLDEN, "memory_model.txt")) if l[0].isdigit()][0]
    cfg = small_cfg(head_dim=int(d), context=40, batch=1, n_kv_heads=1, n_q_heads=1)
    K, _ = W.make_cache(cfg)
    c = oracle.encode(K, cfg.dtype, np.zeros((1, 1, int(d)), np.float32), 0, 40)
    assert c.shape[-1] == int(nbytes) and c.nbytes == 40 * int(d) // 8


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_sign_bits_match_numpy_and_round_trip(oracle, dtype):
    cfg = small_cfg(dtype=dtype, head_dim=64)
    K, _ = W.make_cache(cfg, channel_offset_std=2.0)
    rng = np.random.default_rng(5)
    mu = rng.normal(0, 2, size=(cfg.batch, cfg.n_kv_heads, 64)).astype(np.float32)
    codes = oracle.encode(K, dtype, mu, 0, cfg.context)
    want_bits = f64(K, dtype) >= mu[:, :, None, :].astype(np.float64)
    got_bits = np.unpackbits(codes, axis=-1, bitorder="big").astype(bool)
    assert np.array_equal(got_bits, want_bits)
    assert np.array_equal(np.packbits(got_bits, axis=-1, bitorder="big"), codes)


def test_sign_of_zero_and_ties_with_mu(oracle):
    # K == mu and -0 >= +0 both count as "+"
    k = np.array([0.0, -0.0, 1.0, -1.0, 0.5, 0.5, 0.25, -0.25], np.float32).reshape(1, 1, 1, 8)
    mu = np.array([0.0, 0.0, 1.0, -1.0, 0.5, 0.75, 0.25, 0.0], np.float32).reshape(1, 1, 8)
    c = oracle.encode(bits_of(k, "fp16"), "fp16", mu, 0, 1)
    assert int(c[0, 0, 0, 0]) == 0b11111010


def test_reflection_flips_every_bit(oracle):
    cfg = small_cfg(dtype="fp16", sigma="unit", outlier_frac=0.0, outlier_count=0)
    K, _ = W.make_cache(cfg)
    Kf = W.from_bits(K, "fp16")
    mu = np.zeros((cfg.batch, cfg.n_kv_heads, cfg.head_dim), np.float32)
    c1 = oracle.encode(K, "fp16", mu, 0, cfg.context)
    c2 = oracle.encode(bits_of(-Kf, "fp16"), "fp16", mu, 0, cfg.context)
    nz = np.packbits(Kf != 0, axis=-1, bitorder="big")
    assert np.array_equal((c1 ^ c2) & nz, nz)


def test_encode_range_only_touches_requested_tokens(oracle):
    cfg = small_cfg()
    K, _ = W.make_cache(cfg)
    mu = np.zeros((cfg.batch, cfg.n_kv_heads, cfg.head_dim), np.float32)
    full = oracle.encode(K, cfg.dtype, mu, 0, cfg.context)
    part = np.full_like(full, 0xAA)
    oracle.encode(K, cfg.dtype, mu, 50, 7, part)
    assert np.array_equal(part[:, :, 50:57], full[:, :, 50:57])
    assert np.all(part[:, :, :50] == 0xAA) and np.all(part[:, :, 57:] == 0xAA)


# --------------------------------------------------------------------------- mu
def test_mean_matches_numpy_and_centres(oracle):
    cfg = small_cfg(context=333)
    K, _ = W.make_cache(cfg, capacity=340, channel_offset_std=2.0)
    sl = np.array([333, 150], np.int32)
    mu = oracle.mean(K, cfg.dtype, sl)
    Kd = f64(K, cfg.dtype)
    for b in range(2):
        want = Kd[b, :, :sl[b]].mean(axis=1)
        assert np.array_equal(mu[b], want.astype(np.float32))
        centred = Kd[b, :, :sl[b]] - mu[b][:, None, :]
        assert np.abs(centred.mean(axis=1)).max() <= 1e-6 * np.abs(Kd).max()


def test_centring_balances_signs_max_entropy_condition(oracle):
    L = 4096
    cfg = small_cfg(batch=1, n_kv_heads=1, n_q_heads=1, context=L, head_dim=32, sigma="unit",
                    outlier_frac=0.0, outlier_count=0)
    K, _ = W.make_cache(cfg, channel_offset_std=2.0)
    sl = np.array([L], np.int32)
    mu = oracle.mean(K, cfg.dtype, sl)
    frac = np.unpackbits(oracle.encode(K, cfg.dtype, mu, 0, L), axis=-1, bitorder="big").mean(axis=2)
    assert np.abs(frac - 0.5).max() <= 4 / np.sqrt(L)          # P(+) = P(-) = 1/2 after centring
    raw = np.unpackbits(oracle.encode(K, cfg.dtype, 0 * mu, 0, L), axis=-1, bitorder="big").mean(axis=2)
    assert np.abs(raw - 0.5).max() > 0.2                        # and visibly not without it


# --------------------------------------------------------------------------- codebook
def test_codebook_brute_force_and_invariants(oracle):
    cfg = small_cfg(context=257)
    K, _ = W.make_cache(cfg, capacity=260, channel_offset_std=1.0)
    sl = np.array([257, 31], np.int32)
    mu, codes, cb, cnt = oracle.fit(K, cfg.dtype, sl)
    Kd = f64(K, cfg.dtype)
    G = cfg.head_dim // 4
    for b in range(cfg.batch):
        for h in range(cfg.n_kv_heads):
            Kp = Kd[b, h, :sl[b]] - mu[b, h].astype(np.float64)
            assert cnt[b, h].sum(axis=1).tolist() == [sl[b]] * G
            for g in range(G):
                clusters = {}
                for i in range(sl[b]):
                    sub = Kp[i, 4 * g:4 * g + 4]
                    j = int("".join("1" if x >= 0 else "0" for x in sub), 2)
                    clusters.setdefault(j, []).append(sub)
                for j in range(16):
                    members = clusters.get(j, [])
                    assert cnt[b, h, g, j] == len(members)
                    want = np.mean(members, axis=0) if members else np.zeros(4)
                    assert np.array_equal(cb[b, h, g, j], want.astype(np.float32))
                    # a centroid lies in the orthant of its own sign pattern (or is zero)
                    for e in range(4):
                        c = cb[b, h, g, j, e]
                        assert c == 0 or (c > 0) == bool((j >> (3 - e)) & 1)
            # sum_j |C_j| c_j = sum_i K'_i, which is ~0 after centring
            tot = (cnt[b, h][..., None] * cb[b, h].astype(np.float64)).sum(axis=1).reshape(-1)
            assert np.allclose(tot, Kp.sum(axis=0), atol=1e-4 * sl[b])


def test_codes_passed_to_codebook_are_the_ones_used(oracle):
    # a codebook built from all-zero codes puts every member into cluster 0
    cfg = small_cfg(batch=1, n_kv_heads=1, n_q_heads=1, context=50)
    K, _ = W.make_cache(cfg)
    sl = np.array([50], np.int32)
    mu = oracle.mean(K, cfg.dtype, sl)
    cb, cnt = oracle.codebook(K, cfg.dtype, sl, mu, np.zeros((1, 1, 50, cfg.head_dim // 8), np.uint8))
    assert np.all(cnt[..., 0] == 50) and np.all(cnt[..., 1:] == 0)
    Kp = f64(K, cfg.dtype)[0, 0] - mu[0, 0]
    assert np.allclose(cb[0, 0, :, 0, :].reshape(-1), Kp.mean(axis=0), rtol=1e-6, atol=1e-7)


# --------------------------------------------------------------------------- table + score
def test_score_equals_reconstruct_then_dot(oracle):
    cfg = small_cfg(context=300, head_dim=64)
    K, _ = W.make_cache(cfg, channel_offset_std=1.0)
    sl = np.array([300, 123], np.int32)
    mu, codes, cb, cnt = oracle.fit(K, cfg.dtype, sl)
    q, _, _ = W.make_step_inputs(cfg, 0)
    s = oracle.score(q, cfg.dtype, cb, codes, sl)
    qd = f64(q, cfg.dtype)
    R = cfg.n_q_heads // cfg.n_kv_heads
    G = cfg.head_dim // 4
    nib = np.stack([codes >> 4, codes & 15], axis=-1).reshape(*codes.shape[:3], G)  # [B,H,L,G]
    for b in range(cfg.batch):
        for hq in range(cfg.n_q_heads):
            h = hq // R
            # K_hat_i = concat_g c[g, code_i(g)]
            Khat = cb[b, h][np.arange(G)[None, :], nib[b, h, :sl[b]]].reshape(sl[b], -1).astype(np.float64)
            want = Khat @ qd[b, hq]
            assert np.allclose(s[b, hq, :sl[b]], want, rtol=1e-12, atol=1e-12)
            assert np.all(np.isneginf(s[b, hq, sl[b]:]))


def test_singleton_clusters_make_scores_exact(oracle):
    # 16 keys whose sub-vectors take 16 distinct sign patterns in every group: each occupied
    # cluster has one member, so K_hat = K' and the LUT score is q.K' = q.K - q.mu exactly.
    D, L = 32, 16
    rng = np.random.default_rng(3)
    mag = rng.uniform(0.5, 2.0, size=(L, D)).astype(np.float32)
    K = np.empty((L, D), np.float32)
    for g in range(D // 4):
        perm = rng.permutation(16)
        for i in range(L):
            for e in range(4):
                K[i, 4 * g + e] = mag[i, 4 * g + e] * (1 if (perm[i] >> (3 - e)) & 1 else -1)
    Kb = bits_of(K, "fp16").reshape(1, 1, L, D)
    sl = np.array([L], np.int32)
    mu = np.zeros((1, 1, D), np.float32)  # encode against zero so the patterns are the ones built
    codes = oracle.encode(Kb, "fp16", mu, 0, L)
    cb, cnt = oracle.codebook(Kb, "fp16", sl, mu, codes)
    assert cnt.max() == 1
    q = bits_of(rng.normal(size=(1, 2, D)), "fp16")
    s = oracle.score(q, "fp16", cb, codes, sl)
    exact = f64(q, "fp16")[0] @ f64(Kb, "fp16")[0, 0].T
    assert np.allclose(s[0], exact, rtol=1e-6, atol=1e-6)
    got = oracle.topk(s, sl, 5)
    for hq in range(2):
        assert set(got[0, hq]) == set(np.argsort(-exact[hq])[:5])


def test_gqa_mapping_query_head_reads_its_own_kv_head(oracle):
    cfg = small_cfg(batch=1, n_kv_heads=2, n_q_heads=6, context=64)
    K, V = W.make_cache(cfg)
    sl = np.array([64], np.int32)
    mu, codes, cb, cnt = oracle.fit(K, cfg.dtype, sl)
    q, _, _ = W.make_step_inputs(cfg, 0)
    s = oracle.score(q, cfg.dtype, cb, codes, sl)
    for hq in range(6):
        alone = oracle.score(q[:, hq:hq + 1], cfg.dtype, cb[:, hq // 3:hq // 3 + 1],
                             codes[:, hq // 3:hq // 3 + 1], sl)
        assert np.array_equal(alone[0, 0], s[0, hq])


# --------------------------------------------------------------------------- top-k
def test_topk_matches_full_sort(oracle):
    rng = np.random.default_rng(9)
    s = rng.normal(size=(2, 3, 500))
    s[0, 1, 100:140] = s[0, 1, 7]          # a block of exact ties
    sl = np.array([500, 77], np.int32)
    for k in (1, 5, 77, 130, 500, 600):
        idx = oracle.topk(s, sl, k)
        for b in range(2):
            for h in range(3):
                L = sl[b]
                order = np.lexsort((np.arange(L), -s[b, h, :L]))  # score desc, then index asc
                want = list(order[:k]) + [-1] * max(0, k - L)
                assert idx[b, h].tolist() == want
    assert oracle.topk(s, sl, 1)[0, 0, 0] == np.argmax(s[0, 0])
    assert sorted(oracle.topk(s, sl, 500)[0, 2].tolist()) == list(range(500))


# --------------------------------------------------------------------------- attention
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_attention_over_everything_is_dense_attention(oracle, dtype):
    cfg = small_cfg(dtype=dtype, context=150, head_dim=64, n_kv_heads=2, n_q_heads=6)
    K, V = W.make_cache(cfg, capacity=160)
    q, _, _ = W.make_step_inputs(cfg, 1)
    L = 150
    idx = np.tile(np.arange(L, dtype=np.int32), (cfg.batch, cfg.n_q_heads, 1))
    out = oracle.sparse_attn(q, K, V, dtype, idx)
    Kd, Vd, qd = f64(K, dtype), f64(V, dtype), f64(q, dtype)
    for b in range(cfg.batch):
        for hq in range(cfg.n_q_heads):
            h = hq // 3
            want = dense_attention(qd[b, hq], Kd[b, h, :L], Vd[b, h, :L], 1 / np.sqrt(64))
            assert np.allclose(out[b, hq], want, rtol=1e-12, atol=1e-13)
    # a custom scale is honoured
    out2 = oracle.sparse_attn(q, K, V, dtype, idx, scale=0.37)
    want = dense_attention(qd[0, 0], Kd[0, 0, :L], Vd[0, 0, :L], 0.37)
    assert np.allclose(out2[0, 0], want, rtol=1e-12, atol=1e-13)


def test_attention_special_cases(oracle):
    cfg = small_cfg(context=90)
    K, V = W.make_cache(cfg)
    q, _, _ = W.make_step_inputs(cfg, 2)
    Vd = f64(V, cfg.dtype)
    rng = np.random.default_rng(1)
    # |S| = 1: the output is that V row
    one = rng.integers(0, 90, size=(cfg.batch, cfg.n_q_heads, 1)).astype(np.int32)
    out = oracle.sparse_attn(q, K, V, cfg.dtype, one)
    for b in range(cfg.batch):
        for hq in range(cfg.n_q_heads):
            assert np.array_equal(out[b, hq], Vd[b, hq // 2, one[b, hq, 0]])
    # convex combination, order invariance, -1 padding ignored, empty -> 0
    idx = np.stack([[rng.permutation(90)[:20] for _ in range(cfg.n_q_heads)] for _ in range(cfg.batch)]).astype(np.int32)
    out = oracle.sparse_attn(q, K, V, cfg.dtype, idx)
    for b in range(cfg.batch):
        for hq in range(cfg.n_q_heads):
            sel = Vd[b, hq // 2, idx[b, hq]]
            assert np.all(out[b, hq] <= sel.max(axis=0) + 1e-12) and np.all(out[b, hq] >= sel.min(axis=0) - 1e-12)
    perm = rng.permutation(20)
    assert np.allclose(oracle.sparse_attn(q, K, V, cfg.dtype, idx[:, :, perm]), out, rtol=1e-12, atol=1e-13)
    padded = np.concatenate([idx, -np.ones_like(idx[:, :, :5])], axis=2)
    assert np.allclose(oracle.sparse_attn(q, K, V, cfg.dtype, padded), out, rtol=1e-12, atol=1e-13)
    empty = -np.ones((cfg.batch, cfg.n_q_heads, 3), np.int32)
    assert np.all(oracle.sparse_attn(q, K, V, cfg.dtype, empty) == 0)


def test_attention_unchanged_by_channel_shift_of_keys(oracle):
    # softmax(x - c) = softmax(x): shifting every key by the same vector adds q.c to all logits
    rng = np.random.default_rng(4)
    L, D = 40, 32
    K = rng.integers(-40, 40, size=(1, 1, L, D)).astype(np.float32) / 8
    shift = rng.integers(-16, 16, size=D).astype(np.float32) / 8
    V = rng.normal(size=(1, 1, L, D)).astype(np.float32)
    q = rng.integers(-8, 8, size=(1, 2, D)).astype(np.float32) / 4
    idx = np.tile(np.arange(0, L, 2, dtype=np.int32), (1, 2, 1))
    a = oracle.sparse_attn(bits_of(q, "bf16"), bits_of(K, "bf16"), bits_of(V, "bf16"), "bf16", idx)
    b = oracle.sparse_attn(bits_of(q, "bf16"), bits_of(K - shift, "bf16"), bits_of(V, "bf16"), "bf16", idx)
    assert np.array_equal(W.from_bits(bits_of(K - shift, "bf16"), "bf16"), K - shift)  # exactly representable
    assert np.allclose(a, b, rtol=1e-10, atol=1e-12)


# --------------------------------------------------------------------------- decode step
def test_decode_step_with_k_equal_context_is_dense_attention_and_appends(oracle):
    cfg = small_cfg(context=120, top_k=121)
    K, V = W.make_cache(cfg, capacity=128, channel_offset_std=1.5)
    sl = np.array([120, 120], np.int32)
    mu, codes, cb, cnt = oracle.fit(K, cfg.dtype, sl)
    q, kn, vn = W.make_step_inputs(cfg, 0)
    K0 = K.copy()
    out, idx = oracle.decode_step(q, kn, vn, K, V, cfg.dtype, sl, mu, cb, codes, 121)
    assert sl.tolist() == [121, 121]
    assert np.array_equal(K[:, :, 120], kn) and np.array_equal(V[:, :, 120], vn)
    assert np.array_equal(K[:, :, :120], K0[:, :, :120])
    want_code = np.packbits(f64(kn, cfg.dtype) >= mu.astype(np.float64), axis=-1, bitorder="big")
    assert np.array_equal(codes[:, :, 120], want_code)
    Kd, Vd, qd = f64(K, cfg.dtype), f64(V, cfg.dtype), f64(q, cfg.dtype)
    for b in range(2):
        for hq in range(cfg.n_q_heads):
            assert sorted(idx[b, hq].tolist()) == list(range(121))
            want = dense_attention(qd[b, hq], Kd[b, hq // 2, :121], Vd[b, hq // 2, :121], 1 / np.sqrt(cfg.head_dim))
            assert np.allclose(out[b, hq], want, rtol=1e-11, atol=1e-13)


def test_retrieval_quality_sanity(oracle):
    # not a parity pin (the paper prints no recall value): the compressed-domain top-k must
    # overlap the exact q.K top-k far more than chance.
    cfg = W.scaled(W.CONFIGS["C2"], batch=1, n_kv_heads=2, n_q_heads=8, context=4096, top_k=128)
    K, V = W.make_cache(cfg)
    sl = np.array([4096], np.int32)
    mu, codes, cb, cnt = oracle.fit(K, cfg.dtype, sl)
    q, _, _ = W.make_step_inputs(cfg, 0)
    idx = oracle.topk(oracle.score(q, cfg.dtype, cb, codes, sl), sl, 128)
    Kd, qd = f64(K, cfg.dtype), f64(q, cfg.dtype)
    rec = []
    for hq in range(8):
        exact = set(np.argsort(-(Kd[0, hq // 4] @ qd[0, hq]))[:128])
        rec.append(len(exact & set(idx[0, hq])) / 128)
    assert np.mean(rec) > 10 * 128 / 4096


# =========================================================================== 2-bit token-wise K/V format
def q2_cfg(**kw):
    base = dict(batch=2, n_kv_heads=2, n_q_heads=4, head_dim=128, context=150, top_k=20, dtype="bf16",
                sigma="lognormal", outlier_frac=0.05, outlier_scale=8.0, seed=21)
    base.update(kw)
    return W.scaled(W.CONFIGS["C2"], **base)


def test_fp16_conversion_matches_numpy(oracle):
    rng = np.random.default_rng(3)
    x = np.concatenate([
        rng.normal(0, 1, 4000), rng.normal(0, 1e-5, 2000), rng.normal(0, 3e4, 2000),
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e6, -1e6, 6.103515625e-05, 6.0975552e-05,
                  5.9604645e-08, 2.9802322e-08, 2.98023224e-08 * 1.0001, 8.940697e-08, 1.0009765625,
                  1.00048828125, 1.00146484375, np.inf, -np.inf])]).astype(np.float32)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.to_fp16(x), want)


def test_two_bit_groups_worked_by_hand(oracle):
    rows = [l for l in open(os.path.join(GOLDEN, "eq9_two_bit_groups.txt")) if l[0] not in "#\n"]
    assert len(rows) == 8
    for line in rows:
        vals, par, codes = [np.array(p.split(), np.float64) for p in line.split("|")]
        V = np.tile(vals, 16).astype(np.float32).reshape(1, 1, 1, 128)     # 4 groups of 32, all alike
        Kz = np.zeros((1, 1, 1, 128), np.uint16)
        qkv = oracle.quantize_kv(Kz, bits_of(V, "fp16"), "fp16", np.zeros((1, 1, 128), np.float32),
                                 np.ones((1, 1, 128), np.float32), 0, 1)
        assert np.array_equal(qkv.vq[0, 0, 0], np.tile(codes, 16).astype(np.uint8)), line
        got = oracle.widen(qkv.vpar[0, 0, 0], "fp16")
        assert np.array_equal(got, np.tile(par, (4, 1))), line
        # an all-zero key: zero magnitudes, zero parameters
        assert not qkv.kq.any() and not qkv.kpar.any()


def test_two_bit_memory_model_matches_overhead_analysis(oracle):
    row = [l.split() for l in open(os.path.join(GOLDEN, "memory_model.txt")) if l.startswith("q2")][0]
    sign, val, par, fp16_bits, saving = map(int, row[1:])
    cfg = q2_cfg(batch=1, n_kv_heads=1, context=10)
    qkv = oracle.QuantKV(1, 1, 10, 128)
    # the fields hold exactly the paper's bit counts per token: 2 bits per code, 16 bits per parameter
    assert 2 * (qkv.kq[0, 0, 0].size + qkv.vq[0, 0, 0].size) == val
    assert 16 * (qkv.kpar[0, 0, 0].size + qkv.vpar[0, 0, 0].size) == par
    assert sign == cfg.head_dim and fp16_bits == 2 * 16 * cfg.head_dim
    assert round(100 * (1 - (sign + val + par) / fp16_bits)) == saving
    # the library's record keeps one token in one 128-byte line: the 896 bits plus 16 spare bytes
    rec = oracle.pack_records(np.zeros((1, 1, 10, 16), np.uint8), qkv)
    assert rec.shape[-1] == 128 and (sign + val + par) // 8 + 16 == 128


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_alpha_and_two_bit_quantiser_against_numpy(oracle, dtype):
    # the quantisation and normalisation equations written out plainly in fp64 (true divisions; numpy's own
    # fp64 -> fp16 conversion rounds once, to nearest even)
    cfg = q2_cfg(dtype=dtype)
    K, V = W.make_cache(cfg, channel_offset_std=1.5)
    sl = np.array([150, 97], np.int32)
    mu, codes, _, _ = oracle.fit(K, dtype, sl)
    al, qkv = oracle.fit_q2(K, V, dtype, sl, mu)
    K64, V64 = f64(K, dtype), f64(V, dtype)
    for b in range(2):
        L = int(sl[b])
        Kp = K64[b, :, :L] - mu[b, :, None, :].astype(np.float64)
        assert np.array_equal(al[b], np.abs(Kp).max(axis=1).astype(np.float32))
        a64 = al[b].astype(np.float64)[:, None, :]
        with np.errstate(divide="ignore", invalid="ignore"):
            khat = np.where(a64 > 0, np.abs(Kp) / a64, 0.0)
        for x, q, par in ((khat, qkv.kq, qkv.kpar), (V64[b, :, :L], qkv.vq, qkv.vpar)):
            g = x.reshape(x.shape[0], L, 4, 32)
            lo, hi = g.min(-1), g.max(-1)
            zp16 = lo.astype(np.float16)
            qs16 = ((hi - lo) / 3.0).astype(np.float16)
            assert np.array_equal(par[b, :, :L, :, 0], qs16.view(np.uint16))
            assert np.array_equal(par[b, :, :L, :, 1], zp16.view(np.uint16))
            qs, zp = qs16.astype(np.float64)[..., None], zp16.astype(np.float64)[..., None]
            with np.errstate(divide="ignore", invalid="ignore"):
                want = np.where(qs > 0, np.clip(np.rint((g - zp) / qs), 0, 3), 0).astype(np.uint8)
            assert np.array_equal(q[b, :, :L].reshape(g.shape), want)
        assert not qkv.kq[b, :, L:].any() and not qkv.vpar[b, :, L:].any()   # untouched beyond seq_len


def test_two_bit_code_decision_is_a_true_division(oracle):
    # qs = fp16(1/3) has no exact reciprocal.  x = qs / 2 sits exactly on the tie t = 0.5 (-> 0, ties to even);
    # one fp16 step above it t > 0.5 (-> 1).  A product with a rounded reciprocal, or arithmetic in binary32,
    # may move either: the oracle must not.
    qs = np.float16(1.0 / 3.0).astype(np.float64)
    assert qs == 1365.0 / 4096.0
    for zp in (0.0, -0.25, -0.125):
        v = np.full(32, zp)
        v[1] = zp + 1.0                                  # span 1 -> qs = fp16(1/3)
        v[2] = zp + qs / 2                               # t = 0.5 exactly
        v[3] = zp + qs / 2 + 2.0 ** -13                  # t just above the tie
        v[4] = zp + qs / 2 - 2.0 ** -13
        V = np.tile(v, 4).astype(np.float32).reshape(1, 1, 1, 128)
        assert np.array_equal(V.astype(np.float16).astype(np.float64).ravel(), np.tile(v, 4)), "fp16-exact inputs"
        qkv = oracle.quantize_kv(np.zeros((1, 1, 1, 128), np.uint16), bits_of(V, "fp16"), "fp16",
                                 np.zeros((1, 1, 128), np.float32), np.ones((1, 1, 128), np.float32), 0, 1)
        assert oracle.widen(qkv.vpar[0, 0, 0, 0], "fp16").tolist() == [qs, zp]
        assert qkv.vq[0, 0, 0, :5].tolist() == [0, 3, 0, 1, 0]
    # the K side divides by alpha: |K'| / alpha with alpha = 3 is not |K'| times a rounded 1/3
    Kv = np.zeros(128, np.float32)
    Kv[:4] = [3.0, 0.0, 0.5, 1.5]                        # x = 1, 0, 1/6, 1/2  ->  qs = fp16(1/3), t = 3, 0, 0.50018, 1.50037
    al = np.ones((1, 1, 128), np.float32)
    al[0, 0, :32] = 3.0
    qkv = oracle.quantize_kv(bits_of(Kv.reshape(1, 1, 1, 128), "fp16"), np.zeros((1, 1, 1, 128), np.uint16), "fp16",
                             np.zeros((1, 1, 128), np.float32), al, 0, 1)
    assert oracle.widen(qkv.kpar[0, 0, 0, 0], "fp16").tolist() == [qs, 0.0]
    assert qkv.kq[0, 0, 0, :4].tolist() == [3, 0, 1, 2]


def test_stored_parameters_round_once_from_fp64(oracle):
    # 1 + 2^-11 + 2^-30 lies above the fp16 tie between 1 and 1 + 2^-10: one rounding gives the upper value,
    # rounding to binary32 first lands on the tie and then falls to the even (lower) one
    x = np.array([1 + 2.0 ** -11 + 2.0 ** -30, 1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11 - 2.0 ** -40, 1 / 3, 2 / 3, 1e-7,
                  6.1e-5, 65519.999, 65520.0, -0.0])
    with np.errstate(over="ignore"):
        assert np.array_equal(oracle.f64_to_fp16(x), x.astype(np.float16).view(np.uint16))
    assert oracle.f64_to_fp16(x[:1])[0] == np.float16(1 + 2.0 ** -10).view(np.uint16)
    rng = np.random.default_rng(5)
    y = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 1e-6, 5000), rng.uniform(0, 1, 5000) / 3])
    assert np.array_equal(oracle.f64_to_fp16(y), y.astype(np.float16).view(np.uint16))


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_alpha_from_channel_extremes(oracle, dtype):
    # x -> |x - mu| is largest at an end of the range, and rounding to fp32 is monotone: alpha, a maximum over
    # all fitted tokens, is already fixed by the smallest and the largest key of each channel.  A prefill pass
    # that keeps per-channel minima and maxima next to the column sums therefore has alpha without reading K again.
    cfg = q2_cfg(dtype=dtype, batch=2, context=700)
    K, _ = W.make_cache(cfg, channel_offset_std=2.0)
    sl = np.array([700, 333], np.int32)
    mu = oracle.mean(K, dtype, sl)
    al = oracle.alpha(K, dtype, sl, mu)
    K64 = f64(K, dtype)
    for b in range(2):
        kmin, kmax = K64[b, :, :sl[b]].min(axis=1), K64[b, :, :sl[b]].max(axis=1)
        m = mu[b].astype(np.float64)
        want = np.maximum(np.abs(kmax - m), np.abs(kmin - m)).astype(np.float32)
        assert np.array_equal(al[b], want)
        # and in binary32 arithmetic (what a GPU pass would do): the same bits
        k32min, k32max = kmin.astype(np.float32), kmax.astype(np.float32)
        want32 = np.maximum(np.abs(k32max - mu[b]), np.abs(k32min - mu[b]))
        assert want32.dtype == np.float32 and np.array_equal(al[b], want32)
    assert np.array_equal(oracle.alpha(K, dtype, np.array([0, 0], np.int32), mu), np.zeros_like(mu))


def test_two_bit_reconstruction_error_bound_and_signs(oracle):
    cfg = q2_cfg(batch=1, context=300)
    K, V = W.make_cache(cfg, channel_offset_std=1.0)
    sl = np.array([300], np.int32)
    mu, codes, _, _ = oracle.fit(K, cfg.dtype, sl)
    al, qkv = oracle.fit_q2(K, V, cfg.dtype, sl, mu)
    Kd, Vd = oracle.dequant_kv(codes, qkv, al, 0, 300)
    Kp = (W.from_bits(K, cfg.dtype).astype(np.float32) - mu[:, :, None, :]).astype(np.float64)
    Vf = f64(V, cfg.dtype)
    # codes reach both ends of every non-constant group
    vg = qkv.vq.reshape(1, 2, 300, 4, 32)
    nonconst = oracle.widen(qkv.vpar[..., 0], "fp16") > 0
    assert np.all(vg.min(-1)[nonconst] == 0) and np.all(vg.max(-1)[nonconst] == 3)
    # |x - D(Q(x))| <= qs / 2 plus what rounding qs and zp to 16 bits can add (3 |dqs| + |dzp|)
    vqs = oracle.widen(qkv.vpar[..., 0], "fp16")[..., None]
    span = Vf.reshape(1, 2, 300, 4, 32)
    slack = 4 * 2.0 ** -11 * np.abs(span).max(-1, keepdims=True) + 3 * 2.0 ** -11 * vqs
    assert np.all(np.abs(span - Vd.reshape(span.shape)) <= vqs / 2 + slack)
    kqs = oracle.widen(qkv.kpar[..., 0], "fp16")[..., None]
    a = al.astype(np.float64)[:, :, None, :].reshape(1, 2, 1, 4, 32)
    kerr = np.abs(np.abs(Kp) - np.abs(Kd)).reshape(1, 2, 300, 4, 32)
    assert np.all(kerr <= a * (kqs / 2 + 8 * 2.0 ** -11))
    # the sign of the reconstruction is the code bit, and the code bit is the sign of K - mu
    bits = np.unpackbits(codes, axis=-1, bitorder="big").astype(bool)
    assert np.all((Kd >= 0) | ~bits) and np.all((Kd <= 0) | bits)
    assert np.all(np.abs(Kd) <= a.reshape(1, 2, 1, 128) * (1 + 2.0 ** -9))


def test_two_bit_record_round_trip_and_layout(oracle):
    rng = np.random.default_rng(8)
    qkv = oracle.QuantKV(1, 2, 5, 128)
    qkv.kq[:] = rng.integers(0, 4, qkv.kq.shape)
    qkv.vq[:] = rng.integers(0, 4, qkv.vq.shape)
    qkv.kpar[:] = rng.integers(0, 2 ** 16, qkv.kpar.shape)
    qkv.vpar[:] = rng.integers(0, 2 ** 16, qkv.vpar.shape)
    codes = rng.integers(0, 256, (1, 2, 5, 16)).astype(np.uint8)
    rec = oracle.pack_records(codes, qkv)
    c2, back = oracle.unpack_records(rec)
    assert np.array_equal(c2, codes)
    for f in ("kq", "vq", "kpar", "vpar"):
        assert np.array_equal(getattr(back, f), getattr(qkv, f))
    # spot-check the layout by hand: slot 5 of token 3 of head 1 covers channels 40..47, group 1
    slot = rec[0, 1, 3, 40:48]
    assert slot[0] == codes[0, 1, 3, 5] and slot[1] == 0
    assert (int(slot[2]) | int(slot[3]) << 8) == sum(int(qkv.kq[0, 1, 3, 40 + e]) << (2 * e) for e in range(8))
    assert (int(slot[4]) | int(slot[5]) << 8) == sum(int(qkv.vq[0, 1, 3, 40 + e]) << (2 * e) for e in range(8))
    assert (int(slot[6]) | int(slot[7]) << 8) == int(qkv.kpar[0, 1, 3, 1, 1])       # slot 5 = group 1, K zp


def test_two_bit_attention_all_tokens_equals_dense_on_reconstruction(oracle):
    cfg = q2_cfg(batch=1, n_kv_heads=2, n_q_heads=4, context=90)
    K, V = W.make_cache(cfg, channel_offset_std=0.5)
    sl = np.array([90], np.int32)
    mu, codes, _, _ = oracle.fit(K, cfg.dtype, sl)
    al, qkv = oracle.fit_q2(K, V, cfg.dtype, sl, mu)
    Kd, Vd = oracle.dequant_kv(codes, qkv, al, 0, 90)
    q, _, _ = W.make_step_inputs(cfg, 0)
    qf = f64(q, cfg.dtype)
    idx = np.tile(np.arange(90, dtype=np.int32), (1, 4, 1))
    out = oracle.sparse_attn_q2(q, cfg.dtype, codes, qkv, al, idx)
    for hq in range(4):
        want = dense_attention(qf[0, hq], Kd[0, hq // 2], Vd[0, hq // 2], 1 / np.sqrt(128))
        assert np.allclose(out[0, hq], want, rtol=1e-12, atol=1e-13)
    # one selected token: the output is that token's reconstructed value row; -1 entries are skipped
    one = np.full((1, 4, 3), -1, np.int32)
    one[:, :, 1] = 17
    out1 = oracle.sparse_attn_q2(q, cfg.dtype, codes, qkv, al, one)
    for hq in range(4):
        assert np.array_equal(out1[0, hq], Vd[0, hq // 2, 17])
    # a permutation of the selection changes nothing beyond rounding
    perm = np.random.default_rng(2).permutation(90).astype(np.int32)
    outp = oracle.sparse_attn_q2(q, cfg.dtype, codes, qkv, al, np.tile(perm, (1, 4, 1)))
    assert np.allclose(outp, out, rtol=1e-12, atol=1e-13)


def test_two_bit_decode_step_appends_against_frozen_parameters(oracle):
    cfg = q2_cfg(batch=2, context=64, top_k=12)
    K, V = W.make_cache(cfg, capacity=70, channel_offset_std=1.0)
    sl = np.array([64, 40], np.int32)
    mu, codes, cb, _ = oracle.fit(K, cfg.dtype, sl)
    al, qkv = oracle.fit_q2(K, V, cfg.dtype, sl, mu)
    q, kn, vn = W.make_step_inputs(cfg, 0)
    al0 = al.copy()
    out, idx = oracle.decode_step_q2(q, kn, vn, cfg.dtype, sl, mu, al, cb, codes, qkv, 12)
    assert sl.tolist() == [65, 41] and np.array_equal(al, al0)
    for b, t in ((0, 64), (1, 40)):
        want_bits = f64(kn[b], cfg.dtype) >= mu[b].astype(np.float64)
        assert np.array_equal(np.unpackbits(codes[b, :, t], axis=-1, bitorder="big").astype(bool), want_bits)
        # the new value row obeys the same group rule as a fitted one
        v32 = W.from_bits(vn[b], cfg.dtype).astype(np.float32).reshape(2, 4, 32)
        assert np.array_equal(qkv.vpar[b, :, t, :, 1], v32.min(-1).astype(np.float16).view(np.uint16))
    assert out.shape == (2, 4, 128) and np.all(idx[1] < 41) and np.all(idx[0] < 65)
    ref = oracle.sparse_attn_q2(q, cfg.dtype, codes, qkv, al, idx)
    assert np.array_equal(ref, out)


# =========================================================================== forced-inclusion sets (sink tokens)
def forced_setup(oracle, seed=31, L=400, cap=None, shorter=123):
    cfg = q2_cfg(batch=2, n_kv_heads=2, n_q_heads=8, context=L, top_k=40, seed=seed)
    K, V = W.make_cache(cfg, capacity=cap or L, channel_offset_std=0.7)
    sl = np.array([L, L - shorter], np.int32)
    mu, codes, cb, _ = oracle.fit(K, cfg.dtype, sl)
    q, kn, vn = W.make_step_inputs(cfg, 0)
    rng = np.random.default_rng(seed)
    forced = np.stack([np.stack([rng.choice(int(sl[b]), 12, replace=False) for _ in range(2)]) for b in range(2)])
    forced = forced.astype(np.int32)
    return cfg, K, V, sl, mu, codes, cb, q, kn, vn, forced


def test_forced_set_selection_against_brute_force(oracle):
    cfg, K, V, sl, mu, codes, cb, q, _, _, forced = forced_setup(oracle)
    forced[0, 1, 3] = -1                 # unused slot
    forced[1, 0, 5] = 399                # beyond seq_len[1] = 277: ignored
    out, idx = oracle.decode_step_forced(q, None, None, K, V, cfg.dtype, sl, mu, cb, codes, 40, forced)
    s = oracle.score(q, cfg.dtype, cb, codes, sl)
    for b in range(2):
        for hq in range(8):
            h = hq // 4
            f = [int(i) for i in forced[b, h] if 0 <= i < sl[b]]
            got = [int(i) for i in idx[b, hq] if i >= 0]
            assert len(got) == len(set(got)) == 40 and set(f) <= set(got)
            others = np.array([i for i in range(int(sl[b])) if i not in f])
            order = others[np.lexsort((others, -s[b, hq, others]))]
            assert set(got) - set(f) == set(order[:40 - len(f)].tolist())
    # the result is ordinary sparse attention over that set
    assert np.array_equal(out, oracle.sparse_attn(q, K, V, cfg.dtype, idx))
    # an empty forced set is the plain decode step
    none = np.full((2, 2, 4), -1, np.int32)
    out0, idx0 = oracle.decode_step_forced(q, None, None, K, V, cfg.dtype, sl.copy(), mu, cb, codes, 40, none)
    ref0, ridx0 = oracle.decode_step(q, None, None, K, V, cfg.dtype, sl.copy(), mu, cb, codes, 40)
    assert np.array_equal(np.sort(idx0, -1), np.sort(ridx0, -1)) and np.allclose(out0, ref0, rtol=1e-12, atol=1e-14)


def test_forced_set_with_full_budget_is_dense_attention(oracle):
    cfg, K, V, sl, mu, codes, cb, q, _, _, forced = forced_setup(oracle, seed=32, L=90, shorter=0)
    out, idx = oracle.decode_step_forced(q, None, None, K, V, cfg.dtype, sl, mu, cb, codes, 90, forced)
    Kf, Vf, qf = f64(K, cfg.dtype), f64(V, cfg.dtype), f64(q, cfg.dtype)
    for b in range(2):
        for hq in range(8):
            assert sorted(idx[b, hq].tolist()) == list(range(90))
            want = dense_attention(qf[b, hq], Kf[b, hq // 4, :90], Vf[b, hq // 4, :90], 1 / np.sqrt(128))
            assert np.allclose(out[b, hq], want, rtol=1e-12, atol=1e-13)


def test_forced_rows_in_full_precision_next_to_records(oracle):
    cfg, K, V, sl, mu, codes, cb, q, kn, vn, forced = forced_setup(oracle, seed=33, L=300, cap=304)
    al, qkv = oracle.fit_q2(K, V, cfg.dtype, sl, mu)
    forced[0, 0, 0] = -1
    fK = np.zeros((2, 2, 12, 128), np.uint16)
    fV = np.zeros((2, 2, 12, 128), np.uint16)
    for b in range(2):
        for h in range(2):
            for j in range(12):
                if forced[b, h, j] >= 0:
                    fK[b, h, j], fV[b, h, j] = K[b, h, forced[b, h, j]], V[b, h, forced[b, h, j]]
    out, idx = oracle.decode_step_q2_forced(q, kn, vn, cfg.dtype, sl, mu, al, cb, codes, qkv, 40, forced, fK, fV)
    assert sl.tolist() == [301, 178]
    Kd, Vd = oracle.dequant_kv(codes, qkv, al, 0, 301)
    qf = f64(q, cfg.dtype)
    for b in range(2):
        for hq in range(8):
            h = hq // 4
            f = [int(i) for i in forced[b, h] if i >= 0]
            dyn = [int(i) for i in idx[b, hq] if i >= 0 and i not in f]
            assert len(dyn) == 40 - len(f)
            Kc = np.concatenate([Kd[b, h, dyn], f64(K[b, h, f], cfg.dtype) - mu[b, h].astype(np.float64)])
            Vc = np.concatenate([Vd[b, h, dyn], f64(V[b, h, f], cfg.dtype)])
            want = dense_attention(qf[b, hq], Kc, Vc, 1 / np.sqrt(128))
            assert np.allclose(out[b, hq], want, rtol=1e-12, atol=1e-13)
    # without the side rows everything comes from records
    out_r, idx_r = oracle.decode_step_q2_forced(q, None, None, cfg.dtype, sl, mu, al, cb, codes, qkv, 40, forced)
    assert np.array_equal(idx_r, idx)
    assert np.array_equal(out_r, oracle.sparse_attn_q2(q, cfg.dtype, codes, qkv, al, idx))
    assert not np.allclose(out_r, out, rtol=1e-6, atol=0)      # 2-bit and 16-bit forced rows do differ


def test_budget_that_follows_the_context_length(oracle):
    # 7.5 % of the context ("retains only 7.5 % of the tokens"), integer ceiling, capped by k, at least 1
    assert [oracle.budget(4000, L, 75) for L in (32768, 1000, 13, 1, 0, 100000)] == [2458, 75, 1, 1, 1, 4000]
    assert oracle.budget(64, 999, 0) == 64
    cfg, K, V, sl, mu, codes, cb, q, _, _, forced = forced_setup(oracle, seed=34)
    none = np.full((2, 2, 1), -1, np.int32)
    out, idx = oracle.decode_step_forced(q, None, None, K, V, cfg.dtype, sl, mu, cb, codes, 60, none, k_per_mille=75)
    s = oracle.score(q, cfg.dtype, cb, codes, sl)
    for b, kb in ((0, 30), (1, 21)):            # ceil(400 * 0.075), ceil(277 * 0.075)
        for hq in range(8):
            got = [int(i) for i in idx[b, hq] if i >= 0]
            order = np.lexsort((np.arange(int(sl[b])), -s[b, hq, :sl[b]]))
            assert len(got) == kb and set(got) == set(order[:kb].tolist())
    # forced tokens count towards the budget and may use it up: 12 forced of a budget of 10 leave no pick
    out2, idx2 = oracle.decode_step_forced(q, None, None, K, V, cfg.dtype, sl, mu, cb, codes, 60, forced, k_per_mille=25)
    for b in range(2):
        for hq in range(8):
            assert sorted(i for i in idx2[b, hq] if i >= 0) == sorted(forced[b, hq // 4].tolist())


def test_group_shared_selection_is_the_summed_query(oracle):
    cfg = q2_cfg(batch=2, n_kv_heads=2, n_q_heads=8, context=500, top_k=30, seed=51)
    K, V = W.make_cache(cfg, channel_offset_std=0.8)
    sl = np.array([500, 211], np.int32)
    mu, codes, cb, _ = oracle.fit(K, cfg.dtype, sl)
    q, _, _ = W.make_step_inputs(cfg, 0)
    s_kv = oracle.shared_scores(q, cfg.dtype, cb, codes, sl)
    # the lookup table is linear in the query: summed scores = (sum of the group's queries) . reconstructed key
    qsum = f64(q, cfg.dtype).reshape(2, 2, 4, 128).sum(axis=2)
    for b in range(2):
        for h in range(2):
            L = int(sl[b])
            nib = np.stack([codes[b, h, :L] >> 4, codes[b, h, :L] & 15], axis=-1).reshape(L, 32)
            Khat = cb[b, h][np.arange(32)[None, :], nib].reshape(L, 128).astype(np.float64)
            assert np.allclose(s_kv[b, h, :L], Khat @ qsum[b, h], rtol=1e-12, atol=1e-12)
            assert np.all(np.isneginf(s_kv[b, h, L:]))
    out, idx = oracle.decode_step_shared(q, None, None, K, V, cfg.dtype, sl, mu, cb, codes, 30)
    assert idx.shape == (2, 2, 30)
    for b in range(2):
        for h in range(2):
            L = int(sl[b])
            order = np.lexsort((np.arange(L), -s_kv[b, h, :L]))
            assert idx[b, h].tolist() == order[:30].tolist()
    assert np.array_equal(out, oracle.sparse_attn(q, K, V, cfg.dtype, np.repeat(idx, 4, axis=1)))
    # one query head per KV head: nothing to share, the plain decode step
    cfg1 = q2_cfg(batch=1, n_kv_heads=2, n_q_heads=2, context=300, top_k=20, seed=52)
    K1, V1 = W.make_cache(cfg1)
    sl1 = np.array([300], np.int32)
    mu1, codes1, cb1, _ = oracle.fit(K1, cfg1.dtype, sl1)
    q1, _, _ = W.make_step_inputs(cfg1, 0)
    o_s, i_s = oracle.decode_step_shared(q1, None, None, K1, V1, cfg1.dtype, sl1, mu1, cb1, codes1, 20)
    o_p, i_p = oracle.decode_step(q1, None, None, K1, V1, cfg1.dtype, sl1, mu1, cb1, codes1, 20)
    assert np.array_equal(i_s, i_p) and np.array_equal(o_s, o_p)
