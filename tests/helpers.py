"""Plumbing shared by the GPU parity tests: numpy bit patterns <-> torch device tensors, and a
small state object that runs the oracle's prefill-side quantiser once and mirrors it on the GPU."""
import numpy as np
import torch

import sik_workloads as W

TORCH_DT = {"fp16": torch.float16, "bf16": torch.bfloat16}


def dev(bits: np.ndarray, dtype: str) -> torch.Tensor:
    """uint16 bit patterns -> contiguous device tensor of the 16-bit float type (bit-identical)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16).copy())
    return t.view(TORCH_DT[dtype]).cuda()


def bits_of_tensor(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def f64(bits, dtype):
    return W.from_bits(bits, dtype).astype(np.float64)


def topk_sets_agree(idx_gpu_row, idx_ref_row, s_ref_row, L, k, rel=1e-5):
    """North-star rule: |S| = min(k, L), no duplicates, all < L; every index in the symmetric
    difference has a reference score within rel * |k-th reference score| of the k-th score."""
    kk = min(k, L)
    g = [int(i) for i in idx_gpu_row if i >= 0]
    assert len(g) == kk, (len(g), kk)
    assert sum(1 for i in idx_gpu_row if i < 0) == k - kk
    assert len(set(g)) == kk, "duplicate indices"
    assert all(0 <= i < L for i in g)
    r = [int(i) for i in idx_ref_row if i >= 0]
    diff = set(g) ^ set(r)
    if not diff:
        return 0
    kth = np.sort(s_ref_row[:L])[::-1][kk - 1]
    tol = rel * abs(kth)
    for i in diff:
        assert abs(s_ref_row[i] - kth) <= tol, (i, s_ref_row[i], kth, tol)
    return len(diff)


def half_ulp(x, dtype):
    """Half a unit in the last place of the 16-bit type at |x| (8 significand bits bf16, 11 fp16)."""
    e = np.floor(np.log2(np.maximum(np.abs(x), 1e-30)))
    return np.exp2(e - (8 if dtype == "bf16" else 11))


def check_attention(got, ref, out_f32, dtype="bf16", label=None):
    """fp32 output: max|d| <= 1e-5 * max|ref| per (b, hq).  16-bit output: max|d| <= 2e-3, except
    where the 16-bit grid itself is coarser than that (|out| above ~1 for bf16): there the value must
    be the correctly rounded one up to the fp32 error, |d| <= half-ulp(ref) + 1e-5 * max|ref|.
    For 16-bit outputs the plain max|d| over the whole tensor is printed beside the worst ratio to that bar
    (and how many elements sit above a plain 2e-3, all of them where the 16-bit grid is coarser)."""
    worst_all, above = 0.0, 0
    for b in range(ref.shape[0]):
        for hq in range(ref.shape[1]):
            d = np.abs(got[b, hq] - ref[b, hq])
            scale = max(np.abs(ref[b, hq]).max(), 1e-30)
            if out_f32:
                assert d.max() <= 1e-5 * scale, (b, hq, float(d.max()), scale)
            else:
                bar = np.maximum(2e-3, half_ulp(ref[b, hq], dtype) + 1e-5 * scale)
                worst = float((d / bar).max())
                assert worst <= 1.0, (b, hq, worst, float(d.max()))
                worst_all = max(worst_all, worst)
                above += int((d > 2e-3).sum())
    plain = float(np.abs(got - ref).max())
    if not out_f32:
        print(f"{label or '16-bit output'} ({dtype}): plain max|d| = {plain:.3e} (max|ref| = {float(np.abs(ref).max()):.3g}), "
              f"{above} of {ref.size} elements above 2e-3, worst |d| / bar = {worst_all:.3f}")
    return plain


# --------------------------------------------------------------------------- 2-bit records: oracle (fp64) against binary32
U32 = 2.0 ** -24  # unit roundoff of binary32


def records_agree(oracle, got, K, V, dtype, mu, alpha, codes_ref, qkv_ref, b, t0, t1, base=0):
    """Compare the library's records of tokens [t0, t1) of sequence b with the oracle's fields (got, K and V
    may be slices that start at token `base`; codes_ref and qkv_ref are indexed by the token itself).

    The oracle evaluates the quantisation function in fp64; the library decides in binary32 (subtraction of
    mu, product with a rounded 1/alpha, subtraction of zp, product with a rounded 1/qs: six roundings, each
    at most U32 relative).  Rule:
      * sign bytes and the spare byte: equal;
      * a stored parameter (fp16 qs, zp) equals the oracle's, or is the neighbouring fp16 value while the exact
        fp64 value lies within the library's rounding error of the rounding boundary between the two
        (zp: 4 U32 |min x| on the K side, exact on the V side; qs: (4 U32 (|max x| + |min x|) [K side] +
        3 U32 span) / 3);
      * a code equals round((x - zp) / qs) evaluated in fp64 WITH THE RECORD'S OWN PARAMETERS (where those
        equal the oracle's this is the oracle's code, asserted), or is the other neighbour of t while t lies
        within 4 U32 (x / qs [K side] + |t|) of a half-integer.
    Returns (parameter exceptions, code exceptions, parameters compared, codes compared)."""
    import sik_workloads as W

    g_codes, g = oracle.unpack_records(got[b:b + 1, :, t0 - base:t1 - base])
    n = t1 - t0
    if n <= 0:
        return 0, 0, 0, 0
    H = got.shape[1]
    assert np.array_equal(g_codes[0], codes_ref[b, :, t0:t1]), "sign bytes differ"
    assert not got[b, :, t0 - base:t1 - base].reshape(H, n, 16, 8)[..., 1].any(), "spare byte not zero"
    K64 = W.from_bits(K[b, :, t0 - base:t1 - base], dtype).astype(np.float64)
    V64 = W.from_bits(V[b, :, t0 - base:t1 - base], dtype).astype(np.float64)
    a64 = alpha[b].astype(np.float64)[:, None, :]
    with np.errstate(divide="ignore", invalid="ignore"):
        xk = np.where(a64 > 0, np.abs(K64 - mu[b].astype(np.float64)[:, None, :]) / a64, 0.0)
    n_par = n_code = tot_par = tot_code = 0
    for x, is_k, q_g, p_g, q_o, p_o in ((xk, 1.0, g.kq[0], g.kpar[0], qkv_ref.kq[b, :, t0:t1], qkv_ref.kpar[b, :, t0:t1]),
                                        (V64, 0.0, g.vq[0], g.vpar[0], qkv_ref.vq[b, :, t0:t1], qkv_ref.vpar[b, :, t0:t1])):
        xg = x.reshape(H, n, 4, 32)
        lo, hi = xg.min(-1), xg.max(-1)
        exact = np.stack([(hi - lo) / 3.0, lo + 0.0], axis=-1)                  # what qs, zp round from
        band = np.stack([(4 * U32 * (np.abs(hi) + np.abs(lo)) * is_k + 3 * U32 * (hi - lo)) / 3.0,
                         4 * U32 * np.abs(lo) * is_k], axis=-1)
        vg, vo = oracle.widen(p_g, "fp16"), oracle.widen(p_o, "fp16")
        differ = p_g != p_o
        if differ.any():
            # neighbours in the fp16 grid (same sign, or the two zeros) with the exact value near their midpoint
            step = np.abs(p_g.astype(np.int32) - p_o.astype(np.int32))
            ok = (step == 1) & (np.abs(exact - (vg + vo) / 2) <= band)
            assert ok[differ].all(), ("parameter off", int((differ & ~ok).sum()))
            n_par += int(differ.sum())
        tot_par += differ.size
        qs, zp = vg[..., 0][..., None], vg[..., 1][..., None]
        with np.errstate(divide="ignore", invalid="ignore"):
            t = np.where(qs > 0, (xg - zp) / qs, 0.0)
            want = np.clip(np.rint(t), 0, 3).astype(np.uint8)
            tband = 4 * U32 * (np.where(qs > 0, xg / qs, 0.0) * is_k + np.abs(t))
        same_par = ~differ.any(-1)[..., None]
        qo = q_o.reshape(H, n, 4, 32)
        assert np.array_equal(np.where(same_par, want, qo), qo), "test-side formula disagrees with the oracle"
        qg = q_g.reshape(H, n, 4, 32)
        off = qg != want
        if off.any():
            near = np.abs(t - (np.floor(t) + 0.5)) <= tband
            other = np.clip(np.where(want == np.clip(np.floor(t), 0, 3), np.ceil(t), np.floor(t)), 0, 3)
            ok = near & (qg == other)
            assert ok[off].all(), ("code off", int((off & ~ok).sum()))
            n_code += int(off.sum())
        tot_code += off.size
    return n_par, n_code, tot_par, tot_code
