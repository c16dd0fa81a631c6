"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments before touching a device (no GPU needed: validation happens first)."""
import ctypes
import os
import re

import pytest

import paper_2603_14224_amd as sik

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "sik.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sik_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = sik.lib()
    names = header_symbols()
    assert set(names) == set(sik.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_strerror():
    assert sik.lib().sik_version() >= 100
    for code in range(0, -10, -1):
        assert sik.sik_strerror(code) not in ("", "unknown status")
    assert sik.sik_strerror(-99) == "unknown status"


def L(**kw):
    base = dict(batch=1, n_kv_heads=8, n_q_heads=32, head_dim=128, max_len=4096, kv_dtype=sik.SIK_BF16)
    base.update(kw)
    return sik.make_layout(**base)


def test_workspace_bytes_and_layout_validation():
    assert sik.sik_workspace_bytes(L(), 256) > 0
    assert sik.sik_workspace_bytes(L(), 256) % 256 == 0
    assert sik.sik_workspace_bytes(L(batch=32), 256) > sik.sik_workspace_bytes(L(), 256)
    for bad in (L(head_dim=96), L(n_q_heads=30), L(batch=0), L(max_len=0), L(kv_dtype=sik.SIK_F32),
                L(out_dtype=sik.SIK_F16), L(n_kv_heads=1, n_q_heads=65536)):  # head counts are 16-bit kernel fields
        assert sik.sik_workspace_bytes(bad, 16) == 0
    assert sik.sik_workspace_bytes(L(), 5000) == 0  # k > max_len


FAKE = ctypes.c_void_p(256 * 1000)  # never dereferenced: validation fails first


def test_argument_errors_are_reported_before_any_launch():
    lib = sik.lib()
    lay = L()
    ref = ctypes.byref(lay)
    assert lib.sik_score(ref, None, FAKE, FAKE, FAKE, FAKE, None) == -1
    assert lib.sik_score(ctypes.byref(L(head_dim=64)), FAKE, FAKE, FAKE, FAKE, FAKE, None) == -2
    assert lib.sik_score(ctypes.byref(L(kv_dtype=2)), FAKE, FAKE, FAKE, FAKE, FAKE, None) == -3
    assert lib.sik_topk(ref, FAKE, FAKE, 0, FAKE, FAKE, 1 << 30, None) == -4
    assert lib.sik_topk(ref, FAKE, FAKE, 4097, FAKE, FAKE, 1 << 30, None) == -4
    assert lib.sik_topk(ref, FAKE, FAKE, 16, FAKE, None, 1 << 30, None) == -6
    assert lib.sik_topk(ref, FAKE, FAKE, 16, FAKE, FAKE, 64, None) == -6
    assert lib.sik_topk(ref, FAKE, FAKE, 16, FAKE, ctypes.c_void_p(256 * 1000 + 8), 1 << 30, None) == -6
    assert lib.sik_sparse_attn(ref, FAKE, FAKE, None, FAKE, 16, 0.0, FAKE, FAKE, 1 << 30, None) == -1
    assert lib.sik_sparse_attn(ref, FAKE, FAKE, FAKE, FAKE, 16, 0.0, FAKE, FAKE, 10, None) == -6
    assert lib.sik_quantize_keys(ref, FAKE, FAKE, 0, 1, 7, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == -8
    assert lib.sik_quantize_keys(ref, FAKE, FAKE, 4000, 200, sik.SIK_Q_ENCODE, FAKE, None, None, FAKE, None, 0, None) == -5
    assert lib.sik_quantize_keys(ref, FAKE, FAKE, -1, 2, sik.SIK_Q_ENCODE, FAKE, None, None, FAKE, None, 0, None) == -5
    assert lib.sik_quantize_keys(ref, FAKE, FAKE, 0, 0, sik.SIK_Q_FIT, FAKE, None, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert lib.sik_decode_step(ref, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 16, 0.0, FAKE, None,
                               FAKE, 1 << 30, None) == -1  # k_new without v_new
    assert lib.sik_decode_step(ref, FAKE, None, None, FAKE, FAKE, FAKE, None, FAKE, FAKE, 0, 0.0, FAKE, None,
                               FAKE, 1 << 30, None) == -4
    assert lib.sik_decode_step(None, FAKE, None, None, FAKE, FAKE, FAKE, None, FAKE, FAKE, 4, 0.0, FAKE, None,
                               FAKE, 1 << 30, None) == -1


def test_argument_block_and_workspace_calls_validate_on_the_host():
    lib = sik.lib()
    lay = L()
    ref = ctypes.byref(lay)
    f = FAKE.value
    base = dict(q=f, K=f, V=f, seq_len=f, mu=f, codebook=f, codes=f, k=16, out=f, workspace=f,
                workspace_bytes=1 << 30)

    def call(**kw):
        a = sik.DecodeArgs(**{**base, **kw})
        return lib.sik_decode_step_ex(ref, ctypes.byref(a))

    assert lib.sik_decode_step_ex(ref, None) == -1
    assert call(launches=4) == -8 and call(launches=-1) == -8 and call(spin_limit=-5) == -8
    assert call(q=None, launches=1) == -1
    assert call(k=0, launches=3) == -4
    assert call(k_per_mille=1001) == -4
    assert call(n_forced=4) == -1                       # a forced set without its indices
    assert call(n_forced=200, forced_idx=f) == -2       # more than 128 forced tokens
    assert call(n_forced=16, forced_idx=f, k=16) == -4  # the budget counts the forced tokens
    assert call(forced_K=f, forced_V=f, n_forced=4, forced_idx=f) == -8   # side rows go with the 2-bit cache
    assert call(K=None, V=None, kvq=f) == -1            # records without alpha
    assert call(workspace_bytes=64, launches=1) == -6
    # workspace initialisation and status
    assert lib.sik_workspace_init(ref, 16, None, 1 << 30, None) == -6
    assert lib.sik_workspace_init(ref, 16, FAKE, 64, None) == -6
    assert lib.sik_workspace_init(ref, 5000, FAKE, 1 << 30, None) == -4
    st = ctypes.c_uint32(0)
    assert lib.sik_workspace_status(None, None, ctypes.byref(st)) == -1
    assert lib.sik_workspace_status(FAKE, None, None) == -1
    # prefill compression
    assert lib.sik_prefill_compress(ref, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert lib.sik_prefill_compress(ref, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 64, None) == -6
    assert lib.sik_prefill_compress(ctypes.byref(L(head_dim=64)), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                    FAKE, 1 << 30, None) == -2
    # the entry point on the built-in buffer rejects what does not fit before touching a device
    big = L(batch=32, max_len=16384)
    assert lib.sik_decode_step_static(ctypes.byref(big), FAKE, None, None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 512, 0.0,
                                      FAKE, None, None) == -9


def test_binding_raises_on_error_status():
    import torch
    lay = L()
    with pytest.raises(sik.SikError):
        sik.sik_topk(lay, torch.zeros(4), torch.zeros(1, dtype=torch.int32), 0, torch.zeros(4, dtype=torch.int32),
                     torch.zeros(256, dtype=torch.uint8))


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: any other --gpus exits with a message before anything touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_chunk_plans_stay_inside_their_limits():
    """Every layout the header admits is cut into at most 64 chunks of at most 64512 tokens per head (the
    published histogram counts are 16 bits wide and the forced-token bitmap has one bit per token of a chunk);
    anything else is SIK_ERR_SHAPE from every entry point, and sik_workspace_bytes returns 0."""
    max_len = 4128768
    seen_big = False
    for batch in (1, 2, 7, 64, 512):
        for hkv, hq in ((1, 1), (1, 4), (8, 32), (8, 64), (2, 24)):
            if batch * hq > (1 << 20):
                continue
            for ml in (1, 1000, 4096, 65535, 65536, 66000, 131072, 524288, 524289, 1 << 20, 1 << 21, 4000000, max_len):
                lay = L(batch=batch, n_kv_heads=hkv, n_q_heads=hq, max_len=ml)
                info = sik.sik_plan_info(lay)
                s_n, s_ch, nhb, h_n, h_ch, f_n, f_ch = info[:7]
                assert 1 <= s_n <= 64 and 1024 <= s_ch <= 64512 and s_ch % 1024 == 0 and s_n * s_ch >= ml
                assert nhb == (hq // hkv + 3) // 4
                assert 1 <= h_n <= 64 and h_ch <= 64512 and h_n * h_ch >= ml
                assert (f_n == 0) == (ml > 524288) and (f_n == 0 or (f_n * f_ch >= ml and f_n <= 64))
                seen_big |= s_ch > 32768
                if sik.sik_workspace_bytes(lay, 1) == 0:           # only the sheer size may stop it
                    assert batch * hq * ml > 1 << 36
    assert seen_big
    # one 131072-token chunk used to be planned here (64 x 8 KV heads of 32 query heads): now three chunks
    assert sik.sik_plan_info(L(batch=64, max_len=131072))[:2] == [3, 64512]
    assert sik.sik_plan_info(L(batch=16, n_kv_heads=1, n_q_heads=32, max_len=131072))[3:5] == [3, 64512]
    too_long = L(max_len=max_len + 1)
    with pytest.raises(sik.SikError) as e:
        sik.sik_plan_info(too_long)
    assert e.value.status == -2
    assert sik.sik_workspace_bytes(too_long, 16) == 0
    assert sik.lib().sik_score(ctypes.byref(too_long), FAKE, FAKE, FAKE, FAKE, FAKE, None) == -2
    assert sik.lib().sik_topk(ctypes.byref(too_long), FAKE, FAKE, 16, FAKE, FAKE, 1 << 40, None) == -2
