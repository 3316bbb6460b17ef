"""Host-side checks that need no GPU: the library loads, exports what the header declares, and
rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2512_12131_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "lrboost.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lr_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), f"{n} declared in lrboost.h but not exported"
    assert set(names) == set(B.EXPORTS), "binding and header disagree on the entry points"
    assert lib.lr_version() >= 100


def test_binding_constants_equal_the_headers():
    """Every enumerator and numeric #define of the header that the binding also names has the header's value."""
    text = open(os.path.join(ROOT, "include", "lrboost.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    header = {}
    for body in re.findall(r"typedef\s+enum\s*\{(.*?)\}", text, flags=re.S):
        nxt = 0
        for item in body.split(","):
            item = item.strip()
            if not item:
                continue
            m = re.match(r"(LR_[A-Z0-9_]+)\s*(?:=\s*(-?\d+))?$", item)
            assert m, item
            nxt = int(m.group(2)) if m.group(2) is not None else nxt
            header[m.group(1)] = nxt
            nxt += 1
    for name, val in re.findall(r"#define\s+(LR_[A-Z0-9_]+)\s+\(?(\d+)u?\)?\s*$", text, flags=re.M):
        header[name] = int(val)
    shared = [n for n in header if hasattr(B, n)]
    assert {"LR_BF16", "LR_ACT_SILU", "LR_NORM_ONLINE", "LR_NORM_SHARD_LOCAL", "LR_NORM_ONLINE_GATHER",
            "LR_TAG_ATTN_FWD", "LR_TAG_ATTN_BWD"} <= set(shared), sorted(shared)
    for n in shared:
        assert getattr(B, n) == header[n], (n, getattr(B, n), header[n])


def test_status_strings():
    lib = B.lib()
    for code in (0, -1, -2, -3, -4, -5):
        assert lib.lr_status_string(code).decode().startswith("LR_")
    assert b"unknown" in lib.lr_status_string(-99)


def test_argument_errors_are_detected_on_the_host():
    lib = B.lib()
    fake = C.c_void_p(0x1000)          # 16-byte aligned, never dereferenced on these paths
    odd = C.c_void_p(0x1002)
    null = C.c_void_p(0)
    f = lib.lr_linear_fwd
    # null pointer
    assert f(null, 64, fake, fake, fake, fake, 64, 8, 64, 16, 64, 1, 1, fake, 1 << 20, None) == -1
    # unknown dtype / activation
    assert f(fake, 64, fake, fake, fake, fake, 64, 8, 64, 16, 64, 1, 7, fake, 1 << 20, None) == -1
    assert f(fake, 64, fake, fake, fake, fake, 64, 8, 64, 16, 64, 9, 1, fake, 1 << 20, None) == -1
    # leading dimension smaller than the row
    assert f(fake, 32, fake, fake, fake, fake, 64, 8, 64, 16, 64, 1, 1, fake, 1 << 20, None) == -1
    # bf16 sizes must be multiples of 8, pointers 16-byte aligned
    assert f(fake, 64, fake, fake, fake, fake, 64, 8, 64, 12, 64, 1, 1, fake, 1 << 20, None) == -4
    assert f(odd, 64, fake, fake, fake, fake, 64, 8, 64, 16, 64, 1, 1, fake, 1 << 20, None) == -4
    # workspace too small / missing
    need = lib.lr_linear_workspace_bytes(8, 64, 16, 64, 1, 0)
    assert need > 0
    assert f(fake, 64, fake, fake, fake, fake, 64, 8, 64, 16, 64, 1, 1, fake, need - 1, None) == -3
    assert f(fake, 64, fake, fake, fake, fake, 64, 8, 64, 16, 64, 1, 1, null, 0, None) == -3
    # T = 0 is a valid no-op
    assert f(fake, 64, fake, fake, fake, fake, 64, 0, 64, 16, 64, 1, 1, null, 0, None) == 0
    # attention: sizes the kernels cannot address (32-bit byte offsets inside one batch element), other head
    # sizes and non-causal masks are refused before anything is launched
    a = lib.lr_attention_fwd
    assert a(fake, fake, fake, fake, fake, 4096, 1, 1 << 20, 32, 128, 1, 1, None) == -2
    assert a(fake, fake, fake, fake, fake, 2048, 1, 128, 32, 64, 1, 1, None) == -2
    assert a(fake, fake, fake, fake, fake, 4096, 1, 128, 32, 128, 0, 1, None) == -2
    assert a(fake, fake, fake, fake, null, 4096, 1, 128, 32, 128, 1, 1, None) == -1


def test_lax_entry_points_refuse_on_the_host():
    """The LaX block needs its struct and the identity gate; both are checked before any launch."""
    lib = B.lib()
    fake = C.c_void_p(0x1000)
    desc_id = B.make_block_desc(1, 128, 128, 1, 128, 256, 256, 32, act=B.LR_ACT_IDENTITY)
    desc_silu = B.make_block_desc(1, 128, 128, 1, 128, 256, 256, 32, act=B.LR_ACT_SILU)
    ps = B.BlockParams(*[fake] * len(B.PARAM_NAMES))
    ck = B.BlockCkpt(*[fake] * 6)
    lx = B.BlockLax(*[C.c_void_p(0)] * 12)
    odd = B.BlockLax(*([C.c_void_p(0x1002)] + [C.c_void_p(0)] * 11))
    f = lib.lr_block_lax_fwd
    assert f(C.byref(desc_id), C.byref(ps), fake, fake, C.byref(ck), None, fake, 1 << 30, None) == -1
    assert f(C.byref(desc_silu), C.byref(ps), fake, fake, C.byref(ck), C.byref(lx), fake, 1 << 30, None) == -2
    assert f(C.byref(desc_id), C.byref(ps), fake, fake, C.byref(ck), C.byref(odd), fake, 1 << 30, None) == -4
    assert f(C.byref(desc_id), C.byref(ps), fake, fake, C.byref(ck), C.byref(lx), fake, 16, None) == -3


def test_rope_arguments_are_checked_on_the_host():
    lib = B.lib()
    fake, null, odd = C.c_void_p(0x1000), C.c_void_p(0), C.c_void_p(0x1004)
    f = lib.lr_rope
    assert f(fake, 128, fake, fake, 2, 16, 2, 128, 0, 1, None) == -1           # row shorter than the heads
    assert f(fake, 256, fake, fake, 2, 16, 2, 64, 0, 1, None) == -2            # other head sizes
    assert f(fake, 256, fake, fake, 2, 16, 2, 128, 0, 0, None) == -2           # fp32
    assert f(fake, 256, null, fake, 2, 16, 2, 128, 0, 1, None) == -1
    assert f(odd, 256, fake, fake, 2, 16, 2, 128, 0, 1, None) == -4
    assert f(fake, 256, fake, fake, 0, 16, 2, 128, 0, 1, None) == 0            # nothing to do
    # the block descriptor wants both tables or neither
    d = B.make_block_desc(1, 128, 128, 1, 128, 256, 256, 32)
    assert lib.lr_block_workspace_bytes(C.byref(d), 0) > 0
    d.rope_cos = 0x1000
    assert lib.lr_block_workspace_bytes(C.byref(d), 0) == 0


def test_gqa_attention_arguments_are_checked_on_the_host():
    lib = B.lib()
    fake, odd = C.c_void_p(0x1000), C.c_void_p(0x1004)
    f = lib.lr_attention_gqa_fwd
    # q, k, v, o, lse, ld, ldkv, B, S, H, Hkv, hd, causal, dt, stream
    assert f(fake, fake, fake, fake, fake, 512, 256, 1, 64, 4, 3, 128, 1, 1, None) == -1     # 3 does not divide 4
    assert f(fake, fake, fake, fake, fake, 512, 128, 1, 64, 4, 2, 128, 1, 1, None) == -1     # kv rows too short
    assert f(fake, fake, fake, fake, fake, 512, 256, 1, 64, 4, 0, 128, 1, 1, None) == -1
    assert f(fake, fake, fake, fake, fake, 512, 260, 1, 64, 4, 2, 128, 1, 1, None) == -4     # row stride not x8
    assert f(fake, odd, fake, fake, fake, 512, 256, 1, 64, 4, 2, 128, 1, 1, None) == -4
    assert f(fake, fake, fake, fake, fake, 512, 256, 1, 64, 4, 2, 64, 1, 1, None) == -2      # other head sizes
    assert f(fake, fake, fake, fake, fake, 512, 256, 1, 64, 4, 2, 128, 0, 1, None) == -2     # non-causal
    assert f(fake, fake, fake, fake, None, 512, 256, 1, 64, 4, 2, 128, 1, 1, None) == -1
    w = lib.lr_attention_gqa_bwd_workspace_bytes
    assert w(1, 64, 4, 3, 128) == 0 and w(1, 64, 4, 2, 64) == 0
    mha, gq = w(2, 256, 4, 4, 128), w(2, 256, 4, 2, 128)
    assert mha == lib.lr_attention_bwd_workspace_bytes(2, 256, 4, 128)
    assert gq == mha + 2 * (2 * 256) * (4 * 128) * 2          # one dK and one dV contribution per query head
    g = lib.lr_attention_gqa_bwd
    args = [fake] * 9 + [512, 256, 2, 256, 4, 2, 128, 1, 1]
    assert g(*args, fake, gq - 1, None) == -3                  # short workspace
    assert g(*args, None, gq, None) == -3


def test_block_descriptor_checks_the_kv_head_count():
    lib = B.lib()
    ok = B.make_block_desc(1, 128, 512, 4, 128, 256, 256, 32, n_kv_heads=2)
    mha = B.make_block_desc(1, 128, 512, 4, 128, 256, 256, 32)
    assert 0 < lib.lr_block_workspace_bytes(C.byref(ok), 1)
    assert lib.lr_block_workspace_bytes(C.byref(ok), 0) < lib.lr_block_workspace_bytes(C.byref(mha), 0)   # narrower k, v
    for bad in (3, 8, -1):
        d = B.make_block_desc(1, 128, 512, 4, 128, 256, 256, 32, n_kv_heads=bad)
        want_zero = bad > 0
        assert (lib.lr_block_workspace_bytes(C.byref(d), 0) == 0) == want_zero, bad


def test_mfma_probe_arguments_are_checked_on_the_host():
    f = B.lib().lr_mfma_probe
    tf = C.c_double(0.0)
    assert f(1, 100, 1, None, None) == -1            # nowhere to put the result
    assert f(1, 0, 1, C.byref(tf), None) == -1
    assert f(1, 100, 0, C.byref(tf), None) == -1
    assert f(1, (1 << 20) + 1, 1, C.byref(tf), None) == -1
    assert f(1, 100, 1001, C.byref(tf), None) == -1


def test_workspace_queries_scale_and_reject():
    lib = B.lib()
    a = lib.lr_group_workspace_bytes(3, 1024, 256, 64, 256, 1, 0)
    b = lib.lr_group_workspace_bytes(3, 2048, 256, 64, 256, 1, 0)
    assert 0 < a < b
    assert lib.lr_group_workspace_bytes(0, 1024, 256, 64, 256, 1, 0) == 0
    assert lib.lr_linear_workspace_bytes(16, 64, 16, 64, 5, 0) == 0
    d = B.make_block_desc(2, 256, 256, 2, 128, 344, 344, 64)
    assert lib.lr_block_workspace_bytes(C.byref(d), 0) > 0
    assert lib.lr_block_workspace_bytes(C.byref(d), 1) > lib.lr_block_workspace_bytes(C.byref(d), 0)
    assert lib.lr_block_ckpt_bytes(C.byref(d)) == 7 * 512 * 64 * 2 + 2 * 512 * 4
    bad = B.make_block_desc(2, 256, 256, 4, 128, 344, 344, 64)     # heads * head_dim != d_model
    assert lib.lr_block_workspace_bytes(C.byref(bad), 0) == 0
    f32 = B.make_block_desc(2, 256, 256, 2, 128, 344, 344, 64, dt=B.LR_F32)
    assert lib.lr_block_workspace_bytes(C.byref(f32), 0) == 0


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/liblrboost.so")
    with pytest.raises(B.LrError):
        B.lib()
