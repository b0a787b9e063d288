"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects
bad arguments before touching the GPU (no compute calls here)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "optgqa.h")


@pytest.fixture(scope="module")
def G():
    import paper_2505_02351_amd as G
    if not os.path.exists(G.LIB_PATH):
        from paper_2505_02351_amd import build
        build.build()
    G.load_library()
    return G


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(optgqa_[a-z_]+)\s*\(", text)))


def test_exports_every_declared_symbol(G):
    lib = G.load_library()
    names = declared_symbols()
    assert {"optgqa_reshape_and_cache", "optgqa_paged_attention", "optgqa_paged_prefill"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_status_strings(G):
    assert G.abi_version() >= 1
    assert G.status_string(0) == "ok"
    for code in range(-6, 0):
        assert G.status_string(code) not in ("ok", "unknown status")
    assert G.status_string(-99) == "unknown status"


def test_argument_errors_before_any_launch(G):
    lib = G.load_library()
    one = ctypes.c_void_p(16)       # non-null, aligned, never dereferenced: every call below fails first
    # reshape_and_cache
    f = lib.optgqa_reshape_and_cache
    assert f(one, one, one, one, one, -1, 2, 64, 16, 128, 128, 0, None) == -2
    assert f(one, one, one, one, one, 4, 2, 48, 16, 96, 96, 0, None) == -3          # head_dim
    assert f(one, one, one, one, one, 4, 2, 64, 12, 128, 128, 0, None) == -3         # block_size
    assert f(one, one, one, one, one, 4, 2, 64, 16, 100, 128, 0, None) == -2         # stride < row
    assert f(one, one, one, one, one, 4, 2, 64, 16, 128, 128, 7, None) == -3         # dtype
    assert f(None, one, one, one, one, 4, 2, 64, 16, 128, 128, 0, None) == -1
    assert f(None, None, None, None, None, 0, 2, 64, 16, 128, 128, 0, None) == 0     # no tokens: no-op
    # paged_attention
    g = lib.optgqa_paged_attention
    base = dict(scale=0.125, B=2, Hq=8, Hkv=2, D=64, bs=16, MB=8, Lmax=128, P=0)

    def call(out=one, q=one, kc=one, vc=one, bt=one, cl=one, ws=None, wsb=0, dt=0, **kw):
        a = dict(base, **kw)
        return g(out, q, kc, vc, bt, cl, None, a["scale"], a["B"], a["Hq"], a["Hkv"], a["D"], a["bs"],
                 a["MB"], a["Lmax"], a["P"], ws, wsb, dt, None)

    assert call(Hq=7) == -2                      # Hq % Hkv
    assert call(D=96) == -3
    assert call(bs=8, Lmax=64) == -3
    assert call(Lmax=129) == -2                  # exceeds the table row
    assert call(P=24) == -2                      # not a multiple of block_size / 16
    assert call(P=48, bs=32, MB=4) == -2
    assert call(q=None) == -1
    assert call(out=ctypes.c_void_p(8)) == -3    # misaligned
    assert call(P=32) == -4                      # split forced, no workspace
    assert call(P=-2) == -4 and call(P=-2, D=128) == -4      # the equal-work split needs its workspace
    assert call(B=0) == 0
    assert call(dt=2) == -3
    # prefill
    h = lib.optgqa_paged_prefill
    assert h(one, one, one, one, one, one, None, None, 0.1, 2, 8, 2, 64, 16, 8, 4, 0, None) == -1
    assert h(one, one, one, one, one, one, one, None, 0.1, 2, 8, 3, 64, 16, 8, 4, 0, None) == -2
    assert h(one, one, one, one, one, one, one, None, 0.1, 2, 8, 2, 64, 16, 8, 0, 0, None) == 0
    # gather
    k = lib.optgqa_gather_kv
    assert k(one, one, one, one, one, None, 2, 2, 64, 16, 8, 128, 0, None) == -1
    assert k(one, one, one, one, one, one, 2, 2, 32, 16, 8, 128, 0, None) == -3


def test_more_entry_points_reject_bad_arguments_before_any_launch(G):
    import ctypes
    import numpy as np
    lib = G.load_library()
    one = ctypes.c_void_p(16)
    # decode step: strides shorter than a token row, missing new rows
    d = lib.optgqa_decode_step
    args = lambda k_new=one, ks=128, D=64: (one, one, k_new, one, one, one, one, one, None, 0.1, 2, 8, 2, D, 16, 8, 128,
                                           ks, 128, None, 0, 0, None)
    assert d(*args(ks=64)) == -2
    assert d(*args(k_new=None)) == -1
    assert d(*args(D=96)) == -3
    # 8-bit caches: scales must be positive and finite, head_dim 64 or 128, workspace required
    a = lib.optgqa_paged_attention_fp8
    f = lambda ks=1.0, vs=1.0, D=128, ws=None, wsb=0: a(one, one, one, one, one, one, None, 0.1, ks, vs, 2, 8, 2, D, 16,
                                                        8, 128, ws, wsb, 0, None)
    assert f(ks=0.0) == -2 and f(vs=-1.0) == -2 and f(ks=float("inf")) == -2 and f(ks=float("nan")) == -2
    assert f(D=96) == -3
    assert f() == -4 and f(D=64) == -4
    r = lib.optgqa_reshape_and_cache_fp8
    g = lambda k=one, ks=1.0, stride=256, T=3: r(k, one, one, one, one, T, 2, 128, 16, stride, 256, ks, 1.0, 1, None)
    assert g(ks=0.0) == -2 and g(stride=100) == -2 and g(stride=260) == -3 and g(k=ctypes.c_void_p(8)) == -3
    assert g(T=0) == 0
    sf = lib.optgqa_decode_step_fp8
    h = lambda ks=1.0, D=128, kn=one, st=256, ws=None: sf(one, one, kn, one, one, one, one, one, None, 0.1, ks, 1.0, 2, 8, 2,
                                                          D, 16, 8, 128, st, 256, ws, 0, 0, None)
    assert h(ks=0.0) == -2 and h(D=96) == -3 and h(kn=None) == -1 and h(st=100) == -2 and h() == -4 and h(D=64) == -4
    pf = lib.optgqa_paged_prefill_fp8
    e = lambda ks=1.0, D=128, B=2, cu=one: pf(one, one, one, one, one, one, cu, None, 0.1, ks, 1.0, B, 8, 2, D, 16, 8,
                                             32, 0, None)
    assert e(ks=0.0) == -2 and e(D=96) == -3 and e(cu=None) == -1 and e(B=0) == 0
    # sliding window: positive windows only, decode needs the workspace
    wa = lib.optgqa_paged_attention_window
    f = lambda W=8, D=128: wa(one, one, one, one, one, one, None, 0.1, W, 2, 8, 2, D, 16, 8, 128, None, 0, 0, None)
    assert f(W=0) == -2 and f(W=-5) == -2 and f(D=96) == -3 and f() == -4 and f(D=64) == -4
    wsx = lib.optgqa_decode_step_window
    f = lambda W=8, D=128, ks=256: wsx(one, one, one, one, one, one, one, one, None, 0.1, W, 2, 8, 2, D, 16, 8, 128, ks,
                                       256, None, 0, 0, None)
    assert f(W=0) == -2 and f(D=96) == -3 and f(ks=100) == -2 and f() == -4
    wp = lib.optgqa_paged_prefill_window
    f = lambda W=8, D=128, B=2, cu=one: wp(one, one, one, one, one, one, cu, None, 0.1, W, B, 8, 2, D, 16, 8, 32, 0, None)
    assert f(W=0) == -2 and f(D=96) == -3 and f(cu=None) == -1 and f(B=0) == 0
    # whole-prompt prefill: strides, both caches or neither, head_dim 128 only
    pp = lib.optgqa_prompt_prefill
    f = lambda kc=None, vc=None, D=128, ks=256, cu=one, B=2, bt=None, L=32: pp(
        one, one, one, one, kc, vc, bt, cu, None, 0.1, B, 8, 2, D, 16, 8, L, ks, 256, 0, None)
    assert f(ks=100) == -2 and f(ks=260) == -3 and f(D=96) == -3 and f(cu=None) == -1 and f(B=0) == 0
    assert f(kc=one) == -1                                   # one cache without the other
    assert f(kc=one, vc=one) == -1                           # caches without block tables
    assert f(kc=one, vc=one, bt=one, L=8 * 16 + 1) == -2     # prompts longer than the tables can address
    # one-call prefill step: new rows and caches both required, strides checked like the prompt call's
    ps = lib.optgqa_prefill_step
    f = lambda kn=one, kc=one, D=128, ks=256, vs=256, cu=one, B=2, mq=4, scale=0.1: ps(
        one, one, kn, one, kc, one, one, one, cu, None, scale, B, 8, 2, D, 16, 8, mq, ks, vs, 0, None)
    assert f(kn=None) == -1 and f(kc=None) == -1 and f(cu=None) == -1
    assert f(ks=100) == -2 and f(ks=260) == -3 and f(vs=(1 << 30) + 8) == -2 and f(D=96) == -3
    assert f(scale=float("nan")) == -2 and f(kn=ctypes.c_void_p(18)) == -3
    assert f(B=0) == 0 and f(mq=0) == 0
    pp = lib.optgqa_prompt_prefill
    assert pp(one, one, one, one, None, None, None, one, None, 0.1, 2, 8, 2, 128, 16, 8, 32, (1 << 30) + 8, 256, 0,
              None) == -2
    # streaming probe: the host copy of the tile list is checked against the pool size
    p = lib.optgqa_stream_probe
    lst = np.array([0, 1, 2, 3, 4, 5, 6, 7], np.int32)
    h = lst.ctypes.data_as(ctypes.c_void_p)
    lst[5] = 8                                                              # one piece past the pool
    assert p(one, one, 8 * 4096, one, h, 1, 2, one, None) == -6
    assert p(one, one, 8 * 4096, one, None, 1, 2, one, None) == -1
    assert p(one, one, 100, one, h, 1, 2, one, None) == -2
    # kernel-event hook: both or neither
    assert lib.optgqa_set_kernel_events(one, None) == -1
    assert lib.optgqa_set_kernel_events(None, None) == 0


def test_workspace_query(G):
    # fixed partitions at head_dim 128: two slots per partition of every (sequence, KV head) segment,
    # 8 heads x (128 + 2) floats each, after 4 + 1 plan entries padded to 4
    n, P = G.paged_attention_workspace_bytes(4, 64, 8, 128, 16, 32768, 512)
    assert P == 512 and n == (8 + 2 * 4 * 8 * 64 * 8 * (128 + 2)) * 4
    # ... the same at head_dim 64 with (64 + 2) floats per head
    n, P = G.paged_attention_workspace_bytes(4, 64, 8, 64, 16, 32768, 512)
    assert P == 512 and n == (8 + 2 * 4 * 8 * 64 * 8 * (64 + 2)) * 4
    n, P = G.paged_attention_workspace_bytes(1, 8, 2, 64, 16, 128, 0)
    assert (n, P) == (0, 0)                      # short context: no split
    # head_dim 128 and worth splitting: the equal-work split, one slot per wave (one wave per SIMD
    # of 256 CUs) plus one per (sequence, KV head), each slot 8 heads x (128 + 2) floats, after
    # 64 + 1 plan entries padded to 4
    n, P = G.paged_attention_workspace_bytes(64, 32, 4, 128, 32, 8192, 0)
    slots = 256 * 2 * 4 + 64 * 4                 # sized for two workgroups per CU (the 8-bit cache path)
    assert P == G.SPLIT_BALANCED and n == (68 + slots * 8 * (128 + 2)) * 4
    assert G.paged_attention_workspace_bytes(64, 32, 4, 128, 32, 8192, G.SPLIT_BALANCED) == (n, P)
    # small problems get fewer waves: 2 x 2 segments x 13 tiles -> 52 tiles -> 2 workgroups
    n, P = G.paged_attention_workspace_bytes(2, 8, 2, 128, 16, 200, G.SPLIT_BALANCED)
    assert P == G.SPLIT_BALANCED and n == (4 + (2 * 4 + 4) * 4 * (128 + 2)) * 4
    # head_dim 64: the same split, (64 + 2) floats per head
    n, P = G.paged_attention_workspace_bytes(64, 32, 4, 64, 32, 8192, 0)
    assert P == G.SPLIT_BALANCED and n == (68 + slots * 8 * (64 + 2)) * 4
    assert G.paged_attention_workspace_bytes(64, 32, 4, 64, 32, 8192, G.SPLIT_BALANCED) == (n, P)
    n, P = G.paged_attention_workspace_bytes(64, 32, 4, 128, 32, 8192, -1)
    assert (n, P) == (0, 0)


def test_validate_tables_host(G):
    bt = np.array([[3, 1, -1], [0, 2, 4]], np.int32)
    assert G.validate_tables_host(bt, np.array([20, 48], np.int32), 16, 5) == 0
    assert G.validate_tables_host(bt, np.array([33, 48], np.int32), 16, 5) == -6    # reads the -1
    assert G.validate_tables_host(bt, np.array([20, 48], np.int32), 16, 4) == -6    # id 4 >= 4
    assert G.validate_tables_host(bt, np.array([20, 49], np.int32), 16, 5) == -6    # too long
    assert G.validate_tables_host(bt, np.array([0, 0], np.int32), 16, 5) == 0


def test_missing_library_fails_loudly():
    """No CPU or PyTorch fallback: without the built library the binding raises at load time."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import sys; sys.path.insert(0, %r); import paper_2505_02351_amd as G\n"
            "try:\n    G.load_library('/nonexistent/liboptgqa.so')\n"
            "except ImportError as e:\n    print('raised:', e); sys.exit(7)\n"
            "sys.exit(0)\n" % root)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode == 7 and "is missing" in r.stdout, (r.returncode, r.stdout, r.stderr[-300:])


def test_static_scratch_entry_point_refuses_what_does_not_fit(G):
    """optgqa_paged_attention_static: a shape whose split needs more than the static array is
    refused on the host (no GPU call is made before that decision)."""
    lib = G.load_library()
    one = ctypes.c_void_p(16)
    n, chosen = G.paged_attention_workspace_bytes(500, 32, 2, 128, 16, 4096, 0)
    assert chosen != 0 and n > G.STATIC_SCRATCH_BYTES
    rc = lib.optgqa_paged_attention_static(one, one, one, one, one, one, None, 0.1, 500, 32, 2, 128, 16, 256, 4096,
                                           1, None)
    assert rc == -4
    header = open(HEADER).read()
    m = re.search(r"#define OPTGQA_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", header)
    assert m and int(m.group(1)) << int(m.group(2)) == G.STATIC_SCRATCH_BYTES


def test_binding_refuses_wrong_element_types_and_host_tensors(G):
    """The binding hands raw pointers to the library, so it must refuse - before any pointer is
    taken or anything is launched - index tensors of torch's default int64, slopes that are not
    float32, caches of another 2-byte type than q, and tensors that are not in GPU memory."""
    import torch
    q = torch.zeros(2, 8, 64, dtype=torch.float16)
    out = torch.empty_like(q)
    c = torch.zeros(4, 2, 16, 64, dtype=torch.float16)
    c8 = torch.zeros(4, 2, 16, 64, dtype=torch.uint8)
    bt = torch.zeros(2, 2, dtype=torch.int32)
    cl = torch.ones(2, dtype=torch.int32)
    cu = torch.tensor([0, 1, 2], dtype=torch.int32)
    sl = torch.ones(8, dtype=torch.float32)
    slots = torch.zeros(2, dtype=torch.int64)
    kv = torch.zeros(2, 2, 64, dtype=torch.float16)
    ws = torch.zeros(1024, dtype=torch.float32)

    def refused(exc, fn, *args):
        with pytest.raises(exc):
            fn(*args)

    # element types (checked first, so these need no GPU)
    refused(TypeError, G.paged_attention, out, q, c, c, bt.long(), cl, sl, 0.1, 32)
    refused(TypeError, G.paged_attention, out, q, c, c, bt, cl.long(), sl, 0.1, 32)
    refused(TypeError, G.paged_attention, out, q, c, c, bt, cl, sl.double(), 0.1, 32)
    refused(TypeError, G.paged_attention, out, q, c.bfloat16(), c, bt, cl, sl, 0.1, 32)
    refused(TypeError, G.paged_attention, out.bfloat16(), q, c, c, bt, cl, sl, 0.1, 32)
    refused(TypeError, G.paged_attention, out.float(), q.float(), c.float(), c.float(), bt, cl, sl, 0.1, 32)
    refused(TypeError, G.paged_attention_static, out, q, c, c, bt.long(), cl, sl, 0.1, 32)
    refused(TypeError, G.reshape_and_cache, kv, kv, c, c, slots.int())
    refused(TypeError, G.reshape_and_cache, kv.bfloat16(), kv.bfloat16(), c, c, slots)
    refused(TypeError, G.reshape_and_cache_fp8, kv, kv, c, c, slots, 1.0, 1.0)          # caches must be uint8
    refused(TypeError, G.decode_step, out, q, kv.bfloat16(), kv, c, c, bt, cl, sl, 0.1, 32, None)
    refused(TypeError, G.decode_step_fp8, out, q, kv, kv, c, c, bt, cl, sl, 0.1, 1.0, 1.0, 32, ws)
    refused(TypeError, G.paged_attention_fp8, out, q, c8, c8, bt.long(), cl, sl, 0.1, 1.0, 1.0, 32, ws)
    refused(TypeError, G.paged_prefill, out, q, c, c, bt, cl, cu.long(), sl, 0.1, 1)
    refused(TypeError, G.paged_prefill_fp8, out, q, c, c, bt, cl, cu, sl, 0.1, 1.0, 1.0, 1)
    refused(TypeError, G.paged_attention_window, out, q, c, c, bt, cl.short(), sl, 0.1, 4, 32, ws)
    refused(TypeError, G.decode_step_window, out, q, kv, kv, c, c.bfloat16(), bt, cl, sl, 0.1, 4, 32, ws)
    refused(TypeError, G.paged_prefill_window, out, q, c, c, bt.long(), cl, cu, sl, 0.1, 4, 1)
    refused(TypeError, G.prompt_prefill, out, q, kv, kv, None, None, None, cu.long(), sl, 0.1, 2)
    refused(TypeError, G.prefill_step, out, q, kv, kv, c, c, bt, cl.long(), cu, sl, 0.1, 1)
    refused(TypeError, G.prefill_step, out, q, kv.bfloat16(), kv, c, c, bt, cl, cu, sl, 0.1, 1)
    refused(TypeError, G.gather_kv, torch.zeros(2, 32, 2, 64, dtype=torch.bfloat16),
            torch.zeros(2, 32, 2, 64, dtype=torch.bfloat16), c, c, bt, cl)
    # correctly typed tensors in host memory
    refused(ValueError, G.paged_attention, out, q, c, c, bt, cl, sl, 0.1, 32)
    refused(ValueError, G.reshape_and_cache, kv, kv, c, c, slots)
    refused(ValueError, G.decode_step, out, q, kv, kv, c, c, bt, cl, sl, 0.1, 32, None)
    refused(ValueError, G.paged_prefill, out, q, c, c, bt, cl, cu, sl, 0.1, 1)
    refused(ValueError, G.prompt_prefill, out, q, kv, kv, None, None, None, cu, sl, 0.1, 2)
    refused(ValueError, G.prefill_step, out, q, kv, kv, c, c, bt, cl, cu, sl, 0.1, 1)


def test_non_finite_scale_is_refused(G):
    lib = G.load_library()
    one = ctypes.c_void_p(16)
    for bad in (float("nan"), float("inf"), -float("inf")):
        assert lib.optgqa_paged_attention(one, one, one, one, one, one, None, bad, 2, 8, 2, 64, 16, 8, 128, 0, None, 0,
                                          0, None) == -2
        assert lib.optgqa_paged_prefill(one, one, one, one, one, one, one, None, bad, 2, 8, 2, 128, 16, 8, 4, 0,
                                        None) == -2
        assert lib.optgqa_prompt_prefill(one, one, one, one, None, None, None, one, None, bad, 2, 8, 2, 128, 16, 8, 4,
                                         256, 256, 0, None) == -2


def test_shared_prefix_host_checks(G):
    """Bundle size, workspace size and the host validator of the shared-prefix entry points, and their
    argument errors (nothing here reaches the GPU)."""
    lib = G.load_library()
    one = ctypes.c_void_p(16)
    assert G.shared_prefix_bundle(32, 4, 128) == 2          # group 8
    assert G.shared_prefix_bundle(32, 8, 128) == 4          # group 4
    assert G.shared_prefix_bundle(8, 8, 128) == 16          # multi-head
    assert G.shared_prefix_bundle(12, 2, 128) == 2          # group 6: 12 of the 16 columns
    assert G.shared_prefix_bundle(40, 2, 128) == 1          # group 20 -> 10 heads per pass
    assert lib.optgqa_shared_prefix_bundle(32, 5, 128) == -2
    assert lib.optgqa_shared_prefix_bundle(32, 4, 64) == 2 and lib.optgqa_shared_prefix_bundle(32, 4, 96) == -3
    plain, _ = G.paged_attention_workspace_bytes(64, 32, 4, 128, 32, 8192, G.SPLIT_BALANCED)
    shared = G.shared_prefix_workspace_bytes(64, 32, 4, 128, 32, 8192)
    assert shared > plain > 0                               # twice the segments, 16 columns per slot
    assert 0 < G.shared_prefix_workspace_bytes(64, 32, 4, 64, 32, 8192) < shared
    assert G.shared_prefix_workspace_bytes(64, 32, 4, 96, 32, 8192) == 0
    # entry points: head_dim 96, missing workspace, missing table
    f = lib.optgqa_paged_attention_shared
    args = lambda D=128, sb=one, ws=one, wsb=1 << 30: (one, one, one, one, one, one, sb, None, 0.1, 2, 8, 2, D, 16, 8, 128,
                                                       ws, wsb, 0, None)
    assert f(*args(D=96)) == -3
    assert f(*args(sb=None)) == -1
    assert f(*args(ws=None, wsb=0)) == -4
    g = lib.optgqa_decode_step_shared
    assert g(one, one, one, one, one, one, one, one, None, None, 0.1, 2, 8, 2, 128, 16, 8, 128, 256, 256, one, 1 << 30,
             0, None) == -1
    # validator: two bundles of two, block size 4
    bt = np.array([[5, 6, 7, 8], [5, 6, 9, 10], [1, 2, 3, 4], [1, 11, 12, 13]], np.int32)
    cl = np.array([14, 13, 16, 9], np.int32)
    ok = np.array([0, 2, 0, 1], np.int32)
    v = lambda sb, new=1, bundle=2, lens=cl: G.validate_shared_prefix_host(bt, lens, np.asarray(sb, np.int32), 4, bundle, new)
    assert v(ok) == 0
    assert v([0, 3, 0, 1]) == -6                  # third block differs from the leader's
    assert v([1, 2, 0, 1]) == -6                  # a leader cannot share
    assert v([0, 2, 0, 3]) == -6                  # 3 blocks = 12 tokens > 9 - 1 cached
    assert v([0, 2, 0, 2]) == -6                  # second block differs
    assert v([0, -1, 0, 0]) == -6
    assert v([0, 0, 0, 0]) == 0
    assert v(ok, lens=np.array([14, 8, 16, 9], np.int32)) == -6      # 2 blocks = 8 tokens > 8 - 1 cached
    assert v(ok, new=0, lens=np.array([14, 8, 16, 9], np.int32)) == 0
    assert v(ok, bundle=4) == -6                  # sequence 3 would then share with sequence 0
    assert lib.optgqa_validate_shared_prefix_host(None, None, None, 0, 4, 4, 2, 1) == 0
    assert lib.optgqa_validate_shared_prefix_host(None, one, one, 2, 4, 4, 2, 1) == -1
    assert lib.optgqa_validate_shared_prefix_host(one, one, one, 2, 4, 4, 0, 1) == -2


def test_per_head_scale_entry_points_reject_missing_arrays(G):
    lib = G.load_library()
    one = ctypes.c_void_p(16)
    assert lib.optgqa_reshape_and_cache_fp8_heads(one, one, one, one, one, 4, 2, 128, 16, 256, 256, None, one, 0,
                                                  None) == -1
    assert lib.optgqa_reshape_and_cache_fp8_heads(one, one, one, one, one, 4, 2, 48, 16, 96, 96, one, one, 0,
                                                  None) == -3
    assert lib.optgqa_paged_attention_fp8_heads(one, one, one, one, one, one, None, 0.1, one, None, 2, 8, 2, 128, 16,
                                                8, 128, one, 1 << 30, 0, None) == -1
    assert lib.optgqa_paged_attention_fp8_heads(one, one, one, one, one, one, None, 0.1, one, one, 2, 8, 2, 96, 16,
                                                8, 128, one, 1 << 30, 0, None) == -3          # head_dim 96
    assert lib.optgqa_paged_attention_fp8_heads(one, one, one, one, one, one, None, 0.1, one, one, 2, 8, 2, 128, 16,
                                                8, 128, None, 0, 0, None) == -4               # workspace required
    assert lib.optgqa_decode_step_fp8_heads(one, one, one, one, one, one, one, one, None, 0.1, None, None, 2, 8, 2,
                                            128, 16, 8, 128, 256, 256, one, 1 << 30, 0, None) == -1
    assert lib.optgqa_paged_prefill_fp8_heads(one, one, one, one, one, one, one, None, 0.1, None, one, 2, 8, 2, 128,
                                              16, 8, 4, 0, None) == -1
    assert lib.optgqa_paged_prefill_fp8_heads(one, one, one, one, one, one, one, None, 0.1, one, one, 2, 8, 2, 96,
                                              16, 8, 4, 0, None) == -3
