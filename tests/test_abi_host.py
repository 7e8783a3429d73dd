"""Host-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments before touching a GPU (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", f) for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h")]


@pytest.fixture(scope="module")
def B():
    from paper_2410_23537_amd import binding
    return binding


def _declared_functions():
    text = "\n".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(alise_[a-z0-9_]+)\s*\(", text)))


def test_exports_match_header(B):
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(B):
    for code, name in [(0, "ALISE_OK"), (1, "ALISE_INVALID_ARGUMENT"), (2, "ALISE_UNSUPPORTED"),
                       (3, "ALISE_WORKSPACE_TOO_SMALL"), (4, "ALISE_MISALIGNED"), (5, "ALISE_HIP_ERROR")]:
        assert B.alise_status_string(code) == name
    assert B.alise_status_string(99) == "ALISE_UNKNOWN_STATUS"


def _cache(B, **kw):
    base = dict(k_codes=0x1000, v_codes=0x2000, k_meta=0x3000, v_meta=0x4000, num_pages=10, page_size=16,
                num_kv_heads=8, head_dim=128, bits=8, group_size=64)
    base.update(kw)
    return B.alise_kv_cache(**base)


def test_layout_helpers(B):
    lib = B.raw()
    c = _cache(B)
    assert lib.alise_kv_codes_bytes(ctypes.byref(c)) == 10 * 8 * 16 * 128
    assert lib.alise_kv_meta_bytes(ctypes.byref(c)) == 10 * 8 * 16 * 2 * 4
    c4 = _cache(B, bits=4, group_size=32)
    assert lib.alise_kv_codes_bytes(ctypes.byref(c4)) == 10 * 8 * 16 * 64
    assert lib.alise_kv_meta_bytes(ctypes.byref(c4)) == 10 * 8 * 16 * 4 * 4
    assert lib.alise_kv_codes_bytes(ctypes.byref(_cache(B, bits=5))) == 0
    # interleaved blocks [K codes | V codes | K meta | V meta]: span from the base to the end of the last slab
    blk = 2 * 16 * 128 + 2 * 16 * 2 * 4
    ci = _cache(B, codes_block_stride=blk, meta_block_stride=blk)
    assert lib.alise_kv_codes_bytes(ctypes.byref(ci)) == (10 * 8 - 1) * blk + 16 * 128
    assert lib.alise_kv_meta_bytes(ctypes.byref(ci)) == (10 * 8 - 1) * blk + 16 * 2 * 4


@pytest.mark.parametrize("kw,want", [
    (dict(bits=3), 2), (dict(bits=16), 2), (dict(head_dim=96), 2), (dict(group_size=48), 2),
    (dict(group_size=8), 2), (dict(bits=4, group_size=16), 2), (dict(page_size=12), 2),
    (dict(page_size=4), 2), (dict(page_size=512), 2), (dict(num_pages=0), 1), (dict(num_kv_heads=-1), 1),
    (dict(num_pages=1 << 28, page_size=16), 2),
    (dict(k_codes=0), 1), (dict(v_meta=0), 1), (dict(k_codes=0x1008), 4),
    (dict(codes_block_stride=16 * 128 - 16), 1), (dict(codes_block_stride=16 * 128 + 8), 1),
    (dict(meta_block_stride=64), 1), (dict(codes_block_stride=1 << 31), 2),
    (dict(num_pages=1 << 24, num_kv_heads=128, page_size=8), 2),
])
def test_bad_cache_is_rejected_by_every_entry_point(B, kw, want):
    lib = B.raw()
    c = _cache(B, **kw)
    assert lib.alise_kv_quant_write(ctypes.byref(c), 0x10000, 0x20000, 0x30000, 4, None) == want
    assert lib.alise_kv_dequant_page(ctypes.byref(c), 0, 0x10000, 0x20000, None) == want
    assert lib.alise_paged_decode_attn(ctypes.byref(c), 0x10000, 0x20000, 0x30000, 16, 0x40000, 2, 8, 256,
                                       0.1, 0x50000, 1 << 30, None) == want


def test_quant_write_arguments(B):
    lib = B.raw()
    c = _cache(B)
    assert lib.alise_kv_quant_write(None, 0x10000, 0x20000, 0x30000, 4, None) == 1
    assert lib.alise_kv_quant_write(ctypes.byref(c), 0x10000, 0x20000, 0x30000, -1, None) == 1
    assert lib.alise_kv_quant_write(ctypes.byref(c), 0, 0, 0, 0, None) == 0          # T = 0: no-op
    assert lib.alise_kv_quant_write(ctypes.byref(c), 0, 0x20000, 0x30000, 4, None) == 1
    assert lib.alise_kv_quant_write(ctypes.byref(c), 0x10000, 0x20000, 0, 4, None) == 1
    assert lib.alise_kv_quant_write(ctypes.byref(c), 0x10004, 0x20000, 0x30000, 4, None) == 4
    assert lib.alise_kv_quant_write(ctypes.byref(c), 0x10000, 0x20000, 0x30004, 4, None) == 4


def test_dequant_page_arguments(B):
    lib = B.raw()
    c = _cache(B)
    assert lib.alise_kv_dequant_page(ctypes.byref(c), -1, 0x10000, 0x20000, None) == 1
    assert lib.alise_kv_dequant_page(ctypes.byref(c), 10, 0x10000, 0x20000, None) == 1
    assert lib.alise_kv_dequant_page(ctypes.byref(c), 0, 0, 0x20000, None) == 1
    assert lib.alise_kv_dequant_page(ctypes.byref(c), 0, 0x10002, 0x20000, None) == 4


@pytest.mark.parametrize("entry", ["alise_paged_decode_attn", "alise_paged_decode_attn_planned"])
def test_attention_arguments(B, entry):
    lib = B.raw()
    c = _cache(B)
    f = getattr(lib, entry)
    ok = [ctypes.byref(c), 0x10000, 0x20000, 0x30000, 16, 0x40000, 2, 8, 256, 0.1, 0x50000, 1 << 30, None]

    def call(**kw):
        names = ["c", "q", "out", "bt", "mb", "lens", "B", "H", "maxlen", "scale", "ws", "wsb", "stream"]
        a = list(ok)
        for k, v in kw.items():
            a[names.index(k)] = v
        return f(*a)

    assert call(B=0) == 0                      # empty batch: nothing to do, nothing launched
    assert call(B=-1) == 1
    assert call(H=0) == 1
    assert call(H=12) == 2                     # not a multiple of the 8 KV heads
    assert call(maxlen=-5) == 1
    assert call(mb=0) == 1
    assert call(mb=15) == 1                    # 15 pages of 16 cannot hold 256 tokens
    assert call(scale=0.0) == 1
    assert call(scale=float("nan")) == 1
    assert call(q=0) == 1
    assert call(out=0) == 1
    assert call(bt=0) == 1
    assert call(lens=0) == 1
    assert call(ws=0) == 1
    assert call(q=0x10008) == 4
    assert call(bt=0x30002) == 4
    assert call(ws=0x50010) == 4
    need = lib.alise_paged_decode_attn_workspace_bytes(ctypes.byref(c), 2, 8, 256)
    assert need > 0 and need % 256 == 0
    assert call(wsb=need - 1) == 3
    assert lib.alise_paged_decode_attn_workspace_bytes(ctypes.byref(c), 2, 12, 256) == 0
    # the workspace grows with the batch; with the longest context only as far as the cache's capacity allows
    assert lib.alise_paged_decode_attn_workspace_bytes(ctypes.byref(c), 64, 8, 256) > need
    assert lib.alise_paged_decode_attn_workspace_bytes(ctypes.byref(c), 2, 8, 1 << 16) >= need


def _workspace_model(num_pages, P, Hkv, H, D, B_, max_len, gqa):
    """The documented size of the attention workspace, restated: tiles = min(B ceil(max_len / split),
    B + capacity / split) at the largest split (2048 tokens, at most 128 pages, 64 on the matrix-core path), at least
    the small-batch allowance B + 2 * min_items / items_per_tile, never more than the same bound at 256 tokens."""
    up = lambda v: (v + 255) // 256 * 256
    C = min(2048, (64 if gqa else 128) * P)
    C_min = min(256, C)
    cap = num_pages * P
    bound = lambda c: min(B_ * max(1, -(-max_len // c)), B_ + cap // c)
    ipt = Hkv if gqa else H
    small = B_ + -(-2 * 256 * 8 * (1 if gqa else 4) // ipt)
    tiles = max(1, min(bound(C_min), max(bound(C), small)))
    return 256 + up(4 * (B_ + 1)) + up(4 * B_) + up(16 * tiles) + up(4 * tiles * H * (D + 2))


def test_attention_workspace_is_bounded_by_the_cache_capacity(B):
    lib = B.raw()
    size = lambda c, B_, H, L: lib.alise_paged_decode_attn_workspace_bytes(ctypes.byref(c), B_, H, L)
    # the INT4 stress configuration: 512 requests of up to 16384 tokens in a cache of 1.4 M tokens
    c5 = _cache(B, num_pages=87100, page_size=16, num_kv_heads=32, head_dim=128, bits=4, group_size=32)
    n5 = size(c5, 512, 32, 16384)
    assert n5 == _workspace_model(87100, 16, 32, 32, 128, 512, 16384, False)
    assert n5 < 25 << 20                             # 546 MB when it was sized by B * max_context_len
    # the grouped-query configuration (matrix-core path: items are KV heads)
    c4 = _cache(B, num_pages=16100, page_size=32, num_kv_heads=8, head_dim=128, bits=8, group_size=128)
    assert size(c4, 128, 64, 8192) == _workspace_model(16100, 32, 8, 64, 128, 128, 8192, True)
    # B = 512 at 128 K context in a cache that holds 2 M tokens: bounded by the capacity, not by 4.4 GB
    cl = _cache(B, num_pages=1 << 17, page_size=16, num_kv_heads=32, head_dim=128, bits=4, group_size=32)
    assert size(cl, 512, 32, 1 << 17) == _workspace_model(1 << 17, 16, 32, 32, 128, 512, 1 << 17, False) < 64 << 20
    # small caches and short contexts: B * ceil(max_len / split) is the smaller term
    c = _cache(B)
    assert size(c, 2, 8, 256) == _workspace_model(10, 16, 8, 8, 128, 2, 256, False)
    assert size(c, 2, 8, 100) == _workspace_model(10, 16, 8, 8, 128, 2, 100, False)


def test_static_scratch_entry_checks_sizes_before_any_hip_call(B):
    """The entry point without a workspace argument: same host checks, and a batch whose workspace would not fit the
    library's static array is refused (no GPU here: a status other than these would mean a HIP call was made)."""
    lib = B.raw()
    c = _cache(B)
    f = lambda c_=ctypes.byref(c), q=0x10000, out=0x20000, bt=0x30000, mb=1 << 12, lens=0x40000, B_=2, H=8, maxlen=256, \
        scale=0.1: lib.alise_paged_decode_attn_static(c_, q, out, bt, mb, lens, B_, H, maxlen, scale, None)
    assert f(B_=0) == 0
    assert f(B_=-1) == 1 and f(H=0) == 1 and f(H=12) == 2 and f(q=0) == 1 and f(lens=0) == 1 and f(q=0x10008) == 4
    assert f(mb=15) == 1 and f(scale=0.0) == 1
    limit = B.ALISE_STATIC_SCRATCH_BYTES
    assert limit == 32 << 20
    # sizes whose workspace exceeds the array: refused with ALISE_WORKSPACE_TOO_SMALL
    big = _cache(B, num_pages=1 << 20, num_kv_heads=8)
    assert lib.alise_paged_decode_attn_workspace_bytes(ctypes.byref(big), 4096, 64, 1 << 14) > limit
    assert f(c_=ctypes.byref(big), B_=4096, H=64, maxlen=1 << 14) == 3
    assert lib.alise_paged_decode_attn_workspace_bytes(ctypes.byref(c), 2, 8, 256) <= limit


def test_attention_plan_arguments(B):
    lib = B.raw()
    c = _cache(B)
    need = lib.alise_paged_decode_attn_workspace_bytes(ctypes.byref(c), 2, 8, 256)
    f = lambda c_=ctypes.byref(c), lens=0x40000, B_=2, H=8, maxlen=256, ws=0x50000, wsb=need: \
        lib.alise_paged_decode_attn_plan(c_, lens, B_, H, maxlen, ws, wsb, None)
    assert f(B_=0) == 0
    assert f(B_=-1) == 1 and f(H=0) == 1 and f(maxlen=-1) == 1
    assert f(H=12) == 2
    assert f(lens=0) == 1 and f(ws=0) == 1
    assert f(lens=0x40002) == 4 and f(ws=0x50010) == 4
    assert f(wsb=need - 1) == 3
    assert f(c_=None) == 1
    nop = _cache(B)                                 # the plan looks at no cache pointer
    nop.k_codes = nop.v_codes = nop.k_meta = nop.v_meta = None
    assert f(c_=ctypes.byref(nop), B_=0) == 0


def test_swap_arguments(B):
    lib = B.raw()
    c = _cache(B)                                   # 10 pages of 16 tokens, 8 heads, INT8, D=128, G=64
    blk = 2 * 16 * 128 + 2 * 16 * 2 * 4             # bytes of one (page, head) block
    assert lib.alise_kv_swap_bytes(ctypes.byref(c), 0) == 0
    assert lib.alise_kv_swap_bytes(ctypes.byref(c), 1) == 8 * blk
    assert lib.alise_kv_swap_bytes(ctypes.byref(c), 16) == 8 * blk
    assert lib.alise_kv_swap_bytes(ctypes.byref(c), 17) == 2 * 8 * blk
    assert lib.alise_kv_swap_bytes(ctypes.byref(_cache(B, bits=5)), 17) == 0
    need = 2 * 8 * blk
    for f in (lib.alise_kv_swap_out, lib.alise_kv_swap_in):
        assert f(None, 0x10000, 17, 0x20000, need, None) == 1
        assert f(ctypes.byref(c), 0x10000, -1, 0x20000, need, None) == 1
        assert f(ctypes.byref(c), 0x10000, 161, 0x20000, 1 << 30, None) == 1      # more tokens than the cache holds
        assert f(ctypes.byref(c), 0, 0, 0, 0, None) == 0                            # no tokens: no-op
        assert f(ctypes.byref(c), 0, 17, 0x20000, need, None) == 1
        assert f(ctypes.byref(c), 0x10000, 17, 0, need, None) == 1
        assert f(ctypes.byref(c), 0x10000, 17, 0x20000, need - 1, None) == 1        # buffer too small
        assert f(ctypes.byref(c), 0x10000, 17, 0x20008, need, None) == 4
        assert f(ctypes.byref(c), 0x10002, 17, 0x20000, need, None) == 4
        assert f(ctypes.byref(_cache(B, head_dim=96)), 0x10000, 17, 0x20000, need, None) == 2


def test_prefill_arguments(B):
    lib = B.raw()
    c = _cache(B)                                   # INT8, D=128, G=64, pages of 16: a shape the prefill kernel takes
    f = lib.alise_paged_prefill_attn
    ok = [ctypes.byref(c), 0x10000, 0x20000, 0x60000, 0x30000, 16, 0x40000, 2, 300, 8, 256, 0.1, 0x50000, 1 << 30, None]

    def call(**kw):
        names = ["c", "q", "out", "qs", "bt", "mb", "lens", "B", "tq", "H", "maxlen", "scale", "ws", "wsb", "stream"]
        a = list(ok)
        for k, v in kw.items():
            a[names.index(k)] = v
        return f(*a)

    need = lib.alise_paged_prefill_attn_workspace_bytes(ctypes.byref(c), 2, 300, 8, 256)
    assert need > 0 and need % 256 == 0
    assert call(B=0) == 0 and call(tq=0) == 0       # nothing to do, nothing launched
    assert call(B=-1) == 1 and call(tq=-1) == 1 and call(H=0) == 1 and call(maxlen=-1) == 1
    assert call(H=12) == 2                          # not a multiple of the 8 KV heads
    assert call(H=8 * 32, wsb=0) == 3               # more than 16 query heads per KV head: the single-query kernels, a larger workspace
    assert call(mb=0) == 1 and call(mb=15) == 1     # 15 pages of 16 cannot hold 256 tokens
    assert call(scale=0.0) == 1 and call(scale=float("nan")) == 1
    for name in ("q", "out", "qs", "bt", "lens", "ws"):
        assert call(**{name: 0}) == 1
    assert call(q=0x10008) == 4 and call(out=0x20004) == 4
    assert call(qs=0x60002) == 4 and call(bt=0x30002) == 4 and call(lens=0x40001) == 4
    assert call(ws=0x50010) == 4
    assert call(wsb=need - 1) == 3
    # layouts without a matrix-core kernel run on the single-query kernels: one block-table row per query token
    # (300 rows of 256 / page_size entries) in front of that call's own workspace
    for kw in (dict(head_dim=64), dict(group_size=32), dict(page_size=8)):
        other = _cache(B, **kw)
        n = lib.alise_paged_prefill_attn_workspace_bytes(ctypes.byref(other), 2, 300, 8, 256)
        P = kw.get("page_size", 16)
        inner = lib.alise_paged_decode_attn_workspace_bytes(ctypes.byref(_cache(B, num_pages=1 << 20, **kw)), 300, 8, 256)
        assert n == 1280 + (300 * (256 // P) * 4 + 255) // 256 * 256 + inner and n % 256 == 0
        assert call(c=ctypes.byref(other), mb=256 // P, wsb=n - 1) == 3
    for g in (32, 64, 128):                             # INT4 is taken with groups of 32, 64 and 128
        c4 = _cache(B, bits=4, group_size=g)
        assert 0 < lib.alise_paged_prefill_attn_workspace_bytes(ctypes.byref(c4), 2, 300, 8, 256) < 8192


def test_fused_op_arguments(B):
    lib = B.raw()
    A = 0x1000          # any 16-byte aligned, non-null address: the checks below fail before a pointer is used
    ln = lambda x=A, res=A, g=A, b=A, eps=1e-5, h=A + 64, y=A + 128, rows=4, hidden=64: lib.alise_add_layernorm(
        x, res, g, b, eps, h, y, rows, hidden, None)
    assert ln(x=None) == B.ALISE_INVALID_ARGUMENT
    assert ln(g=None) == B.ALISE_INVALID_ARGUMENT
    assert ln(b=None) == B.ALISE_INVALID_ARGUMENT
    assert ln(y=None) == B.ALISE_INVALID_ARGUMENT
    assert ln(rows=-1) == B.ALISE_INVALID_ARGUMENT
    assert ln(eps=-1.0) == B.ALISE_INVALID_ARGUMENT
    assert ln(eps=float("nan")) == B.ALISE_INVALID_ARGUMENT
    assert ln(eps=float("inf")) == B.ALISE_INVALID_ARGUMENT
    assert ln(h=A + 128) == B.ALISE_INVALID_ARGUMENT            # h_out and y_out the same buffer
    for hidden in (0, 4, 12, 16392, 1 << 20):
        assert ln(hidden=hidden) == B.ALISE_UNSUPPORTED
    assert ln(x=A + 2) == B.ALISE_MISALIGNED
    assert ln(res=A + 8) == B.ALISE_MISALIGNED
    assert ln(y=A + 130) == B.ALISE_MISALIGNED
    assert ln(rows=0) == B.ALISE_OK                               # nothing to do, nothing launched
    assert ln(rows=0, res=None, h=None) == B.ALISE_OK

    relu = lambda x=A, b=A, y=A, rows=4, cols=64: lib.alise_bias_relu(x, b, y, rows, cols, None)
    assert relu(x=None) == B.ALISE_INVALID_ARGUMENT
    assert relu(y=None) == B.ALISE_INVALID_ARGUMENT
    assert relu(rows=-3) == B.ALISE_INVALID_ARGUMENT
    for cols in (0, 7, 20):
        assert relu(cols=cols) == B.ALISE_UNSUPPORTED
    assert relu(b=A + 4) == B.ALISE_MISALIGNED
    assert relu(rows=0) == B.ALISE_OK
    assert relu(rows=0, b=None) == B.ALISE_OK

    probe = lambda src=A, n=4096, out=A: lib.alise_hbm_read_probe(src, n, out, None)
    assert probe(out=None) == B.ALISE_INVALID_ARGUMENT
    assert probe(src=None) == B.ALISE_INVALID_ARGUMENT
    for n in (8, 17, 4100):
        assert probe(n=n) == B.ALISE_UNSUPPORTED                  # whole 16-byte units only
    assert probe(src=A + 8) == B.ALISE_MISALIGNED
    assert probe(out=A + 2) == B.ALISE_MISALIGNED

    issue = lambda mode=3, iters=10, sink=A: lib.alise_issue_overlap_probe(mode, iters, sink, None)
    assert issue(sink=None) == B.ALISE_INVALID_ARGUMENT
    assert issue(iters=-1) == B.ALISE_INVALID_ARGUMENT and issue(iters=(1 << 24) + 1) == B.ALISE_INVALID_ARGUMENT
    assert issue(mode=0) == B.ALISE_UNSUPPORTED and issue(mode=4) == B.ALISE_UNSUPPORTED
    assert issue(sink=A + 2) == B.ALISE_MISALIGNED


def test_build_names_the_compiler_the_kernels_were_validated_with():
    """The hand-placed wait states of the kernels were validated with one compiler; the build warns about any other."""
    import warnings
    from paper_2410_23537_amd import build
    banner = build.compiler_banner()
    assert "clang version" in banner
    with warnings.catch_warnings(record=True) as seen:
        warnings.simplefilter("always")
        ok = build.check_compiler()
    assert ok == banner.startswith(build.VALIDATED_COMPILER)
    assert ok == (not any("validated" in str(w.message) for w in seen))


def test_bench_reports_traffic_only_for_the_sources_it_was_measured_with(tmp_path, monkeypatch):
    """bench.py takes roofline.traffic from the rocprofv3 summary of the workload, which names the hash of the attention
    sources the counters were taken with: a summary of other sources, or none, gives null and a note."""
    import bench
    now = bench.attention_sources_sha256()
    assert len(now) == 16 and int(now, 16) >= 0
    monkeypatch.setattr(bench, "PROFILES", str(tmp_path))
    assert bench.measured_traffic("int4")[0] is None                            # no summary at all
    (tmp_path / "attention_step_int4.md").write_text(f"# x\ntraffic_bytes_per_launch: 7191314368\nattention_sources_sha256: {now}\n")
    got, note = bench.measured_traffic("int4")
    assert got == 7191314368 and now in note
    (tmp_path / "attention_step_int4.md").write_text("# x\ntraffic_bytes_per_launch: 7191314368\nattention_sources_sha256: 0123456789abcdef\n")
    got, note = bench.measured_traffic("int4")
    assert got is None and "profile again" in note
    (tmp_path / "attention_step_int4.md").write_text("# a summary without the two lines\n")
    assert bench.measured_traffic("int4")[0] is None


def test_committed_profiles_match_the_committed_sources():
    """The summaries under profiles/ were taken with the attention sources as they are committed: bench.py will
    report their traffic figures."""
    import bench
    for name in ("int4", "llama7b", "gqa70b", "opt13b"):
        got, note = bench.measured_traffic(name)
        assert got is not None and got > 0, note


def test_replay_arguments(B):
    """alise_replay.h: everything that can be wrong with the configuration is found before any HIP call."""
    lib = B.raw()
    c = _cache(B)
    sc = B.alise_sched_config(3, 4, 6, 0, 1000, 5000, 2, 1, 20)
    h = ctypes.c_void_p()

    def create(cache=c, sched=sc, **kw):
        f = dict(num_q_heads=8, max_context=64, max_iter_tokens=128, overlap_swaps=1, softmax_scale=0.088, reserved=0)
        f.update(kw)
        rc = B.alise_replay_config(**f)
        return lib.alise_replay_create(ctypes.byref(cache) if cache is not None else None,
                                       ctypes.byref(sched) if sched is not None else None, ctypes.byref(rc), None, ctypes.byref(h))

    assert create(cache=None) == B.ALISE_INVALID_ARGUMENT
    assert create(sched=None) == B.ALISE_INVALID_ARGUMENT
    assert create(num_q_heads=0) == B.ALISE_INVALID_ARGUMENT
    assert create(num_q_heads=12) == B.ALISE_INVALID_ARGUMENT           # not a multiple of the 8 KV heads
    assert create(max_context=1) == B.ALISE_INVALID_ARGUMENT
    assert create(max_iter_tokens=0) == B.ALISE_INVALID_ARGUMENT
    assert create(softmax_scale=0.0) == B.ALISE_INVALID_ARGUMENT
    assert create(reserved=1) == B.ALISE_INVALID_ARGUMENT
    assert create(cache=_cache(B, bits=5)) == B.ALISE_UNSUPPORTED
    assert create(sched=B.alise_sched_config(3, 0, 6, 0, 1000, 5000, 2, 1, 20)) == B.ALISE_INVALID_ARGUMENT
    assert create(sched=B.alise_sched_config(0, 4, 6, 0, 1000, 5000, 2, 1, 20)) == B.ALISE_INVALID_ARGUMENT   # the scheduler's own check
    assert h.value is None
    # NULL objects
    lib.alise_replay_destroy(None)
    assert lib.alise_replay_num_jobs(None) == 0
    assert lib.alise_replay_synchronize(None) == B.ALISE_INVALID_ARGUMENT
    assert lib.alise_replay_commit(None, 0, None, 0) == B.ALISE_INVALID_ARGUMENT
    assert lib.alise_replay_add_job(None, 0, 0, 4, 4, 0) == B.ALISE_INVALID_ARGUMENT
    assert lib.alise_replay_get_stats(None, None) == B.ALISE_INVALID_ARGUMENT
    assert lib.alise_replay_iterate(None, None, None, None, None, None) == B.ALISE_INVALID_ARGUMENT
