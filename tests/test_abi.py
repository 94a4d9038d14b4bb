"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and its host
logic (budget rules, validation, error codes) behaves as include/thrift.h says.  No kernel runs."""
import ctypes as C
import os
import re

import pytest

from paper_2605_23081_amd import binding as T

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "thrift.h")).read()
    declared = set(re.findall(r"\b(thrift_[a-z0-9_]+)\s*\(", header))
    assert declared == set(T.EXPORTS), declared ^ set(T.EXPORTS)
    L = T.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_host_budget_helpers_match_the_oracle(oracle):
    for vis in (0, 1, 19, 20, 21, 64, 2048):
        for f in (0.0, 1e-7, 0.01, 0.05, 0.1, 0.25, 0.999999, 1.0):
            assert T.row_budget(vis, f) == oracle.row_k(vis, f)
        assert T.row_budget(vis, 0.5, fixed_k=7) == oracle.row_k(vis, 0.5, 7)
    for Bq, Bk, Tk in ((64, 64, 32), (128, 64, 64), (1, 64, 16)):
        for i in range(0, 16):
            assert T.visible_blocks(i, Tk, Bq, Bk, True) == oracle.visible_blocks(i, Tk, Bq, Bk, True)
    assert T.visible_blocks(0, 2048, 1, 64, True, 131071) == 2048
    for n, f in ((32, 0.05), (512, 0.05), (2048, 0.25)):
        assert T.budget_to_global_k(n, f) == oracle.paper_global_k(n, f)
    assert T.select_kmax(32, 32, 64, 64, True, 0.05) == 2
    assert T.select_kmax(1024, 2048, 128, 64, True, 0.05) == 103
    assert T.select_kmax(8, 8, 64, 64, False, 0.0, fixed_k=3) == 3


def test_validation_errors_come_before_any_launch():
    L = T.lib()
    fake = C.c_void_p(0x1000)   # never dereferenced: every call below must fail validation first
    NULL, SHAPE, DTYPE, BUDGET, WORKSPACE = 1, 2, 3, 4, 5
    assert L.thrift_block_means(None, 0, 1, 1, 64, 128, 64, fake, None) == NULL
    assert L.thrift_block_means(fake, 0, 1, 1, 64, 64, 64, fake, None) == SHAPE      # D != 128
    assert L.thrift_block_means(fake, 0, 1, 1, 100, 128, 0, fake, None) == SHAPE     # block < 1
    assert L.thrift_block_means(fake, 0, 1, 1, 0, 128, 64, fake, None) == SHAPE      # empty sequence
    assert L.thrift_block_means(fake, 7, 1, 1, 64, 128, 64, fake, None) == DTYPE
    assert L.thrift_block_means(fake, 2, 1, 1, 64, 128, 64, fake, None) == DTYPE     # fp32 is output-only
    assert L.thrift_quantize_mxfp4(fake, 0, 1, 1, 0, 128, 1, fake, fake, None) == SHAPE    # empty sequence
    assert L.thrift_quantize_mxfp4(fake, 0, 1, 1, 64, 128, 2, fake, fake, None) == SHAPE
    sel = lambda **kw: L.thrift_select_topk(fake, fake, 1, kw.get("Hq", 4), kw.get("Hkv", 2), 8, kw.get("Tk", 8), 128, 64, 64, 1,
                                            C.c_double(kw.get("budget", 0.05)), kw.get("fixed_k", -1), 0, fake, fake,
                                            kw.get("kmax", 8), None)
    assert sel(Hq=3) == SHAPE
    assert sel(Tk=5000) == SHAPE
    assert sel(budget=1.5) == BUDGET
    assert sel(budget=-0.1) == BUDGET
    assert sel(budget=1.0, kmax=4) == BUDGET           # kmax too small for a 100 % budget
    pre = lambda **kw: L.thrift_attn_prefill(fake, fake, fake, kw.get("dt", 0), fake, fake, fake, fake, fake, fake, fake, fake, 4,
                                             1, 4, kw.get("Hkv", 2), kw.get("N", 256), kw.get("D", 128), kw.get("Bq", 64),
                                             kw.get("Bk", 64), 1, C.c_float(0.0), kw.get("out", fake), kw.get("odt", 0), None,
                                             None, 0, None)
    assert pre(Bq=32) == SHAPE and pre(Bk=128) == SHAPE and pre(D=64) == SHAPE and pre(N=0) == SHAPE and pre(Hkv=3) == SHAPE
    assert pre(out=None) == NULL
    assert pre(odt=5) == DTYPE and pre(dt=2) == DTYPE
    dec = lambda **kw: L.thrift_attn_decode(fake, 0, fake, fake, fake, fake, fake, fake, fake, None, 1, 4, 2, kw.get("N", 1024), 128, 64,
                                            C.c_double(kw.get("budget", 0.05)), -1, kw.get("split", 8), C.c_float(0.0), fake, 0,
                                            None, None, 0, kw.get("ws", fake), kw.get("wsb", 1 << 30), None)
    assert dec(split=0) == SHAPE and dec(N=1000) == SHAPE
    assert dec(budget=2.0) == BUDGET
    assert dec(ws=None) == WORKSPACE and dec(wsb=16) == WORKSPACE
    app = lambda **kw: L.thrift_kv_cache_append(kw.get("k", fake), fake, kw.get("dt", 0), kw.get("n", 1), kw.get("sl", fake), None,
                                                fake, fake, fake, fake, fake, fake, fake, 1, 2, kw.get("N", 1024), kw.get("D", 128),
                                                kw.get("Bk", 64), None)
    assert app(k=None) == NULL and app(sl=None) == NULL
    assert app(n=0) == SHAPE and app(n=2000) == SHAPE and app(N=1000) == SHAPE and app(D=64) == SHAPE and app(Bk=32) == SHAPE
    assert app(dt=2) == DTYPE
    fwd = lambda **kw: L.thrift_attention_forward(kw.get("q", fake), fake, fake, kw.get("dt", 1), 1, 4, kw.get("Hkv", 2), kw.get("N", 300),
                                                  kw.get("D", 128), kw.get("Bq", 128), 64, 1, C.c_double(kw.get("budget", 0.05)), -1, 0,
                                                  C.c_float(0.0), fake, 1, None, kw.get("ws", fake), kw.get("wsb", 16), None)
    assert fwd(q=None) == NULL and fwd(dt=2) == DTYPE and fwd(Hkv=3) == SHAPE and fwd(N=0) == SHAPE and fwd(Bq=32) == SHAPE
    assert fwd(budget=1.5) == BUDGET and fwd(ws=None) == WORKSPACE and fwd(wsb=16) == WORKSPACE
    # an unknown tile order is refused before the first stage of the chain is enqueued (it reaches only the last stage)
    assert L.thrift_attention_forward(fake, fake, fake, 1, 1, 4, 2, 300, 128, 128, 64, 1, C.c_double(0.05), -1, 7, C.c_float(0.0),
                                      fake, 1, None, fake, 1 << 30, None) == SHAPE
    # the entry point without a workspace argument: sizes are checked against its static array first
    sta = lambda **kw: L.thrift_attn_decode_static(fake, 0, fake, fake, fake, fake, fake, fake, fake, None, kw.get("B", 1), 4, 2,
                                                   kw.get("N", 1024), 128, 64, C.c_double(0.05), -1, kw.get("split", 8), C.c_float(0.0),
                                                   fake, 0, None, None, 0, None)
    assert sta(split=0) == SHAPE and sta(N=1000) == SHAPE
    assert sta(B=4096, N=131072, split=256) == WORKSPACE
    wsq = L.thrift_attention_forward_workspace
    assert wsq(1, 4, 2, 300, 128, 128, 64, 1, C.c_double(0.05), -1) > 300 * 128 * 6 // 2
    assert wsq(1, 4, 2, 300, 64, 128, 64, 1, C.c_double(0.05), -1) == 0 and wsq(1, 4, 2, 300, 128, 128, 64, 1, C.c_double(-1.0), -1) == 0
    need = T.decode_workspace_bytes(16, 32, 8, 131072, 128, 64, 256)
    assert 0 < need < (64 << 20)
    assert T.decode_workspace_bytes(16, 32, 8, 131072, 64, 64, 256) == 0
    assert "gfx950" in T.status_string(6)


def test_peak_probe_validates_before_launching():
    L = T.lib()
    fake, work = C.c_void_p(0x1000), C.c_double(0.0)
    probe = lambda kind=4, dt=1, iters=10, buf=fake, size=1 << 30: L.thrift_peak_probe(kind, dt, iters, buf, C.c_size_t(size), C.byref(work), None)
    assert probe(buf=None) == 1
    assert probe(kind=5) == 2 and probe(kind=-1) == 2
    assert probe(iters=0) == 2
    assert probe(size=(16 << 20) - 1) == 2                 # smaller than the probes' result region
    assert probe(buf=C.c_void_p(0x1008)) == 2              # not 16-byte aligned
    assert probe(kind=1, dt=2) == 3                        # the 16-bit MFMA probe needs fp16 or bf16
    assert L.thrift_peak_probe(4, 1, 10, fake, C.c_size_t(1 << 30), None, None) == 1


def test_without_a_gpu_valid_calls_fail_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    fake = C.c_void_p(0x1000)
    assert T.lib().thrift_block_means(fake, 0, 1, 1, 64, 128, 64, fake, None) == 6   # THRIFT_ERR_ARCH, nothing launched


def test_spill_check_reads_the_compiler_listing():
    """The build refuses a fused kernel whose listing touches scratch memory inside a loop (and only then)."""
    from paper_2605_23081_amd.build import scratch_in_loops
    listing = "\n".join([
        "_ZN6thrift4walkEv:",
        "; %bb.0:",
        "\tscratch_store_dword off, v1, off offset:16 ; 4-byte Folded Spill",          # before the loop: fine
        ".LBB0_1:                                ; =>This Inner Loop Header: Depth=1",
        "\tv_add_f32_e32 v0, v0, v1",
        "; %bb.2:                                ;   in Loop: Header=BB0_1 Depth=1",
        "\ts_cbranch_scc1 .LBB0_1",
        ".LBB0_3:",
        "\tscratch_load_dword v1, off, off offset:16 ; 4-byte Folded Reload",           # after it: fine
        "\ts_endpgm",
        "_ZN6thrift3badEv:",
        ".LBB1_1:                                ; =>This Inner Loop Header: Depth=1",
        "; %bb.2:                                ;   in Loop: Header=BB1_1 Depth=1",
        "\tscratch_load_dword v1, off, off ; 4-byte Folded Reload",
        "\ts_cbranch_scc1 .LBB1_1",
        "\ts_endpgm",
    ])
    assert scratch_in_loops(listing) == ["_ZN6thrift3badEv"]
    # a persistent kernel's outermost loop runs over work items: a reload at an item's start is outside the walk, one in
    # a nested loop (whose header line names the parent first and itself on the comment line below) is inside it
    def persistent(name, reload_in_walk):
        return "\n".join([
            name + ":",
            ".LBB2_1:                                ; =>This Loop Header: Depth=1",
            "\tscratch_load_dword v1, off, off offset:8 ; 4-byte Folded Reload",
            ".LBB2_2:                                ;   Parent Loop BB2_1 Depth=1",
            "                                        ; =>  This Inner Loop Header: Depth=2",
            "\tscratch_load_dword v2, off, off ; 4-byte Folded Reload" if reload_in_walk else "\tv_add_f32_e32 v0, v0, v1",
            "\ts_cbranch_scc1 .LBB2_2",
            "; %bb.3:                                ;   in Loop: Header=BB2_1 Depth=1",
            "\ts_cbranch_scc1 .LBB2_1",
            "\ts_endpgm",
        ])
    assert scratch_in_loops(persistent("_ZN6thrift17persistent_kernelEv", False)) == []
    assert scratch_in_loops(persistent("_ZN6thrift17persistent_kernelEv", True)) == ["_ZN6thrift17persistent_kernelEv"]
    assert scratch_in_loops(persistent("_ZN6thrift5otherEv", False)) == ["_ZN6thrift5otherEv"]


def test_listing_checks_refuse_a_format_they_cannot_read():
    """A listing without the labels the checks rely on must not pass for clean."""
    from paper_2605_23081_amd.build import m0_outside_inline_asm, scratch_in_loops
    for text in ("", "kernel_without_mangled_name:\n\tscratch_load_dword v1, off, off\n\ts_endpgm",
                 "_ZN6thrift4walkEv:\n\tv_add_f32_e32 v0, v0, v1\n\ts_endpgm"):          # no basic blocks, no loop annotation
        with pytest.raises(RuntimeError):
            scratch_in_loops(text)
    with pytest.raises(RuntimeError):
        m0_outside_inline_asm("\ts_mov_b32 m0, s10\n\tglobal_load_lds_dwordx4 v1, s[2:3]")   # no inline-assembly markers


def test_m0_check_reads_the_compiler_listing():
    from paper_2605_23081_amd.build import m0_outside_inline_asm
    ok = "\n".join(["\t;;#ASMSTART", "\ts_mov_b32 m0, s10", "\ts_nop 0", "\tglobal_load_lds_dwordx4 v1, s[2:3]", "\t;;#ASMEND",
                    "\tv_add_u32_e32 v0, v1, v2", "; a comment that mentions m0"])
    assert m0_outside_inline_asm(ok) == 0
    assert m0_outside_inline_asm(ok + "\n\ts_mov_b32 m0, -1\n\tds_gws_init v0 gds") == 1
