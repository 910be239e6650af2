"""CPU-side checks of the C-ABI library: it loads, exports what the header
declares, its integer plan equals the oracle's and a brute-force replay of
Alg. 2's IF, and malformed arguments come back as status codes before any
GPU work is attempted."""
import ctypes as C
import os
import re

import numpy as np
import pytest
import torch

from oracle import lococo_oracle as orc
from paper_2406_05317_amd import binding as lb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "lococo.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(lococo_[a-z_]+)\s*\(", hdr))
    assert declared == set(lb.EXPORTS), declared ^ set(lb.EXPORTS)
    L = lb.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert re.fullmatch(r"\d+\.\d+\.\d+", lb.lococo_version())


def test_struct_layouts_match_the_header():
    # sizes the C compiler gives for the header's structs (LP64, natural alignment)
    assert C.sizeof(lb.lococo_config) == 72
    assert C.sizeof(lb.lococo_cache) == 64
    assert C.sizeof(lb.lococo_tensor) == 32
    assert C.sizeof(lb.lococo_qkvo) == 128
    assert C.sizeof(lb.lococo_seg) == 32


def test_plan_is_bit_exact_against_the_oracle_and_a_replay():
    rng = np.random.default_rng(0)
    cases = [(256, 16, 16, 0, 0), (3584, 128, 128, 0, 0), (32768, 512, 512, 0, 0),
             (8192, 64, 128, 0, 0), (16384, 256, 256, 0, 1), (0, 4, 4, 0, 0), (5, 16, 4, 0, 0),
             (3482, 128, 128, 0, 0)]
    for _ in range(300):
        M = int(rng.integers(1, 50))
        cases.append((int(rng.integers(0, 400)), int(rng.integers(1, 60)), M,
                      int(rng.integers(0, M + 1)), int(rng.integers(0, 2))))
    for L, B, M, len0, cur0 in cases:
        got = np.array(lb.lococo_plan(L, B, M, len0, cur0), dtype=np.int64).reshape(-1, 6)
        want = orc.plan(L, B, M, len0, cur0)
        assert np.array_equal(got, want), (L, B, M, len0, cur0)
        # replay of the IF, token counts only
        m, cur = len0, cur0
        for (start, ln, branch, before, after, buf) in got:
            assert before == m and ln == min(B, L - start)
            if m + ln <= M:
                assert branch == 0 and after == m + ln and buf == cur
            else:
                cur ^= 1
                assert branch == 1 and after == M and buf == cur
            m = after
        assert got[:, 1].sum() == L


def _cfg(**kw):
    import torch
    base = dict(dtype=torch.float32, batch=1, n_q_heads=2, n_kv_heads=1, head_dim=8, M=4,
                conv_width=3)
    base.update(kw)
    return lb.make_config(**base)


def test_plan_and_config_errors_are_status_codes():
    n = C.c_int64(0)
    L = lb.lib()
    assert L.lococo_plan(10, 0, 4, 0, 0, None, C.byref(n)) == lb.LOCOCO_EINVAL
    assert L.lococo_plan(10, 2, 4, 5, 0, None, C.byref(n)) == lb.LOCOCO_ESTATE
    assert L.lococo_plan(10, 2, 4, 0, 2, None, C.byref(n)) == lb.LOCOCO_ESTATE
    assert L.lococo_plan(10, 2, 4, 0, 0, None, None) == lb.LOCOCO_EINVAL
    assert b"n_inout" in L.lococo_last_error()
    out = C.c_size_t(0)
    for kw, status in [(dict(conv_width=4), lb.LOCOCO_EUNSUPPORTED),
                       (dict(conv_width=0), lb.LOCOCO_EINVAL),
                       (dict(n_q_heads=3, n_kv_heads=2), lb.LOCOCO_EINVAL),
                       (dict(M=0), lb.LOCOCO_EINVAL), (dict(norm=3), lb.LOCOCO_EINVAL),
                       (dict(conv_in=3), lb.LOCOCO_EINVAL), (dict(impl=7), lb.LOCOCO_EINVAL),
                       (dict(head_dim=4096), lb.LOCOCO_EUNSUPPORTED)]:
        cfg = _cfg(**kw)
        assert L.lococo_workspace_bytes(C.byref(cfg), 16, 4, 0, C.byref(out)) == status, kw
        assert len(L.lococo_last_error()) > 0
    bad = _cfg()
    bad.struct_size = 12
    assert L.lococo_workspace_bytes(C.byref(bad), 16, 4, 0, C.byref(out)) == lb.LOCOCO_EINVAL
    assert L.lococo_workspace_bytes(None, 16, 4, 0, C.byref(out)) == lb.LOCOCO_EINVAL
    with pytest.raises(lb.LococoError):
        lb.lococo_workspace_bytes(_cfg(conv_width=2), 16, 4)


def test_call_argument_errors_enqueue_nothing():
    """Null / aliased / misaligned arguments are refused on the host."""
    L = lb.lib()
    cfg = _cfg()
    x = lb.lococo_qkvo()
    cache = lb.lococo_cache()
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 4, None, None) == lb.LOCOCO_EINVAL
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 4, C.byref(cache), None) == lb.LOCOCO_EINVAL
    fake = [0x10000, 0x20000, 0x30000, 0x40000]        # never dereferenced: validation fails first
    cache = lb.lococo_cache((C.c_void_p * 2)(fake[0], fake[0]), (C.c_void_p * 2)(fake[2], fake[3]), 0, 0)
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 4, C.byref(cache), None) == lb.LOCOCO_EINVAL
    assert b"alias" in L.lococo_last_error()
    cache = lb.lococo_cache((C.c_void_p * 2)(fake[0], fake[1]), (C.c_void_p * 2)(fake[2], fake[3]), 0, 9)
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 4, C.byref(cache), None) == lb.LOCOCO_ESTATE
    cache.len = 0
    cache.cur = 3
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 4, C.byref(cache), None) == lb.LOCOCO_ESTATE
    cache.cur = 0
    cache.protect = 0x70002                            # misaligned mask pointer
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 4, C.byref(cache), None) == lb.LOCOCO_EINVAL
    cache.protect, cache.protect_chain_stride = 0x70000, -1
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 4, C.byref(cache), None) == lb.LOCOCO_EINVAL
    cache.protect, cache.protect_chain_stride = None, 0
    cache.attn_colsum = 0x80002                        # misaligned score accumulator
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 4, C.byref(cache), None) == lb.LOCOCO_EINVAL
    assert b"attn_colsum" in L.lococo_last_error()
    cache.attn_colsum = None
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 0, C.byref(cache), None) == lb.LOCOCO_EINVAL
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 4, C.byref(cache), None) == lb.LOCOCO_EINVAL
    assert b"q pointer" in L.lococo_last_error()
    t = lb.lococo_tensor(0x50000, 64, 32, 4)           # stride_t below head_dim
    x = lb.lococo_qkvo(t, t, t, lb.lococo_tensor(0x60000, 64, 32, 8))
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 4, C.byref(cache), None) == lb.LOCOCO_EINVAL
    t = lb.lococo_tensor(0x50000, 64, 32, 8)
    x = lb.lococo_qkvo(t, t, t, t)                     # o aliases q
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 4, C.byref(cache), None) == lb.LOCOCO_EINVAL
    x = lb.lococo_qkvo(t, t, t, lb.lococo_tensor(0x60000, 64, 32, 8))
    # a compressing step without filters / without workspace
    cache.len = 4
    assert L.lococo_segment_step(C.byref(cfg), C.byref(x), 4, None, None, C.byref(cache), None, 0,
                                 None) == lb.LOCOCO_EINVAL
    assert L.lococo_segment_step(C.byref(cfg), C.byref(x), 4, 0x70000, None, C.byref(cache), None, 0,
                                 None) == lb.LOCOCO_EWORKSPACE
    assert cache.len == 4 and cache.cur == 0           # state untouched on failure
    assert L.lococo_mix_from_logits(C.byref(cfg), C.byref(x), 4, None, C.byref(cache),
                                    None) == lb.LOCOCO_EINVAL


def test_every_export_has_its_argument_types_declared():
    """Without argtypes ctypes passes Python ints as 32-bit C ints and truncates device pointers."""
    L = lb.lib()
    for name in lb.EXPORTS:
        fn = getattr(L, name)
        if name in ("lococo_last_error", "lococo_version"):
            continue
        assert fn.argtypes is not None, name


def test_prepare_filters_rejects_bad_arguments_before_touching_the_gpu():
    cfg = lb.make_config(dtype=torch.bfloat16, batch=1, n_q_heads=4, n_kv_heads=4, head_dim=128, M=128,
                         conv_width=15)
    assert lb.lib().lococo_prepare_filters(C.byref(cfg), None, None, 0, None) == lb.LOCOCO_EINVAL
    cfg.flags = 6
    with pytest.raises(lb.LococoError) as e:
        lb.lococo_workspace_bytes(cfg, 128, 128)
    assert e.value.status == lb.LOCOCO_EINVAL


def test_blocks_that_span_2_gib_are_refused_on_the_mfma_paths():
    """The MFMA kernels address the rows of a block with 32-bit offsets inside buffer resources; a
    token stride that makes a block span 2 GiB or more is refused at validation, and the
    shape-agnostic kernels (64-bit addressing) still take it."""
    L = lb.lib()
    cfg = lb.make_config(dtype=torch.bfloat16, batch=1, n_q_heads=4, n_kv_heads=4, head_dim=128, M=128,
                         conv_width=15)
    fake = [0x100000, 0x200000, 0x300000, 0x400000]    # never dereferenced: validation fails first
    cache = lb.lococo_cache((C.c_void_p * 2)(fake[0], fake[1]), (C.c_void_p * 2)(fake[2], fake[3]), 0, 0)
    huge = 1 << 24                                     # elements between tokens: 128 tokens * 32 MiB = 4 GiB
    t = lambda p: lb.lococo_tensor(p, 0, 128, huge)
    x = lb.lococo_qkvo(t(0x500000), t(0x600000), t(0x700000), t(0x800000))
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 128, C.byref(cache), None) == lb.LOCOCO_EUNSUPPORTED
    assert b"2 GiB" in L.lococo_last_error()
    assert L.lococo_segment_step(C.byref(cfg), C.byref(x), 128, 0x900000, None, C.byref(cache), 0xa00000,
                                 1 << 30, None) == lb.LOCOCO_EUNSUPPORTED
    assert cache.len == 0 and cache.cur == 0
    cache.len = 128
    assert L.lococo_mix_from_logits(C.byref(cfg), C.byref(x), 128, 0xb00000, C.byref(cache),
                                    None) == lb.LOCOCO_EUNSUPPORTED
    assert cache.len == 128 and cache.cur == 0


def test_debug_options_are_validated_and_path_description_needs_no_gpu_for_generic_shapes():
    assert C.sizeof(lb.lococo_path_info) == 32
    L = lb.lib()
    assert L.lococo_debug_option(99, 0) == lb.LOCOCO_EINVAL
    assert L.lococo_debug_option(lb.LOCOCO_OPT_LOGITS_TILES, 100) == lb.LOCOCO_EINVAL
    assert L.lococo_debug_option(lb.LOCOCO_OPT_MAX_RESIDENT, -3) == lb.LOCOCO_EINVAL
    assert L.lococo_debug_option(lb.LOCOCO_OPT_UNFUSED_KV, 2) == lb.LOCOCO_EINVAL
    assert L.lococo_debug_option(lb.LOCOCO_OPT_NO_STEP_PIPELINE, 5) == lb.LOCOCO_EINVAL
    assert L.lococo_debug_option(8, 0) == lb.LOCOCO_EINVAL
    assert L.lococo_debug_option(lb.LOCOCO_OPT_LOGITS_TILES, 128) == lb.LOCOCO_OK
    assert L.lococo_debug_option(lb.LOCOCO_OPT_RESET, 0) == lb.LOCOCO_OK
    info = lb.lococo_describe_path(_cfg(), 4)          # fp32, head_dim 8: the shape-agnostic kernels
    assert info["path"] == 0 and info["tile_slots"] == 0 and info["scan_groups"] == 0
    assert L.lococo_describe_path(C.byref(_cfg()), 0, C.byref(lb.lococo_path_info())) == lb.LOCOCO_EINVAL
    assert L.lococo_describe_path(C.byref(_cfg()), 4, None) == lb.LOCOCO_EINVAL


def test_the_library_reads_no_environment_variable():
    """Behaviour switches are explicit calls (lococo_debug_option), not ambient state."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--undefined-only", lb.LIB_PATH], capture_output=True, text=True).stdout
    assert "getenv" not in out


def test_size_limits_and_the_newer_entry_points_refuse_on_the_host():
    """Block lengths and row counts beyond what the kernels hold, and the argument checks of the scan
    backward and of the entry point that allocates nothing: all status codes, nothing dereferenced."""
    L = lb.lib()
    cfg = _cfg()
    fake = [0x10000, 0x20000, 0x30000, 0x40000]
    cache = lb.lococo_cache((C.c_void_p * 2)(fake[0], fake[1]), (C.c_void_p * 2)(fake[2], fake[3]), 0, 0)
    t = lb.lococo_tensor(0x50000, 1 << 30, 1 << 24, 8)
    x = lb.lococo_qkvo(t, t, t, lb.lococo_tensor(0x60000, 1 << 30, 1 << 24, 8))
    assert L.lococo_segment_step(C.byref(cfg), C.byref(x), 70000, 0x70000, None, C.byref(cache), None, 0,
                                 None) == lb.LOCOCO_EUNSUPPORTED
    assert b"65535" in L.lococo_last_error()
    assert L.lococo_attn_only(C.byref(cfg), C.byref(x), 60000, C.byref(cache), None) == lb.LOCOCO_EUNSUPPORTED
    assert b"exceeds" in L.lococo_last_error()
    # the entry point without allocations: prepared filters make no sense there, and a step whose scratch
    # would not fit the library's own array is refused
    flagged = _cfg(flags=1)
    assert L.lococo_segment_step_noalloc(C.byref(flagged), C.byref(x), 4, 0x70000, None, C.byref(cache),
                                         None) == lb.LOCOCO_EINVAL
    # scan backward
    n = C.c_size_t(0)
    assert L.lococo_sequence_backward_workspace_bytes(C.byref(cfg), -1, 4, C.byref(n)) == lb.LOCOCO_EINVAL
    assert L.lococo_sequence_backward_workspace_bytes(C.byref(cfg), 16, 0, C.byref(n)) == lb.LOCOCO_EINVAL
    assert L.lococo_sequence_backward_workspace_bytes(C.byref(cfg), 16, 4, None) == lb.LOCOCO_EINVAL
    assert L.lococo_sequence_backward_workspace_bytes(C.byref(cfg), 16, 4, C.byref(n)) == lb.LOCOCO_OK and n.value > 0
    g = [0x100000 + 0x1000 * i for i in range(10)]
    args = lambda **kw: dict(dict(L=16, B=4, cw=0x70000, d_o=g[0], dq=g[1], dk=g[2], dv=g[3], ck=g[4], cv=g[5], dW=g[6],
                                  ws=0x200000, ws_bytes=1 << 40), **kw)

    def call(c=cfg, **kw):
        a = args(**kw)
        return L.lococo_sequence_backward(C.byref(c), C.byref(x), a["L"], a["B"], a["cw"], None, C.byref(cache), a["d_o"],
                                          None, None, a["dq"], a["dk"], a["dv"], a["ck"], a["cv"], a["dW"], None,
                                          a["ws"], a["ws_bytes"], None)
    assert call(L=0) == lb.LOCOCO_EINVAL
    assert call(B=0) == lb.LOCOCO_EINVAL
    assert call(d_o=None) == lb.LOCOCO_EINVAL and b"gradient pointer" in L.lococo_last_error()
    assert call(ck=None) == lb.LOCOCO_EINVAL
    assert call(cw=None) == lb.LOCOCO_EINVAL and b"compresses" in L.lococo_last_error()
    assert call(c=flagged) == lb.LOCOCO_EINVAL
    assert call(c=_cfg(norm=2)) == lb.LOCOCO_EUNSUPPORTED
    assert call(ws=None) == lb.LOCOCO_EWORKSPACE
    assert call(ws_bytes=256) == lb.LOCOCO_EWORKSPACE
    assert call(ws=0x200010) == lb.LOCOCO_EWORKSPACE          # not 256-byte aligned


def test_bench_refuses_more_than_one_gpu():
    """Everything here runs on one GPU: `bench.py --gpus N` with N above 1 exits with a message that says so."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
