"""The C-ABI boundary on a machine without a GPU: the library loads, exports every symbol the header
declares, and turns every invalid argument into a status code before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2410_06577_amd import rodimus

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_WS, E_LAUNCH, E_ALIAS, E_SCRATCH = range(9)


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(rodimus.LIB_PATH):
        from paper_2410_06577_amd import build
        build.build()
    return rodimus.lib()


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "rodimus.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(rodimus_[a-z_]+)\s*\(", header))
    assert {"rodimus_chunk_scan_fwd", "rodimus_decode_step", "rodimus_status_string",
            "rodimus_chunk_scan_workspace_bytes", "rodimus_chunk_scan_path", "rodimus_ddts_gates",
            "rodimus_chunk_scan_fwd_zbeta", "rodimus_decode_step_zbeta", "rodimus_chunk_scan_varlen_fwd",
            "rodimus_chunk_scan_bwd", "rodimus_chunk_scan_bwd_workspace_bytes", "rodimus_chunk_scan_bwd_zbeta",
            "rodimus_chunk_scan_fwd_block", "rodimus_decode_step_block",
            "rodimus_short_conv_fwd", "rodimus_short_conv_step",
            "rodimus_chunk_scan_fwd_gated", "rodimus_decode_step_gated",
            "rodimus_chunk_scan_fwd_general", "rodimus_decode_step_general",
            "rodimus_chunk_scan_varlen_bwd", "rodimus_chunk_scan_varlen_bwd_workspace_bytes",
            "rodimus_chunk_scan_fwd_noalloc", "rodimus_chunk_scan_fwd_noalloc_scratch_bytes",
            "rodimus_chunk_scan_bwd_gated", "rodimus_chunk_scan_bwd_gated_workspace_bytes",
            "rodimus_chunk_scan_fwd_gated_block", "rodimus_decode_step_gated_block",
            "rodimus_chunk_scan_varlen_fwd_cut", "rodimus_chunk_scan_varlen_workspace_bytes",
            "rodimus_hbm_stream_probe", "rodimus_chunk_scan_varlen_fwd_gated_block",
            "rodimus_chunk_scan_varlen_bwd_cut", "rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes",
            "rodimus_chunk_scan_varlen_bwd_gated", "rodimus_chunk_scan_varlen_bwd_gated_workspace_bytes"} <= declared
    for name in declared:
        assert hasattr(L, name), name


def test_status_strings(L):
    seen = {rodimus.status_string(s) for s in range(9)}
    assert len(seen) == 9 and "ok" in seen
    assert rodimus.status_string(1234) == "unknown status"


def _scan(L, *, q=0x10000, k=0x20000, v=0x30000, la=0x40000, beta=0x50000, S0=0x60000, o=0x70000, S_T=0x80000,
          B=1, T=4, H=1, dk=16, dv=32, chunk=4, io=rodimus.F32, ws=None, ws_bytes=0):
    p = lambda x: None if x is None else ctypes.c_void_p(x)
    return L.rodimus_chunk_scan_fwd(p(q), p(k), p(v), p(la), p(beta), p(S0), p(o), p(S_T),
                                    B, T, H, dk, dv, chunk, io, p(ws), ws_bytes, None)


def _decode(L, *, q=0x10000, k=0x20000, v=0x30000, la=0x40000, beta=0x50000, S=0x100000, o=0x70000,
            N=2, H=2, dk=16, dv=32, io=rodimus.BF16):
    p = lambda x: None if x is None else ctypes.c_void_p(x)
    return L.rodimus_decode_step(p(q), p(k), p(v), p(la), p(beta), p(S), p(o), N, H, dk, dv, io, None)


def test_scan_rejects_bad_arguments_before_any_launch(L):
    assert _scan(L, io=7) == E_DTYPE
    for bad in (dict(B=-1), dict(T=-1), dict(H=-2), dict(dk=0), dict(dk=129), dict(dv=0),
                dict(chunk=0), dict(chunk=65), dict(dk=128, chunk=64)):
        assert _scan(L, **bad) == E_SHAPE, bad
    for name in ("q", "k", "v", "la", "o"):
        assert _scan(L, **{name: None}) == E_NULL, name
    for name in ("q", "k", "v", "la", "beta", "S0", "o", "S_T"):
        assert _scan(L, **{name: 0x10008 + 0x100000}) == E_ALIGN, name
    # the output may not overlap an input; S_T may be S0 itself but not a shifted view of it
    assert _scan(L, o=0x30000) == E_ALIAS                   # o == v
    assert _scan(L, o=0x10010) == E_ALIAS                   # o inside q
    assert _scan(L, S_T=0x60010) == E_ALIAS                 # S_T partially over S0
    assert _scan(L, S_T=0x10000) == E_ALIAS                 # S_T over q


def test_scan_workspace_may_not_overlap_a_tensor_of_the_call(L):
    # a call that is cut along the sequence (few (batch, head) pairs, long T) writes its workspace while it reads the inputs
    G = 0x100000000
    shape = dict(B=1, T=32768, H=16, dk=64, dv=256, chunk=64, io=rodimus.BF16)
    need = L.rodimus_chunk_scan_workspace_bytes(1, 32768, 16, 64, 256, 64, rodimus.BF16)
    assert need > 0
    ptrs = dict(q=1 * G, k=2 * G, v=3 * G, la=4 * G, beta=5 * G, S0=6 * G, o=7 * G, S_T=8 * G)
    assert _scan(L, **shape, **ptrs, ws=None, ws_bytes=0) == E_WS
    assert _scan(L, **shape, **ptrs, ws=9 * G, ws_bytes=need - 16) == E_WS
    for name, at in ptrs.items():
        assert _scan(L, **shape, **ptrs, ws=at, ws_bytes=need) == E_ALIAS, name
        assert _scan(L, **shape, **ptrs, ws=at - need + 16, ws_bytes=need) == E_ALIAS, name     # its tail reaches into the tensor


def test_noalloc_scan_validates_and_refuses_shapes_beyond_its_scratch(L):
    G = 0x100000000
    p = lambda x: None if x is None else ctypes.c_void_p(x)

    def call(B=1, T=32768, H=16, dk=64, dv=256, chunk=64, io=rodimus.BF16, **ptr):
        a = dict(q=1 * G, k=2 * G, v=3 * G, la=4 * G, beta=5 * G, S0=6 * G, o=7 * G, S_T=8 * G)
        a.update(ptr)
        return L.rodimus_chunk_scan_fwd_noalloc(p(a["q"]), p(a["k"]), p(a["v"]), p(a["la"]), p(a["beta"]), p(a["S0"]), p(a["o"]),
                                                p(a["S_T"]), B, T, H, dk, dv, chunk, io, None)

    limit = L.rodimus_chunk_scan_fwd_noalloc_scratch_bytes()
    assert limit == 10 << 20
    # 95 (batch, head) pairs at dv = 256 are cut in two and need 2 x 95 x 64 KiB of entering states: more than the buffer
    assert L.rodimus_chunk_scan_workspace_bytes(95, 4096, 1, 64, 256, 64, rodimus.BF16) > limit
    assert call(B=95, T=4096, H=1) == E_SCRATCH
    # the usual validation still comes first / still applies
    assert call(io=7) == E_DTYPE and call(dk=0) == E_SHAPE
    assert call(q=None) == E_NULL and call(o=3 * G) == E_ALIAS and call(k=2 * G + 8) == E_ALIGN
    assert call(B=0) == OK and call(T=0, S_T=None) == OK


def test_decode_rejects_bad_arguments_before_any_launch(L):
    assert _decode(L, io=-1) == E_DTYPE
    for bad in (dict(N=-1), dict(H=-1), dict(dk=0), dict(dk=257), dict(dv=0), dict(dv=30)):
        assert _decode(L, **bad) == E_SHAPE, bad
    for name in ("q", "k", "v", "la", "S", "o"):
        assert _decode(L, **{name: None}) == E_NULL, name
    for name in ("q", "k", "v", "la", "beta", "S", "o"):
        assert _decode(L, **{name: 0x900008}) == E_ALIGN, name
    assert _decode(L, o=0x100000) == E_ALIAS                # o over the state
    assert _decode(L, S=0x30000) == E_ALIAS                 # state over v


def _gates(L, *, z_g=0x10000, z_tau=0x20000, z_beta=0x30000, q=0x40000, k=0x50000, la=0x60000, beta=0x70000,
           q_out=0x80000, k_out=0x90000, rows=4, dk=64, dv=256, io=rodimus.BF16):
    p = lambda x: None if x is None else ctypes.c_void_p(x)
    return L.rodimus_ddts_gates(p(z_g), p(z_tau), p(z_beta), p(q), p(k), p(la), p(beta), p(q_out), p(k_out),
                                rows, dk, dv, io, None)


def test_gates_reject_bad_arguments_before_any_launch(L):
    assert _gates(L, io=5) == E_DTYPE
    for bad in (dict(rows=-1), dict(dk=4), dict(dk=24), dict(dk=1024), dict(dv=12), dict(dv=0)):
        assert _gates(L, **bad) == E_SHAPE, bad
    for name in ("z_g", "z_tau", "q", "k", "la", "q_out", "k_out"):
        assert _gates(L, **{name: None}) == E_NULL, name
    assert _gates(L, z_beta=None) == E_NULL and _gates(L, beta=None) == E_NULL      # they come and go together
    for name in ("z_g", "z_tau", "z_beta", "q", "k", "la", "beta", "q_out", "k_out"):
        assert _gates(L, **{name: 0xA00008}) == E_ALIGN, name
    assert _gates(L, q_out=0x50000) == E_ALIAS          # q_out over k
    assert _gates(L, la=0x10000) == E_ALIAS             # log_alpha over z_g
    assert _gates(L, k_out=0x80000) == E_ALIAS          # two outputs on top of each other
    assert _gates(L, rows=0) == OK
    assert _gates(L, rows=0, z_beta=None, beta=None, dv=0) == OK


def test_zbeta_calls_validate_like_the_calls_they_mirror(L):
    p = ctypes.c_void_p

    def scan(z=0x50000, o=0x70000, T=4, io=rodimus.BF16):
        S_T = p(0x80000) if T > 0 else None               # T = 0 with a final state wanted would launch a copy
        return L.rodimus_chunk_scan_fwd_zbeta(p(0x10000), p(0x20000), p(0x30000), p(0x40000), None if z is None else p(z),
                                              p(0x60000), p(o), S_T, 1, T, 1, 16, 32, 4, io, None, 0, None)

    def dec(z=0x50000, S=0x100000, N=2, io=rodimus.BF16):
        return L.rodimus_decode_step_zbeta(p(0x10000), p(0x20000), p(0x30000), p(0x40000), None if z is None else p(z),
                                           p(S), p(0x70000), N, 2, 16, 32, io, None)

    assert scan(z=None) == E_NULL and dec(z=None) == E_NULL            # the pre-activation is required ...
    assert scan(z=None, T=0) == OK and dec(z=None, N=0) == OK          # ... unless the call is empty
    assert scan(z=0x50008) == E_ALIGN and dec(z=0x50008) == E_ALIGN
    assert scan(io=9) == E_DTYPE and dec(io=9) == E_DTYPE
    # z_beta has the I/O element size: 4*32 bf16 = 256 bytes from 0x50000; an output just behind it is fine, on it is not
    assert scan(o=0x50080) == E_ALIAS
    assert dec(S=0x50040) == E_ALIAS


def test_varlen_scan_validation(L):
    p = ctypes.c_void_p

    def call(beta=0x50000, kind=0, cu=0x90000, N=2, total=8, o=0x70000, S_T=0x80000, io=rodimus.F32, dk=16):
        f = lambda x: None if x is None else p(x)
        return L.rodimus_chunk_scan_varlen_fwd(p(0x10000), p(0x20000), p(0x30000), p(0x40000), f(beta), kind, p(0x60000),
                                               f(o), f(S_T), f(cu), N, total, 1, dk, 32, 4, io, None)

    assert call(kind=2) == E_DTYPE and call(io=3) == E_DTYPE
    assert call(cu=None) == E_NULL
    assert call(cu=0x90004) == E_ALIGN
    assert call(kind=1, beta=None) == E_NULL            # a pre-activation is required, plain beta is optional
    assert call(N=-1) == E_SHAPE and call(total=-1) == E_SHAPE and call(dk=0) == E_SHAPE
    assert call(o=0x90000) == E_ALIAS                   # o over the length table
    assert call(S_T=0x90000) == E_ALIAS
    assert call(N=0, total=0, cu=None, S_T=None) == OK  # empty batch
    assert call(total=0, S_T=None) == OK                # sequences of length zero, no state wanted


def test_block_calls_validation(L):
    p = ctypes.c_void_p
    f = lambda x: None if x is None else p(x)

    def scan(beta=0x50000, kind=0, x=0x90000, d=0xA0000, z=0xB0000, act=0, o=0x70000, io=rodimus.F32):
        return L.rodimus_chunk_scan_fwd_block(p(0x10000), p(0x20000), p(0x30000), p(0x40000), f(beta), kind, p(0x60000), f(x),
                                              f(d), f(z), act, f(o), p(0x80000), 1, 4, 1, 16, 32, 4, io, None, 0, None)

    def dec(x=0x90000, d=0xA0000, z=0xB0000, act=1, kind=0, S=0x100000):
        return L.rodimus_decode_step_block(p(0x10000), p(0x20000), p(0x30000), p(0x40000), p(0x50000), kind, f(x), f(d), f(z),
                                           act, f(S), p(0x70000), 2, 2, 16, 32, rodimus.BF16, None)

    assert scan(act=2) == E_DTYPE and scan(kind=3) == E_DTYPE and dec(act=-1) == E_DTYPE and dec(kind=2) == E_DTYPE
    assert scan(d=None) == E_NULL and dec(d=None) == E_NULL            # a feed-through needs its weight
    assert scan(x=0x90008) == E_ALIGN and scan(z=0xB0004) == E_ALIGN and dec(d=0xA0008) == E_ALIGN
    assert scan(o=0x90000) == E_ALIAS and scan(o=0xB0000) == E_ALIAS   # o over x' / over z
    assert dec(S=0x90000) == E_ALIAS


def test_backward_validation(L):
    p = ctypes.c_void_p
    names = ["q", "k", "v", "la", "beta", "S0", "d_o", "dS_T", "dq", "dk_out", "dv_out", "dla", "dbeta", "dS0", "ws"]
    base = {n: 0x100000 * (i + 1) for i, n in enumerate(names)}

    def call(B=1, T=4, H=1, dk=64, dv=128, io=rodimus.BF16, ws_bytes=None, **over):
        a = dict(base)
        a.update(over)
        f = lambda x: None if x is None else p(x)
        need = L.rodimus_chunk_scan_bwd_workspace_bytes(B, T, H, dk, dv, io)
        return L.rodimus_chunk_scan_bwd(*[f(a[n]) for n in names[:14]], B, T, H, dk, dv, io, f(a["ws"]),
                                        need if ws_bytes is None else ws_bytes, None)

    assert call(io=4) == E_DTYPE
    for bad in (dict(dk=0), dict(dk=129), dict(dv=0), dict(dk=128, dv=256), dict(B=-1), dict(T=-1),
                dict(T=1 << 20, H=1 << 12)):
        assert call(**bad) == E_SHAPE, bad
    for name in ("q", "k", "v", "la", "d_o", "dq", "dk_out", "dv_out", "dla"):
        assert call(**{name: None}) == E_NULL, name
    for name in names:
        assert call(**{name: base[name] + 8}) == E_ALIGN, name
    assert call(dq=base["q"]) == E_ALIAS and call(dv_out=base["d_o"]) == E_ALIAS and call(dk_out=base["dq"]) == E_ALIAS
    assert call(ws=base["dla"]) == E_ALIAS
    assert call(ws_bytes=16) == E_WS and call(ws=None) == E_WS
    # q .* dq and k .* dk per token, and per (batch, head, channel): one constant, 32 run totals of the first, 32 x 8 of the second
    assert L.rodimus_chunk_scan_bwd_workspace_bytes(2, 100, 3, 64, 128, rodimus.BF16) == (2 * 2 * 100 * 3 * 64 + 2 * 3 * 64 * 289) * 4
    # few (batch, head) pairs and a long sequence: the call is cut along the sequence (here 2 * 1 * 2 = 4 workgroups, 16 chunks
    # -> 4 segments of 4 chunks); units = (batch, head, segment), plus two sets of state slots and the segment decays
    units = 1 * 2 * 4
    assert L.rodimus_chunk_scan_bwd_workspace_bytes(1, 1000, 2, 64, 256, rodimus.BF16) == (
        2 * 1000 * 2 * 64 + units * 64 * 289 + 2 * units * 64 * 256 + 2 * 3 * 2 * 64) * 4
    # the layer workload fills the chip without a cut; a packed batch is never cut
    assert L.rodimus_chunk_scan_bwd_workspace_bytes(8, 4096, 16, 64, 256, rodimus.BF16) == (2 * 8 * 4096 * 16 * 64 + 128 * 64 * 289) * 4
    assert L.rodimus_chunk_scan_varlen_bwd_workspace_bytes(1, 1000, 2, 64, 256, rodimus.BF16) == (2 * 1000 * 2 * 64 + 2 * 64 * 289) * 4
    # any other shape takes the generic kernels: q .* dq only
    assert L.rodimus_chunk_scan_bwd_workspace_bytes(2, 100, 3, 32, 128, rodimus.BF16) == (2 * 100 * 3 * 32 + 2 * 3 * 32) * 4
    assert L.rodimus_chunk_scan_bwd_workspace_bytes(2, 100, 3, 64, 128, rodimus.F32) == (2 * 100 * 3 * 64 + 2 * 3 * 64) * 4
    assert L.rodimus_chunk_scan_bwd_workspace_bytes(2, 100, 3, 129, 8, rodimus.F32) == 0
    assert call(dk=16, dv=32, io=rodimus.F32, ws_bytes=16) == E_WS
    assert call(B=0) == OK

    # the pre-activation form: the gate is required, and only the matrix-core shapes are served
    def call_z(B=1, T=4, H=1, dk=64, dv=128, io=rodimus.BF16, **over):
        a = dict(base)
        a.update(over)
        f = lambda x: None if x is None else p(x)
        need = L.rodimus_chunk_scan_bwd_workspace_bytes(B, T, H, dk, dv, io)
        return L.rodimus_chunk_scan_bwd_zbeta(*[f(a[n]) for n in names[:14]], B, T, H, dk, dv, io, f(a["ws"]), need, None)

    assert call_z(beta=None) == E_NULL
    assert call_z(dk=16, dv=32, io=rodimus.F32) == E_SHAPE and call_z(dk=64, dv=128, io=rodimus.F32) == E_SHAPE
    assert call_z(dbeta=base["beta"]) == E_ALIAS and call_z(beta=base["beta"] + 8) == E_ALIGN
    assert call_z(B=0) == OK


def test_gated_calls_validation(L):
    p = ctypes.c_void_p
    f = lambda x: None if x is None else p(x)

    def scan(q=0x10000, k=0x20000, v=0x30000, zg=0x40000, zt=0x48000, zb=0x50000, S0=0x60000, o=0x70000, S_T=0x80000,
             B=1, T=4, H=1, dk=16, dv=32, chunk=4, io=rodimus.F32, ws=None, ws_bytes=0):
        return L.rodimus_chunk_scan_fwd_gated(f(q), f(k), f(v), f(zg), f(zt), f(zb), f(S0), f(o), f(S_T), B, T, H, dk, dv,
                                              chunk, io, f(ws), ws_bytes, None)

    def dec(q=0x10000, k=0x20000, v=0x30000, zg=0x40000, zt=0x48000, zb=0x50000, S=0x100000, o=0x70000, N=2, H=2, dk=16,
            dv=32, io=rodimus.BF16):
        return L.rodimus_decode_step_gated(f(q), f(k), f(v), f(zg), f(zt), f(zb), f(S), f(o), N, H, dk, dv, io, None)

    assert scan(io=5) == E_DTYPE and dec(io=-1) == E_DTYPE
    assert scan(dk=0) == E_SHAPE and scan(chunk=0) == E_SHAPE and dec(dv=6) == E_SHAPE
    for name in ("q", "k", "v", "zg", "zt", "o"):
        assert scan(**{name: None}) == E_NULL, name
        assert dec(**{name: None}) == E_NULL, name
    assert dec(S=None) == E_NULL
    for name, val in (("zg", 0x40008), ("zt", 0x48004), ("zb", 0x50002)):
        assert scan(**{name: val}) == E_ALIGN, name
        assert dec(**{name: val}) == E_ALIGN, name
    assert scan(o=0x40000) == E_ALIAS and scan(o=0x48000) == E_ALIAS and scan(S_T=0x48000) == E_ALIAS
    assert dec(o=0x48000) == E_ALIAS and dec(S=0x40000) == E_ALIAS
    # the MFMA shapes need their workspace in this form as well
    need = L.rodimus_chunk_scan_workspace_bytes(1, 32768, 16, 64, 256, 64, rodimus.BF16)
    assert need > 0
    assert scan(B=1, T=32768, H=16, dk=64, dv=256, chunk=64, io=rodimus.BF16, q=0x10000000, k=0x20000000, v=0x30000000,
                zg=0x40000000, zt=0x50000000, zb=0x60000000, S0=None, o=0x80000000, S_T=None) == E_WS
    assert scan(B=0) == OK and dec(N=0) == OK and scan(T=0, S_T=None) == OK


def test_stream_probe_validation(L):
    p = lambda x: None if x is None else ctypes.c_void_p(x)
    call = lambda src=0x100000, dst=0x900000, units=1024, reads=4, wgs=256: L.rodimus_hbm_stream_probe(
        p(src), p(dst), ctypes.c_size_t(units), reads, wgs, None)
    assert call(reads=3) == E_SHAPE and call(wgs=0) == E_SHAPE and call(wgs=(1 << 20) + 1) == E_SHAPE
    assert call(dst=None) == E_NULL and call(src=None) == E_NULL and call(src=0x100008) == E_ALIGN
    assert call(dst=0x100000 + 3 * 16384) == E_ALIAS          # inside the fourth input stream
    assert call(units=0, src=None, dst=None) == OK


def test_packed_cut_workspace_and_validation(L):
    L.rodimus_chunk_scan_varlen_workspace_bytes.restype = ctypes.c_size_t
    need = L.rodimus_chunk_scan_varlen_workspace_bytes(8, 32768, 16, 64, 256, 64, rodimus.BF16)
    # segments of 32768 * 16 * 2 / 256 = 4096 tokens: at most 8 + 8 slots of [16 heads][64][256] fp32 plus their decays
    assert need == 16 * 16 * 64 * (256 + 1) * 4
    assert L.rodimus_chunk_scan_varlen_workspace_bytes(3, 1023, 2, 64, 128, 64, rodimus.BF16) == 0       # too short to cut
    assert L.rodimus_chunk_scan_varlen_workspace_bytes(256, 90000, 2, 64, 128, 64, rodimus.BF16) > 0
    assert L.rodimus_chunk_scan_varlen_workspace_bytes(257, 90000, 2, 64, 128, 64, rodimus.BF16) == 0    # too many sequences: the slot walk
    assert L.rodimus_chunk_scan_varlen_workspace_bytes(3, 9000, 2, 16, 32, 16, rodimus.F32) == 0         # any-shape kernels
    assert L.rodimus_chunk_scan_varlen_workspace_bytes(3, 9000, 2, 64, 128, 64, rodimus.BF16) == (9000 // 512 + 3) * 2 * 64 * 129 * 4
    p = lambda x: None if x is None else ctypes.c_void_p(x)

    def call(ws=0x4000000, ws_bytes=1 << 30, kind=0, cu=0x90000, o=0xA00000, total=9000):
        return L.rodimus_chunk_scan_varlen_fwd_cut(p(0x1000000), p(0x2000000), p(0x3000000), p(0x5000000), p(0x6000000), kind,
                                                   p(0x7000000), p(o), p(0x8000000), p(cu), 3, total, 2, 64, 128, 64, rodimus.BF16,
                                                   p(ws), ctypes.c_size_t(ws_bytes), None)

    assert call(ws=None, ws_bytes=0) == E_WS and call(ws_bytes=1000) == E_WS
    assert call(kind=7) == E_DTYPE and call(cu=None) == E_NULL and call(ws=0x4000008) == E_ALIGN
    assert call(ws=0xA00000) == E_ALIAS                      # the workspace over the output
    assert call(ws=0x8000000 - 4096) == E_ALIAS              # ... or reaching into the state cache


def test_packed_backward_cut_workspace(L):
    for f in (L.rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes, L.rodimus_chunk_scan_varlen_bwd_workspace_bytes):
        f.restype = ctypes.c_size_t
    # 8 sequences, 32768 tokens, 16 heads: segments of 32768 * 16 / 256 = 2048 tokens, at most 16 + 8 slots of 16 units each
    units, rows = 24 * 16, 32768 * 16
    want = (2 * rows * 64 + units * 64 * (1 + 32 + 8 * 32) + 2 * units * 64 * 256 + 2 * units * 64) * 4
    assert L.rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes(8, 32768, 16, 64, 256, rodimus.BF16) == want
    # too short, or a shape of the token-by-token kernels: the uncut call's size
    for args in ((3, 500, 2, 64, 128, rodimus.BF16), (3, 5000, 2, 16, 32, rodimus.F32)):
        assert L.rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes(*args) == L.rodimus_chunk_scan_varlen_bwd_workspace_bytes(*args)


def test_packed_gated_backward_workspace_and_validation(L):
    size = L.rodimus_chunk_scan_varlen_bwd_gated_workspace_bytes
    size.restype = ctypes.c_size_t
    L.rodimus_chunk_scan_varlen_bwd_workspace_bytes.restype = ctypes.c_size_t
    L.rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes.restype = ctypes.c_size_t
    N, total, H, dv = 3, 5000, 2, 128
    front = total * H * 64 * (4 + 2 * 2 + 4)         # log_alpha fp32, prepared q and k bf16, dlog_alpha fp32
    assert size(N, total, H, 64, dv, rodimus.BF16, 0) == front + L.rodimus_chunk_scan_varlen_bwd_workspace_bytes(N, total, H, 64, dv, rodimus.BF16)
    assert size(N, total, H, 64, dv, rodimus.BF16, 1) == front + L.rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes(N, total, H, 64, dv, rodimus.BF16)
    assert size(N, total, H, 16, 32, rodimus.F32, 0) == 0          # matrix-core shapes only
    p = lambda x: None if x is None else ctypes.c_void_p(x)
    G = 0x10000000

    def call(ws_bytes=1 << 30, cu=18 * G, **kw):
        a = dict(q=G, k=2 * G, v=3 * G, zg=4 * G, zt=5 * G, zb=6 * G, S0=7 * G, do=8 * G, dS=9 * G, dq=10 * G, dk=11 * G, dv=12 * G,
                 dzg=13 * G, dzt=14 * G, dzb=15 * G, dS0=16 * G, ws=17 * G)
        a.update(kw)
        return L.rodimus_chunk_scan_varlen_bwd_gated(*(p(a[n]) for n in ("q", "k", "v", "zg", "zt", "zb", "S0", "do", "dS", "dq", "dk", "dv",
                                                                          "dzg", "dzt", "dzb", "dS0")), p(cu), N, total, H, 64, dv, rodimus.BF16,
                                                     1, p(a["ws"]), ctypes.c_size_t(ws_bytes), None)

    assert call(cu=None) == E_NULL and call(zt=None) == E_NULL and call(dzg=None) == E_NULL
    assert call(ws_bytes=1000) == E_WS and call(ws=None) == E_WS
    assert call(dzg=4 * G) == E_ALIAS and call(dzt=13 * G) == E_ALIAS and call(dzg=18 * G) == E_ALIAS       # over z_g, over dz_g, over cu_seqlens
    assert call(zg=4 * G + 8) == E_ALIGN


def test_packed_gated_block_validation(L):
    p = lambda x: None if x is None else ctypes.c_void_p(x)

    def call(act=0, ws=None, ws_bytes=0, total=9000, **kw):
        a = dict(q=0x1000000, k=0x2000000, v=0x3000000, zg=0x4000000, zt=0x5000000, zb=0x6000000, S0=0x7000000, x=0x8000000,
                 d=0x9000000, z=0xA000000, o=0xB000000, S_T=0xC000000, cu=0xD000000)
        a.update(kw)
        return L.rodimus_chunk_scan_varlen_fwd_gated_block(p(a["q"]), p(a["k"]), p(a["v"]), p(a["zg"]), p(a["zt"]), p(a["zb"]), p(a["S0"]),
                                                           p(a["x"]), p(a["d"]), p(a["z"]), act, p(a["o"]), p(a["S_T"]), p(a["cu"]), 3, total,
                                                           2, 64, 128, 64, rodimus.BF16, p(ws), ctypes.c_size_t(ws_bytes), None)

    assert call(act=9) == E_DTYPE and call(cu=None) == E_NULL and call(zt=None) == E_NULL and call(d=None) == E_NULL
    assert call(o=0x8000000) == E_ALIAS and call(S_T=0xA000000) == E_ALIAS and call(z=0xA000004) == E_ALIGN
    assert call(ws=0xE000000, ws_bytes=1000) == E_WS          # a workspace asks for the cut: it must then be large enough
    assert call(ws=0xB000000, ws_bytes=1 << 30) == E_ALIAS    # ... and must not lie over the output


def test_gated_block_calls_validation(L):
    p = lambda x: None if x is None else ctypes.c_void_p(x)

    def scan(o=0xA0000, S_T=0xB0000, act=0, **kw):
        a = dict(q=0x10000, k=0x20000, v=0x30000, zg=0x40000, zt=0x48000, zb=0x50000, S0=0x60000, x=0x70000, d=0x80000, z=0x90000)
        a.update(kw)
        return L.rodimus_chunk_scan_fwd_gated_block(p(a["q"]), p(a["k"]), p(a["v"]), p(a["zg"]), p(a["zt"]), p(a["zb"]), p(a["S0"]),
                                                    p(a["x"]), p(a["d"]), p(a["z"]), act, p(o), p(S_T), 1, 4, 1, 16, 32, 4, rodimus.F32,
                                                    None, 0, None)

    def dec(o=0xA0000, S=0x100000, act=1, **kw):
        a = dict(q=0x10000, k=0x20000, v=0x30000, zg=0x40000, zt=0x48000, zb=0x50000, x=0x70000, d=0x80000, z=0x90000)
        a.update(kw)
        return L.rodimus_decode_step_gated_block(p(a["q"]), p(a["k"]), p(a["v"]), p(a["zg"]), p(a["zt"]), p(a["zb"]), p(a["x"]), p(a["d"]),
                                                 p(a["z"]), act, p(S), p(o), 2, 2, 16, 32, rodimus.BF16, None)

    assert scan(act=5) == E_DTYPE and dec(act=-1) == E_DTYPE
    assert scan(zg=None) == E_NULL and scan(zt=None) == E_NULL and dec(zt=None) == E_NULL
    assert scan(d=None) == E_NULL and dec(d=None) == E_NULL                  # feed-through without its weights
    assert scan(x=0x70008) == E_ALIGN and dec(z=0x90004) == E_ALIGN
    assert scan(o=0x70000) == E_ALIAS and scan(o=0x40000) == E_ALIAS and scan(S_T=0x90000) == E_ALIAS
    assert dec(o=0x90000) == E_ALIAS and dec(S=0x48000) == E_ALIAS


def test_general_transition_calls_validation(L):
    p = ctypes.c_void_p
    f = lambda x: None if x is None else p(x)

    def scan(la=0x40000, lb=0x48000, beta=0x50000, o=0x70000, S_T=0x80000, B=1, T=4, H=1, dk=16, dv=32, chunk=4, io=rodimus.F32):
        return L.rodimus_chunk_scan_fwd_general(p(0x10000), p(0x20000), p(0x30000), f(la), f(lb), f(beta), p(0x60000), f(o),
                                                f(S_T), B, T, H, dk, dv, chunk, io, None)

    def dec(la=0x40000, lb=0x48000, beta=0x50000, S=0x100000, o=0x70000, N=2, H=2, dk=16, dv=32, io=rodimus.BF16):
        return L.rodimus_decode_step_general(p(0x10000), p(0x20000), p(0x30000), f(la), f(lb), f(beta), f(S), f(o), N, H, dk,
                                             dv, io, None)

    assert scan(lb=None) == E_NULL and dec(lb=None) == E_NULL and scan(la=None) == E_NULL
    assert scan(lb=0x48008) == E_ALIGN and dec(lb=0x48004) == E_ALIGN
    assert scan(o=0x48000) == E_ALIAS and scan(S_T=0x48000) == E_ALIAS and dec(o=0x48000) == E_ALIAS and dec(S=0x48000) == E_ALIAS
    assert scan(io=9) == E_DTYPE and scan(dk=0) == E_SHAPE and dec(dv=2) == E_SHAPE
    assert scan(B=0) == OK and dec(N=0) == OK and scan(T=0, S_T=None) == OK


def test_short_conv_validation(L):
    p = ctypes.c_void_p
    f = lambda x: None if x is None else p(x)

    def fwd(x=0x100000, w=0x200000, b=0x300000, si=0x400000, y=0x500000, so=0x600000, B=2, T=5, C=16, W=4, act=1,
            io=rodimus.BF16):
        return L.rodimus_short_conv_fwd(f(x), f(w), f(b), f(si), f(y), f(so), B, T, C, W, act, io, None)

    def step(x=0x100000, w=0x200000, b=0x300000, st=0x400000, y=0x500000, N=2, C=16, W=4, act=1, io=rodimus.F32):
        return L.rodimus_short_conv_step(f(x), f(w), f(b), f(st), f(y), N, C, W, act, io, None)

    assert fwd(io=3) == E_DTYPE and fwd(act=2) == E_DTYPE and step(act=-1) == E_DTYPE
    for bad in (dict(W=0), dict(W=9), dict(C=12), dict(B=-1), dict(T=-1), dict(C=-8)):
        assert fwd(**bad) == E_SHAPE, bad
    assert step(W=9) == E_SHAPE and step(C=4) == E_SHAPE and step(N=-1) == E_SHAPE
    for name in ("x", "w", "y"):
        assert fwd(**{name: None}) == E_NULL, name
        assert step(**{name: None}) == E_NULL, name
    assert step(st=None) == E_NULL and step(st=None, W=1, N=0) == OK
    for name, val in (("x", 0x100008), ("w", 0x200004), ("b", 0x300008), ("si", 0x400002), ("y", 0x500008), ("so", 0x600008)):
        assert fwd(**{name: val}) == E_ALIGN, name
    assert fwd(y=0x100000) == E_ALIAS and fwd(so=0x400000) == E_ALIAS and fwd(so=0x100000) == E_ALIAS
    assert fwd(y=0x600000) == E_ALIAS and step(y=0x400000) == E_ALIAS
    assert fwd(B=0) == OK and fwd(C=0) == OK and fwd(T=0, so=None) == OK and step(N=0) == OK


def test_packed_backward_validation(L):
    p = ctypes.c_void_p
    names = ["q", "k", "v", "la", "beta", "S0", "d_o", "dS_T", "dq", "dk_out", "dv_out", "dla", "dbeta", "dS0", "cu", "ws"]
    base = {n: 0x100000 * (i + 1) for i, n in enumerate(names)}

    def call(N=2, total=10, H=1, dk=64, dv=128, io=rodimus.BF16, ws_bytes=None, **over):
        a = dict(base)
        a.update(over)
        f = lambda x: None if x is None else p(x)
        need = L.rodimus_chunk_scan_varlen_bwd_workspace_bytes(N, total, H, dk, dv, io)
        return L.rodimus_chunk_scan_varlen_bwd(*[f(a[n]) for n in names[:15]], N, total, H, dk, dv, io, f(a["ws"]),
                                               need if ws_bytes is None else ws_bytes, None)

    assert L.rodimus_chunk_scan_varlen_bwd_workspace_bytes(3, 100, 2, 64, 128, rodimus.BF16) == (2 * 100 * 2 * 64 + 3 * 2 * 64 * 289) * 4
    assert L.rodimus_chunk_scan_varlen_bwd_workspace_bytes(3, 100, 2, 16, 32, rodimus.F32) == (100 * 2 * 16 + 3 * 2 * 16) * 4
    assert call(cu=None) == E_NULL and call(cu=base["cu"] + 4) == E_ALIGN and call(q=None) == E_NULL
    assert call(dq=base["cu"]) == E_ALIAS and call(ws=base["cu"]) == E_ALIAS
    assert call(ws_bytes=16) == E_WS and call(io=7) == E_DTYPE and call(dk=0) == E_SHAPE and call(total=-1) == E_SHAPE
    assert call(N=0, total=0, cu=None) == OK


def test_gated_backward_validation(L):
    G = 0x100000000
    p = lambda x: None if x is None else ctypes.c_void_p(x)
    names = ["q", "k", "v", "z_g", "z_tau", "z_beta", "S0", "d_o", "dS_T", "dq", "dk", "dv", "dz_g", "dz_tau", "dz_beta", "dS0"]
    base = {n: (i + 1) * G for i, n in enumerate(names)}
    shape = dict(B=2, T=128, H=2, dk=64, dv=128, io=rodimus.BF16)
    need = L.rodimus_chunk_scan_bwd_gated_workspace_bytes(2, 128, 2, 64, 128, rodimus.BF16)
    inner = L.rodimus_chunk_scan_bwd_workspace_bytes(2, 128, 2, 64, 128, rodimus.BF16)
    assert need == inner + 2 * 128 * 2 * 64 * (4 + 2 + 2 + 4)           # log_alpha, scaled q, folded k, dlog_alpha in front

    def call(ws=20 * G, ws_bytes=need, B=2, T=128, H=2, key_width=64, value_width=128, io=rodimus.BF16, **ptr):
        a = dict(base)
        a.update(ptr)
        return L.rodimus_chunk_scan_bwd_gated(*[p(a[n]) for n in names], B, T, H, key_width, value_width, io, p(ws), ws_bytes, None)

    assert call(io=9) == E_DTYPE
    assert call(key_width=32) == E_SHAPE and call(value_width=64) == E_SHAPE and call(io=rodimus.F32) == E_SHAPE and call(B=-1) == E_SHAPE
    for n in ("q", "k", "v", "z_g", "z_tau", "d_o", "dq", "dk", "dv", "dz_g", "dz_tau"):
        assert call(**{n: None}) == E_NULL, n
    assert call(z_beta=None) == E_NULL                       # dz_beta without z_beta
    assert call(ws=None) == E_WS and call(ws_bytes=need - 16) == E_WS
    assert call(z_g=base["z_g"] + 8) == E_ALIGN and call(dz_tau=base["dz_tau"] + 4) == E_ALIGN
    assert call(dz_g=base["q"]) == E_ALIAS and call(dz_tau=base["dz_g"]) == E_ALIAS and call(dz_g=20 * G + 64) == E_ALIAS
    assert call(dq=base["z_g"]) == E_ALIAS and call(dk=base["z_tau"]) == E_ALIAS
    assert call(B=0) == OK


def test_empty_problems_are_successful_noops(L):
    assert _scan(L, B=0) == OK
    assert _scan(L, H=0) == OK
    assert _scan(L, T=0, S_T=None) == OK
    assert _decode(L, N=0) == OK
    assert _decode(L, H=0) == OK


def test_queries(L):
    assert L.rodimus_chunk_scan_path(1, 64, 1, 16, 32, 16, rodimus.F32) == rodimus.PATH_GENERIC
    assert L.rodimus_chunk_scan_path(1, 64, 1, 0, 32, 16, rodimus.F32) == rodimus.PATH_NONE
    assert L.rodimus_chunk_scan_workspace_bytes(1, 64, 1, 16, 32, 16, rodimus.F32) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 4, 1, 16)
    with pytest.raises(ValueError, match="device tensors"):
        rodimus.rodimus_chunk_scan_fwd(x, x, x, x)
    with pytest.raises(ValueError, match="device tensors"):
        rodimus.rodimus_decode_step(x[0], x[0], x[0], x[0], None, torch.zeros(4, 1, 16, 16))
