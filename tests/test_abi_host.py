"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "hstu_attn.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2508_04711_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2508_04711_amd import build
        build.build()
    return binding.load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hstu_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"hstu_jagged_attn_fwd", "hstu_jagged_attn_bwd", "hstu_jagged_attn_cp_partial",
            "hstu_jagged_attn_workspace_bytes", "hstu_attn_status_string"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_header_is_plain_c_and_cxx(tmp_path):
    """The boundary is a C header: it must compile as strict C99 and as C++ with no warnings."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "hstu_attn.h"\n'
                   'int main(void) { hstu_attn_params p; hstu_cp_desc c; hstu_ts_bias b; hstu_cp_ring_desc r;\n'
                   '  (void)p; (void)c; (void)b; (void)r; return hstu_attn_status_string(0) == 0; }\n')
    inc = os.path.join(ROOT, "include")
    for cmd in (["gcc", "-std=c99", "-x", "c"], ["g++", "-std=c++11", "-x", "c++"]):
        res = subprocess.run(cmd + ["-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(src)],
                             capture_output=True, text=True)
        assert res.returncode == 0, res.stderr


def _params(binding, **kw):
    base = dict(batch=2, num_heads=2, d_qk=64, d_v=64, max_len=16, alpha=0.125, causal=1, dtype=0,
                total_rows=10, out_dtype=0, flags=0)
    base.update(kw)
    return binding._Params(base["batch"], base["num_heads"], base["d_qk"], base["d_v"],
                           base["max_len"], base["alpha"], base["causal"], base["dtype"],
                           base["total_rows"], base["out_dtype"], base["flags"])


def test_status_strings(lib):
    from paper_2508_04711_amd import binding
    assert binding.hstu_attn_status_string(0) == "ok"
    seen = {binding.hstu_attn_status_string(s) for s in range(-7, 1)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert binding.hstu_attn_status_string(-99) == "unknown status"


def test_bad_arguments_are_rejected_on_the_host(lib):
    from paper_2508_04711_amd import binding
    fake = ctypes.c_void_p(0x1000)      # never dereferenced: every call below fails validation first
    def fwd(p, q=fake, ws=fake, ws_bytes=1 << 20):
        return lib.hstu_jagged_attn_fwd(ctypes.byref(p), q, fake, fake, fake, fake, ws, ws_bytes, None)
    assert fwd(_params(binding, d_qk=48)) == -3
    assert fwd(_params(binding, dtype=7)) == -3
    assert fwd(_params(binding, out_dtype=0, dtype=1)) == -3       # fp32 in, bf16 out
    assert fwd(_params(binding, flags=128)) == -3     # an unknown bit
    assert fwd(_params(binding, flags=8 | 16)) == -3  # two forward tile heights at once
    assert fwd(_params(binding, num_heads=0)) == -2
    assert fwd(_params(binding, max_len=0)) == -2
    assert fwd(_params(binding, total_rows=-1)) == -2
    assert fwd(_params(binding, total_rows=1 << 31)) == -2
    assert fwd(_params(binding, alpha=float("nan"))) == -2
    assert fwd(_params(binding), q=None) == -1
    assert fwd(_params(binding), q=ctypes.c_void_p(0x1004)) == -7
    assert fwd(_params(binding), ws_bytes=16) == -4
    assert lib.hstu_jagged_attn_fwd(None, fake, fake, fake, fake, fake, fake, 1 << 20, None) == -1
    # empty problems succeed without a launch, whatever the pointers
    assert fwd(_params(binding, batch=0, total_rows=0), q=None) == 0
    assert fwd(_params(binding, total_rows=0), q=None) == 0
    bwd = lib.hstu_jagged_attn_bwd(ctypes.byref(_params(binding)), fake, fake, fake, None, fake,
                                   fake, fake, fake, fake, 1 << 20, None)
    assert bwd == -1
    cp = binding._CpDesc(2, 2, 0, 0, 5, 5)       # q_rank out of range
    rc = lib.hstu_jagged_attn_cp_partial(ctypes.byref(_params(binding)), ctypes.byref(cp), fake, fake,
                                         fake, None, fake, fake, None, None, None, fake, 1 << 20, None)
    assert rc == -5
    cp = binding._CpDesc(0, 0, 0, 0, 5, 5)
    rc = lib.hstu_jagged_attn_cp_partial(ctypes.byref(_params(binding)), ctypes.byref(cp), fake, fake,
                                         fake, None, fake, fake, None, None, None, fake, 1 << 20, None)
    assert rc == -5


def test_bias_calls_reject_bad_arguments_on_the_host(lib):
    from paper_2508_04711_amd import binding
    fake = ctypes.c_void_p(0x1000)      # never dereferenced: every call below fails validation first

    def desc(ts=0x1000, w=0x1000, dw=0x1000, nb=16, f=2):
        return binding._TsBias(ts, w, dw, nb, f)

    def fwd(p, b, ws_bytes=1 << 20):
        return lib.hstu_jagged_attn_bias_fwd(ctypes.byref(p), ctypes.byref(b) if b is not None else None,
                                             fake, fake, fake, fake, fake, fake, ws_bytes, None)

    def bwd(p, b, ws_bytes=1 << 20):
        return lib.hstu_jagged_attn_bias_bwd(ctypes.byref(p), ctypes.byref(b), fake, fake, fake, fake, fake,
                                             fake, fake, fake, fake, ws_bytes, None)

    ok = _params(binding)
    assert fwd(ok, None) == -1                                   # no descriptor
    assert fwd(ok, desc(ts=None)) == -1 and fwd(ok, desc(w=None)) == -1
    assert bwd(ok, desc(dw=None)) == -1                          # the backward call needs the gradient buffer
    assert fwd(ok, desc(nb=0)) == -2 and fwd(ok, desc(nb=513)) == -2
    assert fwd(ok, desc(f=-1)) == -2 and fwd(ok, desc(f=9)) == -2
    assert fwd(_params(binding, batch=-1), desc()) == -2               # the common checks come first
    assert fwd(ok, desc(), ws_bytes=64) == -4 and bwd(ok, desc(), ws_bytes=64) == -4
    assert fwd(_params(binding, batch=0, total_rows=0), desc()) == 0   # empty batch: nothing to do
    # workspace: the plain call's plus one 16-byte record per row (and 64 rows of padding)
    for which in (0, 1):
        plain = lib.hstu_jagged_attn_workspace_bytes(ctypes.byref(ok), which)
        with_bias = lib.hstu_jagged_attn_bias_workspace_bytes(ctypes.byref(ok), which)
        assert with_bias == plain + 512 * 8 + 16 * (10 + 64) + (-16 * (10 + 64)) % 256   # sums, then records
    # the context-parallel call with bias: records for both sides' rows
    rec = 16 * (10 + 64) + (-16 * (10 + 64)) % 256
    assert lib.hstu_jagged_attn_bias_workspace_bytes(ctypes.byref(ok), 2) == \
        lib.hstu_jagged_attn_workspace_bytes(ctypes.byref(ok), 2) + 512 * 8 + 2 * rec
    assert lib.hstu_jagged_attn_bias_workspace_bytes(ctypes.byref(ok), 3) == 0
    # hstu_jagged_attn_cp_partial_bias: the descriptor's checks come before any device work
    cpd = binding._CpDesc(2, 0, 1, 0, 5, 5)

    def cpb(p, b, ws_bytes=1 << 20, d_o=fake):
        return lib.hstu_jagged_attn_cp_partial_bias(ctypes.byref(p), ctypes.byref(cpd),
                                                    ctypes.byref(b) if b is not None else None, fake, fake,
                                                    fake, d_o, fake, fake, fake, fake, fake, fake, ws_bytes, None)

    def cdesc(tq=0x1000, tk=0x1000, w=0x1000, dw=0x1000, nb=16, f=2):
        return binding._CpTsBias(tq, tk, w, dw, nb, f)

    assert cpb(ok, None) == -1
    assert cpb(ok, cdesc(tq=None)) == -1 and cpb(ok, cdesc(tk=None)) == -1 and cpb(ok, cdesc(w=None)) == -1
    assert cpb(ok, cdesc(dw=None)) == -1                 # backward (d_o given) needs the gradient buffer
    assert cpb(ok, cdesc(nb=600)) == -2 and cpb(ok, cdesc(f=12)) == -2
    assert cpb(ok, cdesc(), ws_bytes=128) == -4
    # hstu_cp_ring_pass_bias: no descriptor, or one without the query timestamps or the table
    ring = binding._RingDesc()
    def rpb(b):
        return lib.hstu_cp_ring_pass_bias(ctypes.byref(ok), ctypes.byref(ring),
                                          ctypes.byref(b) if b is not None else None, fake, None, fake, fake,
                                          None, fake, 1 << 20, ctypes.c_void_p(1), ctypes.c_void_p(2))
    assert rpb(None) == -1
    assert rpb(binding._RingTsBias()) == -1
    assert lib.hstu_jagged_attn_bias_workspace_bytes(ctypes.byref(_params(binding, d_qk=48)), 0) == 0


def test_reorder_rejects_bad_arguments_on_the_host(lib):
    fake = 0x1000
    def call(batch=2, total=100, cp=2, rank=0, n=1, src=(fake,), dst=(fake,), rb=(256,), local=50,
             off=ctypes.cast(fake, ctypes.POINTER(ctypes.c_int32))):
        s = (ctypes.c_void_p * 4)(*src)
        d = (ctypes.c_void_p * 4)(*dst)
        r = (ctypes.c_int64 * 4)(*rb)
        return lib.hstu_cp_reorder(batch, total, cp, rank, 0, n, ctypes.cast(s, ctypes.c_void_p),
                                   ctypes.cast(d, ctypes.c_void_p), ctypes.cast(r, ctypes.c_void_p),
                                   local, off, None)
    assert call(cp=0) == -5 and call(rank=2) == -5 and call(rank=-1) == -5
    assert call(total=-1) == -2 and call(total=1 << 31) == -2 and call(local=-1) == -2
    assert call(n=0) == -2 and call(n=5) == -2
    assert call(rb=(26,)) == -2 and call(rb=(0,)) == -2 and call(rb=(2,)) == -2   # multiples of 4 only
    assert call(src=(None,)) == -1 and call(dst=(None,)) == -1
    assert call(src=(0x1008,)) == -7
    assert call(off=None) == -1
    assert call(total=0, off=None) == 0 and call(local=0, off=None) == 0      # nothing to move


def test_workspace_query(lib):
    from paper_2508_04711_amd import binding
    p = _params(binding, batch=16, total_rows=37117, d_qk=128, d_v=128)
    sizes = [lib.hstu_jagged_attn_workspace_bytes(ctypes.byref(p), k) for k in (0, 1, 2)]
    # schedules only: the forward reads V row-major
    assert all(0 < x < (1 << 20) for x in sizes)
    # with a forced tile height the forward and context-parallel workspaces hold a transposed bf16
    # copy of V: [H, d_v, ~T]
    forced = _params(binding, batch=16, total_rows=37117, d_qk=128, d_v=128, flags=8)
    fsizes = [lib.hstu_jagged_attn_workspace_bytes(ctypes.byref(forced), k) for k in (0, 1, 2)]
    vt = 2 * 128 * 37117 * 2
    assert vt < fsizes[0] < 1.2 * vt and 0 < fsizes[1] < (1 << 20) and vt < fsizes[2] < 1.5 * vt
    # with sequences long enough to be cut along the keys (max_len >= 4096) the query-side passes
    # add room for fp32 partial results: at most (tiles + 1024 / H + 1) slots of 128 rows
    long_p = _params(binding, batch=16, total_rows=37117, d_qk=128, d_v=128, max_len=8192)
    slots = 37117 // 128 + 16 + 1 + 1024 // 2 + 1
    part = slots * 2 * 128 * 128 * 4
    grown = [lib.hstu_jagged_attn_workspace_bytes(ctypes.byref(long_p), k) for k in (0, 1, 2)]
    assert sizes[0] + 0.9 * part < grown[0] < sizes[0] + 1.1 * part
    assert 0.9 * part < grown[1] < 1.1 * part + (1 << 20)
    assert grown[2] > sizes[2] + 1.8 * part
    assert lib.hstu_jagged_attn_workspace_bytes(ctypes.byref(p), 9) == 0
    assert lib.hstu_jagged_attn_workspace_bytes(ctypes.byref(_params(binding, d_v=5)), 0) == 0
    # grows with the batch and with the rows
    big = _params(binding, batch=500, total_rows=10 ** 6, d_qk=128, d_v=128)
    assert lib.hstu_jagged_attn_workspace_bytes(ctypes.byref(big), 0) > sizes[0]
    # batches of short sequences: schedules only
    short = _params(binding, batch=4096, total_rows=600000, d_qk=128, d_v=128)
    # (mean length <= 512: plus 8 bytes per row and two small schedules for the packed tiles)
    assert 0 < lib.hstu_jagged_attn_workspace_bytes(ctypes.byref(short), 0) < (4 << 20) + 8 * 600000 + (1 << 20)


def test_validate_offsets_host(lib):
    from paper_2508_04711_amd import binding
    assert binding.hstu_validate_offsets_host([0, 3, 3, 10], 10) == 0
    assert binding.hstu_validate_offsets_host([1, 3, 10], 10) == -2
    assert binding.hstu_validate_offsets_host([0, 5, 4, 10], 10) == -2
    assert binding.hstu_validate_offsets_host([0, 5, 9], 10) == -2


def test_tile_rows(lib):
    from paper_2508_04711_amd import binding
    for side in (0, 1):
        assert binding.hstu_schedule_tile_rows(0, 128, 128, side) % 32 == 0
        assert binding.hstu_schedule_tile_rows(1, 32, 32, side) > 0


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2508_04711_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libhstu_attn.so")
    with pytest.raises(RuntimeError):
        binding.load_library()


def test_static_scratch_forward_refuses_large_problems_on_the_host(lib):
    """The forward without workspace checks the size before any device call: a problem whose
    workspace exceeds the static array is refused with its own status, and the limit is exported."""
    from paper_2508_04711_amd import binding
    assert lib.hstu_static_scratch_bytes() == 16 << 20
    big = _params(binding, batch=8, num_heads=8, d_qk=128, d_v=128, max_len=32768, total_rows=96016)
    assert lib.hstu_jagged_attn_workspace_bytes(ctypes.byref(big), 0) > (16 << 20)
    one = ctypes.c_void_p(4096)  # never dereferenced: the size check comes first
    assert lib.hstu_jagged_attn_fwd_static(ctypes.byref(big), one, one, one, one, one, None) == -8
    assert b"static" in lib.hstu_attn_status_string(-8)
    bad = _params(binding, d_qk=48)
    assert lib.hstu_jagged_attn_fwd_static(ctypes.byref(bad), one, one, one, one, one, None) == -3
    empty = _params(binding, batch=0, total_rows=0)
    assert lib.hstu_jagged_attn_fwd_static(ctypes.byref(empty), None, None, None, None, None, None) == 0


def test_size_limits_are_those_of_the_pass_that_has_them(lib):
    """Only a forward pass that builds the transposed copy of V is limited to 131071 key tiles; the
    other passes, and batches of short sequences, take any size below 2^31 rows."""
    from paper_2508_04711_amd import binding
    ws = lambda p, which: lib.hstu_jagged_attn_workspace_bytes(ctypes.byref(p), which)
    # 131072 sequences of 40 rows: short sequences, no transposed copy anywhere
    many = _params(binding, batch=131072, num_heads=4, d_qk=128, d_v=128, max_len=64, total_rows=131072 * 40)
    assert ws(many, 0) > 0 and ws(many, 1) > 0
    # 9 million rows in 1000 long sequences: fine by default, out of range for the forward's transposed copy
    long = _params(binding, batch=1000, num_heads=1, d_qk=128, d_v=128, max_len=2000, total_rows=9_000_000)
    assert ws(long, 0) > 0 and ws(long, 1) > 0
    forced = _params(binding, batch=1000, num_heads=1, d_qk=128, d_v=128, max_len=2000, total_rows=9_000_000, flags=8)
    assert ws(forced, 0) == 0 and ws(forced, 1) > 0
    # just inside: (rows / 64 + batch + 1) tiles < 131072
    edge = _params(binding, batch=1000, num_heads=1, d_qk=128, d_v=128, max_len=2000, total_rows=64 * (131071 - 1001),
                   flags=8)
    assert ws(edge, 0) > 0
    over = _params(binding, batch=1000, num_heads=1, d_qk=128, d_v=128, max_len=2000, total_rows=64 * (131072 - 1001),
                   flags=8)
    assert ws(over, 0) == 0
