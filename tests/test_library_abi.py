"""CPU-side checks: the C-ABI library loads, exports what include/kda.h declares, and
rejects malformed calls without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    import paper_2510_26692_amd as kda
    if not os.path.exists(kda.library_path()):
        from paper_2510_26692_amd import build
        build.build(verbose=False)
    return kda, kda.load_library()


def test_every_declared_symbol_is_exported():
    kda, lib = _lib()
    header = open(os.path.join(ROOT, "include", "kda.h")).read() + open(os.path.join(ROOT, "include", "kda_debug.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(kda_[a-z_0-9]+)\s*\(", header))
    assert {"kda_chunk_fwd", "kda_recurrent_step", "kda_chunk_fwd_workspace_size",
            "kda_chunk_fwd_min_workspace_size", "kda_status_string", "kda_last_error",
            "kda_version", "kda_debug_set_producers", "kda_debug_set_wait_limit", "kda_debug_chunk_fwd_plan",
            "kda_chunk_fwd_check", "kda_recurrent_steps_pooled", "kda_chunk_fwd_fused",
            "kda_recurrent_steps_fused", "kda_chunk_fwd_fused_workspace_size",
            "kda_chunk_fwd_fused_min_workspace_size", "kda_debug_set_time_split",
            "kda_chunk_fwd_scalar_gate", "kda_recurrent_steps_pooled_scalar_gate"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_library_imports_no_allocating_or_stream_creating_runtime_call():
    """The boundary's conventions, checked on the built library itself: it allocates nothing, creates no
    stream or event and registers no host memory, so none of those runtime entry points may even be
    imported.  The only calls that wait for the device are hipStreamSynchronize and the blocking hipMemcpy
    of kda_chunk_fwd_check, which exists to wait."""
    import subprocess
    kda, _ = _lib()
    out = subprocess.run(["nm", "-D", "--undefined-only", kda.library_path()], check=True, capture_output=True, text=True).stdout
    imported = {ln.split()[-1].split("@")[0] for ln in out.splitlines() if ln.strip()}
    hip = {n for n in imported if n.startswith("hip")}
    assert "hipLaunchKernel" in hip
    banned = [n for n in hip if re.search(r"Malloc|Free|StreamCreate|EventCreate|HostRegister|HostAlloc|DeviceSynchronize|"
                                          r"EventSynchronize|Graph|MemPool|ModuleLoad", n)]
    assert not banned, banned
    assert hip <= {"hipLaunchKernel", "hipGetDevice", "hipDeviceGetAttribute", "hipFuncSetAttribute", "hipGetLastError",
                   "hipGetErrorString", "hipMemcpyAsync", "hipMemcpy", "hipStreamSynchronize", "hipGetSymbolAddress",
                   "hipPeekAtLastError"}, hip


def test_dims_struct_layout_matches_header():
    kda, _ = _lib()
    # int32, pad, int64, 4 x int32, int32, 2 x enum, float, pad, int64 -> 56 bytes on LP64
    assert ctypes.sizeof(kda.KdaDims) == 56
    assert kda.KdaDims.seqlen.offset == 8 and kda.KdaDims.max_seqlen.offset == 48


def _dims(kda, **kw):
    base = dict(batch=1, seqlen=128, heads=2, dk=128, dv=128, chunk=64, num_seqs=1, in_dtype=1,
                out_dtype=0, scale=1.0, max_seqlen=0)
    base.update(kw)
    return kda.KdaDims(**base)


def test_workspace_sizes_are_consistent():
    kda, lib = _lib()
    d = _dims(kda, batch=4, num_seqs=4, seqlen=4096, heads=16)
    full = kda.kda_chunk_fwd_workspace_size(d)
    small = kda.kda_chunk_fwd_min_workspace_size(d)
    assert full > small > 0 and full % 256 == 0
    # slots + one ready flag per slot, the fp32 state carry, the status word and the sequence order of packed calls
    # (256 + 1024 bytes, with alignment slack), and, for a call
    # of 64 pairs, the area of the time-split scan: 128 words for each of up to 64 pairs and three state arrays for
    # the two ranges such a call may be cut into
    slots = 4 * 16 * (4096 // 64)
    carry = 4 * 16 * 128 * 128 * 4
    fixed = full - slots * (72192 + 4) - carry - (64 * 128 * 4 + 3 * 2 * carry)
    assert 1280 <= fixed <= 1536
    # with the output gate: 16 KiB of staged gate logits per slot on top
    gated = kda.kda_chunk_fwd_workspace_size(d, output_gate=True)
    assert 0 <= gated - full - slots * 16384 < 256
    assert kda.kda_chunk_fwd_min_workspace_size(d, output_gate=True) > small
    assert lib.kda_chunk_fwd_fused_workspace_size(ctypes.byref(d), None) == full
    # fp32 path: two packed C x (C+2) tiles and three C x d operand tiles (+ d) per chunk and head for the
    # fast kernels, none at all for the single sequential kernel
    # (a single row may arrive with cu_seqlens: it is sized for the packed layout, one more slot per sequence)
    f32 = _dims(kda, in_dtype=0)
    n_ch = (f32.seqlen // 64 + f32.num_seqs) * f32.heads
    want = 4 * n_ch * (2 * 64 * 66 + 3 * 64 * f32.dk + f32.dk)
    assert 0 <= kda.kda_chunk_fwd_workspace_size(f32) - want < 2 * 256
    assert kda.kda_chunk_fwd_min_workspace_size(f32) == 0
    assert kda.kda_chunk_fwd_workspace_size(_dims(kda, dk=96, dv=96)) == 0        # unsupported
    assert kda.kda_chunk_fwd_workspace_size(_dims(kda, seqlen=0)) == 0


@pytest.mark.parametrize("kw,status", [
    (dict(dk=96, dv=96), 2), (dict(chunk=32), 2), (dict(out_dtype=1, in_dtype=0), 2), (dict(out_dtype=5), 1),
    (dict(seqlen=-1), 1),
    (dict(num_seqs=3), 1), (dict(in_dtype=7), 1),
])
def test_chunk_fwd_rejects_bad_dims_without_launching(kw, status):
    kda, lib = _lib()
    d = _dims(kda, **kw)
    fake = ctypes.c_void_p(0x1000)
    st = lib.kda_chunk_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, None, None,
                           ctypes.c_void_p(0x2000), None, None, 0, None)
    assert st == status, kda.kda_last_error()
    assert kda.kda_last_error() != ""
    assert kda.kda_status_string(st) not in ("ok", "unknown status")


def test_chunk_fwd_rejects_null_misaligned_and_missing_workspace():
    kda, lib = _lib()
    d = _dims(kda)
    fake = ctypes.c_void_p(0x1000)
    out = ctypes.c_void_p(0x2000)
    assert lib.kda_chunk_fwd(ctypes.byref(d), None, fake, fake, fake, fake, None, None, out, None,
                             None, 0, None) == 1
    assert lib.kda_chunk_fwd(ctypes.byref(d), ctypes.c_void_p(0x1008), fake, fake, fake, fake, None,
                             None, out, None, None, 0, None) == 1
    assert lib.kda_chunk_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, None, None, fake, None,
                             None, 0, None) == 1                                   # o aliases q
    assert lib.kda_chunk_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, None, None, out, None,
                             None, 0, None) == 3                                   # no workspace
    assert lib.kda_chunk_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, None, None, out, None,
                             ctypes.c_void_p(0x3010), 1 << 30, None) == 3          # misaligned
    assert lib.kda_chunk_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, None, None, out, None,
                             ctypes.c_void_p(0x3000), 1024, None) == 3             # too small
    packed = _dims(kda, batch=2, num_seqs=3)
    assert lib.kda_chunk_fwd(ctypes.byref(packed), fake, fake, fake, fake, fake, None, fake, out,
                             None, None, 0, None) == 1                             # packed needs B == 1


def test_chunk_bwd_workspace_size_and_rejections_without_launching():
    kda, lib = _lib()
    d = _dims(kda, batch=2, num_seqs=2)
    D, C = d.dk, 64

    def floats_for(chunks, tokens):
        return chunks * (2 * D * D + D + 2 * C * C + 2 * C * (C + 2) + 3 * C * D + D) + 3 * tokens * D
    chunks = d.num_seqs * ((d.seqlen + C - 1) // C) * d.heads
    tokens = d.batch * d.seqlen * d.heads
    need = kda.kda_chunk_bwd_workspace_size(d)
    assert 0 <= need - 4 * floats_for(chunks, tokens) < 9 * 256      # nine areas, each rounded up to 256 bytes
    # The size entry points never see cu_seqlens.  One row (B = N = 1) may be a packed batch of one
    # sequence, whose chunks are laid out at floor(T / C) + N slots, so it is sized for that layout:
    # the plan of either dispatch then fits what the library asked for.
    for T in (64, 128, 130, 4096):
        one = _dims(kda, seqlen=T)
        packed_slots = (T // C + 1) * one.heads
        plain_slots = ((T + C - 1) // C) * one.heads
        assert packed_slots >= plain_slots
        got = kda.kda_chunk_bwd_workspace_size(one)
        assert 0 <= got - 4 * floats_for(packed_slots, T * one.heads) < 9 * 256, T
        f32 = _dims(kda, seqlen=T, in_dtype=0)
        want = 4 * packed_slots * (2 * C * (C + 2) + 3 * C * D + D)
        assert 0 <= kda.kda_chunk_fwd_workspace_size(f32) - want < 2 * 256, T
    d = _dims(kda)
    need = kda.kda_chunk_bwd_workspace_size(d)
    assert kda.kda_chunk_bwd_workspace_size(_dims(kda, dk=96, dv=96)) == 0
    p = [ctypes.c_void_p(0x1000 * (i + 1)) for i in range(16)]

    def call(dims, q=p[0], d_o=p[5], dq=p[6], dk=p[7], ws=None, ws_bytes=0, cu=None):
        return lib.kda_chunk_bwd(ctypes.byref(dims), q, p[1], p[2], p[3], p[4], None, cu, d_o, None,
                                 dq, dk, p[8], p[9], p[10], None, ws, ws_bytes, None)
    assert call(d) == 3                                                   # no workspace
    assert call(d, ws=ctypes.c_void_p(0x100000), ws_bytes=need - 1) == 3  # too small
    assert call(d, ws=ctypes.c_void_p(0x100010), ws_bytes=need) == 3      # misaligned
    assert call(d, q=None) == 1
    assert call(d, d_o=None) == 1
    assert call(d, dq=p[0]) == 1                                          # gradient aliases an input
    assert call(d, dq=p[7]) == 1                                          # two gradients alias
    assert call(d, q=ctypes.c_void_p(0x1004)) == 1                        # misaligned tensor
    assert call(_dims(kda, dk=96, dv=96)) == 2
    assert call(_dims(kda, chunk=32)) == 2
    assert call(_dims(kda, batch=2, num_seqs=3), cu=p[11]) == 1           # packed needs B == 1
    too_long = _dims(kda, batch=1, num_seqs=1, seqlen=65536 * 64)
    assert call(too_long, ws=ctypes.c_void_p(0x100000), ws_bytes=1 << 62) == 2
    assert call(_dims(kda, seqlen=0)) == 0                                # nothing to do


def test_recurrent_step_rejects_bad_calls():
    kda, lib = _lib()
    d = _dims(kda, seqlen=2)
    fake = ctypes.c_void_p(0x1000)
    assert lib.kda_recurrent_step(ctypes.byref(d), fake, fake, fake, fake, fake, fake, fake, None) == 1
    d = _dims(kda, seqlen=1)
    assert lib.kda_recurrent_step(ctypes.byref(d), fake, fake, fake, fake, fake, None, fake, None) == 1
    d = _dims(kda, seqlen=1, dk=256, dv=256)
    assert lib.kda_recurrent_step(ctypes.byref(d), fake, fake, fake, fake, fake, fake, fake, None) == 2


def test_empty_problems_are_ok_and_launch_nothing():
    kda, lib = _lib()
    d = _dims(kda, heads=0)
    assert lib.kda_chunk_fwd(ctypes.byref(d), None, None, None, None, None, None, None, None, None,
                             None, 0, None) == 0
    d = _dims(kda, seqlen=1, batch=0, num_seqs=0)
    assert lib.kda_recurrent_step(ctypes.byref(d), None, None, None, None, None, None, None, None) == 0


def test_binding_fails_loudly_without_the_library(monkeypatch):
    import paper_2510_26692_amd.kda as binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libkda.so")
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        binding.load_library()


def test_bench_flop_model_matches_the_papers_formula():
    """bench.py's FLOP-per-token constant against the hand-evaluated values of the paper's
    formula (Section 6.3, "Training flops") stored in tests/golden/flops_model.txt."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_mod", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    rows = [tuple(int(x) for x in ln.split()) for ln in open(os.path.join(ROOT, "tests", "golden", "flops_model.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert rows
    for T, C, d, flops in rows:
        assert 6 * T * d * d + 3 * T * C * d + T * C * C == flops
    assert (1, 64, 128, bench.FLOP_PER_TOKHEAD) in rows
