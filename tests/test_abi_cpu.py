"""The C-ABI library on a machine without a GPU: it loads, exports every declared symbol,
and rejects bad arguments before any launch (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tokenring.h")


@pytest.fixture(scope="module")
def tr():
    from paper_2412_20501_amd.build import ensure_built
    ensure_built()          # hipcc cross-compiles without a GPU; an existing library is used as it is
    import paper_2412_20501_amd as m
    m.raw_lib()
    return m


def _t(tr, dtype, B, H, S, D, ptr=0x7F0000000000, strides=None):
    sb, sh, ss = strides if strides else (H * S * D, S * D, D)
    return tr.TrTensor(ptr, dtype, B, H, S, D, sb, sh, ss)


def test_every_declared_symbol_is_exported(tr):
    text = open(HEADER).read()
    names = set(re.findall(r"\b(tr_[a-z_]+)\s*\(", text))
    assert {"tr_block_attn", "tr_block_attn_causal_at", "tr_block_attn_merge", "tr_merge", "tr_merge_n", "tr_ring_attn", "tr_ring_attn_blocks", "tr_ring_attn_noalloc", "tr_ring_attn_blocks_workspace_bytes", "tr_ring_attn_sched", "tr_schedule_steps",
            "tr_ring_attn_workspace_bytes", "tr_time_next_kernel", "tr_last_error", "tr_version"} <= names
    lib = ctypes.CDLL(tr.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in tokenring.h but not exported"
    assert tr.tr_version().startswith("tokenring-gfx950")


def test_struct_layout_matches_header(tr):
    assert ctypes.sizeof(tr.TrTensor) == 8 + 8 + 7 * 8      # ptr, dtype (+pad), 7 x int64
    assert tr.TrTensor.B.offset == 16 and tr.TrTensor.stride_s.offset == 64


def _status(tr, fn, *args):
    st = fn(*args)
    return st, tr.raw_lib().tr_last_error().decode()


def test_block_attn_rejects_bad_arguments(tr):
    lib = tr.raw_lib()
    q = _t(tr, tr.TR_BF16, 1, 4, 128, 128); k = _t(tr, tr.TR_BF16, 1, 2, 128, 128, ptr=0x7F1000000000)
    v = _t(tr, tr.TR_BF16, 1, 2, 128, 128, ptr=0x7F2000000000)
    o = _t(tr, tr.TR_F32, 1, 4, 128, 128, ptr=0x7F3000000000); l = _t(tr, tr.TR_F32, 1, 4, 128, 1, ptr=0x7F4000000000)
    B = ctypes.byref
    call = lambda q=q, k=k, v=v, m=0, s=0.1, o=o, l=l: _status(tr, lib.tr_block_attn, B(q), B(k), B(v), m, s, B(o), B(l), None)
    assert call(q=_t(tr, tr.TR_BF16, 1, 4, 128, 128, ptr=None))[0] == 1                     # NULL data
    assert lib.tr_block_attn(None, B(k), B(v), 0, 0.1, B(o), B(l), None) == 1              # NULL descriptor
    assert call(q=_t(tr, tr.TR_F32, 1, 4, 128, 128))[0] == 2                                # q must be bf16
    assert call(l=_t(tr, tr.TR_BF16, 1, 4, 128, 1, ptr=0x7F4000000000))[0] == 2             # lse must be fp32
    st, msg = call(q=_t(tr, tr.TR_BF16, 1, 4, 128, 96), o=_t(tr, tr.TR_F32, 1, 4, 128, 96, ptr=0x7F3000000000))
    assert st == 3 and "head dim" in msg
    assert call(k=_t(tr, tr.TR_BF16, 1, 3, 128, 128, ptr=0x7F1000000000), v=_t(tr, tr.TR_BF16, 1, 3, 128, 128, ptr=0x7F2000000000))[0] == 3   # 4 % 3
    assert call(v=_t(tr, tr.TR_BF16, 1, 2, 64, 128, ptr=0x7F2000000000))[0] == 3            # k/v length differ
    assert call(o=_t(tr, tr.TR_F32, 1, 4, 127, 128, ptr=0x7F3000000000))[0] == 3            # out shape
    assert call(m=1, k=_t(tr, tr.TR_BF16, 1, 2, 64, 128, ptr=0x7F1000000000), v=_t(tr, tr.TR_BF16, 1, 2, 64, 128, ptr=0x7F2000000000))[0] == 3  # diag needs Sq == Sk
    assert call(m=7)[0] == 6                                                                # unknown mask
    assert call(s=0.0)[0] == 6 and call(s=float("nan"))[0] == 6                             # scale
    assert call(q=_t(tr, tr.TR_BF16, 1, 4, 128, 128, strides=(4 * 128 * 128, 128 * 128, 100)))[0] == 4   # stride_s < D
    assert call(q=_t(tr, tr.TR_BF16, 1, 4, 128, 128, strides=(4 * 128 * 132, 128 * 132, 132)))[0] == 4   # rows not 16-byte multiples
    assert call(q=_t(tr, tr.TR_BF16, 1, 4, 128, 128, ptr=0x7F0000000002))[0] == 4           # misaligned pointer
    big = (1 << 24) + 8                                                                     # K/V row stride beyond the staging offsets
    st, msg = call(k=_t(tr, tr.TR_BF16, 1, 2, 128, 128, ptr=0x7F1000000000, strides=(2 * 128 * big, 128 * big, big)))
    assert st == 4 and "2^24" in msg
    assert call(o=_t(tr, tr.TR_F32, 1, 4, 128, 128, ptr=0x7F0000000000))[0] == 5            # out aliases q
    assert lib.tr_block_attn_causal_at(B(q), B(k), B(v), -1, 0, 0.1, B(o), B(l), None) == 3
    # the fused form merges into fp32 accumulators only
    ob = _t(tr, tr.TR_BF16, 1, 4, 128, 128, ptr=0x7F3000000000)
    assert lib.tr_block_attn_merge(B(q), B(k), B(v), 0, 0.1, B(ob), B(l), None) == 2
    assert lib.tr_block_attn_merge(B(q), B(k), B(v), 9, 0.1, B(o), B(l), None) == 6


def test_merge_rejects_bad_arguments(tr):
    lib = tr.raw_lib()
    B = ctypes.byref
    ao = _t(tr, tr.TR_F32, 1, 2, 64, 128); al = _t(tr, tr.TR_F32, 1, 2, 64, 1, ptr=0x7F1000000000)
    bo = _t(tr, tr.TR_F32, 1, 2, 64, 128, ptr=0x7F2000000000); bl = _t(tr, tr.TR_F32, 1, 2, 64, 1, ptr=0x7F3000000000)
    call = lambda ao=ao, al=al, bo=bo, bl=bl: _status(tr, lib.tr_merge, B(ao), B(al), B(bo), B(bl), None)
    assert call(ao=_t(tr, tr.TR_BF16, 1, 2, 64, 128))[0] == 2                               # accumulator must be fp32
    assert call(bl=_t(tr, tr.TR_BF16, 1, 2, 64, 1, ptr=0x7F3000000000))[0] == 2
    assert call(bo=_t(tr, tr.TR_F32, 1, 2, 63, 128, ptr=0x7F2000000000))[0] == 3
    assert call(al=_t(tr, tr.TR_F32, 1, 2, 64, 2, ptr=0x7F1000000000))[0] == 3
    assert call(ao=_t(tr, tr.TR_F32, 1, 2, 64, 6), bo=_t(tr, tr.TR_F32, 1, 2, 64, 6, ptr=0x7F2000000000))[0] in (3, 4)   # D % 4
    st, msg = call(bo=_t(tr, tr.TR_F32, 1, 2, 64, 128, ptr=0x7F0000000100))
    assert st == 5 and "overlap" in msg                                                     # block aliases accumulator
    assert lib.tr_merge(None, B(al), B(bo), B(bl), None) == 1


def test_ring_attn_rejects_bad_arguments_and_workspace_size(tr):
    lib = tr.raw_lib()
    B = ctypes.byref
    q = _t(tr, tr.TR_BF16, 1, 32, 32768, 128); k = _t(tr, tr.TR_BF16, 1, 32, 32768, 128, ptr=0x7F1000000000)
    v = _t(tr, tr.TR_BF16, 1, 32, 32768, 128, ptr=0x7F2000000000)
    o = _t(tr, tr.TR_F32, 1, 32, 32768, 128, ptr=0x7F3000000000); l = _t(tr, tr.TR_F32, 1, 32, 32768, 1, ptr=0x7F5000000000)
    need = lib.tr_ring_attn_workspace_bytes(B(q), 8)
    assert need == 32 * 4096 * 128 * 4 + 32 * 4096 * 4            # one fp32 block_out + block_lse
    assert lib.tr_ring_attn_workspace_bytes(B(q), 7) == 0 and lib.tr_ring_attn_workspace_bytes(None, 8) == 0
    ws = 0x7F7000000000
    call = lambda q=q, k=k, v=v, n=8, o=o, l=l, ws=ws, nb=need: _status(
        tr, lib.tr_ring_attn, B(q), B(k), B(v), n, 1, B(o), B(l), 0.0, ws, nb, None)
    assert call(n=0)[0] == 3 and call(n=7)[0] == 3                                          # S % n_chunks
    assert call(o=_t(tr, tr.TR_BF16, 1, 32, 32768, 128, ptr=0x7F3000000000))[0] == 2         # out must be fp32
    assert call(k=_t(tr, tr.TR_BF16, 1, 32, 4096, 128, ptr=0x7F1000000000))[0] == 3
    assert call(nb=need - 1)[0] == 7 and call(ws=ws + 16)[0] == 7 and call(nb=0)[0] == 7      # (ws = NULL selects the fused form)
    st, msg = call(ws=0x7F3000000000)
    assert st == 5 and "workspace" in msg


def test_merge_n_and_sched_reject_bad_arguments(tr):
    lib = tr.raw_lib()
    B = ctypes.byref
    P = ctypes.POINTER(tr.TrTensor)
    o = _t(tr, tr.TR_F32, 1, 2, 64, 128); l = _t(tr, tr.TR_F32, 1, 2, 64, 1, ptr=0x7F1000000000)
    bo = [_t(tr, tr.TR_F32, 1, 2, 64, 128, ptr=0x7F2000000000 + i * 0x10000000) for i in range(3)]
    bl = [_t(tr, tr.TR_F32, 1, 2, 64, 1, ptr=0x7F4000000000 + i * 0x10000000) for i in range(3)]
    arr = lambda ts: (P * len(ts))(*[ctypes.pointer(t) for t in ts])
    call = lambda o=o, l=l, bo=bo, bl=bl, n=3: _status(tr, lib.tr_merge_n, B(o), B(l), arr(bo), arr(bl), n, 0, None)
    assert call(n=0)[0] == 3 and call(n=17)[0] == 3
    assert call(o=_t(tr, tr.TR_BF16, 1, 2, 64, 128))[0] == 2
    assert call(bo=bo[:2] + [_t(tr, tr.TR_BF16, 1, 2, 64, 128, ptr=0x7F6000000000)])[0] == 2          # mixed dtypes
    assert call(bo=bo[:2] + [_t(tr, tr.TR_F32, 1, 2, 64, 128, ptr=0x7F6000000000, strides=(2 * 64 * 256, 64 * 256, 256))])[0] == 4
    assert call(bo=bo[:2] + [_t(tr, tr.TR_F32, 1, 2, 63, 128, ptr=0x7F6000000000)])[0] == 3
    assert call(bo=bo[:2] + [_t(tr, tr.TR_F32, 1, 2, 64, 128, ptr=0x7F0000000040)])[0] == 5            # aliases out
    assert lib.tr_merge_n(B(o), B(l), None, arr(bl), 3, 0, None) == 1

    q = _t(tr, tr.TR_BF16, 1, 4, 4096, 128); k = _t(tr, tr.TR_BF16, 1, 4, 4096, 128, ptr=0x7F1000000000)
    v = _t(tr, tr.TR_BF16, 1, 4, 4096, 128, ptr=0x7F2000000000)
    oo = _t(tr, tr.TR_F32, 1, 4, 4096, 128, ptr=0x7F3000000000); ll = _t(tr, tr.TR_F32, 1, 4, 4096, 1, ptr=0x7F5000000000)
    sched = lambda n=8, causal=1, s=0, inner=1, oo=oo: _status(tr, lib.tr_ring_attn_sched, B(q), B(k), B(v), n, causal, s, inner, B(oo), B(ll), 0.0, None)
    assert sched(s=7)[0] == 6 and sched(s=-1)[0] == 6
    assert sched(s=tr.TR_SCHED_ZIGZAG, causal=0)[0] == 6                                               # zigzag is causal only
    assert sched(s=tr.TR_SCHED_HYBRID, inner=3)[0] == 3 and sched(s=tr.TR_SCHED_HYBRID, inner=0)[0] == 3
    assert sched(n=0)[0] == 3 and sched(n=3)[0] == 3                                                   # 4096 % 3
    assert sched(n=24, s=tr.TR_SCHED_ZIGZAG)[0] == 3                                                   # 4096 % 48
    assert sched(oo=_t(tr, tr.TR_BF16, 1, 4, 4096, 128, ptr=0x7F3000000000))[0] == 2


def test_written_tensors_must_not_overlap_themselves(tr):
    """A zero or too small stride on a written tensor would let two waves update one element."""
    lib = tr.raw_lib()
    B = ctypes.byref
    q = _t(tr, tr.TR_BF16, 1, 4, 128, 128); k = _t(tr, tr.TR_BF16, 1, 4, 128, 128, ptr=0x7F1000000000)
    v = _t(tr, tr.TR_BF16, 1, 4, 128, 128, ptr=0x7F2000000000)
    o = _t(tr, tr.TR_F32, 1, 4, 128, 128, ptr=0x7F3000000000); l = _t(tr, tr.TR_F32, 1, 4, 128, 1, ptr=0x7F4000000000)
    o_h0 = _t(tr, tr.TR_F32, 1, 4, 128, 128, ptr=0x7F3000000000, strides=(4 * 128 * 128, 0, 128))       # heads on top of each other
    l_h0 = _t(tr, tr.TR_F32, 1, 4, 128, 1, ptr=0x7F4000000000, strides=(4 * 128, 0, 1))
    o_short = _t(tr, tr.TR_F32, 1, 4, 128, 128, ptr=0x7F3000000000, strides=(4 * 128 * 128, 64 * 128, 128))  # head stride < S*D
    for bad_o, bad_l in ((o_h0, l), (o, l_h0), (o_short, l)):
        st, msg = _status(tr, lib.tr_block_attn, B(q), B(k), B(v), 0, 0.1, B(bad_o), B(bad_l), None)
        assert st == 4 and "overlap itself" in msg
        assert lib.tr_block_attn_merge(B(q), B(k), B(v), 0, 0.1, B(bad_o), B(bad_l), None) == 4
        assert lib.tr_ring_attn(B(q), B(k), B(v), 2, 0, B(bad_o), B(bad_l), 0.0, None, 0, None) == 4
        assert lib.tr_ring_attn_sched(B(q), B(k), B(v), 2, 0, 0, 1, B(bad_o), B(bad_l), 0.0, None) == 4
    bo = _t(tr, tr.TR_F32, 1, 4, 128, 128, ptr=0x7F5000000000); bl = _t(tr, tr.TR_F32, 1, 4, 128, 1, ptr=0x7F6000000000)
    assert lib.tr_merge(B(o_h0), B(l), B(bo), B(bl), None) == 4
    assert lib.tr_merge(B(o), B(l_h0), B(bo), B(bl), None) == 4
    P = ctypes.POINTER(tr.TrTensor)
    assert lib.tr_merge_n(B(o_h0), B(l), (P * 1)(ctypes.pointer(bo)), (P * 1)(ctypes.pointer(bl)), 1, 0, None) == 4
    # a token-major layout (the paper's (N, H, D)) is no overlap: stride_h = D, stride_s = H*D
    o_tm = _t(tr, tr.TR_F32, 1, 4, 0, 128, ptr=0x7F3000000000, strides=(0, 128, 4 * 128))
    l_tm = _t(tr, tr.TR_F32, 1, 4, 0, 1, ptr=0x7F4000000000, strides=(0, 1, 4))
    q0 = _t(tr, tr.TR_BF16, 1, 4, 0, 128)
    assert lib.tr_block_attn(B(q0), B(k), B(v), 0, 0.1, B(o_tm), B(l_tm), None) == 0      # Sq = 0: validated, nothing launched


def test_bf16_partials_need_d_multiple_of_4_only(tr):
    """tr_merge and tr_merge_n read bf16 partials four elements at a time: one rule for both (empty S: no launch)."""
    lib = tr.raw_lib()
    B = ctypes.byref
    P = ctypes.POINTER(tr.TrTensor)
    for D, ok in ((12, True), (20, True), (6, False), (10, False)):
        ao = _t(tr, tr.TR_F32, 1, 2, 0, D); al = _t(tr, tr.TR_F32, 1, 2, 0, 1, ptr=0x7F1000000000)
        bo = _t(tr, tr.TR_BF16, 1, 2, 0, D, ptr=0x7F2000000000); bl = _t(tr, tr.TR_F32, 1, 2, 0, 1, ptr=0x7F3000000000)
        st_pair = lib.tr_merge(B(ao), B(al), B(bo), B(bl), None)
        st_n = lib.tr_merge_n(B(ao), B(al), (P * 1)(ctypes.pointer(bo)), (P * 1)(ctypes.pointer(bl)), 1, 0, None)
        assert (st_pair == 0) == ok and (st_n == 0) == ok, (D, st_pair, st_n)
        assert st_pair == st_n


def test_library_is_rebuilt_when_a_source_changes(tr, tmp_path, monkeypatch):
    """The library carries the hash of its sources; ensure_built() compares it with the sources on disk."""
    import shutil
    from paper_2412_20501_amd import build
    assert build.library_hash() == build.source_hash()
    assert build.source_hash() in tr.tr_version()
    # the same check against a copy of the sources with one byte changed: the hashes differ, so a build is due
    csrc = tmp_path / "csrc"
    shutil.copytree(build.CSRC, csrc)
    with open(csrc / "merge.hip", "a") as f:
        f.write("// touched\n")
    monkeypatch.setattr(build, "CSRC", str(csrc))
    assert build.source_hash() != build.library_hash()
    calls = []
    monkeypatch.setattr(build, "build_library", lambda verbose=False: calls.append(1) or build.LIB_PATH)
    build.ensure_built()
    assert calls == [1]


def test_noalloc_ring_rejects_oversize_before_touching_a_device(tr):
    lib = tr.raw_lib()
    B = ctypes.byref
    q = _t(tr, tr.TR_BF16, 1, 32, 32768, 128); k = _t(tr, tr.TR_BF16, 1, 32, 32768, 128, ptr=0x7F1000000000)
    v = _t(tr, tr.TR_BF16, 1, 32, 32768, 128, ptr=0x7F2000000000)
    o = _t(tr, tr.TR_F32, 1, 32, 32768, 128, ptr=0x7F3000000000); l = _t(tr, tr.TR_F32, 1, 32, 32768, 1, ptr=0x7F5000000000)
    st, msg = _status(tr, lib.tr_ring_attn_noalloc, B(q), B(k), B(v), 8, 1, B(o), B(l), 0.0, None)
    assert st == 7 and "scratch" in msg and "workspace" in msg
    assert lib.tr_ring_attn_noalloc(None, B(k), B(v), 8, 1, B(o), B(l), 0.0, None) == 1
    text = open(HEADER).read()
    assert "#define TR_NOALLOC_SCRATCH_BYTES (8 * 1024 * 1024 + 64 * 1024)" in text


def test_header_and_library_work_from_plain_c(tr, tmp_path):
    """include/tokenring.h compiles as strict C99 and a C program linked against the library gets the
    documented status codes (validation only; nothing is launched)."""
    import subprocess
    src = os.path.join(ROOT, "tests", "c_abi", "abi_check.c")
    exe = str(tmp_path / "abi_check")
    lib_dir = os.path.dirname(tr.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), src,
                    "-L", lib_dir, "-ltokenring", "-Wl,-rpath," + lib_dir, "-o", exe], check=True, capture_output=True, text=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0 and "c abi ok" in res.stdout, res.stdout + res.stderr


def test_binding_fails_loudly_without_library(tmp_path, monkeypatch):
    """No fallback: a missing libtokenring.so is an ImportError, not a silent CPU path."""
    import importlib
    import paper_2412_20501_amd._binding as b
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        b._load()
    importlib.reload(b)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU's share of the path; any other --gpus value ends with a message, before torch is touched."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert res.returncode == 2 and "single-GPU" in res.stderr and res.stdout.strip() == ""
