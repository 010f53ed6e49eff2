"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every function include/mqa.h declares, and rejects bad arguments before
touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1911_02150_amd", "libmqa_decode.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="library not built (run __graft_entry__.build())")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mqa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(m[qh]a_[a-z_]+)\s*\(", text)))


def test_header_functions_are_exported():
    from paper_1911_02150_amd import binding
    lib = ctypes.CDLL(LIB)
    names = declared_functions()
    assert {"mqa_append_kv", "mqa_decode_step", "mha_decode_step", "mqa_project_qkvo"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in mqa.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_missing_library_fails_loudly(tmp_path, monkeypatch):
    from paper_1911_02150_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    with pytest.raises(OSError, match="no CPU or PyTorch fallback"):
        binding.load_library(str(tmp_path / "absent.so"))


def test_host_side_sizes_and_plan():
    import paper_1911_02150_amd as m
    assert m.mqa_decode_workspace_bytes(64, 32, 8192, 128) == 64 * 64 * 32 * 130 * 4 + 16 + 64 * 4
    assert m.mqa_decode_workspace_bytes(2, 3, 40, 8) == 2 * 2 * 3 * 10 * 4 + 16 + 2 * 4
    assert m.mha_decode_workspace_bytes(2, 3, 40, 8) == 2 * 2 * 3 * 10 * 4 + 16 + 6 * 4
    assert m.mqa_decode_workspace_bytes(0, 3, 40, 8) == 0
    assert m.mqa_decode_workspace_bytes(1, 32, 1 << 17, 128) == 256 * 32 * 130 * 4 + 16 + 4     # one sequence: up to 256 ranges
    assert m.mqa_decode_num_splits(1, 32, 1 << 17, 128, 128, m.MQA_BF16) == 256
    assert m.mqa_decode_num_splits(128, 8, 128, 128, 128, m.MQA_BF16) == 1          # short caches: one range
    assert m.mqa_decode_num_splits(64, 32, 8192, 128, 128, m.MQA_BF16) > 1          # long cache: split
    assert m.mqa_decode_num_splits(64, 32, 8192, 128, 128, m.MQA_BF16, tuning=dict(splits=5)) == 5
    assert m.mqa_decode_num_splits(1, 8, 64, 128, 128, m.MQA_BF16, tuning=dict(splits=9)) == 2   # at most cap/32
    assert m.mqa_decode_num_splits(4, 8, 64, 64, 64, m.MQA_BF16, tuning=dict(kernel=2)) == -2    # MFMA kernel needs k=v=128
    assert m.status_string(0) == "ok" and "workspace" in m.status_string(4)
    # the whole plan, and exactly what the default plan of a shape uses
    assert m.mqa_decode_plan(64, 32, 8192, 128, 128, m.MQA_BF16) == (4, 2048, 1)
    assert m.mqa_decode_plan(512, 64, 4096, 128, 128, m.MQA_BF16) == (1, 4096, 1)          # 64 heads per workgroup
    assert m.mqa_decode_plan(512, 64, 4096, 128, 128, m.MQA_BF16, tuning=dict(flags=8)) == (1, 4096, 2)
    assert m.mqa_decode_plan(1, 8, 4096, 128, 128, m.MQA_BF16, window=1024) == (9, 128, 1)
    assert m.mqa_decode_plan(2, 8, 64, 128, 128, m.MQA_BF16, multi_head=True)[0] == 1
    assert m.mqa_decode_workspace_bytes_default(64, 32, 8192, 128, 128, m.MQA_BF16) == 64 * 32 * 4 * 130 * 4 + 64 * 4
    assert m.mqa_decode_workspace_bytes_default(512, 64, 4096, 128, 128, m.MQA_BF16) == 512 * 4
    assert m.mqa_decode_workspace_bytes_default(64, 32, 8192, 128, 128, m.MQA_BF16) <= m.mqa_decode_workspace_bytes(64, 32, 8192, 128)
    assert m.mqa_decode_workspace_bytes_default(2, 4, 64, 128, 128, m.MQA_BF16, multi_head=True) == 8 * 4


def test_argument_validation_without_gpu():
    lib = ctypes.CDLL(LIB)
    vp = ctypes.c_void_p
    A = vp(0x10000)          # non-null, aligned; never dereferenced on these paths
    U = vp(0x10004)          # misaligned
    dec = lib.mqa_decode_step
    dec.argtypes = [vp] * 5 + [ctypes.c_int] * 6 + [ctypes.c_float, vp, ctypes.c_size_t, vp]
    ok = dict(b=2, h=4, cap=4096, k=128, v=128, dt=1)

    def call(q=A, K=A, V=A, lens=A, o=A, ws=A, wsb=1 << 30, **kw):
        a = dict(ok, **kw)
        return dec(q, K, V, lens, o, a["b"], a["h"], a["cap"], a["k"], a["v"], a["dt"], 1.0, ws, wsb, None)

    assert call(q=None) == 1 and call(lens=None) == 1 and call(o=None) == 1
    assert call(b=0) == 2 and call(h=-1) == 2 and call(k=12) == 2 and call(v=264) == 2 and call(cap=0) == 2
    assert call(K=U) == 3 and call(o=U) == 3
    assert call(dt=7) == 5
    assert call(ws=None) == 4 and call(wsb=16) == 4            # this shape needs a split, hence a workspace
    mha = lib.mha_decode_step
    mha.argtypes = dec.argtypes
    assert mha(A, A, None, A, A, 2, 4, 64, 128, 128, 1, 1.0, A, 1 << 20, None) == 1

    app = lib.mqa_append_kv
    app.argtypes = [vp] * 5 + [ctypes.c_int] * 6 + [vp]
    assert app(A, A, A, None, A, 2, 1, 8, 128, 128, 1, None) == 1
    assert app(A, A, A, A, A, 2, 0, 8, 128, 128, 1, None) == 2
    assert app(A, A, A, A, A, 2, 1, 8, 100, 128, 1, None) == 2
    assert app(A, U, A, A, A, 2, 1, 8, 128, 128, 1, None) == 3
    assert app(A, A, A, A, A, 2, 1, 8, 128, 128, 3, None) == 5

    prj = lib.mqa_project_qkvo
    prj.argtypes = [ctypes.c_int, vp, vp, vp] + [ctypes.c_int] * 4 + [vp]
    assert prj(0, None, A, A, 4, 64, 2, 16, None) == 1
    assert prj(9, A, A, A, 4, 64, 2, 16, None) == 5 and prj(5, A, A, A, 4, 64, 2, 16, None) == 5
    assert prj(4, A, A, U, 4, 64, 0, 16, None) == 3          # LINEAR ignores h
    assert prj(0, A, A, A, 4, 60, 2, 16, None) == 2
    assert prj(3, A, A, U, 4, 64, 2, 16, None) == 3

    na = lib.mqa_decode_step_noalloc
    na.argtypes = [vp] * 5 + [ctypes.c_int] * 6 + [ctypes.c_float, vp]
    assert na(A, A, A, A, None, 2, 4, 64, 128, 128, 1, 1.0, None) == 1
    assert na(A, A, A, A, A, 2, 4, 64, 12, 128, 1, 1.0, None) == 2
    assert na(A, U, A, A, A, 2, 4, 64, 128, 128, 1, 1.0, None) == 3
    assert na(A, A, A, A, A, 5_000_000, 1, 32, 128, 128, 1, 1.0, None) == 7   # the length schedule alone outgrows the static buffer

    mem = lib.mqa_project_memory_kv
    mem.argtypes = [vp] * 7 + [ctypes.c_int] * 8 + [vp]
    assert mem(A, A, A, A, A, None, A, 2, 64, 128, 1, 64, 128, 128, 1, None) != 1      # mem_lens may be NULL
    assert mem(A, A, None, A, A, None, A, 2, 64, 128, 1, 64, 128, 128, 1, None) == 1
    assert mem(A, A, A, A, A, None, A, 2, 65, 128, 1, 64, 128, 128, 1, None) == 2      # memory longer than the cache
    assert mem(A, A, A, A, A, U, A, 2, 64, 128, 1, 64, 128, 128, 1, None) == 3
    md = lib.mqa_memory_decode_step
    md.argtypes = [vp] * 5 + [ctypes.c_int] * 7 + [ctypes.c_float, vp, ctypes.c_size_t, vp]
    assert md(A, A, A, A, A, 2, 0, 8, 64, 128, 128, 1, 1.0, None, 0, None) == 2
    assert md(A, A, None, A, A, 2, 4, 8, 64, 128, 128, 1, 1.0, None, 0, None) == 1

    rd = lib.mqa_stream_read
    rd.argtypes = [vp, ctypes.c_size_t, vp, vp]
    assert rd(A, 24, A, None) == 2 and rd(None, 32, A, None) == 1


def test_beam_entry_points_validate_without_gpu():
    import paper_1911_02150_amd as m
    lib = ctypes.CDLL(LIB)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    A, U = vp(0x10000), vp(0x10004)
    step = lib.mqa_decode_step_beams
    step.argtypes = [vp] * 8 + [ci] * 8 + [ctypes.c_float, vp, ctypes.c_size_t, vp]
    need = m.mqa_decode_beams_workspace_bytes(8, 4, 8, 4096, 128, 128, 128, m.MQA_BF16)
    # 8 sources x ceil(32 rows / 32) head groups -> 32 ranges over the source, one over the own rows
    assert need == 8 * 4 * 8 * (32 + 1) * 130 * 4
    assert m.mqa_decode_beams_workspace_bytes(8, 0, 8, 4096, 128, 128, 128, m.MQA_BF16) == 0

    def call(ptrs=None, sizes=(8, 4, 8, 4096, 128, 128, 128, 1), ws=A, wsb=need):
        ptrs = ptrs or [A] * 8
        return step(*ptrs, *sizes, 1.0, ws, wsb, None)

    assert call(ptrs=[A] * 3 + [vp(0)] + [A] * 4) == 1
    assert call(sizes=(8, 4, 8, 4096, 128, 128, 132, 1)) == 2
    assert call(sizes=(8, 4, 8, 4096, 128, 128, 128, 7)) == 5
    assert call(ptrs=[A] * 4 + [U] + [A] * 3) == 3
    assert call(wsb=need - 1) == 4 and call(ws=vp(0)) == 4
    re = lib.mqa_beam_reorder_kv
    re.argtypes = [vp] * 7 + [ci] * 6 + [vp]
    B = vp(0x20000)
    assert re(A, A, A, A, B, B, vp(0), 4, 1, 64, 128, 128, 1, None) == 1
    assert re(A, A, A, A, A, B, B, 4, 1, 64, 128, 128, 1, None) == 2          # in place is refused
    assert re(A, A, A, A, B, B, B, 4, 1, 64, 128, 124, 1, None) == 2
    assert re(A, A, A, U, B, B, B, 4, 1, 64, 128, 128, 1, None) == 3
    assert re(A, A, A, A, B, B, B, 4, 1, 64, 128, 128, 3, None) == 5


def test_header_is_plain_c(tmp_path):
    """include/mqa.h must be usable from C: compile a translation unit that takes the address of
    every declared function, as C99 with warnings as errors."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    names = declared_functions()
    src = tmp_path / "use_mqa.c"
    src.write_text('#include "mqa.h"\n' + "void* table[] = {" + ", ".join(f"(void*){n}" for n in names) + "};\n"
                   "int main(void) { mqa_tuning t = {0, 0, 0}; return (int)(t.splits + MQA_OK + MQA_PROJ_O - 3 + MQA_EPI_STORE); }\n")
    inc = os.path.join(ROOT, "include")
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-Wno-pedantic", "-I", inc, "-c", str(src), "-o",
                        str(tmp_path / "use_mqa.o")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
