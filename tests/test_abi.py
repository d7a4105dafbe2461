"""The C-ABI library loads, exports every symbol the header declares, and rejects bad
arguments on the host before touching the GPU (so these run without one)."""
import ctypes
import os
import re

import pytest

from paper_2512_17077_amd import hcsa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "dllm_hcsa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dllm_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = hcsa.lib()
    names = header_symbols()
    assert set(names) == set(hcsa.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None
    assert L.dllm_hcsa_version() >= 100
    assert hcsa.last_error() == "" or isinstance(hcsa.last_error(), str)


def test_select_form_setter_returns_the_previous_form_and_rejects_unknown_values():
    L = hcsa.lib()
    first = L.dllm_hcsa_set_select_form(hcsa.DLLM_SELECT_FORM_ONE_LAUNCH)
    try:
        assert first in (hcsa.DLLM_SELECT_FORM_AUTO, hcsa.DLLM_SELECT_FORM_TWO_LAUNCHES, hcsa.DLLM_SELECT_FORM_ONE_LAUNCH)
        assert L.dllm_hcsa_set_select_form(hcsa.DLLM_SELECT_FORM_TWO_LAUNCHES) == hcsa.DLLM_SELECT_FORM_ONE_LAUNCH
        assert L.dllm_hcsa_set_select_form(7) == -1 and L.dllm_hcsa_set_select_form(-1) == -1
        assert L.dllm_hcsa_set_select_form(hcsa.DLLM_SELECT_FORM_AUTO) == hcsa.DLLM_SELECT_FORM_TWO_LAUNCHES   # unchanged by the rejects
        with pytest.raises(ValueError):
            hcsa.dllm_hcsa_set_select_form(3)
    finally:
        L.dllm_hcsa_set_select_form(first)


def good_batch():
    b = hcsa.DllmBatch()
    b.dtype = hcsa.DLLM_BF16
    b.batch, b.n_q_heads, b.n_kv_heads, b.head_dim = 2, 8, 2, 128
    b.q = b.k = b.v = 0x10000            # never dereferenced: these calls fail before any launch
    b.q_stride_tok, b.q_stride_head = 8 * 128, 128
    b.kv_stride_tok, b.kv_stride_head = 2 * 128, 128
    b.cu_q = b.cu_kv = 0x20000
    b.total_q, b.total_kv, b.max_q, b.max_kv = 64, 500, 32, 300
    b.softmax_scale = 0.088
    return b


FAKE = ctypes.c_void_p(0x30000)


def shaped_batch(batch, hq, hkv, d, total_kv, max_kv, dtype=None):
    b = good_batch()
    b.dtype = hcsa.DLLM_BF16 if dtype is None else dtype
    b.batch, b.n_q_heads, b.n_kv_heads, b.head_dim = batch, hq, hkv, d
    b.q_stride_tok, b.q_stride_head = hq * d, d
    b.kv_stride_tok, b.kv_stride_head = hkv * d, d
    b.total_q, b.max_q = 32 * batch, 32
    b.total_kv, b.max_kv = total_kv, max_kv
    return b


def test_which_form_selection_takes_follows_the_documented_rule():
    """Host logic only (no GPU: 256 compute units are assumed).  One launch needs per-head selection, at most four
    query heads per KV head, rows of at most 256 bytes, lists of at most 8192, (sequence, KV head) pairs that fill
    the compute units in whole rounds or nearly, and a fairly even batch; the setter overrides the size rule only."""
    ONE, TWO = hcsa.DLLM_SELECT_FORM_ONE_LAUNCH, hcsa.DLLM_SELECT_FORM_TWO_LAUNCHES
    form = lambda b, pool_w=1, head_sum=False: hcsa.dllm_hcsa_select_form_of(b, pool_w, head_sum)
    assert hcsa.lib().dllm_hcsa_set_select_form(hcsa.DLLM_SELECT_FORM_AUTO) >= 0
    try:
        c5 = shaped_batch(32, 32, 8, 128, 24 * 8192 + 8 * 2048, 8192)        # the mixed grouped-query burst: 256 pairs
        assert form(c5) == ONE and form(c5, pool_w=3) == ONE and form(c5, head_sum=True) == TWO
        c3 = shaped_batch(16, 32, 32, 128, 34482, 3411)                       # ragged: mean length 63 % of the longest
        assert form(c3) == TWO
        assert form(shaped_batch(16, 32, 32, 128, 16 * 3411, 3411)) == ONE    # the same, even: two full rounds
        assert form(shaped_batch(4, 32, 8, 128, 4 * 8192, 8192)) == TWO       # 32 pairs: most compute units idle
        assert form(shaped_batch(1, 4, 4, 64, 256, 256, hcsa.DLLM_F32)) == ONE   # tiny: launch latency only
        assert form(shaped_batch(1, 32, 32, 128, 1024, 1024)) == TWO          # one layer-sized sequence
        assert form(shaped_batch(23, 32, 8, 128, 23 * 8192, 8192)) == TWO     # 184 pairs: under 3/4 of a round
        assert form(shaped_batch(24, 32, 8, 128, 24 * 8192, 8192)) == ONE     # 192 pairs
        assert form(shaped_batch(48, 32, 8, 128, 48 * 4096, 4096)) == TWO     # 384 pairs: the second round half empty
        assert form(shaped_batch(52, 32, 8, 128, 52 * 4096, 4096)) == ONE     # 416 pairs: 81 % of two rounds
        assert form(shaped_batch(32, 32, 8, 128, 32 * 8193, 8193)) == TWO     # a list too long for the registers
        assert form(shaped_batch(32, 64, 8, 128, 32 * 8192, 8192)) == TWO     # eight query heads per KV head
        assert form(shaped_batch(32, 32, 8, 128, 32 * 8192, 8192, hcsa.DLLM_F32)) == TWO   # 512-byte rows
        assert form(shaped_batch(32, 32, 8, 64, 32 * 8192, 8192, hcsa.DLLM_F32)) == ONE
        hcsa.dllm_hcsa_set_select_form(TWO)
        assert form(c5) == TWO
        hcsa.dllm_hcsa_set_select_form(ONE)
        assert form(c3) == ONE and form(shaped_batch(4, 32, 8, 128, 4 * 8192, 8192)) == ONE
        assert form(c5, head_sum=True) == TWO and form(shaped_batch(32, 64, 8, 128, 32 * 8192, 8192)) == TWO
        bad = shaped_batch(4, 32, 8, 128, 100, 50)
        bad.head_dim = 96
        assert hcsa.lib().dllm_hcsa_select_form_of(ctypes.byref(bad), 1, 0) == -1 and "head_dim" in hcsa.last_error()
    finally:
        hcsa.dllm_hcsa_set_select_form(hcsa.DLLM_SELECT_FORM_AUTO)




def select_status(b, cu_k=FAKE, total_k=100, max_k=50, pool_w=1, idx=FAKE, ws=FAKE, ws_bytes=1 << 40):
    return hcsa.lib().dllm_hcsa_select(ctypes.byref(b), cu_k, total_k, max_k, pool_w, idx, ws, ws_bytes, None)


def attend_status(b, idx=FAKE, cu_k=FAKE, total_k=100, max_k=50, mode=None, o=FAKE, ws=FAKE, ws_bytes=1 << 40):
    return hcsa.lib().dllm_hcsa_attend(ctypes.byref(b), idx, cu_k, total_k, max_k, mode, o, ws, ws_bytes, None)


@pytest.mark.parametrize("field,value", [
    ("dtype", 7), ("batch", 0), ("n_q_heads", 0), ("n_kv_heads", 3), ("head_dim", 96), ("q", 0), ("k", None),
    ("cu_kv", 0), ("max_kv", 501), ("max_q", -1), ("q_stride_head", 64), ("kv_stride_tok", 257), ("v", 0x10008),
    ("softmax_scale", float("inf")), ("softmax_scale", -0.5), ("softmax_scale", 0.0),
])
def test_bad_batch_descriptor_is_rejected_everywhere(field, value):
    b = good_batch()
    setattr(b, field, value)
    assert select_status(b) == hcsa.DLLM_ERR_INVALID_ARG
    assert hcsa.last_error() != ""
    assert attend_status(b) == hcsa.DLLM_ERR_INVALID_ARG
    assert hcsa.lib().dllm_dense_refresh_attend(ctypes.byref(b), FAKE, None, 0, None) == hcsa.DLLM_ERR_INVALID_ARG
    assert hcsa.lib().dllm_hcsa_select_workspace(ctypes.byref(b), 50) == 0


def test_select_scalar_and_workspace_checks():
    b = good_batch()
    assert select_status(b, max_k=0) == hcsa.DLLM_ERR_INVALID_ARG
    assert select_status(b, max_k=301) == hcsa.DLLM_ERR_INVALID_ARG          # > max_kv
    assert select_status(b, pool_w=2) == hcsa.DLLM_ERR_INVALID_ARG
    assert select_status(b, pool_w=65) == hcsa.DLLM_ERR_INVALID_ARG
    assert select_status(b, cu_k=None) == hcsa.DLLM_ERR_INVALID_ARG
    assert select_status(b, idx=None) == hcsa.DLLM_ERR_INVALID_ARG
    assert select_status(b, total_k=10, max_k=50) == hcsa.DLLM_ERR_INVALID_ARG
    need = hcsa.lib().dllm_hcsa_select_workspace(ctypes.byref(b), 50)
    assert need >= 8 * 500 * 4   # the fp32 scores of every (head, position)
    assert select_status(b, ws=None) == hcsa.DLLM_ERR_WORKSPACE
    assert select_status(b, ws_bytes=need - 1) == hcsa.DLLM_ERR_WORKSPACE
    assert "workspace" in hcsa.last_error()
    assert select_status(b, ws=ctypes.c_void_p(0x30010)) == hcsa.DLLM_ERR_WORKSPACE   # misaligned
    big = good_batch()
    big.total_kv, big.max_kv = 100000, 40000
    assert select_status(big) == hcsa.DLLM_ERR_UNSUPPORTED
    big.max_kv = 20000
    assert select_status(big, pool_w=3) == hcsa.DLLM_ERR_UNSUPPORTED


def test_attend_scalar_checks():
    b = good_batch()
    assert attend_status(b, o=None) == hcsa.DLLM_ERR_INVALID_ARG
    assert attend_status(b, max_k=-1) == hcsa.DLLM_ERR_INVALID_ARG
    assert attend_status(b, max_k=301, total_k=400) == hcsa.DLLM_ERR_INVALID_ARG
    assert attend_status(b, cu_k=None) == hcsa.DLLM_ERR_INVALID_ARG
    assert attend_status(b, o=ctypes.c_void_p(0x30004)) == hcsa.DLLM_ERR_INVALID_ARG
    assert hcsa.lib().dllm_dense_refresh_attend(ctypes.byref(b), None, None, 0, None) == hcsa.DLLM_ERR_INVALID_ARG
    # a long kept list on few (sequence, head) pairs is split into chunks and needs partial-result space
    b.batch, b.total_kv, b.max_kv = 1, 9000, 9000
    need = hcsa.lib().dllm_hcsa_attend_workspace(ctypes.byref(b), 4000)
    assert need > 0
    assert attend_status(b, total_k=4000, max_k=4000, ws=None) == hcsa.DLLM_ERR_WORKSPACE
    assert attend_status(b, total_k=4000, max_k=4000, ws_bytes=need - 1) == hcsa.DLLM_ERR_WORKSPACE


def test_attend_without_cu_k_needs_an_empty_kept_set():
    b = good_batch()
    assert attend_status(b, cu_k=None, total_k=1, max_k=0) == hcsa.DLLM_ERR_INVALID_ARG
    assert "cu_k may be NULL only" in hcsa.last_error()
    # idx may be NULL with cu_k present (identity lists); only the reverse is refused
    assert attend_status(b, idx=None, ws=None, ws_bytes=0, total_k=100, max_k=301) == hcsa.DLLM_ERR_INVALID_ARG
    assert "max_k" in hcsa.last_error()


def test_gather_kernel_row_count_limit():
    """One narrow KV head: 2^24 + 1 rows of 128 bytes stay below 4 GiB, but the row index no longer fits
    the 24-bit multiply that forms the byte offset."""
    b = good_batch()
    b.n_q_heads = b.n_kv_heads = 1
    b.head_dim = 64
    b.q_stride_tok = b.q_stride_head = b.kv_stride_tok = b.kv_stride_head = 64
    b.total_kv, b.max_kv = 1 << 25, (1 << 24) + 1
    assert attend_status(b) == hcsa.DLLM_ERR_UNSUPPORTED
    assert "2^24" in hcsa.last_error()
    b.max_kv = 1 << 24
    b.batch = 2
    assert attend_status(b, ws=None, ws_bytes=0) in (hcsa.DLLM_ERR_WORKSPACE, hcsa.DLLM_ERR_DEVICE)   # past the shape checks


def test_select_ex_option_checks():
    b = good_batch()
    L = hcsa.lib()

    def status(forced_tail=0, head_sum=0, max_k=50):
        return L.dllm_hcsa_select_ex(ctypes.byref(b), FAKE, 100, max_k, 1, forced_tail, head_sum, FAKE, FAKE, 1 << 40, None)

    assert status(forced_tail=-1) == hcsa.DLLM_ERR_INVALID_ARG
    assert status(forced_tail=51) == hcsa.DLLM_ERR_INVALID_ARG
    assert "forced_tail" in hcsa.last_error()
    assert status(head_sum=2) == hcsa.DLLM_ERR_INVALID_ARG
    assert status(head_sum=-1) == hcsa.DLLM_ERR_INVALID_ARG


def test_select_static_checks_and_size_limit():
    """The no-workspace selection makes the same host checks, and refuses batches whose scores do not fit
    its built-in buffer, before any HIP call."""
    L = hcsa.lib()

    def status(b, forced_tail=0, head_sum=0, max_k=50, pool_w=1, cu_k=FAKE):
        return L.dllm_hcsa_select_static(ctypes.byref(b), cu_k, 100, max_k, pool_w, forced_tail, head_sum, FAKE, None)

    b = good_batch()
    assert status(b, forced_tail=51) == hcsa.DLLM_ERR_INVALID_ARG
    assert status(b, head_sum=2) == hcsa.DLLM_ERR_INVALID_ARG
    assert status(b, pool_w=4) == hcsa.DLLM_ERR_INVALID_ARG
    assert status(b, cu_k=None) == hcsa.DLLM_ERR_INVALID_ARG
    b.head_dim = 96
    assert status(b) == hcsa.DLLM_ERR_INVALID_ARG
    big = good_batch()
    big.total_kv = 2_000_000            # 8 heads x 2e6 positions x 4 bytes = 64 MB of scores
    assert L.dllm_hcsa_select_workspace(ctypes.byref(big), 50) > hcsa.DLLM_SELECT_STATIC_BYTES
    assert status(big) == hcsa.DLLM_ERR_WORKSPACE
    assert "built-in buffer" in hcsa.last_error()
    text = open(os.path.join(ROOT, "include", "dllm_hcsa.h")).read()
    assert re.search(r"#define\s+DLLM_SELECT_STATIC_BYTES\s+\(32u\s*<<\s*20\)", text)
    assert hcsa.DLLM_SELECT_STATIC_BYTES == 32 << 20


def test_static_scratch_is_a_global_symbol_of_the_device_image(tmp_path):
    """The HIP runtime finds a device variable by name in the code object's dynamic symbol table, and
    aborts the process if it is not there.  A `static __device__` array that host code names is given
    global binding by the compiler unless something (e.g. a `used` attribute) keeps it local: check
    what was built."""
    import shutil
    import subprocess
    llvm = "/opt/rocm/llvm/bin"
    tools = [os.path.join(llvm, t) for t in ("llvm-objcopy", "clang-offload-bundler", "llvm-readelf")]
    obj = os.path.join(ROOT, "paper_2512_17077_amd", "_build", "api.o")
    if not all(os.path.exists(t) for t in tools) or not os.path.exists(obj):
        pytest.skip("ROCm llvm tools or the build's api.o not present")
    fat, co = str(tmp_path / "api.fatbin"), str(tmp_path / "api.co")
    subprocess.run([tools[0], "-O", "binary", "--only-section=.hip_fatbin", obj, fat], check=True)
    subprocess.run([tools[1], "--unbundle", "--type=o", f"--input={fat}",
                    "--targets=hipv4-amdgcn-amd-amdhsa--gfx950", f"--output={co}"], check=True)
    table = subprocess.run([tools[2], "--dyn-syms", co], check=True, capture_output=True, text=True).stdout
    rows = [l.split() for l in table.splitlines() if l.strip().endswith("scratch")]
    assert rows, "no symbol named *scratch in the device image's dynamic symbols"
    assert all("GLOBAL" in r and "OBJECT" in r for r in rows), rows
    assert any(int(r[2]) == hcsa.DLLM_SELECT_STATIC_BYTES for r in rows), rows
    _ = shutil


def test_pack_argument_checks():
    b = good_batch()
    L = hcsa.lib()

    def pack_status(idx=FAKE, cu_k=FAKE, total_k=100, max_k=50, kp=FAKE, vp=FAKE):
        return L.dllm_hcsa_pack(ctypes.byref(b), idx, cu_k, total_k, max_k, kp, vp, None)

    assert pack_status(idx=None) == hcsa.DLLM_ERR_INVALID_ARG
    assert pack_status(cu_k=None) == hcsa.DLLM_ERR_INVALID_ARG
    assert pack_status(kp=None) == hcsa.DLLM_ERR_INVALID_ARG
    assert pack_status(vp=ctypes.c_void_p(0x30004)) == hcsa.DLLM_ERR_INVALID_ARG
    assert pack_status(total_k=0) == hcsa.DLLM_ERR_INVALID_ARG
    assert pack_status(max_k=0) == hcsa.DLLM_ERR_INVALID_ARG
    assert pack_status(max_k=101) == hcsa.DLLM_ERR_INVALID_ARG
    assert "max_k" in hcsa.last_error()


def test_python_struct_matches_the_header_layout(tmp_path):
    """Compile the header with gcc (as C99) and compare sizeof / offsetof with the ctypes mirror."""
    import subprocess
    fields = [f for f, _ in hcsa.DllmBatch._fields_]
    src = tmp_path / "layout.c"
    prints = "\n".join(f'  printf("{f} %zu\\n", offsetof(dllm_batch, {f}));' for f in fields)
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "dllm_hcsa.h"\nint main(void) {\n'
                   '  printf("sizeof %zu\\n", sizeof(dllm_batch));\n' + prints + "\n  return 0;\n}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    out = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True,
                                                       text=True).stdout.splitlines())
    assert int(out["sizeof"]) == ctypes.sizeof(hcsa.DllmBatch)
    for f in fields:
        assert int(out[f]) == getattr(hcsa.DllmBatch, f).offset, f


def test_generated_dense_step_text_is_current(tmp_path):
    """csrc/attend_dense_step.inc is generated by csrc/gen_dense_step.py and committed: the two must agree."""
    import subprocess
    import sys
    csrc = os.path.join(ROOT, "paper_2512_17077_amd", "csrc")
    subprocess.run([sys.executable, os.path.join(csrc, "gen_dense_step.py"), f"--out={tmp_path}"], check=True,
                   capture_output=True)
    assert open(tmp_path / "attend_dense_step.inc").read() == open(os.path.join(csrc, "attend_dense_step.inc")).read()
