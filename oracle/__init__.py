"""ctypes loader for the CPU oracle (oracle/hcsa_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU package never imports this module and
this module never imports the GPU package's binding.  Arrays are numpy, on the
host: float32 data as float32 arrays, bfloat16 data as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hcsa_oracle.c")
_LIB = os.path.join(_HERE, "libhcsa_oracle.so")
_lib = None
# tests/test_oracle_mutants.py points this at deliberately broken builds to show the pins catch them
_OVERRIDE = os.environ.get("HCSA_ORACLE_LIB_OVERRIDE")

F32, BF16 = 0, 1


def build(force: bool = False, sanitize: bool = False, out: str | None = None) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps every fp32 step of
    the score a separately rounded operation; fmaf comes from libm.

    sanitize=True builds a second library (libhcsa_oracle_san.so, or `out`) with
    -fsanitize=address,undefined for running the pin suite under the sanitizers; a process that loads
    it must have the AddressSanitizer runtime preloaded (see sanitizer_env())."""
    if sanitize:
        lib = out or os.path.join(_HERE, "libhcsa_oracle_san.so")
        cmd = ["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
               "-Wall", "-Wextra", "-o", lib, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        return lib
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def sanitizer_env(lib: str) -> dict:
    """Environment for a child process that loads the sanitized build `lib` in place of the oracle:
    the AddressSanitizer runtime has to be the first library of the process, so it is preloaded (ahead of
    whatever is preloaded already); leak checking is off because the Python interpreter itself never
    frees everything."""
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()
    env = dict(os.environ, HCSA_ORACLE_LIB_OVERRIDE=lib, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    env["LD_PRELOAD"] = asan + ((":" + os.environ["LD_PRELOAD"]) if os.environ.get("LD_PRELOAD") else "")
    return env


def _load():
    global _lib
    if _lib is None:
        if _OVERRIDE:
            lib = ctypes.CDLL(_OVERRIDE)
        else:
            build()
            lib = ctypes.CDLL(_LIB)
        vp, ip, i = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int
        lib.oracle_num_threads.restype = i
        lib.oracle_score.restype = i
        lib.oracle_score.argtypes = [i, i, i, i, i, vp, vp, ip, ip, i, vp, vp]
        lib.oracle_topk.restype = i
        lib.oracle_topk.argtypes = [i, i, vp, ip, ip, vp]
        lib.oracle_select.restype = i
        lib.oracle_select.argtypes = [i, i, i, i, i, vp, vp, ip, ip, ip, i, vp]
        lib.oracle_select_ex.restype = i
        lib.oracle_select_ex.argtypes = [i, i, i, i, i, vp, vp, ip, ip, ip, i, i, i, vp]
        lib.oracle_attend.restype = i
        lib.oracle_attend.argtypes = [i, i, i, i, i, vp, vp, vp, ip, ip, vp, ip, vp, ctypes.c_double, vp]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle takes float32 or uint16 (bf16 bits), got {a.dtype}")


def _c(a, dtype=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected its arguments (code {rc})")


def _dims(q, k, cu_q, cu_kv):
    assert q.ndim == 3 and k.ndim == 3 and q.shape[2] == k.shape[2]
    assert q.shape[0] == cu_q[-1] and k.shape[0] == cu_kv[-1]
    return len(cu_q) - 1, q.shape[1], k.shape[1], q.shape[2]


def score(q, k, cu_q, cu_kv, pool_w: int = 1, want64: bool = False):
    """Eq. (6) scores: fp32 [Hq, total_kv] in the canonical order (and the fp64
    companion if asked)."""
    q, k = _c(q), _c(k)
    cu_q, cu_kv = _c(cu_q, np.int32), _c(cu_kv, np.int32)
    B, Hq, Hkv, D = _dims(q, k, cu_q, cu_kv)
    assert _dtype_code(q) == _dtype_code(k)
    s32 = np.empty((Hq, int(cu_kv[-1])), dtype=np.float32)
    s64 = np.empty((Hq, int(cu_kv[-1])), dtype=np.float64) if want64 else None
    rc = _load().oracle_score(_dtype_code(q), B, Hq, Hkv, D, _p(q), _p(k), _p(cu_q), _p(cu_kv),
                              int(pool_w), _p(s32), _p(s64))
    _check(rc, "oracle_score")
    return (s32, s64) if want64 else s32


def topk(s, cu_kv, cu_k):
    """Per-head TopK of given fp32 scores [Hq, total_kv] -> int32 [Hq, total_k]."""
    s = _c(s, np.float32)
    cu_kv, cu_k = _c(cu_kv, np.int32), _c(cu_k, np.int32)
    assert s.ndim == 2 and s.shape[1] == cu_kv[-1]
    idx = np.empty((s.shape[0], int(cu_k[-1])), dtype=np.int32)
    rc = _load().oracle_topk(len(cu_kv) - 1, s.shape[0], _p(s), _p(cu_kv), _p(cu_k), _p(idx))
    _check(rc, "oracle_topk")
    return idx


def select(q, k, cu_q, cu_kv, cu_k, pool_w: int = 1):
    """Score + per-head TopK -> int32 [Hq, total_k], local positions, ascending."""
    q, k = _c(q), _c(k)
    cu_q, cu_kv, cu_k = _c(cu_q, np.int32), _c(cu_kv, np.int32), _c(cu_k, np.int32)
    B, Hq, Hkv, D = _dims(q, k, cu_q, cu_kv)
    assert _dtype_code(q) == _dtype_code(k)
    idx = np.empty((Hq, int(cu_k[-1])), dtype=np.int32)
    rc = _load().oracle_select(_dtype_code(q), B, Hq, Hkv, D, _p(q), _p(k), _p(cu_q), _p(cu_kv),
                               _p(cu_k), int(pool_w), _p(idx))
    _check(rc, "oracle_select")
    return idx


def select_ex(q, k, cu_q, cu_kv, cu_k, pool_w: int = 1, forced_tail: int = 0, head_sum: bool = False):
    """Selection with the active block's own positions (the last `forced_tail` of every sequence)
    always kept (Eq. 4), and / or with one list shared by all heads from head-summed scores (Eq. 5)."""
    q, k = _c(q), _c(k)
    cu_q, cu_kv, cu_k = _c(cu_q, np.int32), _c(cu_kv, np.int32), _c(cu_k, np.int32)
    B, Hq, Hkv, D = _dims(q, k, cu_q, cu_kv)
    assert _dtype_code(q) == _dtype_code(k)
    idx = np.empty((Hq, int(cu_k[-1])), dtype=np.int32)
    rc = _load().oracle_select_ex(_dtype_code(q), B, Hq, Hkv, D, _p(q), _p(k), _p(cu_q), _p(cu_kv), _p(cu_k),
                                  int(pool_w), int(forced_tail), int(bool(head_sum)), _p(idx))
    _check(rc, "oracle_select_ex")
    return idx


def attend(q, k, v, cu_q, cu_kv, idx, cu_k, seq_mode, softmax_scale: float):
    """Softmax attention over each head's kept rows (or all rows where
    seq_mode is 1) -> float64 [total_q, Hq, D]."""
    q, k, v = _c(q), _c(k), _c(v)
    cu_q, cu_kv = _c(cu_q, np.int32), _c(cu_kv, np.int32)
    B, Hq, Hkv, D = _dims(q, k, cu_q, cu_kv)
    assert v.shape == k.shape and _dtype_code(q) == _dtype_code(k) == _dtype_code(v)
    if cu_k is None:
        cu_k = np.zeros(B + 1, dtype=np.int32)
    cu_k = _c(cu_k, np.int32)
    if idx is None:
        idx = np.zeros((Hq, int(cu_k[-1])), dtype=np.int32)
    idx = _c(idx, np.int32)
    assert idx.shape == (Hq, int(cu_k[-1]))
    if seq_mode is not None:
        seq_mode = _c(seq_mode, np.uint8)
        assert seq_mode.shape == (B,)
    out = np.empty((q.shape[0], Hq, D), dtype=np.float64)
    rc = _load().oracle_attend(_dtype_code(q), B, Hq, Hkv, D, _p(q), _p(k), _p(v), _p(cu_q), _p(cu_kv),
                               _p(idx), _p(cu_k), _p(seq_mode), float(softmax_scale), _p(out))
    _check(rc, "oracle_attend")
    return out


def pack(k, v, cu_kv, idx, cu_k):
    """Section 4.5 packing by its definition: for every query head h, sequence b and list position
    t, packed[h, cu_k[b] + t, :] = X[cu_kv[b] + idx[h, cu_k[b] + t], h // G, :] for X = K and V.
    Plain Python loops over (head, sequence); elements keep their type (fp32, or bf16 bit patterns)."""
    k, v = _c(k), _c(v)
    cu_kv, cu_k, idx = _c(cu_kv, np.int32), _c(cu_k, np.int32), _c(idx, np.int32)
    assert k.ndim == 3 and v.shape == k.shape and idx.ndim == 2 and idx.shape[1] == cu_k[-1]
    Hq, Hkv, D = idx.shape[0], k.shape[1], k.shape[2]
    assert Hq % Hkv == 0
    G = Hq // Hkv
    kp = np.zeros((Hq, int(cu_k[-1]), D), dtype=k.dtype)
    vp = np.zeros((Hq, int(cu_k[-1]), D), dtype=v.dtype)
    for h in range(Hq):
        for b in range(len(cu_k) - 1):
            for t in range(int(cu_k[b]), int(cu_k[b + 1])):
                row = int(cu_kv[b]) + int(idx[h, t])
                assert int(cu_kv[b]) <= row < int(cu_kv[b + 1])
                kp[h, t, :] = k[row, h // G, :]
                vp[h, t, :] = v[row, h // G, :]
    return kp, vp
