"""CPU-side checks of the C-ABI library: it loads, exports what the header declares, and its
host-only logic (the "top rho%" count, the dense-step count, argument validation) behaves.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

import oracle
from oracle import schedule as oracle_schedule
from paper_2509_24014_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
            names |= set(re.findall(r"\b(sparsed_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    names = _declared_functions()
    assert "sparsed_attn_dense" in names and "sparsed_select_pattern" in names and "sparsed_attn_sparse" in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in sparsed.h but not exported"
    assert sorted(binding.EXPORTS) == names
    assert binding.version() >= 100


def test_kept_blocks_and_dense_steps_agree_with_the_written_rule():
    for n in range(0, 70):
        for pct in range(1, 101):
            want = max(1, -((-pct * n) // 100)) if n > 0 else 0
            assert binding.kept_blocks(pct / 100.0, n) == want
            if n > 0:
                assert binding.kept_blocks(pct / 100.0, n) == oracle.kept_blocks(pct / 100.0, n)
    for rho, n, k in [(0.3, 8, 3), (0.2, 64, 13), (0.1, 256, 26), (0.1, 512, 52), (0.05, 1024, 52)]:
        assert binding.kept_blocks(rho, n) == k
    for T, skip, nd in [(1024, 0.2, 205), (64, 0.125, 8), (5, 0.2, 1), (10, 0.3, 3), (10, 0.0, 1), (10, 1.0, 10)]:
        assert binding.n_dense_steps(T, skip) == nd == oracle_schedule.n_dense_steps(T, skip)


def _t(B=1, H=2, L=256, D=64, dtype=binding.SPARSED_F32, data=0x1000, sl=None, sh=None, sb=None):
    sl = D if sl is None else sl
    sh = L * sl if sh is None else sh
    sb = H * sh if sb is None else sb
    return binding._Tensor(data, dtype, B, H, L, D, sb, sh, sl)


def _ix(B=1, H=2, nqb=8, nkb=8, bq=32, bk=32, cap=24, rp=0x2000, ci=0x3000):
    return binding._BlockIndex(B, H, nqb, nkb, bq, bk, cap, rp, ci)


def test_argument_validation_rejects_before_any_launch():
    # every call below fails validation on the host; the fake device pointers are never touched
    lib = binding.load_library()
    R = ctypes.byref
    q, k, v, o = _t(), _t(), _t(), _t()
    assert lib.sparsed_attn_dense(None, R(k), R(v), R(o), None) == 1                       # NULL
    assert lib.sparsed_attn_dense(R(_t(data=None)), R(k), R(v), R(o), None) == 1
    assert lib.sparsed_attn_dense(R(_t(D=96)), R(k), R(v), R(o), None) == 6                # head dim
    assert lib.sparsed_attn_dense(R(_t(dtype=7)), R(k), R(v), R(o), None) == 3             # dtype
    assert lib.sparsed_attn_dense(R(q), R(_t(dtype=binding.SPARSED_BF16)), R(v), R(o), None) == 3
    assert lib.sparsed_attn_dense(R(q), R(_t(L=128)), R(v), R(o), None) == 2               # shapes
    assert lib.sparsed_attn_dense(R(_t(H=3)), R(k), R(v), R(_t(H=3)), None) == 2           # 3 % 2 != 0
    assert lib.sparsed_attn_dense(R(_t(data=0x1004)), R(k), R(v), R(o), None) == 4         # alignment
    assert lib.sparsed_attn_dense(R(_t(sl=66)), R(k), R(v), R(o), None) == 4               # stride
    big = _t(L=1 << 20, sl=1 << 12)                                                        # slab of 2^34 bytes
    assert lib.sparsed_attn_dense(R(big), R(big), R(big), R(big), None) == 4
    # a length that is not a block multiple is legal; its index must count the partial last blocks
    r = _t(L=250)
    assert lib.sparsed_attn_sparse(R(r), R(r), R(r), R(_ix(nqb=7, nkb=7)), R(r), None) == 8    # floor(250/32) is one short
    assert b"does not describe" in lib.sparsed_last_error()
    ix = _ix()
    assert lib.sparsed_select_pattern(R(q), R(k), 32, 32, 0.0, R(ix), None) == 5           # rho
    assert lib.sparsed_select_pattern(R(q), R(k), 32, 32, 1.5, R(ix), None) == 5
    assert lib.sparsed_select_pattern(R(q), R(k), 48, 32, 0.3, R(ix), None) == 6           # block sizes
    assert lib.sparsed_select_pattern(R(q), R(k), 32, 32, 0.3, R(_ix(cap=23)), None) == 8  # capacity < nqb*k
    assert lib.sparsed_select_pattern(R(q), R(k), 32, 32, 0.3, R(_ix(nkb=4)), None) == 8   # index vs q
    assert lib.sparsed_select_pattern(R(q), R(k), 32, 32, 0.3, None, None) == 1
    qb = _t(dtype=binding.SPARSED_BF16, D=128)
    assert lib.sparsed_select_pattern(R(qb), R(qb), 64, 16, 0.3, R(_ix(nqb=4, nkb=16, bq=64, bk=16)), None) == 6   # bf16 bk
    ex = binding._Exec(None, 0x4000, 16, None, None, None)
    assert lib.sparsed_select_pattern(R(q), R(k), 32, 32, 0.3, R(ix), R(ex)) == 7          # workspace too small
    assert lib.sparsed_select_pattern(R(q), R(k), 32, 32, 0.3, R(ix), None) == 7           # no workspace: the library has none of its own
    assert b"workspace" in lib.sparsed_last_error()
    assert lib.sparsed_select_pattern(R(q), R(k), 32, 32, 0.3, R(ix), R(binding._Exec(None, 0x4010, 1 << 20, None, None, None))) == 7   # misaligned
    assert lib.sparsed_index_validate(R(ix), None) == 7
    assert lib.sparsed_index_validate(R(ix), R(ex)) == 7
    assert lib.sparsed_attn_sparse(R(q), R(k), R(v), None, R(o), None) == 1
    assert lib.sparsed_attn_sparse(R(q), R(k), R(v), R(_ix(H=4)), R(o), None) == 8
    assert lib.sparsed_select_pattern_isolated(R(q), R(k), 32, 32, 0.3, 9, R(_ix(cap=64)), None) == 5
    assert lib.sparsed_select_pattern_isolated_tokens(R(q), R(k), 32, 32, 0.3, 300, R(_ix(cap=64)), None) == 5   # boundary past L
    assert lib.sparsed_select_pattern_isolated_tokens(R(q), R(k), 32, 32, 0.3, 50, R(_ix(cap=8)), None) == 8    # capacity
    assert lib.sparsed_select_pattern_isolated_tokens(R(q), R(k), 32, 32, 0.3, 50, R(_ix(cap=64)), None) == 7   # workspace
    assert lib.sparsed_index_fill_window(R(_ix(cap=4)), 256, 64, 0, None) == 8                                   # capacity
    assert lib.sparsed_index_fill_window(R(_ix()), 300, 64, 0, None) == 8                                        # 8 blocks do not describe 300 tokens
    assert lib.sparsed_index_window_entries(256, 32, 32, 0, 0) == 8
    out = ctypes.c_double(0.0)
    assert lib.sparsed_probe_mfma_bf16(1, 0, ctypes.byref(out), None) == 5                                       # iters
    assert lib.sparsed_probe_mfma_bf16(1, 10, None, None) == 1
    assert lib.sparsed_probe_mfma_bf16(1, 10, ctypes.byref(out), None) == 7                                       # workspace
    assert lib.sparsed_probe_mix_bf16(7, 1, 10, ctypes.byref(out), None) == 5                                     # mix
    assert lib.sparsed_probe_mix_bf16(5, 1, 10, ctypes.byref(out), None) == 7                                     # workspace
    assert lib.sparsed_probe_valu_f32(2, 10, ctypes.byref(out), None) == 5                                        # op
    assert lib.sparsed_probe_valu_f32(1, 0, ctypes.byref(out), None) == 5                                         # iters
    assert lib.sparsed_probe_valu_f32(1, 10, None, None) == 1
    assert lib.sparsed_probe_valu_f32(1, 10, ctypes.byref(out), None) == 7                                        # workspace
    assert lib.sparsed_status_string(8) == b"malformed block index"


def test_workspace_size_formula():
    lib = binding.load_library()
    lib.sparsed_select_workspace_min_bytes.argtypes = lib.sparsed_select_workspace_bytes.argtypes
    lib.sparsed_select_workspace_min_bytes.restype = ctypes.c_size_t
    t = _t(B=1, H=32, L=65536, D=128, dtype=binding.SPARSED_BF16)
    least = lib.sparsed_select_workspace_min_bytes(ctypes.byref(t), 128, 64)
    assert least == 32 * 65536 * 4 + 32 * 512 * 1024 * 4                                # row statistics + pooled scores
    full = lib.sparsed_select_workspace_bytes(ctypes.byref(t), 128, 64)
    slab = 128 * 1024 * 4                                                               # block_q x nkb floats per resident work-group
    assert full > least and (full - least) % slab == 0 and 256 <= (full - least) // slab <= 1024
    r = _t(B=1, H=2, L=250, D=64)                                                       # fp32: two passes only
    assert lib.sparsed_select_workspace_bytes(ctypes.byref(r), 32, 32) == 2048 + 2 * 8 * 8 * 4   # ceil(250/32) = 8 blocks each way
    assert lib.sparsed_select_workspace_min_bytes(ctypes.byref(r), 32, 32) == 2048 + 2 * 8 * 8 * 4
    assert lib.sparsed_select_workspace_bytes(ctypes.byref(t), 0, 64) == 0


def test_no_fallback_when_the_library_is_missing(monkeypatch, tmp_path):
    """Without libsparsed.so (and with nothing to build it from) every entry point must raise: there is no CPU path."""
    import torch
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libsparsed.so"))
    with pytest.raises(FileNotFoundError):
        binding.load_library(build_if_missing=False)

    def no_compiler(force=True, verbose=False):
        raise RuntimeError("hipcc failed")

    from paper_2509_24014_amd import build as build_mod
    monkeypatch.setattr(build_mod, "build", no_compiler)
    x = torch.zeros(1, 1, 64, 64)
    for call in (lambda: binding.kept_blocks(0.3, 8), lambda: binding.attn_dense(x, x, x)):
        with pytest.raises((RuntimeError, FileNotFoundError, OSError, ValueError)):
            call()
    assert binding._lib is None


def test_product_never_touches_the_oracle():
    """The oracle is test infrastructure: nothing under the package or the workload generator may import,
    link or read it (only tests, the smoke check and the benchmark's CPU baseline do)."""
    pkg = os.path.join(ROOT, "paper_2509_24014_amd")
    offenders = []
    for base in (pkg, os.path.join(ROOT, "workload"), os.path.join(ROOT, "include")):
        for dirpath, _, files in os.walk(base):
            for f in files:
                if f.endswith((".py", ".hip", ".hpp", ".h", ".c", ".cpp")):
                    text = open(os.path.join(dirpath, f), errors="ignore").read()
                    if re.search(r"import\s+oracle|from\s+oracle|oracle\.|liboracle|oracle/", text):
                        offenders.append(os.path.join(dirpath, f))
    assert offenders == []
    # and the oracle shares nothing with the product either
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2509_24014_amd" not in text and "sparsed.h" not in text and "csrc" not in text
