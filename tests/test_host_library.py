"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, its host
functions (codebook, search table) agree with the oracle, and argument validation returns
error codes before anything touches a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_2412_01195_amd import q8opt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "q8opt.h")).read()
    declared = sorted(set(re.findall(r"Q8_API[^;]*?\b(q8_[a-z0-9_]+)\s*\(", hdr)))
    assert declared == sorted(q8opt.EXPORTS)
    L = q8opt.lib()
    for name in declared:
        assert hasattr(L, name), name
    # the benchmark's traffic probe lives in a library of its own, not in the product
    assert not hasattr(L, "q8_probe_adam8bit_traffic")
    assert q8opt.status_str(0) == "Q8_OK" and "Q8_EBLOCK" in q8opt.status_str(q8opt.EBLOCK)


def test_binding_argument_lists_follow_the_header():
    """Every entry point's ctypes argument list has the kinds the header declares, in order:
    pointer, 64-bit integer, int, float (a swapped pair would still load and run)."""
    hdr = open(os.path.join(ROOT, "include", "q8opt.h")).read()
    hdr = re.sub(r"/\*.*?\*/", " ", hdr, flags=re.S)                 # comments carry commas and names

    def kind_of_decl(d):
        d = d.strip()
        if "*" in d:
            return "ptr"
        if d.startswith("int64_t"):
            return "i64"
        if d.startswith("float"):
            return "f32"
        if d.startswith("int ") or d.startswith("q8_status"):
            return "i32"
        raise AssertionError("unexpected parameter declaration: %r" % d)

    def kind_of_ctype(t):
        if t is C.c_void_p or (isinstance(t, type) and issubclass(t, C._Pointer)):
            return "ptr"
        return {C.c_int64: "i64", C.c_int: "i32", C.c_float: "f32"}[t]

    L = q8opt.lib()
    seen = 0
    for m in re.finditer(r"Q8_API\s+[^;(]*?\b(q8_[a-z0-9_]+)\s*\(([^;]*?)\)\s*;", hdr, flags=re.S):
        name, params = m.group(1), m.group(2).strip()
        declared = [] if params == "void" else [kind_of_decl(d) for d in params.split(",")]
        bound = [kind_of_ctype(t) for t in getattr(L, name).argtypes]
        assert bound == declared, name
        seen += 1
    assert seen == len(q8opt.EXPORTS)


@pytest.mark.parametrize("signed", [True, False])
def test_codebook_bit_equal_to_oracle(signed):
    assert np.array_equal(q8opt.build_codebook(signed).view(np.uint32), oracle.build_codebook(signed).view(np.uint32))


def _critical_points(q):
    pts = [np.float32(v) for v in (0.0, -0.0, 1.0, -1.0, 1e-45, -1e-45, 1e-38, 2.0 ** -24, 2.0 ** -25, -(2.0 ** -24))]
    for j in range(256):
        v = q[j]
        for _ in range(3):
            pts.append(v); v = np.nextafter(v, np.float32(2))
        v = q[j]
        for _ in range(3):
            pts.append(v); v = np.nextafter(v, np.float32(-2))
        if j < 255:
            mid = np.float32((np.float64(q[j]) + np.float64(q[j + 1])) / 2)
            lo = hi = mid
            pts.append(mid)
            for _ in range(4):
                lo = np.nextafter(lo, np.float32(-2)); hi = np.nextafter(hi, np.float32(2))
                pts += [lo, hi]
    return [p for p in pts if abs(float(p)) <= 1.0]


@pytest.mark.parametrize("signed", [True, False])
def test_table_lookup_equals_oracle_search(signed):
    q = oracle.build_codebook(signed)
    tab = q8opt.build_qtable(q8opt.build_codebook(signed))
    for x in _critical_points(q):
        assert q8opt.host_nearest_code(tab, x) == oracle.nearest_code(q, x), float(x)
    # every bucket edge of the table: all binary32 values with a zero lower half, +-1 ulp
    hdr = tab[:64].view(np.uint32)
    assert int(hdr[1]) == 16 and int(hdr[2]) == (127 if signed else 0)
    keys = np.arange(0, 0x3F80 + 1, dtype=np.uint32) << np.uint32(16)
    for sign in (0, 0x80000000):
        for d in (-1, 0, 1):
            xs = ((keys + np.uint32(d & 0xFFFFFFFF)) | np.uint32(sign)).astype(np.uint32).view(np.float32)
            xs = xs[np.isfinite(xs) & (np.abs(xs) <= 1)]
            got = np.array([q8opt.host_nearest_code(tab, x) for x in xs])
            ref = np.array([oracle.nearest_code(q, x) for x in xs])
            assert np.array_equal(got, ref), xs[got != ref][:5]
    rng = np.random.default_rng(1)
    xs = np.concatenate([rng.uniform(-1, 1, 20000), 10.0 ** rng.uniform(-10, 0, 20000) * rng.choice([-1, 1], 20000)])
    for x in xs.astype(np.float32):
        assert q8opt.host_nearest_code(tab, x) == oracle.nearest_code(q, x), float(x)


def test_qtable_accepts_other_codebooks_and_rejects_bad_ones():
    lin = np.linspace(-1, 1, 256).astype(np.float32)
    tab = q8opt.build_qtable(lin)
    rng = np.random.default_rng(2)
    for x in rng.uniform(-1, 1, 5000).astype(np.float32):
        assert q8opt.host_nearest_code(tab, x) == oracle.nearest_code(lin, x)
    bad = lin.copy(); bad[10] = bad[9]
    with pytest.raises(q8opt.Q8Error) as e:
        q8opt.build_qtable(bad)
    assert e.value.status == q8opt.ECODEBOOK
    bad = lin.copy(); bad[255] = 1.5
    with pytest.raises(q8opt.Q8Error):
        q8opt.build_qtable(bad)
    fine = np.sort(np.concatenate([[0.0], 1e-9 * np.arange(1, 256)])).astype(np.float32)   # too fine near zero
    with pytest.raises(q8opt.Q8Error):
        q8opt.build_qtable(fine)
    # a non-zero entry below 2^-99 would put a decision threshold among quotients whose last bits
    # the kernels' short division does not guarantee: refused; 2^-99 itself is accepted
    for v, ok in ((2.0 ** -100, False), (1e-40, False), (-(2.0 ** -120), False), (2.0 ** -99, True)):
        tiny = lin.copy()
        tiny[127], tiny[128] = (0.0, np.float32(v)) if v > 0 else (np.float32(v), 0.0)
        assert tiny[126] < tiny[127] < tiny[128] < tiny[129]
        if ok:
            q8opt.build_qtable(tiny)
        else:
            with pytest.raises(q8opt.Q8Error) as e:
                q8opt.build_qtable(tiny)
            assert e.value.status == q8opt.ECODEBOOK


def test_argument_validation_needs_no_gpu():
    L = q8opt.lib()
    a = 0x1000  # fake, aligned, never dereferenced: validation fails first
    assert L.q8_quantize_blockwise(a, a, -1, 2048, a, a, None) == q8opt.EINVAL
    assert L.q8_quantize_blockwise(a, a, 10, 100, a, a, None) == q8opt.EBLOCK
    assert L.q8_quantize_blockwise(a, a, 10, 32, a, a, None) == q8opt.EBLOCK
    assert L.q8_quantize_blockwise(a, a, 10, 8192, a, a, None) == q8opt.EBLOCK
    assert L.q8_quantize_blockwise(a, None, 10, 256, a, a, None) == q8opt.EINVAL
    assert L.q8_quantize_blockwise(a, a + 4, 10, 256, a, a, None) == q8opt.EALIGN
    assert L.q8_quantize_blockwise(a, a, 0, 256, a, a, None) == q8opt.OK          # n == 0: no-op
    assert L.q8_dequantize_blockwise(a, a, a, 10, 256, a + 8, None) == q8opt.EALIGN
    assert L.q8_dequantize_blockwise(a, a + 1, a, 10, 256, a, None) == q8opt.EALIGN
    adam = lambda *p, n=10, B=2048, flags=0, t=1: L.q8_adam8bit_step(*p, n, B, 1e-3, 0.9, 0.999, 1e-8, 0.0, t, flags, None)
    assert adam(a, a, a, a, a, a, a, a, n=-5) == q8opt.EINVAL
    assert adam(a, a, a, a, a, a, a, a, B=1000) == q8opt.EBLOCK
    assert adam(a, a, a, a, a, a, a, a, flags=8) == q8opt.EINVAL
    assert adam(a, a, a, a, a, a, a, a, flags=1, t=0) == q8opt.EINVAL
    assert adam(None, a, a, a, a, a, a, a) == q8opt.EINVAL
    assert adam(a, a + 8, a, a, a, a, a, a) == q8opt.EALIGN
    assert adam(a, a, a + 2, a, a, a, a, a) == q8opt.EALIGN
    assert adam(a, a, a, a, a, a, a + 8, a) == q8opt.EALIGN
    assert adam(a, a, a, a, a, a, a, a, n=0) == q8opt.OK
    assert L.q8_sgd8bit_step(a, a, a, a, a, 10, 48, 0.1, 0.9, 0.0, None) == q8opt.EBLOCK
    assert L.q8_sgd8bit_step(a, a, None, a, a, 10, 64, 0.1, 0.9, 0.0, None) == q8opt.EINVAL
    assert L.q8_sgd8bit_step(a + 4, a, a, a, a, 10, 64, 0.1, 0.9, 0.0, None) == q8opt.EALIGN
    h = C.c_void_p()
    assert L.q8_plan_create(None, 1, 2048, C.byref(h)) == q8opt.EINVAL
    t = (q8opt.q8_tensor * 1)()
    t[0].w = a; t[0].g = a; t[0].n = 5
    assert L.q8_plan_create(t, 1, 2048, C.byref(h)) == q8opt.EINVAL      # no state storage given
    t[0].m_q = a; t[0].N_m = a + 2
    assert L.q8_plan_create(t, 1, 2048, C.byref(h)) == q8opt.EALIGN
    assert L.q8_plan_create(t, 0, 2048, C.byref(h)) == q8opt.EINVAL
    assert L.q8_plan_create(t, 1, 3, C.byref(h)) == q8opt.EBLOCK
    assert L.q8_plan_destroy(None) == q8opt.EINVAL
    assert L.q8_multi_sgd8bit_step(None, a, 0.1, 0.9, 0.0, None) == q8opt.EINVAL


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as strict C99 and a C program must link
    against the library's host entry points (no GPU is touched)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "c_abi.c"
    src.write_text('#include <stdio.h>\n#include "q8opt.h"\n'
                   "int main(void) {\n"
                   "    float q[256];\n"
                   "    if (q8_build_codebook(1, q) != Q8_OK) return 1;\n"
                   "    if (sizeof(q8_tensor) != 72) return 2;\n"
                   '    printf("%s %.9g %.9g\\n", q8_status_str(Q8_EBLOCK), (double)q[127], (double)q[255]);\n'
                   "    return 0;\n}\n")
    exe = tmp_path / "c_abi"
    libdir = os.path.dirname(q8opt.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(root, "include"),
                           "-o", str(exe), str(src), "-L", libdir, "-lq8opt", "-Wl,-rpath," + libdir])
    out = subprocess.check_output([str(exe)], text=True).split()
    assert float(out[-2]) == 0.0 and float(out[-1]) == 1.0
