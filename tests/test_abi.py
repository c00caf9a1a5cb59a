"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
that include/kunlun.h declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def kb():
    from paper_2602_10016_amd import build
    build.build()
    from paper_2602_10016_amd import binding
    return binding


def test_exports_match_header(kb):
    header = open(os.path.join(ROOT, "include", "kunlun.h")).read()
    declared = set(re.findall(r"^(?:int|size_t|const char\*)\s+(kunlun_\w+)\(", header, flags=re.M))
    assert len(declared) == 16
    assert declared == set(kb.EXPORTS)
    lib = kb.raw()
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror_and_workspace(kb):
    assert kb.strerror(0) == "ok"
    for code in range(-6, 0):
        assert kb.strerror(code) not in ("ok", "unknown status")
    assert kb.strerror(-99) == "unknown status"
    n = kb.workspace_bytes(kb.OP_GDPA_FWD, 1024, 8, 128, 64, 4096, 65536, 1144603)
    assert n >= 4 * 1024 and n % 256 == 0
    assert kb.workspace_bytes(99, 1, 1, 64, 1, 1, 1, 1) == 0
    assert kb.workspace_bytes(kb.OP_GDPA_FWD, -1, 1, 64, 1, 1, 1, 1) == 0


def _fwd(lib, q=0x1000, k=0x1000, v=0x1000, o=0x1000, lse=None, qo=None, kvo=0x1000, B=2, H=2, d=64, max_q=8,
         max_kv=64, total_q=16, total_kv=100, scale=0.1, act=3, head_act=None, dtype=0, ws=0x1000, ws_bytes=1 << 20):
    vp = lambda x: None if x is None else ctypes.c_void_p(x)
    return lib.kunlun_gdpa_fwd(vp(q), vp(k), vp(v), vp(o), vp(lse), vp(qo), vp(kvo), B, H, d, max_q, max_kv,
                               total_q, total_kv, scale, act, head_act, dtype, vp(ws), ws_bytes, None)


def test_gdpa_fwd_rejects_bad_arguments(kb):
    lib = kb.raw()
    assert _fwd(lib, q=None) == kb.ERR_NULL
    assert _fwd(lib, o=None) == kb.ERR_NULL
    assert _fwd(lib, kvo=None) == kb.ERR_NULL
    assert _fwd(lib, k=None) == kb.ERR_NULL
    assert _fwd(lib, B=-1) == kb.ERR_SHAPE
    assert _fwd(lib, total_q=15) == kb.ERR_SHAPE          # dense Q: B * max_q rows
    assert _fwd(lib, total_kv=-5) == kb.ERR_SHAPE
    assert _fwd(lib, d=60) == kb.ERR_UNSUPPORTED
    assert _fwd(lib, d=512) == kb.ERR_UNSUPPORTED
    assert _fwd(lib, H=65) == kb.ERR_UNSUPPORTED
    assert _fwd(lib, act=9) == kb.ERR_UNSUPPORTED
    assert _fwd(lib, act=7) == kb.ERR_UNSUPPORTED and _fwd(lib, act=-1) == kb.ERR_UNSUPPORTED  # 0..6 are the score functions
    assert _fwd(lib, dtype=7) == kb.ERR_UNSUPPORTED
    assert _fwd(lib, scale=float("nan")) == kb.ERR_UNSUPPORTED
    assert _fwd(lib, head_act=(ctypes.c_int32 * 2)(3, 17)) == kb.ERR_UNSUPPORTED
    assert _fwd(lib, q=0x1008) == kb.ERR_ALIGN
    assert _fwd(lib, ws=0x1010) == kb.ERR_ALIGN
    assert _fwd(lib, ws=None) == kb.ERR_WORKSPACE
    assert _fwd(lib, ws_bytes=16) == kb.ERR_WORKSPACE
    assert _fwd(lib, B=0, total_q=0, q=None, o=None) == kb.OK   # empty batch: nothing to do


def test_swa_and_bwd_reject_bad_arguments(kb):
    lib = kb.raw()
    vp = lambda x: None if x is None else ctypes.c_void_p(x)
    P = 0x1000
    swa = lambda **kw: lib.kunlun_swa_fwd(vp(kw.get("q", P)), vp(P), vp(P), vp(kw.get("o", P)), None,
                                          vp(kw.get("off", P)), kw.get("B", 2), 2, kw.get("d", 128), 100,
                                          kw.get("total", 150), 255, 0, 0.1, kw.get("dtype", 0), vp(kw.get("ws", P)),
                                          kw.get("ws_bytes", 1 << 20), None)
    assert swa(q=None) == kb.ERR_NULL
    assert swa(off=None) == kb.ERR_NULL
    assert swa(total=-1) == kb.ERR_SHAPE
    assert swa(d=12) == kb.ERR_UNSUPPORTED
    assert swa(ws_bytes=0) == kb.ERR_WORKSPACE
    assert swa(B=0) == kb.OK
    sbwd = lambda **kw: lib.kunlun_swa_bwd(vp(P), vp(P), vp(P), vp(kw.get("o", P)), vp(kw.get("lse", P)), vp(P),
                                           vp(kw.get("dq", P)), vp(P), vp(P), vp(P), kw.get("B", 2), 2,
                                           kw.get("d", 128), 100, 150, 255, 0, 0.1, 0, vp(kw.get("ws", P)), 1 << 20, None)
    assert sbwd(lse=None) == kb.ERR_NULL
    assert sbwd(o=None) == kb.ERR_NULL
    assert sbwd(dq=None) == kb.ERR_NULL
    assert sbwd(d=20) == kb.ERR_UNSUPPORTED
    assert sbwd(ws=None) == kb.ERR_WORKSPACE
    assert sbwd(B=0) == kb.OK
    bwd = lambda **kw: lib.kunlun_gdpa_bwd(vp(P), vp(P), vp(P), vp(kw.get("o", P)), vp(kw.get("lse", P)),
                                           vp(kw.get("d_o", P)), vp(kw.get("dq", P)), vp(P), vp(P), None, vp(P), 2, 2,
                                           64, 8, 64, kw.get("total_q", 16), 100, 0.1, kw.get("act", 3), None, 0,
                                           vp(kw.get("ws", P)), 1 << 20, None)
    assert bwd(d_o=None) == kb.ERR_NULL
    assert bwd(dq=None) == kb.ERR_NULL
    assert bwd(act=0, lse=None) == kb.ERR_NULL     # softmax backward needs the forward statistics
    assert bwd(act=3, lse=None, o=None, ws=None) == kb.ERR_WORKSPACE  # no softmax head: o, lse optional
    assert bwd(total_q=17) == kb.ERR_SHAPE
    assert bwd(ws=None) == kb.ERR_WORKSPACE


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_sumkron_argument_validation_without_gpu(kb):
    lib = kb.raw()
    call = lambda x=0x1000, z=0x1000, w=0x1000, y=0x1000, B=2, S=32, T=4, D=128, k=2, dtype=kb.BF16, ws=0x1000, n=1 << 30: \
        lib.kunlun_sumkron_fwd(x, z, w, y, B, S, T, D, k, dtype, ws, n, None)
    assert call(S=0) == kb.ERR_SHAPE and call(k=0) == kb.ERR_SHAPE and call(B=-1) == kb.ERR_SHAPE
    assert call(dtype=7) == kb.ERR_UNSUPPORTED
    assert call(D=12) == kb.ERR_UNSUPPORTED
    assert call(B=0) == kb.OK  # nothing to do, nothing launched
    assert call(x=None) == kb.ERR_NULL and call(y=None) == kb.ERR_NULL
    assert call(z=0x1004) == kb.ERR_ALIGN
    assert call(ws=None) == kb.ERR_WORKSPACE and call(n=16) == kb.ERR_WORKSPACE
    assert call(ws=0x1010) == kb.ERR_ALIGN
    # the paper's shape runs as one kernel: the workspace holds the prepared copies of Z and W, nothing per example
    need = kb.sumkron_workspace_bytes(1024, 256, 32, 384, 8)
    assert 8 * 32 * 256 * 2 + 8 * 384 * 384 * 2 <= need < 1024 * 32 * 8 * 384 * 2
    assert kb.sumkron_workspace_bytes(1, 256, 32, 384, 8) == need
    # two-GEMM shapes (T != 32 here): the transposed Z and the bf16 intermediate of every example
    assert kb.sumkron_workspace_bytes(1024, 256, 16, 384, 8) >= 1024 * 16 * 8 * 384 * 2
    assert kb.sumkron_workspace_bytes(4, 0, 1, 8, 1) == 0


def test_sumkron_bwd_argument_validation_without_gpu(kb):
    lib = kb.raw()
    call = lambda x=0x1000, z=0x1000, w=0x1000, dy=0x1000, dx=0x1000, dz=0x1000, dw=0x1000, B=2, S=32, T=4, D=128, k=2, \
        dtype=kb.BF16, ws=0x1000, n=1 << 30: lib.kunlun_sumkron_bwd(x, z, w, dy, dx, dz, dw, B, S, T, D, k, dtype, ws, n, None)
    assert call(S=0) == kb.ERR_SHAPE and call(k=0) == kb.ERR_SHAPE and call(B=-1) == kb.ERR_SHAPE
    assert call(dtype=7) == kb.ERR_UNSUPPORTED
    assert call(D=12) == kb.ERR_UNSUPPORTED
    assert call(x=None) == kb.ERR_NULL and call(dy=None) == kb.ERR_NULL and call(dx=None) == kb.ERR_NULL
    assert call(dz=None) == kb.ERR_NULL and call(dw=None) == kb.ERR_NULL and call(w=None) == kb.ERR_NULL
    assert call(dz=None, B=0) == kb.ERR_NULL      # an empty batch still writes zero weight gradients
    assert call(dw=0x1004) == kb.ERR_ALIGN
    assert call(ws=None) == kb.ERR_WORKSPACE and call(n=16) == kb.ERR_WORKSPACE
    assert call(ws=0x1010) == kb.ERR_ALIGN
    # tiled path: Zt, Zc, U, G in bf16 and the larger of the two partial-sum buffers
    need = kb.sumkron_bwd_workspace_bytes(1024, 256, 32, 384, 8)
    assert need >= 2 * 1024 * 32 * 8 * 384 * 2 and kb.sumkron_bwd_workspace_bytes(4, 0, 1, 8, 1) == 0
    # plain path: U and G in fp32
    assert kb.sumkron_bwd_workspace_bytes(3, 40, 6, 24, 3, kb.FP32) >= 2 * 3 * 6 * 3 * 24 * 4
    assert kb.sumkron_bwd_workspace_bytes(0, 256, 32, 384, 8) > 0     # an empty batch is a legal size


def test_backward_workspace_covers_the_partial_sums_of_the_few_keys_path(kb):
    B, H, d, T = 128, 4, 128, 150000
    two_pass = kb.workspace_bytes(kb.OP_GDPA_BWD, B, H, d, 2048, 33, T, B * 33)
    one_pass = kb.workspace_bytes(kb.OP_GDPA_BWD, B, H, d, 2048, 32, T, B * 32)
    # (T/128 + B) * H = 5200 tile-heads: chunks of 4 tiles, one fp32 [2][32][d] partial tile per chunk and head
    assert one_pass - two_pass >= (T // 512) * H * 2 * 32 * d * 4
    # at most 64 queries per example: the fused kernel, no partial sums; the window op never takes this path
    assert kb.workspace_bytes(kb.OP_GDPA_BWD, B, H, d, 64, 32, B * 64, B * 32) < (1 << 20)
    assert kb.workspace_bytes(kb.OP_SWA_BWD, B, H, d, 32, 32, B * 32, B * 32) < (1 << 20)


def test_check_offsets_argument_validation_without_gpu(kb):
    lib = kb.raw()
    call = lambda off=0x1000, B=4, total=100, max_len=64, out=0x1000: lib.kunlun_check_offsets(off, B, total, max_len, out, None)
    assert call(B=-1) == kb.ERR_SHAPE and call(total=-1) == kb.ERR_SHAPE and call(max_len=-1) == kb.ERR_SHAPE
    assert call(off=None) == kb.ERR_NULL and call(out=None) == kb.ERR_NULL
    assert call(off=0x1002) == kb.ERR_ALIGN and call(out=0x1001) == kb.ERR_ALIGN


def test_static_scratch_entry_point_validates_on_the_host(kb):
    """kunlun_gdpa_fwd_static: the checks of kunlun_gdpa_fwd, then its own size limit - all before any device is
    touched (this test runs without a GPU)."""
    lib = kb.raw()
    vp = lambda x: None if x is None else ctypes.c_void_p(x)

    def call(q=0x1000, kvo=0x1000, B=2, d=64, max_q=8, total_q=16, total_kv=100, act=3):
        return lib.kunlun_gdpa_fwd_static(vp(q), vp(0x1000), vp(0x1000), vp(0x1000), None, None, vp(kvo), B, 2, d, max_q, 64,
                                          total_q, total_kv, 0.1, act, None, 0, None)

    assert call(q=None) == kb.ERR_NULL
    assert call(kvo=None) == kb.ERR_NULL
    assert call(q=0x1004) == kb.ERR_ALIGN
    assert call(d=60) == kb.ERR_UNSUPPORTED
    assert call(act=9) == kb.ERR_UNSUPPORTED
    assert call(total_q=15) == kb.ERR_SHAPE
    assert call(B=0, total_q=0) == kb.OK
    big = 200_000
    assert kb.workspace_bytes(kb.OP_GDPA_FWD, big, 2, 64, 8, 64, big * 8, 100) > kb.STATIC_SCRATCH_BYTES
    assert call(B=big, total_q=big * 8) == kb.ERR_WORKSPACE


def test_polynomial_gelu_coefficients_agree_everywhere():
    """The polynomial GELU is defined by seven coefficients and a clamp that are written out four times (the ABI
    header, the HIP kernels, the oracle, the oracle's pins): the copies must be the same numbers."""
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    read = lambda *p: open(os.path.join(root, *p)).read()
    num = r"[-+]?\d\.\d{10}e[-+]\d\d"
    header = read("include", "kunlun.h")
    h = header[header.index("gelu_poly(x) ="):header.index("(C q(C^2) = 1/2")]
    from_header = [float(x.replace(" ", "")) for x in re.findall(r"[-+]?\s?" + num[5:], h)]
    kernels = read("paper_2602_10016_amd", "csrc", "common.h")
    k = kernels[kernels.index("constexpr float A0"):kernels.index("const float t = __builtin_amdgcn_fmed3f")]
    from_kernels = [float(x) for x in re.findall(num, k)]
    oracle_c = read("oracle", "kunlun_oracle.c")
    o = oracle_c[oracle_c.index("GELU_POLY_Q[7]"):oracle_c.index("/* cdf(x) of the polynomial GELU")]
    from_oracle = [float(x) for x in re.findall(num, o)]
    from tests.test_oracle_pins import GELU_POLY_C, GELU_POLY_Q
    assert len(from_oracle) == 7 and from_oracle == from_kernels == GELU_POLY_Q
    assert [abs(x) for x in from_header] == [abs(x) for x in from_oracle]  # (the header writes the signs as operators)
    assert "C = 3.875" in header and "GELU_POLY_C = 3.875f" in kernels and "GELU_POLY_C = 3.875;" in oracle_c and GELU_POLY_C == 3.875


def test_header_is_plain_c_and_links_from_a_c_program(tmp_path):
    """include/kunlun.h compiles as strict C99 (no C++-only construct in the ABI) and a C program linked against the
    library reaches the host-side argument checks (a negative size: refused before any device is touched)."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.join(root, "paper_2602_10016_amd")
    src = tmp_path / "use_kunlun.c"
    src.write_text(
        '#include "kunlun.h"\n#include <stdio.h>\n#include <string.h>\n'
        "int main(void) {\n"
        "    if (strlen(kunlun_strerror(KUNLUN_ERR_SHAPE)) == 0) return 2;\n"
        "    if (kunlun_workspace_bytes(KUNLUN_OP_GDPA_FWD, 4, 2, 64, 8, 100, 32, 400) == 0) return 3;\n"
        "    return kunlun_gdpa_fwd(0, 0, 0, 0, 0, 0, 0, -1, 1, 64, 1, 1, 0, 0, 1.0f, KUNLUN_ACT_GELU_POLY, 0, KUNLUN_BF16, 0, 0, 0)\n"
        "               == KUNLUN_ERR_SHAPE ? 0 : 1;\n"
        "}\n")
    exe = tmp_path / "use_kunlun"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-lkunlun", f"-Wl,-rpath,{libdir}"], check=True)
    assert subprocess.run([str(exe)]).returncode == 0
