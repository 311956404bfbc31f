"""CPU-only checks of the C-ABI library: it loads, exports what the header declares, its host
tables equal the oracle's, and its argument checks reject bad calls before anything is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import dynamic_code as dc
from paper_2407_19775_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not os.path.exists(binding.LIB_PATH),
                                reason="libmmd8.so not built (python -m paper_2407_19775_amd.build)")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mmd8.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mmd8_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert len(names) >= 12
    L = ctypes.CDLL(binding.LIB_PATH)
    for name in names:
        assert hasattr(L, name), name
    for name in binding.EXPORTS:
        assert name in names


def test_every_exported_symbol_is_declared():
    """The other direction: the library exports no mmd8_* function that the header does not declare."""
    import shutil
    import subprocess
    if shutil.which("nm") is None:
        pytest.skip("no nm")
    out = subprocess.run(["nm", "-D", "--defined-only", binding.LIB_PATH], capture_output=True, text=True, check=True).stdout
    exported = sorted({line.split()[-1] for line in out.splitlines() if re.search(r"\s[TW]\s+mmd8_", line)})
    assert exported, "no mmd8_* symbols found"
    assert exported == declared_functions()


def test_packed_weights_of_another_layout_are_refused():
    """A blob written under another layout tag is not multiplied: MMD8_E_VERSION before anything is launched."""
    L = binding.lib()
    fake, y = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x2000)
    tag = L.mmd8_packed_weight_layout()
    ws = L.mmd8_linear_workspace_bytes(8, 128, 64)
    for bad in (0, tag - 1, tag + 1, tag ^ 0x00010000):
        assert L.mmd8_mixed_int8_linear(fake, 8, 128, 128, fake, bad, fake, 64, None, 6.0, y, 64, fake, ws, None, None) == -5
        assert L.mmd8_mixed_int8_linear_gelu(fake, 8, 128, 128, fake, bad, fake, 64, None, 6.0, y, 64, fake, ws, None, None) == -5
        assert L.mmd8_mixed_int8_linear_residual(fake, 8, 128, 128, fake, bad, fake, 64, None, 6.0, fake, 64, y, 64, fake, ws,
                                                 None, None) == -5
        assert L.mmd8_mixed_int8_linear_to_codes(fake, 8, 128, 128, fake, bad, fake, 64, None, 6.0, None, 64, 64, y, y, None,
                                                 fake, L.mmd8_linear_to_codes_workspace_bytes(8, 128, 64, 64), None, None) == -5
        assert L.mmd8_mixed_int8_linear_lora(fake, 8, 128, 128, fake, bad, fake, 64, None, 6.0, fake, fake, 16, None, y, 64, fake,
                                             L.mmd8_linear_lora_workspace_bytes(8, 128, 64, 16), None, None) == -5
        assert L.mmd8_mixed_int8_linear_from_codes(fake, fake, 64, 8, 128, y, fake, bad, fake, 64, None, 6.0,
                                                   ctypes.c_void_p(0x4000), 64, fake, ws, None, None) == -5
        assert L.mmd8_unpack_weight(fake, bad, 128, 64, y, None) == -5
        assert L.mmd8_mixed_int8_linear(None, 0, 128, 128, None, bad, None, 64, None, 6.0, None, 64, None, 0, None, None) == -5
    assert b"layout" in L.mmd8_status_string(-5)
    pw = binding.PackedWeight(None, None, 128, 64, layout=tag + 1)       # the binding hands the stored tag back
    assert pw.layout == tag + 1 and binding.PackedWeight(None, None, 128, 64).layout == tag


def test_host_tables_equal_the_oracle_bit_for_bit():
    T = binding.code_table().numpy()
    Mid = binding.code_midpoints().numpy()
    assert T.tobytes() == dc.code_table().tobytes()
    assert Mid.tobytes() == dc.midpoints().tobytes()


def test_threshold_pattern_is_the_fp16_ceiling():
    L = binding.lib()
    finite = np.arange(0, 0x7c00, dtype=np.uint16)
    vals = finite.view(np.float16).astype(np.float64)
    rng = np.random.default_rng(0)
    taus = np.concatenate([
        vals[rng.integers(0, vals.size, 300)],                           # exactly representable
        vals[rng.integers(1, vals.size, 300)] * (1 - 1e-4),              # just below a value
        vals[rng.integers(0, vals.size - 1, 300)] * (1 + 1e-4) + 1e-12,  # just above a value
        [6.0, 0.0, -1.0, 1e-9, 5.96e-8, 6.0e-8, 65504.0, 65505.0, 1e9, np.inf, 6.1e-5, 6.2e-5],
    ]).astype(np.float32)
    for tau in taus:
        got = L.mmd8_threshold_fp16_pattern(float(tau))
        if tau <= 0:
            want = 0
        else:
            above = np.flatnonzero(vals >= np.float64(tau))
            want = int(above[0]) if above.size else 0x7c00
        assert got == want, (tau, got, want)


def test_sizes_and_layout_tag():
    L = binding.lib()
    assert L.mmd8_packed_weight_layout() != 0
    assert L.mmd8_packed_weight_bytes(4096, 12288) >= 4096 * 12288
    assert L.mmd8_packed_weight_bytes(4096, 12288) % 256 == 0
    assert L.mmd8_packed_weight_bytes(4095, 12288) == 0        # K % 16
    assert L.mmd8_packed_weight_bytes(4096, 12) == 0           # N % 8
    assert L.mmd8_packed_weight_bytes(1 << 20, 64) == 0        # K too large
    assert L.mmd8_linear_workspace_bytes(2048, 4096, 4096) >= 2048 * 4096
    assert L.mmd8_linear_workspace_bytes(0, 4096, 4096) > 0
    assert L.mmd8_linear_workspace_bytes(-1, 4096, 4096) == 0


def test_bad_arguments_are_rejected_before_any_launch():
    L = binding.lib()
    fake = ctypes.c_void_p(0x1000)         # aligned, never dereferenced: every call below must fail first
    odd = ctypes.c_void_p(0x1002)
    assert L.mmd8_quantize_blockwise(fake, 1024, 100, fake, fake, None) == -2      # block % 64
    assert L.mmd8_quantize_blockwise(fake, 1024, 8192, fake, fake, None) == -2     # block > 4096
    assert L.mmd8_quantize_blockwise(None, 1024, 256, fake, fake, None) == -1
    assert L.mmd8_quantize_blockwise(odd, 1024, 256, fake, fake, None) == -1
    assert L.mmd8_quantize_blockwise(None, 0, 256, None, None, None) == 0          # empty is fine
    assert L.mmd8_dequantize_blockwise(fake, None, 1024, 256, fake, None) == -1
    assert L.mmd8_dequantize_blockwise(None, None, 0, 64, None, None) == 0
    assert L.mmd8_prequantize_weight(fake, 100, 64, 64, fake, fake, None) == -2    # K % 16
    assert L.mmd8_prequantize_weight(fake, 128, 64, 32, fake, fake, None) == -1    # ldw < N
    assert L.mmd8_prequantize_weight(fake, 128, 64, 64, None, fake, None) == -1
    ws = L.mmd8_linear_workspace_bytes(8, 128, 64)
    tag = L.mmd8_packed_weight_layout()
    args = dict(X=fake, M=8, K=128, ldx=128, W=fake, c=fake, N=64, bias=None, tau=6.0, Y=ctypes.c_void_p(0x2000),
                ldy=64, ws=fake, wsb=ws)

    def call(**kw):
        a = dict(args, **kw)
        return L.mmd8_mixed_int8_linear(a["X"], a["M"], a["K"], a["ldx"], a["W"], tag, a["c"], a["N"], a["bias"],
                                        a["tau"], a["Y"], a["ldy"], a["ws"], a["wsb"], None, None)

    assert call(K=100) == -2
    assert call(N=60) == -2
    assert call(tau=float("nan")) == -1
    assert call(ldx=64) == -1
    assert call(ldy=60) == -1
    assert call(Y=fake) == -1                                                      # aliasing X
    assert call(Y=ctypes.c_void_p(0x1000 + 16)) == -1                              # overlapping X (8 x 128 fp16 = 2 KB)
    assert call(Y=ctypes.c_void_p(0x1000 + 2032)) == -1                            # its last 16 bytes
    assert call(Y=ctypes.c_void_p(0x1000 + 2048), wsb=ws - 1) == -3                # right behind X: passes that check
    assert call(wsb=ws - 1) == -3
    assert call(X=None) == -1
    assert call(M=-1) == -1
    assert call(M=0, X=None, Y=None, ws=None, wsb=0) == 0                          # empty is fine
    assert b"workspace" in L.mmd8_status_string(-3)


def test_adapter_arguments_are_rejected_before_any_launch():
    L = binding.lib()
    fake, y = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x2000)
    odd = ctypes.c_void_p(0x1008)
    assert L.mmd8_linear_lora_workspace_bytes(8, 128, 64, 16) > L.mmd8_linear_workspace_bytes(8, 128, 64)
    assert L.mmd8_linear_lora_workspace_bytes(2048, 4096, 4096, 64) > L.mmd8_linear_workspace_bytes(2048, 4096, 4096)
    for bad_r in (0, 4, 12, 72, -8):
        assert L.mmd8_linear_lora_workspace_bytes(8, 128, 64, bad_r) == 0
    ws = L.mmd8_linear_lora_workspace_bytes(8, 128, 64, 16)

    def call(A=fake, B=fake, r=16, T=None, wsb=ws, K=128):
        return L.mmd8_mixed_int8_linear_lora(fake, 8, K, 128, fake, L.mmd8_packed_weight_layout(), fake, 64, None, 6.0, A, B, r,
                                             T, y, 64, fake, wsb, None, None)

    assert call(r=4) == -2 and call(r=20) == -2 and call(r=128) == -2
    assert call(A=None) == -1 and call(B=None) == -1
    assert call(A=odd) == -1 and call(T=odd) == -1
    assert call(K=100) == -2
    assert call(wsb=L.mmd8_linear_workspace_bytes(8, 128, 64)) == -3               # sized without the adapter


def test_coded_output_arguments_are_rejected_before_any_launch():
    L = binding.lib()
    fake, out = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x2000)
    odd = ctypes.c_void_p(0x1008)
    base = L.mmd8_linear_workspace_bytes
    wsb = L.mmd8_linear_to_codes_workspace_bytes
    # the layer's last kernel encodes: nothing beyond what the decode path keeps for its partial outputs
    assert wsb(300, 128, 512, 256) == base(300, 128, 512)
    assert wsb(8, 128, 520, 4096) >= base(8, 128, 520)
    # the encoder runs after the layer: room for the fp16 tensor it reads
    assert wsb(300, 128, 512, 1024) >= base(300, 128, 512) + 300 * 512 * 2
    assert wsb(300, 128, 520, 64) >= base(300, 128, 520) + 300 * 520 * 2
    assert wsb(100, 128, 520, 4096) >= base(100, 128, 520) + 100 * 520 * 2
    for bad_block in (0, 32, 100, 8192, -64):
        assert wsb(8, 128, 64, bad_block) == 0
    ws = wsb(8, 128, 64, 64)

    def call(res=None, ldr=64, block=64, codes=out, absmax=out, H=None, wsb_=ws, K=128):
        return L.mmd8_mixed_int8_linear_to_codes(fake, 8, K, 128, fake, L.mmd8_packed_weight_layout(), fake, 64, None, 6.0, res,
                                                 ldr, block, codes, absmax, H, fake, wsb_, None, None)

    assert call(block=48) == -2 and call(block=8192) == -2 and call(K=100) == -2
    assert call(codes=None) == -1 and call(absmax=None) == -1 and call(codes=odd) == -1
    assert call(res=fake, ldr=56) == -1 and call(res=fake, ldr=68) == -1 and call(res=odd) == -1
    assert call(H=odd) == -1
    assert call(wsb_=ws - 256) == -3


def test_residual_arguments_are_rejected_before_any_launch():
    L = binding.lib()
    fake, y = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x2000)
    odd = ctypes.c_void_p(0x1008)
    ws = L.mmd8_linear_workspace_bytes(8, 128, 64)

    def call(res=fake, ldr=64, Y=y, K=128):
        return L.mmd8_mixed_int8_linear_residual(fake, 8, K, 128, fake, L.mmd8_packed_weight_layout(), fake, 64, None, 6.0, res, ldr,
                                                 Y, 64, fake, ws, None, None)

    assert call(res=None) == -1 and call(res=odd) == -1 and call(ldr=56) == -1 and call(ldr=68) == -1
    assert call(Y=None) == -1 and call(K=100) == -2


def test_public_headers_are_plain_c():
    """The boundary is a C ABI: both headers must go through a C99 compiler on their own."""
    import shutil
    import subprocess
    import tempfile
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    with tempfile.TemporaryDirectory() as d:
        src = os.path.join(d, "use.c")
        with open(src, "w") as f:
            f.write('#include "mmd8.h"\n#include "mtpp.h"\nint main(void) { return mmd8_status_string(0) == 0; }\n')
        r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                            "-I", os.path.join(ROOT, "include"), src], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_gelu_coefficients_in_the_kernel_header_reproduce_erfc():
    """The GPU's GELU is x Phi(x) with Phi(-|x|) = t exp(-z^2 + g(t)) / 2, t = 1 / (1 + z / 2), z = |x| / sqrt 2, g a
    degree-8 polynomial whose coefficients are written out in csrc/common.h.  Re-evaluated here in float64 from
    the header's own text and compared with math.erfc over the whole range in which the result is a nonzero fp16
    number: the constants are pinned to the function, not to the script that once fitted them."""
    import math
    text = open(os.path.join(ROOT, "paper_2407_19775_amd", "csrc", "common.h")).read()
    body = text[text.index("gelu_to_half_bits(float x)"):]
    body = body[:body.index("return float_to_half_bits")]
    lead = float(re.search(r"float g = ([-+0-9.e]+)f;", body).group(1))
    rest = [float(v) for v in re.findall(r"g = __builtin_fmaf\(g, t, ([-+0-9.e]+)f\);", body)]
    assert len(rest) == 8
    worst = 0.0
    for i in range(0, 5501):
        x = i * 1e-3
        z = x / math.sqrt(2.0)
        t = 1.0 / (1.0 + 0.5 * z)
        g = lead
        for c in rest:
            g = g * t + c
        phi = 0.5 * t * math.exp(-z * z + g)
        exact = 0.5 * math.erfc(z)
        worst = max(worst, abs(phi - exact) / exact)
    assert worst < 1e-5, worst


def test_the_entry_point_without_a_workspace_refuses_sizes_beyond_its_array():
    L = binding.lib()
    fake, y = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x40000000)
    tag = L.mmd8_packed_weight_layout()

    def call(M, K, N, layout=tag, tau=6.0):
        return L.mmd8_mixed_int8_linear_static(fake, M, K, K, fake, layout, fake, N, None, tau, y, N, None, None)

    assert L.mmd8_linear_workspace_bytes(2048, 28672, 8192) > binding.STATIC_WORKSPACE_BYTES
    assert call(2048, 28672, 8192) == -3                          # before any HIP call: no GPU needed to be told so
    assert call(4096, 8192, 8192) == -3
    assert call(8, 100, 64) == -2 and call(-1, 128, 64) == -1
    assert call(8, 128, 64, layout=tag + 1) == -5
    assert call(0, 128, 64) == 0 and call(0, 128, 64, tau=float("nan")) == -1


def test_variant_entry_points_check_their_arguments():
    L = binding.lib()
    fake, y = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x40000000)
    odd1 = ctypes.c_void_p(0x1001)
    # block scales stored as fp16: 2-byte alignment is enough, odd addresses are not
    assert L.mmd8_quantize_blockwise_h(fake, 1024, 100, fake, fake, None) == -2
    assert L.mmd8_quantize_blockwise_h(fake, 1024, 256, fake, odd1, None) == -1
    assert L.mmd8_quantize_blockwise_h(None, 0, 256, None, None, None) == 0
    assert L.mmd8_dequantize_blockwise_h(fake, odd1, 1024, 256, fake, None) == -1
    assert L.mmd8_dequantize_blockwise_h(fake, None, 1024, 256, fake, None) == -1
    assert L.mmd8_dequantize_blockwise_h(None, None, 0, 64, None, None) == 0
    # the other readings of the layer
    tag = L.mmd8_packed_weight_layout()
    ws = L.mmd8_linear_workspace_bytes(8, 128, 64)

    def call(rd, layout=tag, wsb=ws):
        return L.mmd8_mixed_int8_linear_readings(fake, 8, 128, 128, fake, layout, fake, 64, None, 6.0, rd, y, 64, fake, wsb,
                                                 None, None)

    R = binding.Readings
    assert call(None) == -1
    assert call(ctypes.byref(R(2, None, 0))) == -1 and call(ctypes.byref(R(-1, None, 0))) == -1
    assert call(ctypes.byref(R(0, 0x2000, 60))) == -1          # ldw < N
    assert call(ctypes.byref(R(0, 0x2000, 68))) == -1          # ldw % 8
    assert call(ctypes.byref(R(1, 0x2008, 64))) == -1          # misaligned
    assert call(ctypes.byref(R(1, 0x2000, 64)), layout=tag + 1) == -5
    assert call(ctypes.byref(R(1, 0x2000, 64)), wsb=ws - 1) == -3
