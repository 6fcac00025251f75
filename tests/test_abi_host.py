"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mxfp4.h")


@pytest.fixture(scope="module")
def L():
    from paper_2502_20853_amd import binding, build
    if build.is_stale():
        build.build()
    return binding.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mx_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_exported(L):
    from paper_2502_20853_amd import binding
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for six in ("mx_quantize", "mx_quantize_transposed", "mx_linear_fwd", "mx_linear_bwd_dx",
                "mx_linear_bwd_dw", "mx_ema_weight_quant"):
        assert six in names
    for n in names:
        assert hasattr(L, n), n
    assert L.mx_version().decode().startswith("mxfp4-gfx950")
    assert L.mx_last_hip_error() == 0


def test_binding_and_oracle_are_independent():
    pkg = os.path.join(ROOT, "paper_2502_20853_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            assert "paper_2502_20853_amd" not in open(os.path.join(ROOT, "oracle", f)).read(), f


P = ctypes.c_void_p
FAKE = 0x7F0000000000          # never dereferenced: every call below fails validation first


def q(L, src=FAKE, dtype=1, rows=64, cols=64, ld=64, codes=FAKE, scales=FAKE, rnd=0, mode=0,
      seed=0, tid=0, base=0):
    return L.mx_quantize(P(src), dtype, rows, cols, ld, P(codes), P(scales), rnd, mode, seed, tid, base, P(0))


def test_quantize_rejects(L):
    assert q(L, src=0) == -1 and q(L, codes=0) == -1 and q(L, scales=0) == -1
    assert q(L, dtype=2) == -3
    assert q(L, mode=2) == -4 and q(L, rnd=5) == -4
    assert q(L, cols=48) == -2 and q(L, rows=0) == -2 and q(L, ld=32) == -2 and q(L, cols=0) == -2
    assert q(L, rows=1 << 40, cols=1 << 20, ld=1 << 20) == -2
    assert q(L, src=FAKE + 2) == -5 and q(L, codes=FAKE + 1) == -5
    assert q(L, ld=68) == -5                       # bf16 rows must start 16-byte aligned
    assert q(L, rnd=1, base=4) == -5               # Philox blocks of 8 elements


def qt(L, src=FAKE, dtype=1, rows=64, cols=64, ld=64, ct=FAKE, st=FAKE, rt=1, tidt=6, pre=1,
       cr=FAKE, sr=FAKE, rr=0, tidr=1, rci=0, rsi=0, mode=0, seed=0, base=0):
    return L.mx_quantize_transposed(P(src), dtype, rows, cols, ld, P(ct), P(st), rt, tidt, pre,
                                    P(cr), P(sr), rr, tidr, P(rci), P(rsi), mode, seed, base, P(0))


def test_quantize_transposed_rejects(L):
    assert qt(L, ct=0) == -1 and qt(L, src=0) == -1
    assert qt(L, cr=0) == -1 and qt(L, sr=0) == -1             # half-set optional pair
    assert qt(L, rci=FAKE) == -1
    assert qt(L, rows=48) == -2 and qt(L, cols=16) == -2 and qt(L, ld=32) == -2
    assert qt(L, pre=2) == -4 and qt(L, rt=3) == -4 and qt(L, rr=-1) == -4 and qt(L, mode=9) == -4
    assert qt(L, rci=FAKE, rsi=FAKE) == -4                      # given row result excludes a row output
    assert qt(L, rci=FAKE, rsi=FAKE, cr=0, sr=0, pre=0) == -4   # and needs pre_quant
    assert qt(L, dtype=7) == -3
    assert qt(L, base=3) == -5 and qt(L, ct=FAKE + 2) == -5


def g(L, fn, a=FAKE, as_=FAKE, b=FAKE, bs=FAKE, N=64, C=64, D=64, out=FAKE, dt=0, ldo=64, ws=0, wsb=0):
    return getattr(L, fn)(P(a), P(as_), P(b), P(bs), N, C, D, P(out), dt, ldo, P(ws), wsb, P(0))


def test_linear_fwd_bias_rejects(L):
    def call(bias=FAKE, a=FAKE, C=64, ldo=64, D=64):
        return L.mx_linear_fwd_bias(P(a), P(FAKE), P(FAKE), P(FAKE), 64, C, D, P(bias), P(FAKE), 0, ldo, P(0), 0, P(0))
    assert call(bias=0) == -1 and call(a=0) == -1
    assert call(C=66, ldo=66) == -2                   # the bias is read four columns at a time
    assert call(bias=FAKE + 8) == -5
    assert call(D=48) == -2                           # everything else as mx_linear_fwd


def test_linear_rejects(L):
    for fn in ("mx_linear_fwd", "mx_linear_bwd_dx", "mx_linear_bwd_dw"):
        assert g(L, fn, a=0) == -1 and g(L, fn, bs=0) == -1 and g(L, fn, out=0) == -1
        assert g(L, fn, dt=3) == -3
        assert g(L, fn, N=0) == -2 and g(L, fn, ldo=8) == -2
        assert g(L, fn, a=FAKE + 8) == -5
    assert g(L, "mx_linear_fwd", D=48) == -2          # contraction dims must be multiples of 32
    assert g(L, "mx_linear_bwd_dx", C=48) == -2
    assert g(L, "mx_linear_bwd_dw", N=48) == -2
    assert g(L, "mx_linear_fwd", D=(1 << 24) + 32) == -2      # contraction dimension above 2^24
    # a product that splits K demands its workspace
    need = L.mx_linear_workspace_bytes(2, 50432, 768, 768)
    assert need > 0 and need % (768 * 768 * 4) == 0
    assert g(L, "mx_linear_bwd_dw", N=50432, C=768, D=768, ldo=768) == -6
    assert g(L, "mx_linear_bwd_dw", N=50432, C=768, D=768, ldo=768, ws=FAKE, wsb=need - 1) == -6
    assert L.mx_linear_workspace_bytes(0, 50432, 2304, 768) == 0
    assert L.mx_linear_workspace_bytes(9, 64, 64, 64) == 0


def test_ema_rejects(L):
    def e(w=FAKE, dtype=0, ema=FAKE, beta=0.998, upd=1, rows=64, cols=64, ld=64, codes=FAKE, scales=FAKE, mode=0):
        return L.mx_ema_weight_quant(P(w), dtype, P(ema), beta, upd, rows, cols, ld, P(codes), P(scales), mode, P(0))
    assert e(ema=0) == -1 and e(w=0) == -1
    assert e(upd=3) == -4 and e(beta=1.0) == -4 and e(beta=-0.1) == -4 and e(beta=float("nan")) == -4
    assert e(cols=40) == -2
    assert e(ema=FAKE + 4) == -5


def test_calibration_copy_rejects(L):
    assert L.mx_calibration_copy(P(0), P(FAKE), 64, P(0)) == -1
    assert L.mx_calibration_copy(P(FAKE), P(FAKE), 60, P(0)) == -2
    assert L.mx_calibration_copy(P(FAKE + 4), P(FAKE), 64, P(0)) == -5


def test_dequantize_rejects(L):
    assert L.mx_dequantize(P(0), P(FAKE), 4, 32, P(FAKE), P(0)) == -1
    assert L.mx_dequantize(P(FAKE), P(FAKE), 4, 33, P(FAKE), P(0)) == -2


def test_oscillation_and_ramping_rejects(L):
    def o(w=FAKE, dtype=0, rows=64, cols=64, ld=64, codes=FAKE, scales=FAKE, wp=FAKE, cp=FAKE, sp=FAKE,
          dw=FAKE, dq=FAKE, init=0):
        return L.mx_oscillation_accumulate(P(w), dtype, rows, cols, ld, P(codes), P(scales), P(wp), P(cp), P(sp),
                                           P(dw), P(dq), init, P(0))
    assert o(w=0) == -1 and o(wp=0) == -1 and o(cp=0) == -1 and o(dq=0) == -1
    assert o(dtype=5) == -3 and o(cols=40) == -2 and o(ld=32) == -2
    assert o(init=2) == -4
    assert o(dw=FAKE + 4) == -5 and o(cp=FAKE + 2) == -5

    def r(dw=FAKE, dq=FAKE, n=64, k1=16.0, k2=5, nmax=16, out=FAKE):
        return L.mx_ramping_factor(P(dw), P(dq), n, k1, k2, nmax, P(out), P(0))
    assert r(dw=0) == -1 and r(out=0) == -1
    assert r(n=0) == -2
    assert r(k1=0.0) == -4 and r(k1=float("nan")) == -4 and r(k2=-1) == -4 and r(nmax=0) == -4


def test_diagnostics_rejects(L):
    def c(w=FAKE, dtype=0, rows=64, cols=64, ld=64, mode=0, conf=FAKE, hist=FAKE, bins=16):
        return L.mx_quant_confidence(P(w), dtype, rows, cols, ld, mode, P(conf), P(hist), bins, P(0))
    assert c(w=0) == -1 and c(conf=0, hist=0) == -1
    assert c(dtype=7) == -3 and c(mode=2) == -4
    assert c(cols=48) == -2 and c(ld=32) == -2 and c(rows=0) == -2
    assert c(bins=0) == -4 and c(bins=1025) == -4
    assert c(conf=FAKE + 8) == -5 and c(hist=FAKE + 4) == -5 and c(w=FAKE + 4) == -5

    need = L.mx_rate_of_change_workspace_bytes()
    assert need > 0

    def r(x=FAKE, dtype=0, rows=64, cols=64, ld=64, xp=FAKE, init=0, ws=FAKE, wsb=None, res=FAKE):
        return L.mx_rate_of_change_step(P(x), dtype, rows, cols, ld, P(xp), init, P(ws),
                                        need if wsb is None else wsb, P(res), P(0))
    assert r(x=0) == -1 and r(xp=0) == -1 and r(res=0) == -1
    assert r(dtype=3) == -3 and r(init=-1) == -4
    assert r(cols=60) == -2 and r(ld=56) == -2
    assert r(ws=0) == -6 and r(wsb=need - 1) == -6
    assert r(xp=FAKE + 4) == -5 and r(res=FAKE + 4) == -5


def test_ramping_adamw_rejects(L):
    import ctypes
    f = ctypes.c_float

    def a(w=FAKE, g=FAKE, gd=0, n=64, m=FAKE, v=FAKE, u=FAKE, fac=FAKE, acc=FAKE, st=FAKE,
          lr=1e-3, b1=0.9, b2=0.999, eps=1e-8, wd=0.01):
        return L.mx_ramping_adamw_step(P(w), P(g), gd, n, P(m), P(v), P(u), P(fac), P(acc), P(st),
                                       f(lr), f(b1), f(b2), f(eps), f(wd), P(0))
    assert a(w=0) == -1 and a(g=0) == -1 and a(m=0) == -1 and a(u=0) == -1
    assert a(acc=0) == -1 and a(st=0) == -1            # a factor needs its accumulators
    assert a(gd=2) == -3
    assert a(n=0) == -2 and a(n=66) == -2
    assert a(b1=1.0) == -4 and a(b2=0.0) == -4 and a(lr=-1.0) == -4 and a(eps=float("nan")) == -4 and a(wd=-0.1) == -4
    assert a(w=FAKE + 4) == -5 and a(u=FAKE + 8) == -5 and a(fac=FAKE + 4) == -5 and a(g=FAKE + 8) == -5
    assert a(g=FAKE + 8, gd=1) != -5                   # BF16 gradients need 8-byte alignment only


def test_transposed_batch_rejects(L):
    import ctypes
    from paper_2502_20853_amd.binding import _TransposedJob

    def job(**kw):
        j = _TransposedJob()
        j.src, j.dtype, j.rows, j.cols, j.ld = FAKE, 0, 64, 64, 64
        j.codes_t, j.scales_t, j.codes_row, j.scales_row = FAKE, FAKE, FAKE, FAKE
        j.tensor_id_t, j.tensor_id_row, j.pre_quant = 6, 1, 1
        j.row_codes_in = j.row_scales_in = None
        j.seed, j.index_base, j.seed_dev = 0, 0, None
        j.col_sums = j.col_sum_workspace = None
        for k, v in kw.items():
            setattr(j, k, v)
        return j

    def call(jobs, round_t=1, round_row=0, mode=0):
        arr = (_TransposedJob * max(1, len(jobs)))(*jobs)
        return L.mx_quantize_transposed_batch(arr, len(jobs), round_t, round_row, mode, P(0))
    assert L.mx_quantize_transposed_batch(None, 1, 1, 0, 0, P(0)) == -1
    assert call([]) == -2 and call([job()] * 5) == -2
    assert call([job(), job(codes_t=None)]) == -1                  # a job's own error comes back as is
    assert call([job(), job(rows=48)]) == -2
    assert call([job(), job(src=FAKE + 4)]) == -5
    assert call([job()], round_t=7) == -4 and call([job()], mode=3) == -4
    assert call([job(), job(dtype=1, ld=64)]) == -3                # F32 and BF16 sources do not mix
    given = job(src=None, codes_row=None, scales_row=None, row_codes_in=FAKE, row_scales_in=FAKE)
    assert call([job(), given]) == -4                              # nor a source with a given row result
    assert call([job(index_base=4)]) == -5                         # stochastic streams start on a block of 8
    assert call([job(seed_dev=FAKE + 4)]) == -5                    # a device seed is a 64-bit word, 8-byte aligned
    given2 = job(src=None, codes_row=None, scales_row=None, row_codes_in=FAKE, row_scales_in=FAKE, col_sums=FAKE, col_sum_workspace=FAKE)
    assert call([given2]) == -4                                    # column sums are those of a source tensor
    assert call([job(col_sums=FAKE)]) == -6                        # and need their scratch
    assert call([job(col_sums=FAKE + 2, col_sum_workspace=FAKE)]) == -5
    assert L.mx_column_sum_workspace_bytes(50432, 2304) == 197 * 2304 * 4 and L.mx_column_sum_workspace_bytes(0, 64) == 0


def test_header_is_plain_c(tmp_path):
    """include/mxfp4.h compiles as C99 on its own (no C++ or HIP types at the boundary), and a C
    translation unit can name every declared entry point."""
    import re
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    header = os.path.join(ROOT, "include", "mxfp4.h")
    names = sorted(set(re.findall(r"\b(mx_[a-z0-9_]+)\s*\(", open(header).read())))
    assert "mx_linear_fwd" in names and "mx_quantize_transposed_batch" in names
    src = tmp_path / "use.c"
    src.write_text('#include "mxfp4.h"\n' + "".join("void* p_%s = (void*)%s;\n" % (n, n) for n in names)
                   + "int main(void) { mx_transposed_job j; (void)j; return 0; }\n")
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-Wno-pedantic", "-I", os.path.dirname(header),
                    "-c", str(src), "-o", str(tmp_path / "use.o")], check=True)


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message before it touches a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)


def test_no_alloc_dw_validates_like_the_workspace_entry_point(L):
    """mx_linear_bwd_dw_noalloc returns the argument errors of mx_linear_bwd_dw before it touches the GPU
    (null pointers, contraction length not a multiple of 32, bad dtype, misaligned operands), and the
    K-split workspace of any shape the policy can choose fits the library's own array."""
    from paper_2502_20853_amd import binding
    f = L.mx_linear_bwd_dw_noalloc
    ok = dict(a=FAKE, a_s=FAKE, b=FAKE, b_s=FAKE, N=4096, C=256, D=256, out=FAKE, dt=0, ld=256)

    def call(**kw):
        v = dict(ok, **kw)
        return f(P(v["a"]), P(v["a_s"]), P(v["b"]), P(v["b_s"]), v["N"], v["C"], v["D"], P(v["out"]), v["dt"], v["ld"], P(0))

    assert call(a=0) == binding.MX_ERR_NULL and call(out=0) == binding.MX_ERR_NULL
    assert call(N=4100) == binding.MX_ERR_SHAPE and call(N=0) == binding.MX_ERR_SHAPE and call(ld=128) == binding.MX_ERR_SHAPE
    assert call(dt=7) == binding.MX_ERR_DTYPE
    assert call(a=FAKE + 4) == binding.MX_ERR_ALIGN and call(out=FAKE + 4) == binding.MX_ERR_ALIGN
    import random
    rng = random.Random(0)
    worst = 0
    for _ in range(20000):
        C, D = rng.randint(1, 6000), rng.randint(1, 6000)
        N = 32 * rng.randint(1, 1 << 14)
        worst = max(worst, L.mx_linear_workspace_bytes(binding.GEMM_BWD_DW, N, C, D))
    assert 0 < worst <= binding.NOALLOC_MAX_WORKSPACE_BYTES
