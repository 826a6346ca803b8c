"""Do the pins bite?  Each case plants one plausible mistake in a COPY of the CPU oracle (a dropped
term, a wrong sign, a flipped or transposed index, a precision slip), builds it with gcc, and runs
the pin suite against that build in a subprocess: at least one pin must fail.  Every mutation keeps
all memory accesses in bounds.  CPU only; nothing here touches the GPU library.
"""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "lg_oracle.c")

# (function the edit is confined to, original text, planted mistake)
MUTANTS = [
    ("lgo_matmul", "for (int64_t k = 0; k < K; ++k)", "for (int64_t k = 1; k < K; ++k)"),
    ("lgo_matmul", "s += (double)A[m * lda + k] * (double)B[k * ldb + n];",
     "s -= (double)A[m * lda + k] * (double)B[k * ldb + n];"),
    ("lgo_matmul", "(double)B[k * ldb + n]", "(double)B[k * ldb + (N - 1 - n)]"),
    ("lgo_matmul", "(double)A[m * lda + k]", "(double)A[(M - 1 - m) * lda + k]"),
    ("lgo_matmul", "if (accumulate) s += (double)C[m * ldc + n];", "if (accumulate) s -= (double)C[m * ldc + n];"),
    ("lgo_matmul", "double s = 0.0;", "float s = 0.0f;"),
    ("lgo_matmul_t", "double a = transA ? (double)A[k * lda + m] : (double)A[m * lda + k];",
     "double a = transA ? (double)A[k * lda + (M - 1 - m)] : (double)A[m * lda + k];"),
    ("lgo_matmul_t", "double b = transB ? (double)B[n * ldb + k] : (double)B[k * ldb + n];",
     "double b = transB ? (double)B[(N - 1 - n) * ldb + k] : (double)B[k * ldb + n];"),
    ("lgo_matmul_t", "for (int64_t k = 0; k < K; ++k) {", "for (int64_t k = 0; k + 1 < K; ++k) {"),
    ("lgo_conv_out_extent", "return (in - span) / s + 1;", "return (in - span) / s;"),
    ("lgo_conv2d_nhwc_hwcf", "Kf[((kh * KW + kw) * C + c) * F + f]", "Kf[(((KH - 1 - kh) * KW + kw) * C + c) * F + f]"),
    ("lgo_conv2d_nhwc_hwcf", "Kf[((kh * KW + kw) * C + c) * F + f]", "Kf[((kw * KH + kh) * C + c) * F + f]"),
    ("lgo_conv2d_nhwc_hwcf", "int64_t ih = h * SH + kh * DH;", "int64_t ih = h * SH + kh;"),
    ("lgo_conv2d_nhwc_hwcf", "int64_t iw = w * SW + kw * DW;", "int64_t iw = w + kw * DW;"),
    ("lgo_conv2d_nhwc_hwcf", "for (int64_t c = 0; c < C; ++c) {", "for (int64_t c = 1; c < C; ++c) {"),
    ("lgo_im2col_nhwc", "col[row * Kg + (kh * KW + kw) * C + c]", "col[row * Kg + (kw * KH + kh) * C + c]"),
    ("lgo_dwconv1d_nwc_wc", "(double)Kf[kw * C + c]", "(double)Kf[(KW - 1 - kw) * C + c]"),
    ("lgo_dwconv1d_nwc_wc", "I[(n * W + w * SW + kw * DW) * C + c]", "I[(n * W + w * SW + kw) * C + c]"),
    ("lgo_dwconv2d_nhwc_hwc", "(double)Kf[(kh * KW + kw) * C + c]", "(double)Kf[(kw * KH + kh) * C + c]"),
    ("lgo_dwconv2d_nhwc_hwc", "w * SW + kw * DW) * C + c]", "w + kw * DW) * C + c]"),
    ("lgo_reduce_rows", "for (int64_t j = 0; j < Cn; ++j) s += (double)in[i * ld + j];",
     "for (int64_t j = 1; j < Cn; ++j) s += (double)in[i * ld + j];"),
    ("lgo_reduce_rows", "double s = 0.0;", "float s = 0.0f;"),
    ("lgo_reduce_cols", "for (int64_t i = 0; i < R; ++i) s += (double)in[i * ld + j];",
     "for (int64_t i = 0; i < R; ++i) s += (double)in[i * ld + (Cn - 1 - j)];"),
    ("lgo_reduce_cols", "if (accumulate) s += (double)out[j];", "if (accumulate) s += 0.0;"),
    ("lgo_transpose", "memcpy(&out[j * ld_out + i], &in[i * ld_in + j], sizeof(float));",
     "memcpy(&out[j * ld_out + i], &in[i * ld_in + (Cn - 1 - j)], sizeof(float));"),
    ("lgo_transpose", "memcpy(&out[j * ld_out + i], &in[i * ld_in + j], sizeof(float));",
     "out[j * ld_out + i] = in[i * ld_in + j] + 0.0f;"),
    ("lgo_conv1d_nwc_wcf", "int64_t x = w * SW + kw * DW;", "int64_t x = w * SW + kw;"),
    ("lgo_conv1d_nwc_wcf", "int64_t x = w * SW + kw * DW;", "int64_t x = w + kw * DW;"),
    ("lgo_conv1d_nwc_wcf", "(double)Kf[(kw * C + c) * F + f]", "(double)Kf[((KW - 1 - kw) * C + c) * F + f]"),
    ("lgo_conv1d_nwc_wcf", "(double)Kf[(kw * C + c) * F + f]", "(double)Kf[(kw * C + c) * F + (F - 1 - f)]"),
    ("lgo_transpose_batched", "&in[b0 * is0 + b1 * is1 + i * ld_in + j]", "&in[b1 * is1 + i * ld_in + j]"),
    ("lgo_transpose_batched", "memcpy(&out[b0 * os0 + b1 * os1 + j * ld_out + i]", "memcpy(&out[b0 * os0 + b1 * os1 + i * ld_out + j]"),
    ("lgo_copy2d", "memcpy(&out[i * ld_out + j], &in[i * ld_in + j], sizeof(float));",
     "memcpy(&out[i * ld_out + j], &in[(R - 1 - i) * ld_in + j], sizeof(float));"),
]


def mutate(text, func, old, new):
    start = text.index("\nint " + func + "(") if ("\nint " + func + "(") in text else text.index("\nint64_t " + func + "(")
    nxt = text.find("\nint ", start + 5)
    end = nxt if nxt != -1 else len(text)
    body = text[start:end]
    assert body.count(old) == 1, f"{func}: edit site must be unique ({body.count(old)} matches)"
    return text[:start] + body.replace(old, new) + text[end:]


@pytest.mark.parametrize("func,old,new", MUTANTS, ids=[f"{m[0]}-{i}" for i, m in enumerate(MUTANTS)])
def test_planted_mistake_is_caught(func, old, new, tmp_path):
    text = open(SRC).read()
    c_file = tmp_path / "mutant.c"
    so_file = tmp_path / "libmutant.so"
    c_file.write_text(mutate(text, func, old, new))
    subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                    "-o", str(so_file), str(c_file)], check=True)
    env = dict(os.environ, LGO_ORACLE_LIB=str(so_file), OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        "-x", "-q", "-p", "no:cacheprovider"], env=env, cwd=ROOT,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode != 0, f"no pin noticed: {func}: {old!r} -> {new!r}"
    assert "failed" in r.stdout or "error" in r.stdout.lower()
