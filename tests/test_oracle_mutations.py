"""Do the pins bite?  Each case plants one plausible mistake in a COPY of the oracle's C source (a dropped
scale, a wrong sign, a transposed index, a wrong window, ...), builds it on the CPU, and runs the pin
suites against that copy in a subprocess: at least one pin has to fail.  The unmodified copy has to
pass, so a failure is due to the planted mistake and not to the harness."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "agent_attn_oracle.c")

# (name, text in the source, replacement, which occurrence)
MUTATIONS = [
    ("scale dropped from the scores", "double v = scale * dot;", "double v = dot;", 0),
    ("bias subtracted", "if (bias) v += bias[(size_t)i * L + j];", "if (bias) v -= bias[(size_t)i * L + j];", 0),
    ("pooling window ends at the floor", "return (int)((((long long)(i + 1)) * L + La - 1) / La);",
     "return (int)((((long long)(i + 1)) * L) / La);", 0),
    ("pooling divides by the window height", "= acc / cnt;", "= acc / (double)(y1 - y0);", 0),
    ("bilinear without the half-pixel shift", "* ((double)L0 / (double)L) - 0.5;", "* ((double)L0 / (double)L);", 0),
    ("bias-2 column component read transposed", "if (col2) v += col2[(size_t)x * n + a];",
     "if (col2) v += col2[(size_t)a * w + x];", 0),
    ("bias-1 row component indexed by x", "if (row1) v += row1[(size_t)a * h + y];",
     "if (row1) v += row1[(size_t)a * h + (x < h ? x : h - 1)];", 0),
    ("DWC as a true convolution (flipped taps)", "int yy = y + u, xx = x + v;", "int yy = y - u, xx = x - v;", 0),
    ("broadcast uses V instead of V_A", "oracle_softmax_attention(Qu, A, VA, B2 ?", "oracle_softmax_attention(Qu, A, Vu, B2 ?", 0),
    ("aggregation and broadcast share scale1", "scale2, N, n, d, d, Ou, NULL);", "scale1, N, n, d, d, Ou, NULL);", 0),
    ("k*V residual dropped", "Ou[e] += vk * Vu[e];", "Ou[e] += 0.0 * Vu[e];", 0),
    ("merge weights the sums with the wrong sign", "ll += l[(size_t)s * n + a] * exp(m[(size_t)s * n + a] - mm);",
     "ll += l[(size_t)s * n + a] * exp(mm - m[(size_t)s * n + a]);", 0),
    ("softmax gradient without the row term", "* (dS[(size_t)i * L + j] - inner);", "* (dS[(size_t)i * L + j]);", 0),
    ("dQ without the scale", "dQm[(size_t)i * d + c] = scale * acc;", "dQm[(size_t)i * d + c] = acc;", 0),
    ("dK from the wrong operand", "acc += dS[(size_t)i * L + j] * Qm[(size_t)i * d + c];",
     "acc += dS[(size_t)i * L + j] * Km[(size_t)j * d + c];", 0),
    ("pooling gradient not divided by the window", "dA[((size_t)ay * aw + ax) * d + c] / cnt;",
     "dA[((size_t)ay * aw + ax) * d + c];", 0),
    ("DWC gradient with unflipped taps", "int yy = y + u, xx = x + v;", "int yy = y - u, xx = x - v;", 1),
    ("dA of the two stages not added", "dA_keys[e] += dA_queries[e];", "dA_keys[e] += 0.0;", 0),
    ("bias-block gradient misses one bilinear corner", "gsrc[((size_t)y1 * w0 + x1) * stride] += gv * fy * fx;",
     "gsrc[((size_t)y1 * w0 + x1) * stride] += 0.0;", 0),
    ("projection reads its weight transposed", "acc += X[(size_t)r * K + k] * W[(size_t)o * K + k];",
     "acc += X[(size_t)r * K + k] * W[(size_t)k * O + o];", 0),
    ("projection bias dropped", "if (b) acc += b[o];", "if (b) acc += 0.0 * b[o];", 0),
    ("agent-axis resize walks the agent grid transposed", "oracle_resize_bilinear(src + (size_t)o * ah * aw * inner + i, ah, aw,",
     "oracle_resize_bilinear(src + (size_t)o * ah * aw * inner + i, aw, ah,", 0),
    ("agent-axis resize scatters with the wrong stride", "dst[((size_t)o * ah2 * aw2 + a) * inner + i] = plane[a];",
     "dst[((size_t)o * ah2 * aw2 + a) + (size_t)i * ah2 * aw2] = plane[a];", 0),
]


def _build(tmp_path, name, text):
    c = tmp_path / (name + ".c")
    so = tmp_path / (name + ".so")
    c.write_text(text)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"], check=True)
    return str(so)


def _pins_pass(lib):
    env = dict(os.environ, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "tests/test_oracle_bwd_pins.py", "-x",
                        "-q", "-p", "no:cacheprovider", "--oracle-lib", lib], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, timeout=600)
    return r.returncode == 0, r.stdout.decode()[-400:]


def test_unmodified_copy_passes(tmp_path):
    ok, tail = _pins_pass(_build(tmp_path, "plain", open(SRC).read()))
    assert ok, tail


@pytest.mark.parametrize("name,old,new,which", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, old, new, which):
    src = open(SRC).read()
    parts = src.split(old)
    assert len(parts) > which + 1, "mutation target not found in the oracle source: " + old
    mutated = old.join(parts[:which + 1]) + new + old.join(parts[which + 1:])
    assert mutated != src
    ok, tail = _pins_pass(_build(tmp_path, "mutant", mutated))
    assert not ok, "no pin noticed: " + name
