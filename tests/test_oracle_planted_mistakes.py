"""The pins must catch mistakes: thirty-eight deliberately wrong copies of the oracle (a flipped sign, a dropped term,
a wrong index, a transposed operand, ...) are compiled one by one and the pin files that cover the changed function are
run against each copy in a child process; every copy has to fail at least one pin.  CPU only; the mistakes are planted
in the oracle's source, nothing here touches the GPU path."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = os.path.join(ROOT, "oracle", "spectre_oracle.c")

# (what is planted, text in the source, its replacement, pin files that must notice)
MISTAKES = [
    ('sign of the root of unity',
     'cplx r = { cos(ang), sign * sin(ang) };',
     'cplx r = { cos(ang), -sign * sin(ang) };',
     ('tests/test_oracle_transforms.py',)),
    ('Nyquist bin counted twice in the inverse',
     'if (2 * k == n) acc += Yc[k].re * w.re;',
     'if (2 * k == n) acc += 2.0 * Yc[k].re * w.re;',
     ('tests/test_oracle_transforms.py',)),
    ('Hermitian extension without the conjugate',
     'buf[n - k].im = -Yc[k].im;',
     'buf[n - k].im = Yc[k].im;',
     ('tests/test_oracle_transforms.py',)),
    ('unbiased instead of biased LayerNorm variance',
     'var /= d;',
     'var /= (d - 1);',
     ('tests/test_oracle_mixer_gate.py', 'tests/test_oracle_wrm.py')),
    ('tanh approximation instead of the exact GELU',
     'hid[j] = 0.5 * a * (1.0 + erf(a / sqrt(2.0)));',
     'hid[j] = 0.5 * a * (1.0 + tanh(0.7978845608 * (a + 0.044715 * a * a * a)));',
     ('tests/test_oracle_mixer_gate.py', 'tests/test_oracle_wrm.py')),
    ('sign of the positional phase',
     'u = c_mul(u, root_of_unity((long long)k * pm, n, +1));',
     'u = c_mul(u, root_of_unity((long long)k * pm, n, -1));',
     ('tests/test_oracle_mixer_gate.py',)),
    ('eviction of the old value row dropped',
     'double v_old = (t >= N) ? v_buf[slot] : 0.0;',
     'double v_old = 0.0;',
     ('tests/test_oracle_prefix.py',)),
    ('eviction of the old query row dropped',
     'double q_old = (t >= N) ? q_buf[slot] : 0.0;',
     'double q_old = 0.0;',
     ('tests/test_oracle_prefix.py',)),
    ('sign of the imaginary part in the single-row readout',
     'else acc += 2.0 * (Y.re * w.re - Y.im * w.im);',
     'else acc += 2.0 * (Y.re * w.re + Y.im * w.im);',
     ('tests/test_oracle_prefix.py', 'tests/test_oracle_transforms.py')),
    ('window readout returns the first rows instead of the last',
     'out[(((size_t)b * Lw + i) * H + h) * d + c] = x[N - Lw + i];',
     'out[(((size_t)b * Lw + i) * H + h) * d + c] = x[i];',
     ('tests/test_oracle_prefix.py',)),
    ("first MLP layer's weights transposed",
     'a += qbar[i] * W1[((size_t)hp * d + i) * dg + j];',
     'a += qbar[i] * W1[((size_t)hp * dg + j) * d + i];',
     ('tests/test_oracle_mixer_gate.py',)),
    ('imaginary part of a bin taken from its real weight row',
     'u.im += hid[j] * w[1];',
     'u.im += hid[j] * w[0];',
     ('tests/test_oracle_mixer_gate.py',)),
    ('chirp of the arbitrary-length transform not conjugated',
     'cplx cc = { chirp[m].re, -chirp[m].im };',
     'cplx cc = { chirp[m].re, chirp[m].im };',
     ('tests/test_oracle_transforms.py',)),
    ('slot one ahead',
     'long long s = t % N;',
     'long long s = (t + 1) % N;',
     ('tests/test_oracle_prefix.py',)),
    ('gate conjugated in the mixer',
     'for (int k = 0; k < F; ++k) X[k] = c_mul(gg[k], X[k]);',
     'for (int k = 0; k < F; ++k) { cplx gc = { gg[k].re, -gg[k].im }; X[k] = c_mul(gc, X[k]); }',
     ('tests/test_oracle_mixer_gate.py', 'tests/test_oracle_transforms.py')),
    ('ring slot without the memory offset',
     'long long s = Nmem + t % Nmax;',
     'long long s = t % Nmax;',
     ('tests/test_oracle_memory.py',)),
    ('ring slot wraps over the whole window',
     'long long s = Nmem + t % Nmax;',
     'long long s = Nmem + t % (Nmem + Nmax);',
     ('tests/test_oracle_memory.py',)),
    ('eviction starts one window late',
     'double v_old = (t >= Nmax) ? v_buf[slot] : 0.0;',
     'double v_old = (t >= Nmem + Nmax) ? v_buf[slot] : 0.0;',
     ('tests/test_oracle_memory.py',)),
    ('root of unity of the ring length instead of the window length',
     'cplx w = root_of_unity((long long)k * s, n, -1);',
     'cplx w = root_of_unity((long long)k * s, Nmax, -1);',
     ('tests/test_oracle_memory.py',)),
    ('window gather without the memory offset',
     '= x[Nmem + tok % Nmax];',
     '= x[tok % Nmax];',
     ('tests/test_oracle_memory.py',)),
    ('window gather one token ahead',
     'long long tok = t - Lw + i;',
     'long long tok = t - Lw + i + 1;',
     ('tests/test_oracle_memory.py',)),
    ('prefill writes over the memory rows',
     'size_t dst = (bh * n + Nmem + l) * d + c;',
     'size_t dst = (bh * n + l) * d + c;',
     ('tests/test_oracle_memory.py',)),
    ('prefill transform input without the memory offset',
     'x[Nmem + l] = V[src];',
     'x[l] = V[src];',
     ('tests/test_oracle_memory.py',)),
    ('sign of the Haar detail coefficients',
     'w[half + i] = (cur[2 * i] - cur[2 * i + 1]) / sqrt(2.0);',
     'w[half + i] = (cur[2 * i + 1] - cur[2 * i]) / sqrt(2.0);',
     ('tests/test_oracle_wrm.py',)),
    ('Haar synthesis adds instead of subtracts',
     'cur[2 * i + 1] = (x[i] - x[len + i]) / sqrt(2.0);',
     'cur[2 * i + 1] = (x[i] + x[len + i]) / sqrt(2.0);',
     ('tests/test_oracle_wrm.py',)),
    ('band boundaries shifted by one level',
     'while (i >= (n >> (l - 1))) --l;',
     'while (i >= (n >> l)) --l;',
     ('tests/test_oracle_wrm.py',)),
    ('coarse band mapped to the finest gate',
     'if (i < (n >> J)) return 0;',
     'if (i < (n >> J)) return J;',
     ('tests/test_oracle_wrm.py',)),
    ("second MLP layer's weights transposed",
     'a += hid[j] * W2[((size_t)hp * dw + j) * nout + o];',
     'a += hid[j] * W2[((size_t)hp * nout + o) * dw + j];',
     ('tests/test_oracle_wrm.py',)),
    ('residual term dropped',
     '= x[t] + ref[t];',
     '= ref[t];',
     ('tests/test_oracle_wrm.py',)),
    ('gate table indexed channel-major',
     'w[i] *= sb[(size_t)haar_band(i, L, J) * d + c];',
     'w[i] *= sb[(size_t)c * (J + 1) + haar_band(i, L, J)];',
     ('tests/test_oracle_wrm.py',)),
    ('averaging instead of orthonormal scaling',
     'w[i] = (cur[2 * i] + cur[2 * i + 1]) / sqrt(2.0);',
     'w[i] = (cur[2 * i] + cur[2 * i + 1]) / 2.0;',
     ('tests/test_oracle_wrm.py',)),
    ('Toeplitz taps applied mirrored',
     'int src = k - m;',
     'int src = k + m;',
     ('tests/test_oracle_mixer_gate.py',)),
    ('Toeplitz update without the identity term',
     'cplx acc = raw[k];',
     'cplx acc = { 0.0, 0.0 };',
     ('tests/test_oracle_mixer_gate.py',)),
    ('projection weights transposed',
     'av += x[i] * wv[(size_t)i * d + j];',
     'av += x[i] * wv[(size_t)j * d + i];',
     ('tests/test_oracle_mixer_gate.py',)),
    ('per-coefficient wavelet gate taken from the mirrored coefficient',
     'for (int i = 0; i < L; ++i) w[i] *= sc[(size_t)i * d + c];',
     'for (int i = 0; i < L; ++i) w[i] *= sc[(size_t)(L - 1 - i) * d + c];',
     ('tests/test_oracle_wrm.py',)),
    ('per-coefficient wavelet gates read channel-major',
     'for (int i = 0; i < L; ++i) w[i] *= sc[(size_t)i * d + c];',
     'for (int i = 0; i < L; ++i) w[i] *= sc[(size_t)c * L + i];',
     ('tests/test_oracle_wrm.py',)),
    ('per-coefficient wavelet module without the residual',
     'for (int t = 0; t < L; ++t) out[(((size_t)b * L + t) * H + h) * d + c] = x[t] + ref[t];\n        free(x);\n    }\n    return fail ? -2 : 0;\n}\n\n/* Steps (a), (c), (d): for every column, analyse, scale every coefficient by the',
     'for (int t = 0; t < L; ++t) out[(((size_t)b * L + t) * H + h) * d + c] = ref[t];\n        free(x);\n    }\n    return fail ? -2 : 0;\n}\n\n/* Steps (a), (c), (d): for every column, analyse, scale every coefficient by the',
     ('tests/test_oracle_wrm.py',)),
    ('query pooled over the wrong axis stride',
     'for (int l = 0; l < L; ++l) s += Q[(((size_t)b * L + l) * H + h) * d + c];',
     'for (int l = 0; l < L; ++l) s += Q[(((size_t)b * L + l) * H + c % H) * d + c];',
     ('tests/test_oracle_mixer_gate.py',)),
]


def _run_pins(tmp, tag, text, files):
    """Compile `text` as the oracle and run the given pin files against it; returns pytest's exit status."""
    src = os.path.join(tmp, f"{tag}.c")
    lib = os.path.join(tmp, f"lib{tag}.so")
    with open(src, "w") as fh:
        fh.write(text)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", lib, src, "-lm"])
    env = dict(os.environ, SPECTRE_ORACLE_SOURCE=src, SPECTRE_ORACLE_LIBRARY=lib, OMP_NUM_THREADS="2")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu", *files]
    return subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL).returncode


def test_every_planted_mistake_fails_a_pin(tmp_path):
    original = open(SOURCE).read()
    tmp = str(tmp_path)
    # the harness itself: an unchanged copy passes the pins of every file used below
    every_file = sorted({f for _, _, _, files in MISTAKES for f in files})
    assert _run_pins(tmp, "unchanged", original, every_file) == 0

    def attempt(item):
        i, (what, old, new, files) = item
        assert original.count(old) >= 1, f"the source no longer contains: {old}"
        return what, _run_pins(tmp, f"mistake{i}", original.replace(old, new), list(files))

    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(attempt, enumerate(MISTAKES)))
    survivors = [what for what, status in results if status == 0]
    assert not survivors, f"no pin noticed: {survivors}"
    shutil.rmtree(tmp, ignore_errors=True)
