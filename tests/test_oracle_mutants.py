"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source (a dropped term, a
wrong sign or index, a swapped operand, an off-by-one), builds that copy with gcc and runs the oracle's pin tests
against it: at least one pin must fail for every planted mistake.  Everything here runs on the CPU; the mistakes
live only in temporary copies.  (Changes that cannot show are left out: the clips of Eq. 2's result are implied by
the clamp of r, and the loader hands the scan a zeroed y, so dropping them changes nothing observable.)
"""
import ctypes
import importlib
import itertools
import os
import subprocess

import pytest

import oracle

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "corey_oracle.c")
PIN_MODULES = ("test_oracle_entropy", "test_oracle_chunk", "test_oracle_scan", "test_oracle_conv", "test_oracle_decode")

# (name, text in the source, replacement)
MUTANTS = [
    # ---- Eq. 1 and r
    ("hist: bins scaled by K - 1", "(float)((double)K / ((double)hi - (double)lo));\n            j = 0;",
     "(float)((double)(K - 1) / ((double)hi - (double)lo));\n            j = 0;"),
    ("hist: top edge not clamped into the last bin", "if (k > K - 1) k = K - 1;", "if (k > K - 1) continue;"),
    ("hist: bin index rounded instead of truncated", "int64_t k = (int64_t)q;                            /* truncate, q >= 0 */",
     "int64_t k = (int64_t)(q + 0.5f);"),
    ("hist: range taken from the first value only", "if (v < lo) lo = v;", "if (v < lo && nsamp == 0) lo = v;"),
    ("entropy: sign", "double h = -acc;", "double h = acc;"),
    ("entropy: eps outside the logarithm", "acc += p * log(p + eps);", "acc += p * (log(p) + eps);"),
    ("entropy: base-2 logarithm in the normaliser", "double rr = h / log((double)K);", "double rr = h / log2((double)K);"),
    ("entropy: an empty bin evaluated as 0 * log(0 + eps)", "if (c[k] == 0) continue;", ""),
    ("entropy: probabilities not normalised", "double p = (double)c[k] / n;", "double p = (double)c[k];"),
    ("sampling: stride applied to elements, not blocks", "const int sampled = (j / block) % stride == 0;",
     "const int sampled = j % stride == 0;"),
    ("sampling: count pass off by one block", "if ((j / block) % stride) continue;\n                        const float tt",
     "if (((j / block) + 1) % stride) continue;\n                        const float tt"),
    ("per-sequence: padded positions counted", "int64_t len = seqlens ? seqlens[b] : L;\n                for (int64_t d = 0; d < D; ++d)\n                    for (int64_t t = 0; t < len; ++t, ++j) {\n                        if (",
     "int64_t len = L;\n                for (int64_t d = 0; d < D; ++d)\n                    for (int64_t t = 0; t < len; ++t, ++j) {\n                        if ("),
    ("ema: weights swapped", "return lambda * prev + (1.0 - lambda) * H;", "return (1.0 - lambda) * prev + lambda * H;"),
    # ---- Eq. 2 and the scheduler family
    ("rule: floor instead of round", "double k = floor(lg + 0.5);", "double k = floor(lg);"),
    ("rule: c_min dropped from the interpolation", "double v = (double)p->c_min + re * (double)(p->c_max - p->c_min);",
     "double v = re * (double)p->c_max;"),
    ("rule: interpolation towards c_max + c_min", "re * (double)(p->c_max - p->c_min);", "re * (double)(p->c_max + p->c_min);"),
    ("rule: H_ref scale ignored", "double re = r * p->h_ref_scale;", "double re = r;"),
    ("table: strict comparison at the short length", "c = (L <= p->short_len) ? p->short_chunk : p->long_chunk;",
     "c = (L < p->short_len) ? p->short_chunk : p->long_chunk;"),
    ("guard: distance compared with <=", "if (dist < p->guard_buckets) c = p->safe_chunk;", "if (dist <= p->guard_buckets) c = p->safe_chunk;"),
    ("cap: by the power of two below L", "int64_t cap = pow2ceil(L);", "int64_t cap = pow2ceil(L) > L ? pow2ceil(L) / 2 : L;"),
    # ---- the scan
    ("scan: first-order decay 1 + dl A", "const double abar = exp(dl * (double)A[d * N + n]);", "const double abar = 1.0 + dl * (double)A[d * N + n];"),
    ("scan: A indexed transposed", "exp(dl * (double)A[d * N + n]);\n                    const double bbar_u", "exp(dl * (double)A[n * D + d]);\n                    const double bbar_u"),
    ("scan: step size dropped from the input term", "const double bbar_u = dl * (double)Bm[(b * N + n) * L + t] * uu;",
     "const double bbar_u = (double)Bm[(b * N + n) * L + t] * uu;"),
    ("scan: B and C swapped", "acc += (double)Cm[(b * N + n) * L + t] * h[n];", "acc += (double)Bm[(b * N + n) * L + t] * h[n];"),
    ("scan: read-out before the update", "h[n] = abar * h[n] + bbar_u;\n                    acc += (double)Cm[(b * N + n) * L + t] * h[n];",
     "acc += (double)Cm[(b * N + n) * L + t] * h[n];\n                    h[n] = abar * h[n] + bbar_u;"),
    ("scan: B of the previous step", "dl * (double)Bm[(b * N + n) * L + t] * uu;", "dl * (double)Bm[(b * N + n) * L + (t > 0 ? t - 1 : 0)] * uu;"),
    ("scan: skip term dropped", "double yv = acc + (Dv ? (double)Dv[d] * uu : 0.0);\n                if (z) {\n                    const double zz = (double)z[row * L + t];",
     "double yv = acc;\n                if (z) {\n                    const double zz = (double)z[row * L + t];"),
    ("scan: gate is the logistic function alone", "yv *= zz / (1.0 + exp(-zz));\n                }\n                y[row * L + t] = yv;",
     "yv *= 1.0 / (1.0 + exp(-zz));\n                }\n                y[row * L + t] = yv;"),
    ("scan: softplus without the linear branch", "dl = (dl > 0.0 ? dl : 0.0) + log1p(exp(-fabs(dl)));   /* log(1 + e^dl) */",
     "dl = log1p(exp(-fabs(dl)));"),
    ("scan: bias added after the softplus", "double dl = (double)delta[row * L + t] + (dbias ? (double)dbias[d] : 0.0);\n                if (delta_softplus)\n                    dl = (dl > 0.0 ? dl : 0.0) + log1p(exp(-fabs(dl)));   /* log(1 + e^dl) */",
     "double dl = (double)delta[row * L + t];\n                if (delta_softplus)\n                    dl = (dl > 0.0 ? dl : 0.0) + log1p(exp(-fabs(dl)));\n                dl += (dbias ? (double)dbias[d] : 0.0);"),
    ("scan: initial state ignored", "h[n] = h0 ? (double)h0[row * N + n] : 0.0;", "h[n] = 0.0;"),
    ("scan: state reset at every tile", "const int64_t t1 = (t0 + chunk < len) ? t0 + chunk : len;",
     "const int64_t t1 = (t0 + chunk < len) ? t0 + chunk : len;\n            if (t0 > 0) for (int64_t n = 0; n < N; ++n) h[n] = 0.0;"),
    ("scan: B and C taken from sequence 0", "const int64_t b = row / D, d = row % D;\n        const int64_t len = seqlens ? seqlens[b] : L;\n        double h[1024];",
     "const int64_t b = 0, d = row % D;\n        const int64_t len = seqlens ? seqlens[row / D] : L;\n        double h[1024];"),
    # ---- the producer of u
    ("conv: taps applied newest first", "v += (double)weight[d * W + k] * xv;", "v += (double)weight[d * W + (W - 1 - k)] * xv;"),
    ("conv: bias dropped", "double v = bias ? (double)bias[d] : 0.0;", "double v = 0.0;"),
    ("conv: one step too late", "const int64_t s = t - (W - 1) + k;", "const int64_t s = t - W + k;"),
    ("conv: carried inputs reversed", "else if (state_in) xv = (double)state_in[r * (W - 1) + (s + (W - 1))];\n                v +=",
     "else if (state_in) xv = (double)state_in[r * (W - 1) + (-1 - s)];\n                v +="),
    ("conv: weights of channel 0 for every channel", "(double)weight[d * W + k] * xv;", "(double)weight[k] * xv;"),
    ("conv: activation is the logistic function alone", "u[r * L + t] = v / (1.0 + exp(-v));", "u[r * L + t] = 1.0 / (1.0 + exp(-v));"),
    ("conv: state_out holds the first inputs", "const int64_t s = L - (W - 1) + k;", "const int64_t s = k;"),
    # ---- one generated token
    ("decode: read-out from the old state", "acc += (double)Ct[b * N + n] * hn;", "acc += (double)Ct[b * N + n] * (double)state_in[row * N + n];"),
    ("decode: decay applied to the input term too", "const double hn = exp(dl * (double)A[d * N + n]) * (double)state_in[row * N + n]\n                                  + dl * (double)Bt[b * N + n] * xx;",
     "const double hn = exp(dl * (double)A[d * N + n]) * ((double)state_in[row * N + n]\n                                  + dl * (double)Bt[b * N + n] * xx);"),
    ("decode: skip term dropped", "double yv = acc + (Dv ? (double)Dv[d] * xx : 0.0);", "double yv = acc;"),
    ("decode: no softplus", "if (delta_softplus) dl = (dl > 0.0 ? dl : 0.0) + log1p(exp(-fabs(dl)));", ""),
]


def _load(path):
    lib = ctypes.CDLL(path)
    lib.oracle_entropy_hist.restype = ctypes.c_int
    lib.oracle_select_chunk.restype = ctypes.c_int
    lib.oracle_selective_scan.restype = ctypes.c_int
    lib.oracle_max_threads.restype = ctypes.c_int
    return lib


def _pin_calls():
    """Every pin test of the oracle as (label, zero-argument callable); parametrised ones are expanded."""
    calls = []
    for modname in PIN_MODULES:
        mod = importlib.import_module(modname)
        for name in sorted(vars(mod)):
            fn = getattr(mod, name)
            if not (name.startswith("test_") and callable(fn)):
                continue
            if "library" in name:                              # compares with the GPU library's host code, not a pin
                continue
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            if not marks:
                calls.append((f"{modname}.{name}", fn))
                continue
            axes = []
            for m in marks:
                names = [s.strip() for s in m.args[0].split(",")]
                axes.append([dict(zip(names, v if len(names) > 1 else (v,))) for v in m.args[1]])
            for combo in itertools.product(*axes):
                kw = {}
                for part in combo:
                    kw.update(part)
                calls.append((f"{modname}.{name}{sorted(kw.items())}", (lambda f=fn, k=kw: f(**k))))
    return calls


def _first_failure(calls):
    for label, fn in calls:
        try:
            fn()
        except BaseException as e:                             # noqa: BLE001 - any failure of a pin counts
            if isinstance(e, (KeyboardInterrupt, SystemExit)):
                raise
            return label
    return None


def test_pins_pass_on_the_oracle_as_it_stands():
    assert _first_failure(_pin_calls()) is None


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(name, old, new, tmp_path, monkeypatch):
    src = open(SRC).read()
    assert src.count(old) == 1, f"{name}: the text to replace occurs {src.count(old)} times in the oracle's source"
    mutated = tmp_path / "mutant.c"
    mutated.write_text(src.replace(old, new))
    so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fopenmp", "-w", "-o", str(so), str(mutated), "-lm"],
                   check=True)
    oracle.lib()                                               # the real one is loaded (and built) first
    monkeypatch.setattr(oracle, "_lib", _load(str(so)))
    killed_by = _first_failure(_pin_calls())
    assert killed_by is not None, f"no pin notices: {name}"
