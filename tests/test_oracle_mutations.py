"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of the oracle's C source (a dropped term, a
wrong sign or index, a swapped operand, an off-by-one), builds it into a separate library, and runs the pin tests
against it in a child process: they must fail.  The unmodified oracle passing the same tests is the rest of the CPU
suite.  Everything here runs on the CPU; the HIP path is not involved."""
import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = {n: os.path.join(ROOT, "oracle", n) for n in ("moe_oracle.c", "moe_oracle_fp8.c")}

# (name, file, text to find (its FIRST occurrence is replaced), replacement, pin files that must reject it)
MUTANTS = [
    ("router: bias dropped", "moe_oracle.c", "if (bias) acc += (double)bias[e];", "(void)bias;", ["test_oracle_router.py"]),
    ("router: W indexed by token", "moe_oracle.c", "ld(w_router, (size_t)e * H + h, dt);", "ld(w_router, (size_t)(e ? e - 1 : 0) * H + h, dt);",
     ["test_oracle_router.py"]),
    ("top-k: ties to the higher index", "moe_oracle.c", "return ia < ib; /* equal", "return ia > ib; /* equal", ["test_oracle_router.py"]),
    ("top-k: softmax without the max shift and a wrong sign", "moe_oracle.c", "p[e] = exp((double)l[e] - m);", "p[e] = exp(m - (double)l[e]);",
     ["test_oracle_router.py"]),
    ("top-k: renormalisation divides by the sum over one slot less", "moe_oracle.c",
     "for (int k = 0; k < K; ++k) s += gate[(size_t)t * K + k];", "for (int k = 0; k + 1 < K; ++k) s += gate[(size_t)t * K + k];",
     ["test_oracle_router.py"]),
    ("capacity: rounded down", "moe_oracle.c", "return (int)ceil(capacity_factor", "return (int)floor(capacity_factor", ["test_oracle_permute.py"]),
    ("permute: keeps one assignment too many", "moe_oracle.c", "if (capacity > 0 && rank >= capacity) {", "if (capacity > 0 && rank > capacity) {",
     ["test_oracle_permute.py"]),
    ("permute: copies the row of the wrong token", "moe_oracle.c", "(const char*)x + (a / (size_t)K) * row_bytes, row_bytes);\n    }\n    free(n);",
     "(const char*)x + (a % (size_t)T) * row_bytes, row_bytes);\n    }\n    free(n);", ["test_oracle_permute.py", "test_oracle_layer.py"]),
    ("experts: gate and up swapped in SiLU", "moe_oracle.c", "double silu = g / (1.0 + exp(-g));\n            h[(size_t)r * F + f] = silu * u;",
     "double silu = u / (1.0 + exp(-u));\n            h[(size_t)r * F + f] = silu * g;", ["test_oracle_layer.py"]),
    ("experts: W_down read transposed", "moe_oracle.c", "acc += h[(size_t)r * F + f] * ld(w_down, (size_t)n * F + f, dt);",
     "acc += h[(size_t)r * F + f] * ld(w_down, ((size_t)f * H + n) % ((size_t)H * F), dt);", ["test_oracle_layer.py"]),
    ("experts: every expert uses expert 0's gate weights", "moe_oracle.c", "(const char*)w_gate + (size_t)e * F * H * es,",
     "(const char*)w_gate + (size_t)0 * F * H * es,", ["test_oracle_layer.py"]),
    ("combine: gate of the neighbouring slot", "moe_oracle.c", "acc += gate[(size_t)t * K + k] * y_perm[(size_t)row * H + n];",
     "acc += gate[(size_t)t * K + (k + 1 < K ? k + 1 : k)] * y_perm[(size_t)row * H + n];", ["test_oracle_layer.py", "test_oracle_permute.py"]),
    ("experts backward: derivative of SiLU without its second term", "moe_oracle.c",
     "dg[(size_t)r * F + f] = dh * uv * sg * (1.0 + gv * (1.0 - sg));", "dg[(size_t)r * F + f] = dh * uv * sg;", ["test_oracle_backward.py"]),
    ("experts backward: dW_up from dg", "moe_oracle.c", "au += du[(size_t)r * F + f] * xv;", "au += dg[(size_t)r * F + f] * xv;", ["test_oracle_backward.py"]),
    ("router backward: renormalisation without the projection term", "moe_oracle.c",
     "q[k] = renormalize ? (dgate[(size_t)t * K + k] - a) / S : dgate[(size_t)t * K + k];",
     "q[k] = renormalize ? dgate[(size_t)t * K + k] / S : dgate[(size_t)t * K + k];", ["test_oracle_backward.py"]),
    ("router backward: softmax Jacobian without its diagonal", "moe_oracle.c",
     "if (e >= 0 && e < E) dlogits[(size_t)t * E + e] += q[k] * p[e];", "(void)e;", ["test_oracle_backward.py"]),
    ("router backward: dW_g and dx swapped operands", "moe_oracle.c",
     "for (int t = 0; t < T; ++t) acc += dlogits[(size_t)t * E + e] * ld(x, (size_t)t * H + n, dt);",
     "for (int t = 0; t < T; ++t) acc += dlogits[(size_t)t * E + e] * ld(x, (size_t)t * H + (n + 1) % H, dt);", ["test_oracle_backward.py"]),
    ("fp8 experts: up projection dequantised with the gate's factor", "moe_oracle_fp8.c", "u *= dq_up;", "u *= dq_gate;", ["test_oracle_fp8.py"]),
    ("fp8 experts: SiLU applied after the dequantisation of the wrong operand", "moe_oracle_fp8.c", "double hv = (g / (1.0 + exp(-g))) * u;",
     "double hv = (u / (1.0 + exp(-u))) * g;", ["test_oracle_fp8.py"]),
    ("fp8 experts: h quantised without its scale", "moe_oracle_fp8.c", "volatile float p = (float)hv * scale_h;", "volatile float p = (float)hv;",
     ["test_oracle_fp8.py"]),
    ("fp8 experts: amax of the quantised instead of the real h", "moe_oracle_fp8.c", "if (fabs(hv) > am) am = fabs(hv);",
     "if (fabs(hv * scale_h) > am) am = fabs(hv * scale_h);", ["test_oracle_fp8.py"]),
    ("fp8: delayed scale with the margin's sign flipped", "moe_oracle_fp8.c", "ldexp(1.0, margin)", "ldexp(1.0, -margin)", ["test_oracle_fp8.py"]),
    ("fp8: history maximum replaced by the last entry", "moe_oracle_fp8.c", "if (amax_history[i] > m && isfinite(amax_history[i])) m = amax_history[i];",
     "if (isfinite(amax_history[i])) m = amax_history[i];", ["test_oracle_fp8.py"]),
    ("combine backward: dy_perm without the gate", "moe_oracle.c", "dy_perm[(size_t)row * H + n] = gate[a] * dy[(size_t)t * H + n];",
     "dy_perm[(size_t)row * H + n] = dy[(size_t)t * H + n];", ["test_oracle_backward.py"]),
    ("combine backward: dgate against the gradient of the wrong token", "moe_oracle.c", "dot += dy[(size_t)t * H + n] * y_perm[(size_t)row * H + n];",
     "dot += dy[(size_t)(t ? t - 1 : 0) * H + n] * y_perm[(size_t)row * H + n];", ["test_oracle_backward.py"]),
    ("permute backward: the other gradient path dropped", "moe_oracle.c", "if (addend) acc += addend[(size_t)t * H + n];\n            dx[",
     "(void)addend;\n            dx[", ["test_oracle_backward.py"]),
    ("permute variant: ties to the higher index", "moe_oracle.c", "return (a->a > b->a) - (a->a < b->a);", "return (a->a < b->a) - (a->a > b->a);",
     ["test_oracle_permute_variants.py"]),
    ("permute variant: lowest scores kept", "moe_oracle.c", "if (a->score > b->score) return -1;\n    if (a->score < b->score) return 1;",
     "if (a->score > b->score) return 1;\n    if (a->score < b->score) return -1;", ["test_oracle_permute_variants.py"]),
    ("fp8: decode with exponent bias 8", "moe_oracle_fp8.c", "v = ldexp(1.0 + (double)m / 8.0, e - 7);", "v = ldexp(1.0 + (double)m / 8.0, e - 8);",
     ["test_oracle_fp8.py"]),
    ("fp8: encode saturates one code early", "moe_oracle_fp8.c", "if (a > 448.0) return (uint8_t)(sign | 0x7e);", "if (a > 416.0) return (uint8_t)(sign | 0x7e);",
     ["test_oracle_fp8.py"]),
    ("chunk gather: source chunks start one chunk late", "moe_oracle.c", "const long long from = src_start[c] + i, to = d + i;",
     "const long long from = src_start[c + 1] + i, to = d + i;", ["test_oracle_sort_chunks.py"]),
    ("chunk gather: destination chunk takes the size of its own position", "moe_oracle.c",
     "const long long n = (c >= 0 && c < n_src) ? src_start[c + 1] - src_start[c] : 0;",
     "const long long n = (c >= 0 && c < n_src && p < n_src) ? src_start[p + 1] - src_start[p] : 0;", ["test_oracle_sort_chunks.py"]),
    ("chunk gather: group offsets one chunk early", "moe_oracle.c", "if (group_offsets && group > 0 && p % group == 0) group_offsets[p / group] = (int32_t)d;",
     "if (group_offsets && group > 0 && (p + 1) % group == 0) group_offsets[p / group] = (int32_t)d;", ["test_oracle_sort_chunks.py"]),
]


def _resolve(m):
    name, fname, find, repl, pins = m
    return name, fname, find, repl, pins, open(SRC[fname]).read()


def _run_mutant(m, tmp):
    name, fname, find, repl, pins, text = _resolve(m)
    if text.count(find) < 1:
        return name, "anchor", "anchor text not found in the source"
    d = os.path.join(tmp, str(abs(hash(name))))
    os.makedirs(d, exist_ok=True)
    srcs = []
    for n, path in SRC.items():
        out = os.path.join(d, n)
        body = open(path).read()
        if n == fname:
            body = body.replace(find, repl, 1)
        open(out, "w").write(body)
        srcs.append(out)
    lib = os.path.join(d, "libmutant.so")
    cc = subprocess.run(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-w", "-o", lib, *srcs, "-lm"], capture_output=True, text=True)
    if cc.returncode != 0:
        return name, "compile", cc.stderr[-400:]
    env = dict(os.environ, MOE_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                        *[os.path.join(ROOT, "tests", p) for p in pins]], cwd=ROOT, env=env, capture_output=True, text=True)
    # a mutant that writes past a buffer may also take the child down (signal, or a non-1 status after a test
    # already failed): that run has failed a pin just the same
    crashed = r.returncode < 0 or r.returncode in (134, 139)
    caught = r.returncode == 1 or crashed or (r.returncode != 0 and " failed" in r.stdout)
    return name, ("caught" if caught else "survived" if r.returncode == 0 else "error"), r.stdout[-300:]


def test_every_planted_mistake_is_caught_by_a_pin():
    with tempfile.TemporaryDirectory() as tmp, ThreadPoolExecutor(4) as pool:
        results = list(pool.map(lambda m: _run_mutant(m, tmp), MUTANTS))
    bad = [(n, s, info) for n, s, info in results if s != "caught"]
    assert not bad, "\n".join(f"{n}: {s}: {info}" for n, s, info in bad)
