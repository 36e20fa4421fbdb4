"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer: a second build of oracle/*.c with
-fsanitize=address,undefined runs a small case of every exported function in a child process (the sanitizer runtime
has to be loaded before the interpreter starts).  Any out-of-bounds access, use after free, signed overflow,
misaligned access or invalid shift in the oracle ends the child with a report."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import sys
import numpy as np
sys.path.insert(0, %(root)r)
import oracle as orc
import synth

C, D, B, K, M = 300, 32, 24, 6, 64
W = synth.unit_rows(1, synth.TID_W, C, D, bf16=True)
X = synth.unit_rows(1, synth.TID_X, B, D, bf16=True)
y = synth.labels_uniform(1, B, C)
names = []

G, S = orc.graph_bruteforce(W, K); names.append("orc_graph_bruteforce")
G2, _ = orc.graph_bruteforce(W, K, np.array([0, 5, C - 1], dtype=np.int32))
assert (G2 == G[[0, 5, C - 1]]).all()
g0 = np.full((100, K), -1, dtype=np.int32); s0 = np.full((100, K), -np.inf)
g1, s1 = orc.graph_update(W[:100], W[100:], 0, 100, g0, s0); names.append("orc_graph_update")
g1, s1 = orc.graph_update(W[:100], W[:100], 0, 0, g1, s1)
assert (g1 == G[:100]).all()
act, A, tpos = orc.select_active(y, G, C, M); names.append("orc_select_active")
act2, A2, _ = orc.select_active(y, G, C, B + 3)                       # the cut bites
assert A2 == B + 3 and A > A2
ref = orc.knn_softmax_fwd_bwd(W, X, act[:A], tpos, 30.0, 4.0, want_P=True); names.append("orc_knn_softmax_fwd_bwd")
assert abs(ref["P"].sum(axis=1) - 1).max() < 1e-12
full = orc.full_softmax_fwd_bwd(W, X, y, 30.0, 4.0); names.append("orc_full_softmax_fwd_bwd")
idx = np.array([3, 7, 3, 299, 0], dtype=np.int32)
orc.apply_weight_grad(W, idx, synth.grad_rows(1, 5, D), -0.1); names.append("orc_apply_weight_grad")
orc.normalize_rows(3.0 * W); names.append("orc_normalize_rows")
orc.norm_backward(3.0 * W[:5], synth.grad_rows(2, 5, D).astype(np.float64)); names.append("orc_norm_backward")
orc.apply_weight_grad_normalized(3.0 * W, idx, synth.grad_rows(1, 5, D), -0.1); names.append("orc_apply_weight_grad_normalized")
counts, offsets, flat = orc.graph_compress(G, 100, 120); names += ["orc_graph_compress"]
orc.pad_draws(120, 5, 300); names.append("orc_pad_draws")
a, n, nf, t = orc.select_active_csr(y, counts, offsets, flat, 100, 120, 64, pad=True, seed=5); names.append("orc_select_active_csr")
assert n == 64 and nf <= n
a, n, nf, t = orc.select_active_csr(y, counts, offsets, flat, 100, 120, 64, pad=False)
if n:
    m, l, tz = orc.softmax_node_stats(W[100:220], X, a[:n], t, 30.0); names.append("orc_softmax_node_stats")
    orc.softmax_node_bwd(W[100:220], X, a[:n], t, 30.0, 4.0, m, l + 1.0, tz); names.append("orc_softmax_node_bwd")
g = synth.normal(3, synth.TID_MISC, 0, 5000).astype(np.float32)
g[::7] = 0.0
i1, v1 = orc.topk_abs(g, 40); names.append("orc_topk_abs")
i2, v2 = orc.topk_dc(g, 40, 9); names.append("orc_topk_dc")
assert (i1 == i2).all()
offs = np.array([0, 1000, 1001, 5000], dtype=np.int64)
kk = np.array([10, 1, 50], dtype=np.int32)
i3, _ = orc.topk_group(g, offs, kk); names.append("orc_topk_group")
i4, _ = orc.topk_group(g, offs, kk, M=np.array([3, 1, 8], dtype=np.int32))
assert (i3 == i4).all()
assert orc.num_threads() >= 1; names.append("orc_num_threads")
assert orc.lib()._name.endswith("liboracle_sanitized.so"), orc.lib()._name
print("EXERCISED " + " ".join(names))
"""


def _sanitizer_env():
    sys.path.insert(0, ROOT)
    from oracle.build import sanitizer_runtime
    runtime = sanitizer_runtime()
    assert os.path.isabs(runtime) and os.path.exists(runtime), "gcc's libasan.so not found"
    env = dict(os.environ)
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "2"
    return env


def test_the_sanitizer_set_up_reports_a_planted_mistake(tmp_path):
    """The same flags and the same way of loading, on a five-line C file that reads one element past a heap block:
    the child must end with an AddressSanitizer report (otherwise a clean run of the oracle would prove nothing)."""
    src = tmp_path / "bad.c"
    src.write_text("#include <stdlib.h>\nint bad(int n) { int *p = (int *)malloc(sizeof(int) * (size_t)n); "
                   "for (int i = 0; i < n; ++i) p[i] = i; int v = p[n]; free(p); return v; }\n")
    lib = tmp_path / "libbad.so"
    subprocess.check_call(["gcc", "-O1", "-g", "-fPIC", "-shared", "-fsanitize=address,undefined",
                           "-fno-omit-frame-pointer", "-o", str(lib), str(src)])
    r = subprocess.run([sys.executable, "-c", f"import ctypes; ctypes.CDLL({str(lib)!r}).bad(8)"], env=_sanitizer_env(),
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "AddressSanitizer: heap-buffer-overflow" in r.stderr


def test_every_oracle_function_runs_clean_under_address_and_ub_sanitizers():
    env = _sanitizer_env()
    from oracle.build import build_sanitized
    env["ORACLE_LIB_PATH"] = build_sanitized()
    r = subprocess.run([sys.executable, "-c", CHILD % dict(root=ROOT)], env=env, capture_output=True, text=True, timeout=600)
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    line = [l for l in r.stdout.splitlines() if l.startswith("EXERCISED ")][-1]
    exercised = set(line.split()[1:])
    # every function the library exports (the child really loaded the sanitized build: same symbol list)
    import re
    exported = set()
    for src in ("knn_softmax_oracle.c", "topk_oracle.c"):
        text = open(os.path.join(ROOT, "oracle", src)).read()
        exported |= set(re.findall(r"^int (orc_[a-z0-9_]+)\(", text, flags=re.M))
    assert exported <= exercised, f"not exercised: {sorted(exported - exercised)}"
