"""Would the pins notice a mistake in the oracle?  One plausible mistake at a time (a dropped
term, a wrong sign, index or tie rule, a transposed operand) is planted in a copy of an oracle
file, on the CPU, and the pin tests are run against that copy: every planted mistake must
fail at least one pin.  The copies live in a temporary directory; the repository's files are
never touched, and nothing here runs on a GPU.

Each entry: (what is wrong, text in the oracle file, what it is replaced with)."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

LAYER_MISTAKES = [
 ("bias sign", "logits + b[rows]", "logits - b[rows]"),
 ("bias row modulo", "pos // bias_group_tokens if", "pos % bias_group_tokens if"),
 ("tie to highest index", "e = np.argmax(cand, axis=1)", "e = E - 1 - np.argmax(cand[:, ::-1], axis=1)"),
 ("picked not marked", "picked[tt, e] = True", "pass"),
 ("gates not renormalised", "denom = w.sum(axis=1, keepdims=True)", "denom = 1.0"),
 ("gates normalised over batch", "denom = w.sum(axis=1, keepdims=True)", "denom = w.sum()"),
 ("softmax-all denominator over picked", "denom = np.exp(logits.astype(np.float64) - sel[:, :1]).sum(axis=1, keepdims=True)", "denom = w.sum(axis=1, keepdims=True) * 1.5"),
 ("counts only slot 0", "        for j in range(k):\n            counts[idx[t, j]] += 1", "        for j in range(1):\n            counts[idx[t, j]] += 1"),
 ("argmin instead of argmax", "e = np.argmax(cand, axis=1)", "e = np.argmin(np.where(picked, np.inf, logits.astype(np.float64)), axis=1)"),
 ("mask inverted", "(loc if mask[e] else rem)[e]", "(rem if mask[e] else loc)[e]"),
 ("buckets descending", "for a in range(flat.shape[0]):", "for a in reversed(range(flat.shape[0])):"),
 ("bytes without elem size", "nbytes = np.array([R * hidden * elem_size, R * hidden * elem_size]", "nbytes = np.array([R * hidden, R * hidden]"),
 ("bytes one way only", "nbytes = np.array([R * hidden * elem_size, R * hidden * elem_size]", "nbytes = np.array([R * hidden * elem_size, 0]"),
 ("remote offsets from local", "ro[e + 1] = ro[e] + len(rem[e])", "ro[e + 1] = ro[e] + len(loc[e])"),
 ("silu sign", "h = (g / (1.0 + np.exp(-g))) * u", "h = (g / (1.0 + np.exp(g))) * u"),
 ("sigmoid instead of silu", "h = (g / (1.0 + np.exp(-g))) * u", "h = (1.0 / (1.0 + np.exp(-g))) * u"),
 ("gate and up swapped", "h = (g / (1.0 + np.exp(-g))) * u", "h = (u / (1.0 + np.exp(-u))) * g"),
 ("up dropped", "h = (g / (1.0 + np.exp(-g))) * u", "h = (g / (1.0 + np.exp(-g)))"),
 ("token = a % k", "tok = np.asarray(local_src[b:en]) // k", "tok = np.asarray(local_src[b:en]) % k"),
 ("wrong expert weights", "wg, wu, wd = experts(e)\n", "wg, wu, wd = experts((e + 1) % E)\n"),
 ("shared rows misplaced", "y[n_local + s * T: n_local + (s + 1) * T] = swiglu_rows(x, wg, wu, wd)", "y[n_local + s * T: n_local + (s + 1) * T] = swiglu_rows(x[::-1], wg, wu, wd)"),
 ("combine drops gate", "out[t] += float(topk_gate[t, j]) * y[r]\n        for s", "out[t] += y[r]\n        for s"),
 ("combine slot reversed gate", "out[t] += float(topk_gate[t, j]) * y[r]\n        for s", "out[t] += float(topk_gate[t, k - 1 - j]) * y[r]\n        for s"),
 ("combine drops shared", "for s in range(n_shared):", "for s in range(0):"),
 ("combine shared index", "out[t] += y[n_local + s * T + t]", "out[t] += y[n_local + t]"),
 ("bf16 truncation", "r = ((u + half + lsb) >> drop) << drop", "r = (u >> drop) << drop"),
 ("bf16 round half up", "r = ((u + half + lsb) >> drop) << drop", "r = ((u + half + np.uint64(1)) >> drop) << drop"),
 ("bf16 one more bit", "drop = np.uint64(52 - 7)", "drop = np.uint64(52 - 8)"),
 ("pack_remote token", "x[int(a) // k] for a in remote_src", "x[int(a) % k] for a in remote_src"),
 ("combine_remote drops gate", "out[t] += float(topk_gate[t, j]) * y_remote[r]", "out[t] += y_remote[r]"),
 ("combine_remote no rounding", "                out[t] += float(topk_gate[t, j]) * y_remote[r]\n    return round_to_dtype(out, dtype)", "                out[t] += float(topk_gate[t, j]) * y_remote[r]\n    return out.astype(np.float32)"),
 ("router sum pairs the wrong elements", "acc += x64[:, h:h + 1] * w64[:, h][None, :]", "acc += x64[:, H - 1 - h:H - h] * w64[:, h][None, :]"),
 ("router sum drops the last element", "for h in range(H):    ", "for h in range(H - 1):"),
 ("logits not rounded to fp32", "logits = acc.astype(np.float32)", "logits = acc"),
 ("gate max not subtracted first slot", "w = np.exp(sel - sel[:, :1])", "w = np.exp(sel - sel[:, -1:]) * 0 + np.exp(sel)"),
]

PLACEMENT_MISTAKES = [
 ("entropy natural log", "h -= p * math.log2(p)", "h -= p * math.log(p)"),
 ("entropy sign", "h -= p * math.log2(p)", "h += p * math.log2(p)"),
 ("entropy unnormalised p", "p = c / total", "p = c / E"),
 ("alloc floor->round", "int(math.floor(server_mem[n] / expert_mem * share))", "int(round(server_mem[n] / expert_mem * share))"),
 ("alloc ceil", "int(math.floor(server_mem[n] / expert_mem * share))", "int(math.ceil(server_mem[n] / expert_mem * share))"),
 ("alloc no cap", "cnt[n, l] = min(E, int(math.floor(server_mem[n] / expert_mem * share)))", "cnt[n, l] = int(math.floor(server_mem[n] / expert_mem * share))"),
 ("alloc share by max", "vsum = float(sum(v[n, l] for l in range(L)))", "vsum = float(max(v[n, l] for l in range(L)))"),
 ("alloc zero entropy -> 0 share", "if vsum > 0.0 else 1.0 / L", "if vsum > 0.0 else 0.0"),
 ("servers ascending memory", "key=lambda n: (-server_mem[n], n))", "key=lambda n: (server_mem[n], n))"),
 ("servers index order", "order = sorted(range(N), key=lambda n: (-server_mem[n], n))", "order = list(range(N))"),
 ("donor may drop to E-1", "if lp != l and total[lp] > E]", "if lp != l and total[lp] >= E]"),
 ("donor smallest total", "lp = max(donors, key=lambda j: (total[j], -j))", "lp = min(donors, key=lambda j: (total[j], j))"),
 ("donor tie highest index", "lp = max(donors, key=lambda j: (total[j], -j))", "lp = max(donors, key=lambda j: (total[j], j))"),
 ("donor fixed per pass", "            for n in order:\n                donors = [lp for lp in range(L) if lp != l and total[lp] > E]        # R3\n                if not donors:\n                    break\n                lp = max(donors, key=lambda j: (total[j], -j))",
                          "            donors = [lp for lp in range(L) if lp != l and total[lp] > E]\n            if not donors:\n                feasible = False\n                break\n            lp = max(donors, key=lambda j: (total[j], -j))\n            for n in order:\n                if total[lp] <= E:\n                    break"),
 ("receiver cap ignored", "if cnt[n, lp] > 0 and cnt[n, l] < E:", "if cnt[n, lp] > 0:"),
 ("donor count not checked", "if cnt[n, lp] > 0 and cnt[n, l] < E:", "if cnt[n, l] < E:"),
 ("no stop at E", "                    if total[l] == E:\n                        break\n", ""),
 ("preference ascending", "key=lambda e: (-int(f_nl[e]), e))", "key=lambda e: (int(f_nl[e]), e))"),
 ("preference tie high index", "key=lambda e: (-int(f_nl[e]), e))", "key=lambda e: (-int(f_nl[e]), -e))"),
 ("top-N off by one", "[: int(cnt[n, l])]", "[: max(int(cnt[n, l]) - 1, 0)]"),
 ("duplicates = any held", "if place[n, l, e] and holders(e) >= 2]", "if place[n, l, e]]"),
 ("servers most duplicates first", "key=lambda n: (len(duplicates(n)), n))", "key=lambda n: (-len(duplicates(n)), n))"),
 ("candidate least frequent", "e_new = min(unassigned, key=lambda e: (-int(f[n, l, e]), e))", "e_new = min(unassigned, key=lambda e: (int(f[n, l, e]), e))"),
 ("candidate tie high index", "e_new = min(unassigned, key=lambda e: (-int(f[n, l, e]), e))", "e_new = min(unassigned, key=lambda e: (-int(f[n, l, e]), -e))"),
 ("replace most frequent duplicate", "e_rep = min(dup, key=lambda e: (int(f[n, l, e]), -e))", "e_rep = max(dup, key=lambda e: (int(f[n, l, e]), -e))"),
 ("replace tie low index", "e_rep = min(dup, key=lambda e: (int(f[n, l, e]), -e))", "e_rep = min(dup, key=lambda e: (int(f[n, l, e]), e))"),
 ("order recomputed never / stale U", "                unassigned.remove(e_new)\n", "                pass\n"),
 ("proxy cost counts hosted", "if not place[n, l, e]:\n                    cost", "if place[n, l, e]:\n                    cost"),
 ("migration additions only", "if bool(old[n, l, e]) != bool(new[n, l, e]):", "if not bool(old[n, l, e]) and bool(new[n, l, e]):"),
 ("migration speed of server 0", "seconds += expert_mem / speed[n]", "seconds += expert_mem / speed[0]"),
 ("migration mem*speed", "seconds += expert_mem / speed[n]", "seconds += expert_mem * speed[n]"),
 ("eq4 non-strict", "+ t_mig < cost_old * seconds_per_remote_call", "+ t_mig <= cost_old * seconds_per_remote_call"),
 ("eq4 ignores t_mig", "cost_new * seconds_per_remote_call + t_mig < cost_old", "cost_new * seconds_per_remote_call < cost_old"),
 ("eq4 unscaled cost", "return cost_new * seconds_per_remote_call + t_mig <", "return cost_new + t_mig <"),
]


# A server can only receive an expert of a layer that is short of experts, so it holds fewer
# than E of that layer anyway: dropping that condition of Alg. 1's step 2 changes no result.
NOT_A_MISTAKE = {"receiver cap ignored"}


def _run_against_copy(tmp_root, n, target, pins, mistake):
    """Copies the oracle and the pin tests into a directory of their own, plants the mistake
    there, runs the pins with that directory first on the import path; True = a pin failed."""
    name, old, new = mistake
    d = os.path.join(tmp_root, f"m{n}")
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(d, "oracle"),
                    ignore=shutil.ignore_patterns("__pycache__"))
    os.makedirs(os.path.join(d, "tests"))
    for f in ("conftest.py", pins):
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(d, "tests", f))
    path = os.path.join(d, "oracle", target)
    text = open(path).read()
    assert text.count(old) >= 1, f"the oracle no longer contains the text of mistake {name!r}"
    open(path, "w").write(text.replace(old, new, 1))
    # one thread per run (several runs share the cores); a mistake that makes an iteration of
    # the placement algorithms run on for ever ends at the per-test limit, i.e. fails its pin
    env = dict(os.environ, PYTHONPATH=d + os.pathsep + ROOT, PYTHONDONTWRITEBYTECODE="1",
               OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1")
    try:
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p",
                            "no:cacheprovider", "--timeout", "20", os.path.join(d, "tests", pins)],
                           cwd=d, env=env, capture_output=True, text=True, timeout=300)
    except subprocess.TimeoutExpired:
        return name, True, "did not finish"
    shutil.rmtree(d, ignore_errors=True)
    failed = r.returncode == 1            # 1 = tests failed; anything else is a broken run
    assert r.returncode in (0, 1), (name, r.stdout[-2000:], r.stderr[-2000:])
    return name, failed, ""


@pytest.mark.parametrize("target,pins,mistakes", [
    ("prism_oracle.py", "test_oracle_pins.py", LAYER_MISTAKES),
    ("placement_oracle.py", "test_placement_pins.py", PLACEMENT_MISTAKES),
])
def test_every_planted_mistake_fails_a_pin(tmp_path, target, pins, mistakes):
    # the unchanged copy passes (so a failure below is the mistake's doing)
    name, failed, _ = _run_against_copy(str(tmp_path), 9999, target, pins, ("none", "import", "import"))
    assert not failed
    workers = max(1, min(8, len(os.sched_getaffinity(0))))
    with ThreadPoolExecutor(max_workers=workers) as ex:
        results = list(ex.map(lambda a: _run_against_copy(str(tmp_path), a[0], target, pins, a[1]),
                              enumerate(mistakes)))
    survivors = sorted(name for name, failed, _ in results if not failed)
    assert set(survivors) <= NOT_A_MISTAKE, f"no pin notices: {survivors}"
    print(f"{target}: {len(mistakes) - len(survivors)} of {len(mistakes)} planted mistakes fail a pin"
          + (f"; no mistake at all: {survivors}" if survivors else ""))
