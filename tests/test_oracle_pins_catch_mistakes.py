"""The pins of the C oracle are only worth something if a plausible mistake in the oracle trips one of
them.  Each case plants one mistake (a wrong sign, a dropped term, an off-by-one, a swapped tie rule, a
transposed index) in a copy of oracle/kvq_oracle.c, builds it, and runs the oracle's pin tests against
that build in a child process: the run must fail.  The unmodified source, built the same way, must pass.
Everything here runs on the CPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "kvq_oracle.c")

PINS_QUANT = ["tests/test_oracle_quant.py", "tests/test_oracle_fp16_pack.py", "tests/test_oracle_signposts.py"]
PINS_MATVEC = ["tests/test_oracle_rope_matvec.py", "tests/test_oracle_sink.py"]

# (name, text in the source, mistaken text, pin files that must notice)
MISTAKES = [
    ("rope: sign of the sine term of the lower channel",
     "y[i] = x[i] * c - x[i + half] * sn;", "y[i] = x[i] * c + x[i + half] * sn;", PINS_MATVEC),
    ("rope: sign of the sine term of the upper channel",
     "y[i + half] = x[i + half] * c + x[i] * sn;", "y[i + half] = x[i + half] * c - x[i] * sn;", PINS_MATVEC),
    ("rope: frequency exponent halved",
     "pow(base, -2.0 * (double)i / (double)d)", "pow(base, -1.0 * (double)i / (double)d)", PINS_MATVEC),
    ("rope: position off by one",
     "double phi = (double)n * theta;", "double phi = (double)(n + 1) * theta;", PINS_MATVEC),
    ("nearest signpost: ties to the larger index",
     "if (dj < bestd) { bestd = dj; best = j; }", "if (dj <= bestd) { bestd = dj; best = j; }", PINS_QUANT),
    ("dequantisation: zero-point dropped",
     "*deq = fmaf(s, lut[code], z);", "*deq = s * lut[code];", PINS_QUANT),
    ("normalisation: zero-point not subtracted",
     "float diff = x - z;", "float diff = x;", PINS_QUANT),
    ("Key outlier test: non-strict comparison",
     "if (xv < kvqo_h2f(lo[c]) || xv > kvqo_h2f(hi[c])) {", "if (xv <= kvqo_h2f(lo[c]) || xv >= kvqo_h2f(hi[c])) {",
     PINS_QUANT),
    ("Value scale: full range instead of half range",
     "uint16_t sb = kvqo_f2h(dif * 0.5f);", "uint16_t sb = kvqo_f2h(dif);", PINS_QUANT),
    ("Value zero-point: minimum instead of mid-range",
     "uint16_t zb = kvqo_f2h(sum * 0.5f);", "uint16_t zb = kvqo_f2h(mn);", PINS_QUANT),
    ("Value lower outliers: off by one in the sorted rest",
     "is_out[w[k_side + k].i] = 1;", "is_out[w[k_side + k + 1].i] = 1;", PINS_QUANT),
    ("Value upper outliers: equal values taken from the larger index",
     "    if (p->v < q->v) return 1;\n    return (p->i > q->i) - (p->i < q->i);      /* equal values: smaller index first */",
     "    if (p->v < q->v) return 1;\n    return (p->i < q->i) - (p->i > q->i);", PINS_QUANT),
    ("sparse residual: stored without subtracting the dense part",
     "val[total] = kvqo_f2h(xv - deq);\n                }\n                ++total;\n                ++c_t;\n            }\n        }\n        cnt[t] = c_t;\n    }\n    return total;",
     "val[total] = kvqo_f2h(xv);\n                }\n                ++total;\n                ++c_t;\n            }\n        }\n        cnt[t] = c_t;\n    }\n    return total;",
     PINS_QUANT),
    ("reconstruction: Key outliers not added back",
     "khat[t * D + idx[e]] += (double)kvqo_h2f(val[e]);", "(void)val;", PINS_MATVEC),
    ("reconstruction: Value outliers added at the neighbouring channel",
     "vhat[t * D + idx[e]] += (double)kvqo_h2f(val[e]);", "vhat[t * D + (idx[e] ^ 1)] += (double)kvqo_h2f(val[e]);",
     PINS_MATVEC),
    ("scores: softmax scale dropped",
     "scores[h * ld + n] = (float)((double)scale * acc);", "scores[h * ld + n] = (float)acc;", PINS_MATVEC),
    ("scores: query heads of a group read the next KV head",
     "kvqo_rope(khat + hk * d, d, n, rope_base, krot);",
     "kvqo_rope(khat + ((hk + 1) % n_kv_heads) * d, d, n, rope_base, krot);", PINS_MATVEC),
    ("outputs: Value channels read transposed within the head",
     "acc[h * d + c] += p * vhat[hk * d + c];", "acc[h * d + c] += p * vhat[hk * d + (d - 1 - c)];", PINS_MATVEC),
    ("packing: the two codes of a Key field swapped",
     "put_bits(buf, k_chunk_base(bits, cap, n, h), 2 * bits * field + upper * bits, bits, code);",
     "put_bits(buf, k_chunk_base(bits, cap, n, h), 2 * bits * field + (1 - upper) * bits, bits, code);", PINS_QUANT),
    ("packing: Value pieces of a token pair at the wrong stride",
     "return (int64_t)(h * 2 + g) * (cap / 2) * 16 * bits + (m / 64) * 64 * 16 * bits + (m % 64) * 16;",
     "return (int64_t)(h * 2 + g) * (cap / 2) * 16 * bits + (m / 64) * 64 * 16 * bits + (m % 64) * 8;", PINS_QUANT),
    ("fp16 decoding: subnormals scaled as normal numbers",
     "v = ldexp((double)m, -24);", "v = ldexp((double)m, -25);", PINS_QUANT),
    ("fp16 decoding: exponent bias off by one",
     "v = ldexp((double)(m + 1024u), e - 25);", "v = ldexp((double)(m + 1024u), e - 24);", PINS_QUANT),
    ("packing: Key token blocks of 32 instead of 64",
     "return (int64_t)h * cap * 16 * bits + (n / 64) * 64 * 16 * bits + (n % 64) * 16;",
     "return (int64_t)h * cap * 16 * bits + (n / 32) * 32 * 16 * bits + (n % 32) * 16;", PINS_QUANT),
    ("packing: pieces 512 bytes apart",
     "*byte = base + (int64_t)piece * 1024 + inpiece / 8;", "*byte = base + (int64_t)piece * 512 + inpiece / 8;",
     PINS_QUANT),
    ("packing: bits of a code written most significant first",
     "unsigned b = (value >> k) & 1u;", "unsigned b = (value >> (nbits - 1 - k)) & 1u;", PINS_QUANT),
    ("packing: Value token parity ignored (both tokens of a pair in the low half of a field)",
     "int g = c / 64, field = c % 64, upper = (int)(n % 2);\n    put_bits(", "int g = c / 64, field = c % 64, upper = 0;\n    put_bits(",
     PINS_QUANT),
    ("Value scale: a zero range left at zero",
     "if (sf == 0.0f) { sf = 1.0f; sb = 0x3c00u; }", "if (sf == 0.0f) { sf = 0.0f; }", PINS_QUANT),
    ("Value outliers: guard against too many outliers dropped",
     "if (2 * k_side >= D) return -1;", "if (2 * k_side > D) return -1;", PINS_QUANT),
    ("softmax: maximum not subtracted",
     "for (int64_t n = 0; n < L; ++n) sum += exp((double)scores[h * ld_in + n] - mx);\n        for (int64_t n = 0; n < L; ++n)\n            probs[h * ld_out + n] = (float)(exp((double)scores[h * ld_in + n] - mx) / sum);",
     "mx = 0.0;\n        for (int64_t n = 0; n < L; ++n) sum += exp((double)scores[h * ld_in + n] - mx);\n        for (int64_t n = 0; n < L; ++n)\n            probs[h * ld_out + n] = (float)(exp((double)scores[h * ld_in + n] - mx) / sum);",
     PINS_MATVEC),
    ("softmax: normalised by the maximum term instead of the sum",
     "probs[h * ld_out + n] = (float)(exp((double)scores[h * ld_in + n] - mx) / sum);",
     "probs[h * ld_out + n] = (float)(exp((double)scores[h * ld_in + n] - mx));", PINS_MATVEC),
    ("attention sink: one token too many read from the fp16 rows (scores)",
     "            if (n < n_sink)\n                for (int c = 0; c < D; ++c) khat[c] = (double)kvqo_h2f(sink_k[n * D + c]);",
     "            if (n < n_sink + 1 && n_sink > 0)\n                for (int c = 0; c < D; ++c) khat[c] = (double)kvqo_h2f(sink_k[(n < n_sink ? n : n_sink - 1) * D + c]);",
     PINS_MATVEC),
    ("attention sink: Value rows of sink tokens taken from the quantized cache",
     "            if (n < n_sink)\n                for (int c = 0; c < D; ++c) vhat[c] = (double)kvqo_h2f(sink_v[n * D + c]);\n            else\n                kvqo_reconstruct_v(",
     "            if (0)\n                for (int c = 0; c < D; ++c) vhat[c] = (double)kvqo_h2f(sink_v[n * D + c]);\n            else\n                kvqo_reconstruct_v(",
     PINS_MATVEC),
    ("outputs: grouped-query heads all read KV head 0",
     "int hk = h / group;", "int hk = 0; (void)group;", PINS_MATVEC),
    ("signposts: stored as handed over instead of as fp16 numbers",
     "lut_stored[j] = kvqo_h2f(kvqo_f2h(lut_in[j]));", "lut_stored[j] = lut_in[j];", PINS_QUANT),
    ("fp16 rounding: truncation instead of round-to-nearest-even",
     "double r = nearbyint(q);", "double r = floor(q);", PINS_QUANT),
]


def _build(src_text, out_dir, name):
    c_path = os.path.join(out_dir, name + ".c")
    so_path = os.path.join(out_dir, name + ".so")
    with open(c_path, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", "-O1", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", so_path, c_path, "-lm"],
                   check=True)
    return so_path


def _pins_pass(lib, files):
    env = dict(os.environ, KVQ_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu", *files],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return r.returncode == 0, r.stdout[-1500:]


def _run_all(jobs):
    """jobs: name -> callable returning (passed, output tail).  A few at a time: each is a child pytest."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=max(1, min(6, (os.cpu_count() or 2) - 1))) as pool:
        futures = {name: pool.submit(fn) for name, fn in jobs.items()}
        return {name: f.result() for name, f in futures.items()}


@pytest.fixture(scope="module")
def c_oracle_runs(tmp_path_factory):
    text = open(SRC).read()
    out = str(tmp_path_factory.mktemp("c_oracle"))

    def job(i, good, bad, files):
        def run():
            if good is not None and text.count(good) < 1:
                return None, "the source no longer contains the line this case edits"
            lib = _build(text if good is None else text.replace(good, bad, 1), out, f"variant{i}")
            return _pins_pass(lib, files)
        return run

    jobs = {"unmodified": job(0, None, None, PINS_QUANT + PINS_MATVEC)}
    for i, (name, good, bad, files) in enumerate(MISTAKES, 1):
        jobs[name] = job(i, good, bad, files)
    return _run_all(jobs)


def test_the_unmodified_oracle_built_this_way_passes_its_pins(c_oracle_runs):
    ok, tail = c_oracle_runs["unmodified"]
    assert ok, tail


@pytest.mark.parametrize("name", [m[0] for m in MISTAKES])
def test_a_planted_mistake_trips_a_pin(c_oracle_runs, name):
    ok, tail = c_oracle_runs[name]
    assert ok is not None, f"{name}: {tail}"
    assert not ok, f"no pin noticed: {name}\n{tail}"


# ---- the calibration oracle (numpy): the same exercise on a copy of the tree ------------------------
CALIB_SRC = os.path.join(ROOT, "oracle", "kvq_calib_oracle.py")

CALIB_MISTAKES = [
    ("k-means: weights ignored in the update",
     "c[j] = np.float32(float(np.sum(w64[m] * x64[m])) / sw)", "c[j] = np.float32(float(np.mean(x64[m])))"),
    ("k-means: ties to the larger index", "closer = d < bestd", "closer = d <= bestd"),
    ("k-means: a signpost without weight jumps to zero",
     "        if sw > 0.0:\n            c[j] = np.float32(float(np.sum(w64[m] * x64[m])) / sw)",
     "        c[j] = np.float32(float(np.sum(w64[m] * x64[m])) / sw) if sw > 0.0 else np.float32(0.0)"),
    ("k-means: one iteration too few", "for _ in range(int(iters)):", "for _ in range(int(iters) - 1):"),
    ("objective: weights left out",
     "return float(np.sum(np.asarray(w, dtype=np.float64) * (x.astype(np.float64) - q) ** 2))",
     "return float(np.sum((x.astype(np.float64) - q) ** 2))"),
    ("thresholds: outlier count rounded down", "k = int(np.floor(float(outlier_fraction) / 2.0 * T + 0.5))",
     "k = int(np.floor(float(outlier_fraction) / 2.0 * T))"),
    ("thresholds: one order statistic too far out",
     "lo[c], hi[c] = np.float16(xs[k - 1]), np.float16(xs[T - k])", "lo[c], hi[c] = np.float16(xs[max(k - 2, 0)]), np.float16(xs[min(T - k + 1, T - 1)])"),
    ("range: includes the thresholds themselves", "a, b = xs[k], xs[T - k - 1]", "a, b = xs[k - 1], xs[T - k]"),
    ("scale: full range", "sc = np.float16((np.float32(b) - np.float32(a)) * np.float32(0.5))",
     "sc = np.float16(np.float32(b) - np.float32(a))"),
    ("zero-point: lower end instead of mid-range",
     "z[c] = np.float16((np.float32(b) + np.float32(a)) * np.float32(0.5))", "z[c] = np.float16(np.float32(a))"),
]


def _run_calib_pins(tree):
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu",
                        "tests/test_oracle_calib.py"], cwd=tree, env=dict(os.environ, OMP_NUM_THREADS="2"),
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return r.returncode == 0, r.stdout[-1500:]


def _copy_tree(dst, calib_text):
    import shutil
    for d in ("oracle", "kvq_synth"):
        shutil.copytree(os.path.join(ROOT, d), os.path.join(dst, d), ignore=shutil.ignore_patterns("__pycache__"))
    os.makedirs(os.path.join(dst, "tests"))
    for f in ("conftest.py", "kvq_testlib.py", "test_oracle_calib.py"):
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(dst, "tests", f))
    with open(os.path.join(dst, "oracle", "kvq_calib_oracle.py"), "w") as f:
        f.write(calib_text)


@pytest.fixture(scope="module")
def calib_oracle_runs(tmp_path_factory):
    text = open(CALIB_SRC).read()
    out = tmp_path_factory.mktemp("calib_oracle")

    def job(i, good, bad):
        def run():
            if good is not None and text.count(good) != 1:
                return None, "the source no longer contains the line this case edits"
            tree = str(out / f"tree{i}")
            _copy_tree(tree, text if good is None else text.replace(good, bad, 1))
            return _run_calib_pins(tree)
        return run

    jobs = {"unmodified": job(0, None, None)}
    for i, (name, good, bad) in enumerate(CALIB_MISTAKES, 1):
        jobs[name] = job(i, good, bad)
    return _run_all(jobs)


def test_the_unmodified_calibration_oracle_passes_its_pins_in_a_copied_tree(calib_oracle_runs):
    ok, tail = calib_oracle_runs["unmodified"]
    assert ok, tail


@pytest.mark.parametrize("name", [m[0] for m in CALIB_MISTAKES])
def test_a_planted_mistake_in_the_calibration_oracle_trips_a_pin(calib_oracle_runs, name):
    ok, tail = calib_oracle_runs[name]
    assert ok is not None, f"{name}: {tail}"
    assert not ok, f"no pin noticed: {name}\n{tail}"
