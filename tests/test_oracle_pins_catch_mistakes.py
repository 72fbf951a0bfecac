"""Do the pins pin?  Each case plants one plausible mistake in a COPY of the oracle's source (on the
CPU, in a temporary build), runs the pin suite against it in a subprocess and expects it to fail.
The oracle itself is never modified."""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "saps_oracle.cpp")

MISTAKES = [
    ("philox multipliers swapped", "const uint64_t M0 = 0xD2511F53ull, M1 = 0xCD9E8D57ull;",
     "const uint64_t M0 = 0xCD9E8D57ull, M1 = 0xD2511F53ull;"),
    ("philox nine rounds", "for (int r = 0; r < 10; ++r) {", "for (int r = 0; r < 9; ++r) {"),
    ("philox key bump dropped", "k1 += 0xBB67AE85u;", "k1 += 0u;"),
    ("philox words permuted", "c0 = n0; c1 = n1; c2 = n2; c3 = n3;", "c0 = n2; c1 = n1; c2 = n0; c3 = n3;"),
    ("wrong output word", "return out[j & 3];", "return out[(j + 1) & 3];"),
    ("round in the key instead of the counter", "static_cast<uint32_t>(round), static_cast<uint32_t>(round >> 32)};",
     "static_cast<uint32_t>(seed), static_cast<uint32_t>(round >> 32)};"),
    ("block index not shifted", "const uint64_t blk = static_cast<uint64_t>(j) >> 2;", "const uint64_t blk = static_cast<uint64_t>(j) >> 1;"),
    ("threshold off by a factor", "return static_cast<uint64_t>(std::floor(4294967296.0 / c));",
     "return static_cast<uint64_t>(std::floor(2147483648.0 / c));"),
    ("replace instead of average", "const float s = msg[i * msg_ld + k] + msg[p * msg_ld + k];",
     "const float s = 2.0f * msg[p * msg_ld + k];"),
    ("average only on one side", "if (p == i) continue;", "if (p <= i) continue;"),
    ("halving forgotten", "X[i * ld + idx[k]] = s * 0.5f;", "X[i * ld + idx[k]] = s;"),
    ("step with the wrong sign", "X[e] = std::fmaf(-lr, v, X[e]);", "X[e] = std::fmaf(lr, v, X[e]);"),
    ("step uses the gradient, not the buffer", "X[e] = std::fmaf(-lr, v, X[e]);", "X[e] = std::fmaf(-lr, G[e], X[e]);"),
    ("momentum not fused", "const float v = std::fmaf(mu, V[e], G[e]);", "const float t_ = mu * V[e]; const float v = t_ + G[e];"),
    ("message taken from the wrong row", "msg[i * msg_ld + kk] = X[i * ld + idx[kk]];", "msg[i * msg_ld + kk] = X[((i + 1) % n) * ld + idx[kk]];"),
    ("index list off by one", "idx[k++] = static_cast<uint32_t>(j);", "idx[k++] = static_cast<uint32_t>(j + 1);"),
    ("exchange before the local step", """    if (G) {
        rc = oracle_sgd_step(n, N, ld, X, G, V, lr, mu);
        if (rc) return rc;
    }
    rc = oracle_mask_compact(n, N, ld, n_seg, seg_off, seg_c, X, seed, round, idx, msg, msg_ld, K_out);
    if (rc) return rc;
    return oracle_merge(n, N, ld, X, peer, idx, msg, msg_ld, *K_out);""",
     """    rc = oracle_mask_compact(n, N, ld, n_seg, seg_off, seg_c, X, seed, round, idx, msg, msg_ld, K_out);
    if (rc) return rc;
    rc = oracle_merge(n, N, ld, X, peer, idx, msg, msg_ld, *K_out);
    if (rc) return rc;
    if (G) rc = oracle_sgd_step(n, N, ld, X, G, V, lr, mu);
    return rc;"""),
    ("Eq. (7) order steps first", """    if (rc) return rc;                                  // capacity overflow: nothing was written
    rc = oracle_merge(n, N, ld, X, peer, idx, msg, msg_ld, *K_out);
    if (rc) return rc;
    if (G) rc = oracle_sgd_step(n, N, ld, X, G, V, lr, mu);
    return rc;""", """    if (rc) return rc;
    if (G) rc = oracle_sgd_step(n, N, ld, X, G, V, lr, mu);
    if (rc) return rc;
    return oracle_merge(n, N, ld, X, peer, idx, msg, msg_ld, *K_out);"""),
    ("capacity found only after the local step", "    *K_out = K;\n    if (K > msg_ld) return ORACLE_ECAPACITY;\n    int rc = ORACLE_OK;",
     "    *K_out = K;\n    int rc = ORACLE_OK;"),
    ("consensus divides by n - 1", "mean[j] /= static_cast<double>(n);", "mean[j] /= static_cast<double>(n > 1 ? n - 1 : 1);"),
    ("disagreement without the square", "row += d * d;", "row += d < 0 ? -d : d;"),
]

# The per-segment loop appears four times in the oracle (mask; count and fill of the compaction; count of
# the round).  Each site gets each slip on its own: (name, old, new, which occurrence of `old`).
_T = "const uint64_t T = threshold(seg_c[s]);"
_LOOP = "for (int64_t j = seg_off[s]; j < seg_off[s + 1]; ++j)"
_SEGS = "for (int s = 0; s < n_seg; ++s) {\n        const uint64_t T"
_SITES = ["mask", "compaction count", "compaction fill", "round count"]
SEGMENT_MISTAKES = []
for k, site in enumerate(_SITES):
    SEGMENT_MISTAKES += [
        (f"{site}: first segment's ratio for every segment", _T, "const uint64_t T = threshold(seg_c[0]);", k),
        (f"{site}: next segment's ratio", _T, "const uint64_t T = threshold(seg_c[s + 1 < n_seg ? s + 1 : s]);", k),
        (f"{site}: segment starts one late", _LOOP, "for (int64_t j = seg_off[s] + 1; j < seg_off[s + 1]; ++j)", k),
        (f"{site}: segment ends one early", _LOOP, "for (int64_t j = seg_off[s]; j + 1 < seg_off[s + 1]; ++j)", k),
        (f"{site}: last segment skipped", _SEGS, "for (int s = 0; s + 1 < n_seg || s == 0; ++s) {\n        const uint64_t T", k),
    ]
# "<=" at a segment end: every cut is decided twice, once with the wrong ratio.  Planted where the extra
# coordinate cannot run past a buffer (the two counting loops and the mask are pure reads/own array of N).
SEGMENT_MISTAKES += [
    ("compaction count: <= at the segment end", _LOOP, "for (int64_t j = seg_off[s]; j <= seg_off[s + 1] && j < N; ++j)", 1),
    ("compaction fill: <= at the segment end", _LOOP, "for (int64_t j = seg_off[s]; j <= seg_off[s + 1] && j < N && k < K; ++j)", 2),
    ("round count: <= at the segment end", _LOOP, "for (int64_t j = seg_off[s]; j <= seg_off[s + 1] && j < N; ++j)", 3),
]


def _replace_nth(text, old, new, k):
    pos = -1
    for _ in range(k + 1):
        pos = text.find(old, pos + 1)
        assert pos >= 0, "mutation site not found"
    return text[:pos] + new + text[pos + len(old):]


PIN_FILES = ["test_oracle_mask.py", "test_oracle_round.py", "test_oracle_segments.py"]


def _pins_reject(mutant_text, name):
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "mutant.cpp"); lib = os.path.join(tmp, "libmutant.so")
        open(src, "w").write(mutant_text)
        subprocess.run(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-mfma", "-shared", "-fPIC", src, "-o", lib], check=True)
        env = dict(os.environ, SAPS_ORACLE_LIB=lib, SAPS_ORACLE_MUTATION_RUN="1")
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                            *[os.path.join(ROOT, "tests", f) for f in PIN_FILES]],
                           env=env, cwd=ROOT, capture_output=True, text=True, timeout=300)
        assert r.returncode == 1, f"pin suite exit code {r.returncode} (1 = a pin failed) for: {name}\n{r.stdout[-800:]}"


@pytest.mark.parametrize("name,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_pin_suite_rejects_a_planted_mistake(name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{name}' must occur exactly once in the oracle source"
    _pins_reject(text.replace(old, new), name)


@pytest.mark.parametrize("name,old,new,k", SEGMENT_MISTAKES, ids=[m[0] for m in SEGMENT_MISTAKES])
def test_pin_suite_rejects_a_slip_in_a_segment_loop(name, old, new, k):
    text = open(SRC).read()
    assert text.count(old) == len(_SITES), "the oracle's four segment loops changed shape: update the sites"
    _pins_reject(_replace_nth(text, old, new, k), name)


def test_the_oracle_override_needs_the_mutation_marker():
    # a stray SAPS_ORACLE_LIB alone must not swap the checker under any test
    env = {k: v for k, v in os.environ.items() if k != "SAPS_ORACLE_MUTATION_RUN"}
    env["SAPS_ORACLE_LIB"] = "/nonexistent/libother.so"
    r = subprocess.run([sys.executable, "-c", "from oracle import saps_oracle"], env=env, cwd=ROOT, capture_output=True, text=True)
    assert r.returncode != 0 and "SAPS_ORACLE_MUTATION_RUN" in r.stderr
