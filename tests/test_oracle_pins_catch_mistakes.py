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
    ("Eq. (6) order steps first", """    if (rc) return rc;                                  // capacity overflow: nothing was written
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


@pytest.mark.parametrize("name,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_pin_suite_rejects_a_planted_mistake(name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{name}' must occur exactly once in the oracle source"
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "mutant.cpp"); lib = os.path.join(tmp, "libmutant.so")
        open(src, "w").write(text.replace(old, new))
        subprocess.run(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-mfma", "-shared", "-fPIC", src, "-o", lib], check=True)
        env = dict(os.environ, SAPS_ORACLE_LIB=lib)
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                            os.path.join(ROOT, "tests", "test_oracle_mask.py"), os.path.join(ROOT, "tests", "test_oracle_round.py")],
                           env=env, cwd=ROOT, capture_output=True, text=True, timeout=300)
        assert r.returncode == 1, f"pin suite exit code {r.returncode} (1 = a pin failed) for: {name}\n{r.stdout[-800:]}"
