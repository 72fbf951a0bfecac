// CPU oracle for one SAPS-PSGD round.  TEST INFRASTRUCTURE ONLY.
//
// This file is the slow, plain, single-threaded definition that the GPU library is
// checked against.  It shares no code, header, table or helper with the GPU path and
// must never be called from it: only tests, the smoke check and the benchmark's
// cpu_baseline leg may load it.
//
// What it computes (worker model matrix X stored n x ld row-major, row = worker):
//   update   Alg. 2 line 5 and procedure SGD:  x <- x - gamma * grad, here with a
//            heavy-ball momentum buffer v (v <- mu*v + g ; x <- x - lr*v); mu = 0 and no
//            buffer gives the paper's plain step.  The paper has no momentum; this form
//            (two correctly rounded fp32 fused multiply-adds) is this build's reading.
//   mask     Sec. II-B, Eq. (3): m[j] = 1 with probability 1/c, the same vector on every
//            worker because all use the round's seed.  The paper fixes no generator; this
//            build defines m[j] from Philox4x32-10 (Salmon et al., SC'11) keyed by the
//            seed, counter (j>>2, round), output word j&3, compared with floor(2^32/c).
//   compact  Eq. (2) and the sentence after Eq. (3): only the non-zeros of x o m travel;
//            they are packed in ascending coordinate order.
//   merge    Alg. 2 lines 8-10 read with the prose of Sec. II-A (the worker averages
//            what it received with its own values) and GenerateW (weights 1/2, 1/2):
//            masked coordinates of matched rows become (own + peer)/2, everything else
//            is unchanged.  Matrix form: Eq. (7) without the gradient term.
//   round    Alg. 2 order: update, then mask/compact, then merge.
//   consensus  Sec. II-C: the average model and sum_i ||x_i - mean||^2 (the quantity Theorem 1
//            bounds), by the two-pass textbook definition in fp64.
//
// Pinned by tests/test_oracle_*.py (known-answer vectors, brute force against the
// explicit matrices M and W, closed forms and invariants).
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -mfma -shared -fPIC (no fast-math).

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

// Philox4x32-10 from its published definition: ten rounds of two 32x32->64 multiplies
// with word permutation and key injection, key bumped by two Weyl constants per round.
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    const uint64_t M0 = 0xD2511F53ull, M1 = 0xCD9E8D57ull;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = M0 * c0;
        const uint64_t p1 = M1 * c2;
        const uint32_t n0 = static_cast<uint32_t>(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = static_cast<uint32_t>(p1);
        const uint32_t n2 = static_cast<uint32_t>(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = static_cast<uint32_t>(p0);
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// floor(2^32 / c) as an integer in [0, 2^32]; c = 1 keeps every coordinate.
uint64_t threshold(double c) {
    return static_cast<uint64_t>(std::floor(4294967296.0 / c));
}

// The 32 random bits that decide coordinate j in this round.
uint32_t coord_bits(uint64_t seed, uint64_t round, int64_t j) {
    const uint64_t blk = static_cast<uint64_t>(j) >> 2;
    const uint32_t ctr[4] = {static_cast<uint32_t>(blk), static_cast<uint32_t>(blk >> 32),
                             static_cast<uint32_t>(round), static_cast<uint32_t>(round >> 32)};
    const uint32_t key[2] = {static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
    uint32_t out[4];
    philox4x32_10(ctr, key, out);
    return out[j & 3];
}

bool layout_ok(int32_t n, int64_t N, int64_t ld, int32_t n_seg, const int64_t* seg_off, const double* seg_c) {
    if (n < 1 || N < 0 || ld < N || n_seg < 1 || !seg_off || !seg_c) return false;
    if (seg_off[0] != 0 || seg_off[n_seg] != N) return false;
    for (int s = 0; s < n_seg; ++s) {
        if (seg_off[s + 1] < seg_off[s]) return false;
        if (!(seg_c[s] >= 1.0)) return false;
    }
    return true;
}

bool matching_ok(int32_t n, const int32_t* peer) {
    for (int32_t i = 0; i < n; ++i) {
        if (peer[i] < 0 || peer[i] >= n) return false;
        if (peer[peer[i]] != i) return false;
    }
    return true;
}

}  // namespace

extern "C" {

enum { ORACLE_OK = 0, ORACLE_EINVAL = 1, ORACLE_EMATCH = 2, ORACLE_ECAPACITY = 3 };

void oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    philox4x32_10(ctr, key, out);
}

uint64_t oracle_threshold(double c) { return threshold(c); }

uint32_t oracle_coord_bits(uint64_t seed, uint64_t round, int64_t j) { return coord_bits(seed, round, j); }

// Eq. (3): keep[j] in {0,1} for j in [0, N).
int oracle_mask(int64_t N, int32_t n_seg, const int64_t* seg_off, const double* seg_c,
                uint64_t seed, uint64_t round, uint8_t* keep) {
    if (!layout_ok(1, N, N, n_seg, seg_off, seg_c)) return ORACLE_EINVAL;
    for (int s = 0; s < n_seg; ++s) {
        const uint64_t T = threshold(seg_c[s]);
        for (int64_t j = seg_off[s]; j < seg_off[s + 1]; ++j)
            keep[j] = static_cast<uint64_t>(coord_bits(seed, round, j)) < T ? 1 : 0;
    }
    return ORACLE_OK;
}

// Alg. 2 line 5 (procedure SGD), with momentum.  V may be null iff mu == 0.
int oracle_sgd_step(int32_t n, int64_t N, int64_t ld, float* X, const float* G, float* V, float lr, float mu) {
    if (n < 1 || N < 0 || ld < N || !X || !G) return ORACLE_EINVAL;
    if (!V && mu != 0.0f) return ORACLE_EINVAL;
    for (int32_t i = 0; i < n; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            const int64_t e = i * ld + j;
            if (V) {
                const float v = std::fmaf(mu, V[e], G[e]);
                V[e] = v;
                X[e] = std::fmaf(-lr, v, X[e]);
            } else {
                X[e] = std::fmaf(-lr, G[e], X[e]);
            }
        }
    }
    return ORACLE_OK;
}

// Eq. (2): pack the masked coordinates of every row, ascending j.  On capacity
// overflow nothing is written except *K.
int oracle_mask_compact(int32_t n, int64_t N, int64_t ld, int32_t n_seg, const int64_t* seg_off,
                        const double* seg_c, const float* X, uint64_t seed, uint64_t round,
                        uint32_t* idx, float* msg, int64_t msg_ld, int64_t* K_out) {
    if (!layout_ok(n, N, ld, n_seg, seg_off, seg_c) || !X || !idx || !msg || !K_out || msg_ld < 0)
        return ORACLE_EINVAL;
    int64_t K = 0;
    for (int s = 0; s < n_seg; ++s) {
        const uint64_t T = threshold(seg_c[s]);
        for (int64_t j = seg_off[s]; j < seg_off[s + 1]; ++j)
            if (static_cast<uint64_t>(coord_bits(seed, round, j)) < T) ++K;
    }
    *K_out = K;
    if (K > msg_ld) return ORACLE_ECAPACITY;
    int64_t k = 0;
    for (int s = 0; s < n_seg; ++s) {
        const uint64_t T = threshold(seg_c[s]);
        for (int64_t j = seg_off[s]; j < seg_off[s + 1]; ++j)
            if (static_cast<uint64_t>(coord_bits(seed, round, j)) < T) idx[k++] = static_cast<uint32_t>(j);
    }
    for (int32_t i = 0; i < n; ++i)
        for (int64_t kk = 0; kk < K; ++kk) msg[i * msg_ld + kk] = X[i * ld + idx[kk]];
    return ORACLE_OK;
}

// Alg. 2 line 10 (averaging reading), GenerateW weights 1/2: masked coordinates of a
// matched row become the mean of the two packed messages.
int oracle_merge(int32_t n, int64_t N, int64_t ld, float* X, const int32_t* peer, const uint32_t* idx,
                 const float* msg, int64_t msg_ld, int64_t K) {
    if (n < 1 || N < 0 || ld < N || !X || !peer || !idx || !msg || K < 0 || K > msg_ld) return ORACLE_EINVAL;
    if (!matching_ok(n, peer)) return ORACLE_EMATCH;
    for (int32_t i = 0; i < n; ++i) {
        const int32_t p = peer[i];
        if (p == i) continue;
        for (int64_t k = 0; k < K; ++k) {
            const float s = msg[i * msg_ld + k] + msg[p * msg_ld + k];
            X[i * ld + idx[k]] = s * 0.5f;
        }
    }
    return ORACLE_OK;
}

// One round in Alg. 2 order.  G == null: exchange only.
int oracle_round(int32_t n, int64_t N, int64_t ld, int32_t n_seg, const int64_t* seg_off, const double* seg_c,
                 float* X, const float* G, float* V, float lr, float mu, uint64_t seed, uint64_t round,
                 const int32_t* peer, uint32_t* idx, float* msg, int64_t msg_ld, int64_t* K_out) {
    if (!layout_ok(n, N, ld, n_seg, seg_off, seg_c) || !X || !peer || !idx || !msg || !K_out) return ORACLE_EINVAL;
    if (!matching_ok(n, peer)) return ORACLE_EMATCH;
    // Count first so that a capacity error leaves every buffer untouched.
    int64_t K = 0;
    for (int s = 0; s < n_seg; ++s) {
        const uint64_t T = threshold(seg_c[s]);
        for (int64_t j = seg_off[s]; j < seg_off[s + 1]; ++j)
            if (static_cast<uint64_t>(coord_bits(seed, round, j)) < T) ++K;
    }
    *K_out = K;
    if (K > msg_ld) return ORACLE_ECAPACITY;
    int rc = ORACLE_OK;
    if (G) {
        rc = oracle_sgd_step(n, N, ld, X, G, V, lr, mu);
        if (rc) return rc;
    }
    rc = oracle_mask_compact(n, N, ld, n_seg, seg_off, seg_c, X, seed, round, idx, msg, msg_ld, K_out);
    if (rc) return rc;
    return oracle_merge(n, N, ld, X, peer, idx, msg, msg_ld, *K_out);
}

// One round in the order of Eq. (7): X_{t+1} = X_t o notM + (X_t o M) W - gamma G(X_t).
// The models of the start of the round are packed and averaged; the local step (with the
// build's momentum form) is applied afterwards to the mixed models.
int oracle_round_mix_then_step(int32_t n, int64_t N, int64_t ld, int32_t n_seg, const int64_t* seg_off, const double* seg_c,
                     float* X, const float* G, float* V, float lr, float mu, uint64_t seed, uint64_t round,
                     const int32_t* peer, uint32_t* idx, float* msg, int64_t msg_ld, int64_t* K_out) {
    if (!layout_ok(n, N, ld, n_seg, seg_off, seg_c) || !X || !peer || !idx || !msg || !K_out) return ORACLE_EINVAL;
    if (!matching_ok(n, peer)) return ORACLE_EMATCH;
    if (G && !V && mu != 0.0f) return ORACLE_EINVAL;
    int rc = oracle_mask_compact(n, N, ld, n_seg, seg_off, seg_c, X, seed, round, idx, msg, msg_ld, K_out);
    if (rc) return rc;                                  // capacity overflow: nothing was written
    rc = oracle_merge(n, N, ld, X, peer, idx, msg, msg_ld, *K_out);
    if (rc) return rc;
    if (G) rc = oracle_sgd_step(n, N, ld, X, G, V, lr, mu);
    return rc;
}

// Sec. II-C / Theorem 1: average model (rounded to fp32) and total disagreement, two passes in fp64.
int oracle_consensus(int32_t n, int64_t N, int64_t ld, const float* X, float* mean_out, double* D_out) {
    if (n < 1 || N < 0 || ld < N || !X || !D_out) return ORACLE_EINVAL;
    std::vector<double> mean(static_cast<size_t>(N), 0.0);
    for (int32_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < N; ++j) mean[j] += static_cast<double>(X[i * ld + j]);
    for (int64_t j = 0; j < N; ++j) {
        mean[j] /= static_cast<double>(n);
        if (mean_out) mean_out[j] = static_cast<float>(mean[j]);
    }
    double D = 0.0;
    for (int32_t i = 0; i < n; ++i) {
        double row = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            const double d = static_cast<double>(X[i * ld + j]) - mean[j];
            row += d * d;
        }
        D += row;
    }
    *D_out = D;
    return ORACLE_OK;
}

}  // extern "C"
