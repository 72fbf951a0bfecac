// Stand-alone user of the C ABI (no Python, no torch): device memory from hipMalloc, one fused round,
// checks that need no oracle:  c = 1 with a perfect matching makes paired rows bit-identical, the packed
// message of a row is that row after its local step, K equals N, padding columns are untouched, and a
// round with too small a capacity changes nothing.  Exit code 0 = all checks passed.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/saps.h"
#include "../../include/saps_select.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); return 2; } } while (0)
#define REQUIRE(cond) do { if (!(cond)) { std::printf("FAILED: %s (line %d)\n", #cond, __LINE__); return 1; } } while (0)

int main() {
    const int32_t n = 6;
    const int64_t N = 70001, ld = 70016, cap = 70004;
    std::vector<float> X((size_t)n * ld, 9.5f), G((size_t)n * ld, 0.25f), V((size_t)n * ld, 0.0f);
    for (int i = 0; i < n; ++i)
        for (int64_t j = 0; j < N; ++j) {
            X[(size_t)i * ld + j] = std::sin(0.001f * (float)j + (float)i);
            G[(size_t)i * ld + j] = 0.01f * std::cos(0.002f * (float)j - (float)i);
        }
    float *dX, *dG, *dV, *dmsg; uint32_t* didx; int64_t* dK;
    CHECK_HIP(hipMalloc(&dX, X.size() * 4)); CHECK_HIP(hipMalloc(&dG, X.size() * 4)); CHECK_HIP(hipMalloc(&dV, X.size() * 4));
    CHECK_HIP(hipMalloc(&dmsg, (size_t)n * cap * 4)); CHECK_HIP(hipMalloc(&didx, cap * 4)); CHECK_HIP(hipMalloc(&dK, 8));
    CHECK_HIP(hipMemcpy(dX, X.data(), X.size() * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dG, G.data(), X.size() * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dV, V.data(), X.size() * 4, hipMemcpyHostToDevice));

    // a perfect matching from the library's own peer selection (complete bandwidth graph)
    std::vector<double> B((size_t)n * n, 10.0);
    saps_selector* sel = nullptr;
    REQUIRE(saps_selector_create(&sel, n, B.data(), 5.0, 4, 1) == 0);
    std::vector<int32_t> peer(n);
    saps_select_info info;
    REQUIRE(saps_selector_next(sel, 1, peer.data(), &info) == 0);
    for (int i = 0; i < n; ++i) REQUIRE(peer[i] != i && peer[peer[i]] == i);
    saps_selector_destroy(sel);

    const int64_t seg_off[2] = {0, N};
    const double seg_c[1] = {1.0};
    saps_layout L{n, N, ld, 1, seg_off, seg_c};
    saps_ctx* ctx = nullptr;
    hipStream_t stream; CHECK_HIP(hipStreamCreate(&stream));
    REQUIRE(saps_create(&ctx, &L, cap, stream) == SAPS_OK);
    REQUIRE(saps_round(ctx, dX, dG, dV, 0.1f, 0.9f, 7, 1, peer.data(), didx, dmsg, dK) == SAPS_OK);
    int64_t K = -1;
    REQUIRE(saps_poll_status(ctx, &K) == SAPS_OK);
    REQUIRE(K == N);
    std::vector<float> X1(X.size()), V1(X.size()), msg((size_t)n * cap);
    std::vector<uint32_t> idx(cap);
    CHECK_HIP(hipMemcpy(X1.data(), dX, X.size() * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(V1.data(), dV, X.size() * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(msg.data(), dmsg, msg.size() * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(idx.data(), didx, idx.size() * 4, hipMemcpyDeviceToHost));
    for (int i = 0; i < n; ++i) {
        const int p = peer[i];
        REQUIRE(std::memcmp(&X1[(size_t)i * ld], &X1[(size_t)p * ld], N * 4) == 0);          // pairs identical
        for (int64_t j = N; j < ld; ++j) REQUIRE(X1[(size_t)i * ld + j] == 9.5f && V1[(size_t)i * ld + j] == 0.0f);
        for (int64_t j = 0; j < N; j += 997) {
            const float v = std::fmaf(0.9f, 0.0f, G[(size_t)i * ld + j]);
            const float x = std::fmaf(-0.1f, v, X[(size_t)i * ld + j]);
            REQUIRE(V1[(size_t)i * ld + j] == v);
            REQUIRE(msg[(size_t)i * cap + j] == x);                                            // message = stepped model
            const float xp = std::fmaf(-0.1f, G[(size_t)p * ld + j], X[(size_t)p * ld + j]);
            REQUIRE(X1[(size_t)i * ld + j] == (x + xp) * 0.5f);
        }
    }
    for (int64_t j = 0; j < N; ++j) REQUIRE(idx[j] == (uint32_t)j);
    saps_destroy(ctx);

    // capacity overflow: the round is skipped on the device and reported by the poll
    REQUIRE(saps_create(&ctx, &L, 64, stream) == SAPS_OK);
    REQUIRE(saps_round(ctx, dX, dG, dV, 0.1f, 0.9f, 7, 2, peer.data(), didx, dmsg, dK) == SAPS_OK);
    REQUIRE(saps_poll_status(ctx, &K) == SAPS_ECAPACITY && K == N);
    std::vector<float> X2(X.size());
    CHECK_HIP(hipMemcpy(X2.data(), dX, X.size() * 4, hipMemcpyDeviceToHost));
    REQUIRE(std::memcmp(X1.data(), X2.data(), X.size() * 4) == 0);
    // host-side argument errors
    std::vector<int32_t> bad(peer); bad[0] = bad[1];
    REQUIRE(saps_round(ctx, dX, dG, dV, 0.1f, 0.9f, 7, 3, bad.data(), nullptr, nullptr, nullptr) == SAPS_EMATCH);
    REQUIRE(saps_round(ctx, dX + 1, dG, dV, 0.1f, 0.9f, 7, 3, peer.data(), nullptr, nullptr, nullptr) == SAPS_EINVAL);
    saps_destroy(ctx);
    (void)hipFree(dX); (void)hipFree(dG); (void)hipFree(dV); (void)hipFree(dmsg); (void)hipFree(didx); (void)hipFree(dK);
    std::printf("abi_smoke ok: n=%d N=%lld\n", n, (long long)N);
    return 0;
}
