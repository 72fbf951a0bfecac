// Device kernels of the SAPS-PSGD round for gfx950 (wave64).  Included by saps_api.hip only.
//
// Work decomposition shared by all mask-driven kernels: the coordinate axis is cut into
// tiles of TILE = 1024 coordinates; a workgroup of 256 lanes owns one tile and lane l owns
// the four coordinates 4*(256*tile + l) .. +3, which are exactly one Philox4x32-10 block,
// one 16-byte access per row, and one nibble of mask bits.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace saps {

constexpr int BLOCK = 256;          // lanes per workgroup (4 waves)
constexpr int TILE = BLOCK * 4;     // coordinates per tile
constexpr int WAVES = BLOCK / 64;

typedef float f4 __attribute__((ext_vector_type(4)));

// Everything needed to evaluate Eq. (3) for any coordinate.
struct MaskParams {
    uint32_t key0, key1;      // seed, low and high word
    uint32_t rnd0, rnd1;      // round, low and high word
    uint32_t N;               // coordinates per model
    int32_t n_seg;            // segments after merging equal thresholds; 1 = one threshold
    uint64_t T0;              // floor(2^32 / c) of the only segment when n_seg == 1
    const uint32_t* seg_end;  // device: exclusive end of each segment, seg_end[n_seg-1] == N
    const uint64_t* seg_T;    // device: threshold of each segment
};

// Philox4x32-10 (Salmon et al., SC'11): ten rounds, each two 32x32->64 products, a word
// permutation with key injection, and a Weyl step of the key.
__device__ __forceinline__ void philox4x32_10(uint32_t& c0, uint32_t& c1, uint32_t& c2, uint32_t& c3,
                                              uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
}

// First segment that intersects [start, ...): wave-uniform binary search (start is uniform).
__device__ __forceinline__ int first_segment(const MaskParams& P, uint32_t start) {
    int lo = 0, hi = P.n_seg - 1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (P.seg_end[mid] > start) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// Mask nibble of Philox block q (coordinates 4q..4q+3): bit r set iff coordinate 4q+r < N is kept.
// seg0 = first_segment(tile start), only read when there are several thresholds.
__device__ __forceinline__ uint32_t mask4(const MaskParams& P, uint32_t q, int seg0) {
    const uint32_t j0 = q << 2;
    if (j0 >= P.N) return 0u;
    uint32_t u0 = q, u1 = 0u, u2 = P.rnd0, u3 = P.rnd1;
    philox4x32_10(u0, u1, u2, u3, P.key0, P.key1);
    uint32_t m;
    if (P.n_seg == 1) {
        const uint64_t T = P.T0;
        m = (uint32_t)((uint64_t)u0 < T) | ((uint32_t)((uint64_t)u1 < T) << 1) |
            ((uint32_t)((uint64_t)u2 < T) << 2) | ((uint32_t)((uint64_t)u3 < T) << 3);
    } else {
        const uint32_t u[4] = {u0, u1, u2, u3};
        int s = seg0;
        const int last = P.n_seg - 1;
        m = 0u;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t j = j0 + r;
            while (s < last && j >= P.seg_end[s]) ++s;
            m |= (uint32_t)((uint64_t)u[r] < P.seg_T[s]) << r;
        }
    }
    const uint32_t left = P.N - j0;              // >= 1
    if (left < 4u) m &= (1u << left) - 1u;
    return m;
}

// Exclusive prefix (in ascending coordinate order) of the kept coordinates in front of this
// lane's nibble inside the workgroup, and the workgroup total.  One call per kernel: wave
// ballots give the in-wave part, one LDS word per wave the rest.
__device__ __forceinline__ uint32_t block_prefix(uint32_t m, uint32_t* wave_tot /* LDS[WAVES] */, uint32_t& total) {
    uint32_t excl = 0u, wsum = 0u;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint64_t b = __ballot((m >> r) & 1u);
        excl += __builtin_amdgcn_mbcnt_hi((uint32_t)(b >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b, 0u));
        wsum += (uint32_t)__popcll(b);
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) wave_tot[wave] = wsum;
    __syncthreads();
    uint32_t before = 0u, all = 0u;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
        const uint32_t t = wave_tot[w];
        before += (w < wave) ? t : 0u;
        all += t;
    }
    total = all;
    return excl + before;
}

// ------------------------------------------------------------------ K1: per-tile counts
__global__ __launch_bounds__(BLOCK) void mask_count_kernel(MaskParams P, uint32_t* __restrict__ tile_cnt) {
    __shared__ uint32_t wave_tot[WAVES];
    const uint32_t tile = blockIdx.x;
    const int seg0 = (P.n_seg > 1) ? first_segment(P, tile * (uint32_t)TILE) : 0;
    const uint32_t m = mask4(P, tile * BLOCK + threadIdx.x, seg0);
    uint32_t total;
    (void)block_prefix(m, wave_tot, total);
    if (threadIdx.x == 0) tile_cnt[tile] = total;
}

// ------------------------------------------- K2: counts -> exclusive tile bases, K, flag
// One workgroup of 1024 lanes; lane t scans the contiguous chunk [t*L, (t+1)*L).
__global__ __launch_bounds__(1024) void tile_scan_kernel(uint32_t* __restrict__ tile_cnt, uint32_t ntiles,
                                                         int64_t cap, int64_t* __restrict__ K_int,
                                                         int64_t* __restrict__ K_user, int32_t* __restrict__ flag) {
    __shared__ uint32_t wsum[16];
    const uint32_t t = threadIdx.x;
    const uint32_t L = (ntiles + 1023u) / 1024u;
    const uint32_t lo = min(t * L, ntiles), hi = min(lo + L, ntiles);
    uint32_t s = 0u;
    for (uint32_t k = lo; k < hi; ++k) s += tile_cnt[k];
    // inclusive scan of s over the 1024 lanes
    uint32_t inc = s;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(inc, d, 64);
        if ((int)(t & 63u) >= d) inc += o;
    }
    if ((t & 63u) == 63u) wsum[t >> 6] = inc;
    __syncthreads();
    uint32_t before = 0u, all = 0u;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const uint32_t v = wsum[w];
        before += (w < (int)(t >> 6)) ? v : 0u;
        all += v;
    }
    uint32_t run = before + inc - s;
    for (uint32_t k = lo; k < hi; ++k) {
        const uint32_t c = tile_cnt[k];
        tile_cnt[k] = run;
        run += c;
    }
    if (t == 0) {
        tile_cnt[ntiles] = all;
        *K_int = (int64_t)all;
        if (K_user) *K_user = (int64_t)all;
        if ((int64_t)all > cap) *flag = 1;
    }
}

// --------------------------------------------------------- K3: ascending index list idx
__global__ __launch_bounds__(BLOCK) void idx_scatter_kernel(MaskParams P, const uint32_t* __restrict__ tile_base,
                                                            const int64_t* __restrict__ K_int, int64_t cap,
                                                            uint32_t* __restrict__ idx) {
    __shared__ uint32_t wave_tot[WAVES];
    if (*K_int > cap) return;
    const uint32_t tile = blockIdx.x;
    const int seg0 = (P.n_seg > 1) ? first_segment(P, tile * (uint32_t)TILE) : 0;
    const uint32_t q = tile * BLOCK + threadIdx.x;
    const uint32_t m = mask4(P, q, seg0);
    uint32_t total;
    uint32_t pos = tile_base[tile] + block_prefix(m, wave_tot, total);
    if (m) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if ((m >> r) & 1u) idx[pos++] = (q << 2) + r;
    }
}

// ----------------------------------------------------------------- memory access helpers
template <bool NT> __device__ __forceinline__ f4 ld4(const float* p) {
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
    return *reinterpret_cast<const f4*>(p);
}
template <bool NT> __device__ __forceinline__ void st4(float* p, f4 v) {
    if (NT) __builtin_nontemporal_store(v, reinterpret_cast<f4*>(p));
    else *reinterpret_cast<f4*>(p) = v;
}

// Local step on one value (Alg. 2 line 5 with momentum): two correctly rounded FMAs.
template <bool HAS_V> __device__ __forceinline__ void step1(float& x, float g, float& v, float lr, float mu) {
    if (HAS_V) {
        v = __fmaf_rn(mu, v, g);
        x = __fmaf_rn(-lr, v, x);
    } else {
        x = __fmaf_rn(-lr, g, x);
    }
}

// --------------------------------------------------------------------- K4: local update
template <bool HAS_V, bool NT>
__global__ __launch_bounds__(BLOCK) void sgd_kernel(float* __restrict__ X, const float* __restrict__ G,
                                                    float* __restrict__ V, int64_t ld, uint32_t N, float lr, float mu) {
    const uint32_t q = blockIdx.x * BLOCK + threadIdx.x;
    const uint32_t j0 = q << 2;
    if (j0 >= N) return;
    const int64_t e = (int64_t)blockIdx.y * ld + j0;
    if (N - j0 >= 4u) {
        f4 x = ld4<NT>(X + e), g = ld4<NT>(G + e), v = {0.f, 0.f, 0.f, 0.f};
        if (HAS_V) v = ld4<NT>(V + e);
#pragma unroll
        for (int r = 0; r < 4; ++r) { float xr = x[r], vr = v[r]; step1<HAS_V>(xr, g[r], vr, lr, mu); x[r] = xr; v[r] = vr; }
        st4<NT>(X + e, x);
        if (HAS_V) st4<NT>(V + e, v);
    } else {
        for (uint32_t r = 0; r < N - j0; ++r) {
            float x = X[e + r], v = HAS_V ? V[e + r] : 0.f;
            step1<HAS_V>(x, G[e + r], v, lr, mu);
            X[e + r] = x;
            if (HAS_V) V[e + r] = v;
        }
    }
}

// ------------------------------------------------- K5: packed message rows from the list
__global__ __launch_bounds__(BLOCK) void compact_values_kernel(const float* __restrict__ X, int64_t ld,
                                                               const uint32_t* __restrict__ idx,
                                                               const int64_t* __restrict__ K_int, int64_t cap,
                                                               float* __restrict__ msg, int64_t msg_ld) {
    const int64_t K = *K_int;
    if (K > cap) return;
    const float* x = X + (int64_t)blockIdx.y * ld;
    float* m = msg + (int64_t)blockIdx.y * msg_ld;
    for (int64_t k = (int64_t)blockIdx.x * BLOCK + threadIdx.x; k < K; k += (int64_t)gridDim.x * BLOCK)
        m[k] = x[idx[k]];
}

// -------------------------------------------------- K6: average the two packed messages
__global__ __launch_bounds__(BLOCK) void merge_kernel(float* __restrict__ X, int64_t ld, const int32_t* __restrict__ peer,
                                                      const uint32_t* __restrict__ idx, const float* __restrict__ msg,
                                                      int64_t msg_ld, const int64_t* __restrict__ K_dev, int64_t cap) {
    const int64_t K = *K_dev;
    if (K > cap || K < 0) return;
    const int32_t i = blockIdx.y, p = peer[i];
    if (p == i) return;
    float* x = X + (int64_t)i * ld;
    const float* a = msg + (int64_t)i * msg_ld;
    const float* b = msg + (int64_t)p * msg_ld;
    for (int64_t k = (int64_t)blockIdx.x * BLOCK + threadIdx.x; k < K; k += (int64_t)gridDim.x * BLOCK)
        x[idx[k]] = (a[k] + b[k]) * 0.5f;
}

// -------------------------- K8: exchange-only round through the index list (sparse masks)
// unit u = (i, p): a matched pair with i < p, or an unmatched worker with i == p.
__global__ __launch_bounds__(BLOCK) void exchange_list_kernel(float* __restrict__ X, int64_t ld,
                                                              const int32_t* __restrict__ units,
                                                              const uint32_t* __restrict__ idx,
                                                              const int64_t* __restrict__ K_int, int64_t cap,
                                                              float* __restrict__ msg, int64_t msg_ld) {
    const int64_t K = *K_int;
    if (K > cap) return;
    const int32_t i = units[2 * blockIdx.y], p = units[2 * blockIdx.y + 1];
    float* xi = X + (int64_t)i * ld;
    float* xp = X + (int64_t)p * ld;
    for (int64_t k = (int64_t)blockIdx.x * BLOCK + threadIdx.x; k < K; k += (int64_t)gridDim.x * BLOCK) {
        const uint32_t j = idx[k];
        const float a = xi[j];
        if (msg) msg[(int64_t)i * msg_ld + k] = a;
        if (p != i) {
            const float b = xp[j];
            if (msg) msg[(int64_t)p * msg_ld + k] = b;
            const float avg = (a + b) * 0.5f;
            xi[j] = avg;
            xp[j] = avg;
        }
    }
}

// ------------------------------------------------------------------ K7: fused dense round
// MODE 0: update with momentum buffer, 1: update without buffer, 2: no update (exchange only).
// Grid: x = tiles (optionally remapped so that each XCD walks one contiguous range),
//       y = chunks of PPB units.  The mask nibble and the packed position of a lane's four
//       coordinates are computed once and reused for all PPB units of the chunk.
struct FusedArgs {
    float* X; const float* G; float* V;
    int64_t ld;
    const int32_t* units; int32_t n_units;
    float lr, mu;
    const uint32_t* tile_base; const int64_t* K_int; int64_t cap;
    uint32_t* idx; float* msg; int64_t msg_ld;
    uint32_t ntiles; int32_t xcd_remap;
};

template <int MODE, int PPB, bool NT>
__global__ __launch_bounds__(BLOCK) void fused_round_kernel(MaskParams P, FusedArgs A) {
    __shared__ uint32_t wave_tot[WAVES];
    if (*A.K_int > A.cap) return;
    uint32_t tile = blockIdx.x;
    if (A.xcd_remap) {
        // workgroups are dealt round-robin to the 8 XCDs; give XCD x the tiles [x*per, (x+1)*per)
        const uint32_t per = (A.ntiles + 7u) >> 3;
        tile = (blockIdx.x & 7u) * per + (blockIdx.x >> 3);
        if (tile >= A.ntiles) return;
    }
    const int seg0 = (P.n_seg > 1) ? first_segment(P, tile * (uint32_t)TILE) : 0;
    const uint32_t q = tile * BLOCK + threadIdx.x;
    const uint32_t j0 = q << 2;
    const uint32_t m = mask4(P, q, seg0);
    uint32_t total;
    const uint32_t pos0 = A.tile_base[tile] + block_prefix(m, wave_tot, total);
    if (MODE == 2 && total == 0u) return;                    // nothing of this tile is exchanged
    if (blockIdx.y == 0 && A.idx && m) {
        uint32_t pos = pos0;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if ((m >> r) & 1u) A.idx[pos++] = j0 + r;
    }
    if (j0 >= P.N) return;
    const bool full = (P.N - j0) >= 4u;
    const uint32_t nval = full ? 4u : (P.N - j0);
    const int u_lo = blockIdx.y * PPB;
    const int u_hi = min(u_lo + PPB, A.n_units);
    if (MODE == 2 && m == 0u) return;                        // this lane exchanges nothing

#pragma unroll 1
    for (int u = u_lo; u < u_hi; ++u) {
        const int32_t i = A.units[2 * u], p = A.units[2 * u + 1];
        const bool paired = (p != i);
        const int64_t ei = (int64_t)i * A.ld + j0, ep = (int64_t)p * A.ld + j0;
        f4 xi = {0.f, 0.f, 0.f, 0.f}, gi = xi, vi = xi, xp = xi, gp = xi, vp = xi;
        if (full) {
            xi = ld4<NT>(A.X + ei);
            if (MODE != 2) gi = ld4<NT>(A.G + ei);
            if (MODE == 0) vi = ld4<NT>(A.V + ei);
            if (paired) {
                xp = ld4<NT>(A.X + ep);
                if (MODE != 2) gp = ld4<NT>(A.G + ep);
                if (MODE == 0) vp = ld4<NT>(A.V + ep);
            }
        } else {
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                if ((uint32_t)r < nval) {
                    xi[r] = A.X[ei + r];
                    if (MODE != 2) gi[r] = A.G[ei + r];
                    if (MODE == 0) vi[r] = A.V[ei + r];
                    if (paired) {
                        xp[r] = A.X[ep + r];
                        if (MODE != 2) gp[r] = A.G[ep + r];
                        if (MODE == 0) vp[r] = A.V[ep + r];
                    }
                }
            }
        }
        if (MODE != 2) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float x = xi[r], v = vi[r];
                step1<MODE == 0>(x, gi[r], v, A.lr, A.mu);
                xi[r] = x; vi[r] = v;
                x = xp[r]; v = vp[r];
                step1<MODE == 0>(x, gp[r], v, A.lr, A.mu);
                xp[r] = x; vp[r] = v;
            }
        }
        if (m) {
            uint32_t pos = pos0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if ((m >> r) & 1u) {
                    if (A.msg) {
                        A.msg[(int64_t)i * A.msg_ld + pos] = xi[r];
                        if (paired) A.msg[(int64_t)p * A.msg_ld + pos] = xp[r];
                    }
                    ++pos;
                    if (paired) {
                        const float avg = (xi[r] + xp[r]) * 0.5f;
                        xi[r] = avg; xp[r] = avg;
                    }
                }
            }
        }
        if (full) {
            if (MODE != 2 || paired) st4<NT>(A.X + ei, xi);
            if (MODE == 0) st4<NT>(A.V + ei, vi);
            if (paired) {
                st4<NT>(A.X + ep, xp);
                if (MODE == 0) st4<NT>(A.V + ep, vp);
            }
        } else {
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                if ((uint32_t)r < nval) {
                    if (MODE != 2 || paired) A.X[ei + r] = xi[r];
                    if (MODE == 0) A.V[ei + r] = vi[r];
                    if (paired) {
                        A.X[ep + r] = xp[r];
                        if (MODE == 0) A.V[ep + r] = vp[r];
                    }
                }
            }
        }
    }
}

// --------------------------------------------------------- bandwidth yardstick (a copy)
template <bool NT>
__global__ __launch_bounds__(BLOCK) void stream_copy_kernel(float* __restrict__ dst, const float* __restrict__ src,
                                                            int64_t count4) {
    const int64_t q = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (q < count4) st4<NT>(dst + 4 * q, ld4<NT>(src + 4 * q));
}

}  // namespace saps
