// Device kernels of the SAPS-PSGD round for gfx950 (wave64).  Included by saps_api.hip only.
//
// Work decomposition shared by all mask-driven kernels: the coordinate axis is cut into
// tiles of TILE = 256 coordinates; one wave owns one tile and lane l owns the four
// coordinates 4*(64*tile + l) .. +3, which are exactly one Philox4x32-10 block, one 16-byte
// access per row, and one nibble of mask bits.  Packed positions inside a tile come from
// wave ballots alone; LDS and a barrier appear only where waves have to meet (the group sum of the
// counting kernel, the swap of a tile between the two rows of a pair).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace saps {

constexpr int BLOCK = 256;          // lanes per workgroup (4 waves)
constexpr int WAVES = BLOCK / 64;
constexpr int TILE = 64 * 4;        // coordinates per tile: one wave, one Philox block per lane
constexpr int GROUP = 16;           // tiles per group: the counting kernel's workgroup of 16 waves
constexpr int STREAM_BLOCK = 64;    // lanes per workgroup of the plain streaming kernels (local step, copy): one wave
constexpr int MAX_INLINE_UNITS = 128;
constexpr int FUSED_BLOCK = 128;    // lanes per workgroup of the fused round kernels (2 waves)
constexpr int FUSED_WAVES = FUSED_BLOCK / 64;
// Independent waves per workgroup of fused_round_kernel: the plain-SGD round (MODE 1, six streams per wave) runs 4 % faster
// with one-wave workgroups (32 x 6.65 M: 0.394 against 0.411 ms); with the momentum buffer the two shapes measure alike.
constexpr int fused_round_waves(int mode) { return mode == 1 ? 1 : FUSED_WAVES; }
#ifndef SAPS_CONS_ROWS
#define SAPS_CONS_ROWS 8
#endif
constexpr int CONS_ROWS = SAPS_CONS_ROWS;   // rows a lane of the consensus kernel keeps in flight

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
    const uint32_t* grp_seg;  // device: first segment that intersects each group of 16 tiles
};

// Philox4x32-10 (Salmon et al., SC'11): ten rounds, each two 32x32->64 products, a word
// permutation with key injection, and a Weyl step of the key.  The products are written as
// 64-bit multiplies of zero-extended words so that each becomes one v_mad_u64_u32.
__device__ __forceinline__ void philox4x32_10(uint32_t& c0, uint32_t& c1, uint32_t& c2, uint32_t& c3,
                                              uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
}

// First segment that intersects tile `tile` (wave-uniform): start from the group's entry of the
// host-built table and step over the segments that end before the tile begins.
__device__ __forceinline__ int first_segment(const MaskParams& P, uint32_t tile) {
    int s = (int)P.grp_seg[tile / GROUP];
    const uint32_t start = tile * (uint32_t)TILE;
    const int last = P.n_seg - 1;
    while (s < last && P.seg_end[s] <= start) ++s;
    return s;
}

// Mask nibble of lane `lane` of tile `tile` (coordinates 4q..4q+3, q = 64*tile + lane): bit r set
// iff coordinate 4q+r < N is kept.  seg0 = first_segment(tile), only read when there are
// several thresholds.
__device__ __forceinline__ uint32_t mask4(const MaskParams& P, uint32_t tile, uint32_t lane, int seg0) {
    const uint32_t q = tile * 64u + lane;
    const uint32_t j0 = q << 2;
    if (j0 >= P.N) return 0u;
    uint32_t u0 = q, u1 = 0u, u2 = P.rnd0, u3 = P.rnd1;
    philox4x32_10(u0, u1, u2, u3, P.key0, P.key1);
    uint32_t m;
    const int last = P.n_seg - 1;
    if (P.n_seg == 1 || seg0 == last || P.seg_end[seg0] - tile * (uint32_t)TILE >= (uint32_t)TILE) {
        // one threshold for the whole tile (always, when the model has a single ratio)
        const uint64_t T = (P.n_seg == 1) ? P.T0 : P.seg_T[seg0];
        m = (uint32_t)((uint64_t)u0 < T) | ((uint32_t)((uint64_t)u1 < T) << 1) |
            ((uint32_t)((uint64_t)u2 < T) << 2) | ((uint32_t)((uint64_t)u3 < T) << 3);
    } else {
        // a segment boundary falls inside the tile: look the threshold up per coordinate
        const uint32_t u[4] = {u0, u1, u2, u3};
        int s = seg0;
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
// lane's nibble inside its wave tile, and the tile total, from four ballots.
__device__ __forceinline__ uint32_t wave_prefix(uint32_t m, uint32_t& total) {
    uint32_t excl = 0u, wsum = 0u;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint64_t b = __ballot((m >> r) & 1u);
        excl += __builtin_amdgcn_mbcnt_hi((uint32_t)(b >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b, 0u));
        wsum += (uint32_t)__popcll(b);
    }
    total = wsum;
    return excl;
}

// The matching as a list of units (i, p): a matched pair with i < p, or an unmatched worker
// with i == p.  Small lists travel inside the kernel arguments (no upload, no extra launch);
// longer ones are read from device memory.
struct Units {
    const int32_t* dev;                    // 2 ints per unit, or null when the list is inline
    uint32_t packed[MAX_INLINE_UNITS];     // i | p << 16
};

__device__ __forceinline__ void unit_at(const Units& U, int u, int32_t& i, int32_t& p) {
    if (U.dev) {
        i = U.dev[2 * u]; p = U.dev[2 * u + 1];
    } else {
        const uint32_t w = U.packed[u];
        i = (int32_t)(w & 0xFFFFu); p = (int32_t)(w >> 16);
    }
}

// One word per tile: its kept count (at most 256) in the low half and, in the high half, the kept count of
// the tiles in front of it inside its group of 16 (at most 3840), so that a wave finds the packed position
// of its tile with one uniform load per level (tile word, group base) and no exchange between lanes.
__device__ __forceinline__ uint32_t tile_word(uint32_t count, uint32_t before_in_group) { return count | (before_in_group << 16); }
__device__ __forceinline__ uint32_t tile_count(uint32_t word) { return word & 0xFFFFu; }
__device__ __forceinline__ uint32_t tile_before(uint32_t word) { return word >> 16; }

// ------------------------------------------------ K1: per-tile and per-group kept counts
// One workgroup of 16 waves per group of 16 tiles.
__global__ __launch_bounds__(64 * GROUP) void mask_count_kernel(MaskParams P, uint32_t ntiles,
                                                                uint32_t* __restrict__ tile_cnt,
                                                                uint32_t* __restrict__ grp_cnt) {
    __shared__ uint32_t wsum[GROUP];
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t tile = blockIdx.x * GROUP + wave;
    uint32_t total = 0u;
    if (tile < ntiles) {
        const int seg0 = (P.n_seg > 1) ? first_segment(P, tile) : 0;
        const uint32_t m = mask4(P, tile, threadIdx.x & 63u, seg0);
        (void)wave_prefix(m, total);
    }
    if ((threadIdx.x & 63u) == 0u) wsum[wave] = total;
    __syncthreads();
    if (threadIdx.x < (uint32_t)GROUP) {
        // the first 16 lanes write the group's 16 tile words with one store and the group count
        const uint32_t cnt = wsum[threadIdx.x];
        uint32_t inc = cnt;
#pragma unroll
        for (int d = 1; d < GROUP; d <<= 1) {
            const uint32_t o = __shfl_up(inc, d, 64);
            if ((int)threadIdx.x >= d) inc += o;
        }
        const uint32_t t = blockIdx.x * GROUP + threadIdx.x;
        if (t < ntiles) tile_cnt[t] = tile_word(cnt, inc - cnt);
        if (threadIdx.x == (uint32_t)GROUP - 1u) grp_cnt[blockIdx.x] = inc;
    }
}

// ------------------------------------ K2: group counts -> exclusive group bases, K, flag
// One workgroup of 1024 lanes walks the group counts 4096 at a time with a running carry.
__global__ __launch_bounds__(1024) void group_scan_kernel(uint32_t* __restrict__ grp, uint32_t ngroups,
                                                          int64_t cap, int64_t* __restrict__ K_int,
                                                          int64_t* __restrict__ K_user, int32_t* __restrict__ flag) {
    __shared__ uint32_t wsum[16];
    const uint32_t t = threadIdx.x;
    uint32_t carry = 0u;
    for (uint32_t base = 0u; base < ngroups; base += 4096u) {
        const uint32_t k0 = base + 4u * t;
        uint32_t c[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) c[r] = (k0 + r < ngroups) ? grp[k0 + r] : 0u;
        const uint32_t s = c[0] + c[1] + c[2] + c[3];
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
        uint32_t run = carry + before + inc - s;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (k0 + r < ngroups) grp[k0 + r] = run;
            run += c[r];
        }
        carry += all;
        __syncthreads();
    }
    if (t == 0) {
        *K_int = (int64_t)carry;
        if (K_user) *K_user = (int64_t)carry;
        if ((int64_t)carry > cap) *flag = 1;
    }
}

// ----------------------------------------- counts of the NEXT round, computed inside another kernel
// The counts depend on (seed, round) only, so the kernels of round t can compute those of round t + 1 on
// the side: the Philox arithmetic then hides under a kernel that waits for memory, and the next call starts
// without K1.  One wave counts one whole group of 16 tiles by itself (no LDS, no barrier), waves take
// groups round-robin by their index in the grid, and the low indices, which are dispatched first, come first.
struct NextCounts {
    uint32_t* tile_cnt;   // null: nothing to do
    uint32_t* grp_cnt;
    uint32_t rnd0, rnd1;  // the next round (same seed, thresholds and segments as the running one)
    uint32_t ngroups;
};

__device__ __forceinline__ void count_next_round(const MaskParams& Pcur, const NextCounts& Nx, uint32_t ntiles,
                                                 uint32_t wave_index, uint32_t waves_in_grid) {
    if (!Nx.tile_cnt) return;
    MaskParams P = Pcur;
    P.rnd0 = Nx.rnd0; P.rnd1 = Nx.rnd1;
    const uint32_t lane = threadIdx.x & 63u;
    for (uint32_t g = wave_index; g < Nx.ngroups; g += waves_in_grid) {
        const uint32_t t0 = g * GROUP;
        uint32_t mine = 0u;                                   // lane r keeps the count of tile t0 + r
#pragma unroll 1
        for (uint32_t r = 0; r < (uint32_t)GROUP; ++r) {
            const uint32_t tile = t0 + r;
            if (tile >= ntiles) break;                        // wave-uniform
            const int seg0 = (P.n_seg > 1) ? first_segment(P, tile) : 0;
            const uint32_t m = mask4(P, tile, lane, seg0);
            uint32_t total;
            (void)wave_prefix(m, total);
            if (lane == r) mine = total;
        }
        uint32_t inc = mine;                                  // inclusive prefix over the 16 tiles (lanes >= 16 hold zero)
#pragma unroll
        for (int d = 1; d < GROUP; d <<= 1) {
            const uint32_t o = __shfl_up(inc, d, 64);
            if ((int)lane >= d) inc += o;
        }
        if (lane < (uint32_t)GROUP && t0 + lane < ntiles) Nx.tile_cnt[t0 + lane] = tile_word(mine, inc - mine);
        if (lane == (uint32_t)GROUP - 1u) Nx.grp_cnt[g] = inc;
    }
}

// Where the packed positions and K of the round come from.
//   direct == 0: K2 ran; grp holds exclusive group bases and *K_int the total.
//   direct == 1: small models (at most 256 groups): no K2 launch; grp still holds the group
//                counts and every wave adds up the ones in front of its group itself; the first
//                wave of the grid also publishes K and raises the capacity flag.
struct Bases {
    const uint32_t* grp;
    const uint32_t* tile_cnt;
    int64_t* K_int;
    int64_t* K_user;      // caller's copy of K, written in direct mode only (K2 writes it otherwise)
    int32_t* flag;
    int64_t cap;
    uint32_t ngroups;
    int32_t direct;
};
constexpr uint32_t DIRECT_MAX_GROUPS = 256;

// Wave-uniform words that no kernel writes while it reads them (the counts and bases of the running round; the
// kernels that count the next round on the side write the other buffer): read as constant memory, so that they
// travel through the scalar cache and neither queue behind the wave's 16-byte streams nor wait for them (vector
// loads return in order).  A wave then gets to its stores sooner, and fewer resident waves keep the memory busy.
__device__ __forceinline__ uint32_t uniform_u32(const uint32_t* p, uint32_t index) {
    typedef const __attribute__((address_space(4))) uint32_t* cptr;
    return ((cptr)(uintptr_t)p)[__builtin_amdgcn_readfirstlane(index)];
}
__device__ __forceinline__ int64_t uniform_i64(const int64_t* p) {
    typedef const __attribute__((address_space(4))) int64_t* cptr;
    return *(cptr)(uintptr_t)p;
}

// Packed position of the first kept coordinate of group g and the round's K.  Wave-uniform; every
// lane of the wave must call it.
__device__ __forceinline__ uint32_t group_base_and_K(const Bases& Bp, uint32_t g, bool first_wave, int64_t& K) {
    if (Bp.direct) {
        const uint32_t lane = threadIdx.x & 63u;
        uint32_t before = 0u, all = 0u;
#pragma unroll
        for (uint32_t k = 0; k < DIRECT_MAX_GROUPS / 64u; ++k) {
            const uint32_t gi = lane + 64u * k;
            const uint32_t c = (gi < Bp.ngroups) ? Bp.grp[gi] : 0u;
            all += c;
            before += (gi < g) ? c : 0u;
        }
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { before += __shfl_xor(before, d, 64); all += __shfl_xor(all, d, 64); }
        K = (int64_t)all;
        if (first_wave && lane == 0u) {
            *Bp.K_int = K;
            if (Bp.K_user) *Bp.K_user = K;
            if (K > Bp.cap) *Bp.flag = 1;
        }
        return __builtin_amdgcn_readfirstlane(before);
    }
    K = uniform_i64(Bp.K_int);
    return uniform_u32(Bp.grp, g);
}

// Packed position of the first kept coordinate of a tile (its group's base plus the count of the
// tiles in front of it inside the group, which its tile word carries) and the round's K.
// Wave-uniform; every lane of the wave must call it.
__device__ __forceinline__ uint32_t tile_base_and_K(const Bases& Bp, uint32_t tile, bool first_wave, int64_t& K) {
    const uint32_t word = uniform_u32(Bp.tile_cnt, tile);
    const uint32_t gbase = group_base_and_K(Bp, tile / GROUP, first_wave, K);
    return gbase + tile_before(word);
}

// --------------------------------------------------------- K3: ascending index list idx
// A wave owns TPW consecutive tiles of one group of 16.  The group's tile counts arrive with one load
// (together with the group base and K), then only the tiles that keep something are visited.  TPW = 1
// gives every tile its own wave (dense masks: the Philox blocks are the work); TPW = 16 lets one wave
// step over a whole group when most tiles keep nothing (at c = 1000 three quarters of them), so that the
// memory latency is paid once per group and not once per tile.
template <int TPW>
__global__ __launch_bounds__(BLOCK) void idx_scatter_kernel(MaskParams P, uint32_t ntiles, Bases Bp,
                                                            uint32_t* __restrict__ idx) {
    static_assert(TPW == 1 || TPW == 2 || TPW == 4 || TPW == 8 || TPW == 16, "TPW divides the group");
    const uint32_t w = blockIdx.x * WAVES + (threadIdx.x >> 6);      // wave-uniform
    const uint32_t tfirst = w * (uint32_t)TPW;                       // first tile of this wave
    if (tfirst >= ntiles) return;
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t g = tfirst / GROUP, t0 = g * GROUP;
    const uint32_t word = (lane < (uint32_t)GROUP && t0 + lane < ntiles) ? Bp.tile_cnt[t0 + lane] : 0u;
    const uint32_t cnt = tile_count(word), excl = tile_before(word);
    int64_t K;
    const uint32_t gbase = group_base_and_K(Bp, g, w == 0u, K);
    if (K > Bp.cap) return;
    const uint32_t r0 = tfirst - t0;
    uint64_t todo = __ballot(cnt != 0u) & ((TPW == 16) ? 0xFFFFull : (((1ull << TPW) - 1ull) << r0));
    while (todo) {
        const int r = __builtin_ctzll(todo);
        todo &= todo - 1;
        const uint32_t tile = t0 + (uint32_t)r;
        const uint32_t tbase = gbase + (uint32_t)__shfl((int)excl, r, 64);
        const int seg0 = (P.n_seg > 1) ? first_segment(P, tile) : 0;
        const uint32_t q = tile * 64u + lane;
        const uint32_t m = mask4(P, tile, lane, seg0);
        uint32_t total;
        uint32_t pos = tbase + wave_prefix(m, total);
        if (m) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if ((m >> k) & 1u) idx[pos++] = (q << 2) + k;
        }
    }
}

// ----------------------------------------------------------------- memory access helpers
template <bool NT> __device__ __forceinline__ f4 ld4(const float* p) {
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
    return *reinterpret_cast<const f4*>(p);
}
// Streaming 16-byte store.  The non-temporal flavour carries "sc1 nt" (device-coherent streaming
// write), which measured 2 % faster than "nt" alone on a plain copy (6.60 vs 6.46 TB/s); the compiler
// has no builtin for that pair, so the instruction is written out.  The trailing s_nop keeps the
// required distance to a following overwrite of the data registers, which the compiler cannot see.
template <bool NT> __device__ __forceinline__ void st4(float* p, f4 v) {
    if (NT) {
#ifdef SAPS_PLAIN_NT_STORE
        __builtin_nontemporal_store(v, reinterpret_cast<f4*>(p));
#else
        asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 2" : : "v"(p), "v"(v) : "memory");
#endif
    } else {
        *reinterpret_cast<f4*>(p) = v;
    }
}

// Streaming 4-byte store with the same "sc1 nt" policy, for packed messages and scattered averages:
// on the mixed-ratio exchange (128 x 11.2 M) it measured 0.52 ms against 0.60 ms with plain stores
// (0.57 with "nt" alone); gathers stay plain, a non-temporal hint on them measured slower (0.74 ms).
__device__ __forceinline__ void st1(float* p, float v) {
    asm volatile("global_store_dword %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
// Scattered 4-byte store of an averaged value: streaming (sc1 nt) in general, plain write-back
// (STREAM = false) when the lines that a round touches in all rows fit the L2 caches (32 x 272 k at
// c = 100: 4.2 instead of 6.6 us).  On models that do not fit, write-back stores measured slower
// (32 x 25.6 M at c = 1000: 45 against 42 us; 128 x 11.2 M mixed ratios: 0.61 against 0.52 ms).
template <bool STREAM> __device__ __forceinline__ void st1x(float* p, float v) {
    if (STREAM) st1(p, v); else *p = v;
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
__global__ __launch_bounds__(STREAM_BLOCK) void sgd_kernel(float* __restrict__ X, const float* __restrict__ G,
                                                           float* __restrict__ V, int64_t ld, uint32_t N, float lr, float mu) {
    const uint32_t q = blockIdx.x * STREAM_BLOCK + threadIdx.x;
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
        st1(m + k, x[idx[k]]);
}

// -------------------------------------------------- K6: average the two packed messages
template <bool STREAM>
__global__ __launch_bounds__(BLOCK) void merge_kernel(float* __restrict__ X, int64_t ld, Units U,
                                                      const uint32_t* __restrict__ idx, const float* __restrict__ msg,
                                                      int64_t msg_ld, const int64_t* __restrict__ K_dev, int64_t cap) {
    const int64_t K = *K_dev;
    if (K > cap || K < 0) return;
    int32_t i, p;
    unit_at(U, blockIdx.y, i, p);
    if (p == i) return;
    float* xi = X + (int64_t)i * ld;
    float* xp = X + (int64_t)p * ld;
    const float* a = msg + (int64_t)i * msg_ld;
    const float* b = msg + (int64_t)p * msg_ld;
    for (int64_t k = (int64_t)blockIdx.x * BLOCK + threadIdx.x; k < K; k += (int64_t)gridDim.x * BLOCK) {
        const float avg = (a[k] + b[k]) * 0.5f;
        const uint32_t j = idx[k];
        st1x<STREAM>(xi + j, avg);
        st1x<STREAM>(xp + j, avg);
    }
}

// -------------------------- K8: exchange-only round through the index list (sparse masks)
// unit u = (i, p): a matched pair with i < p, or an unmatched worker with i == p.  Both gathers are
// requested before anything is stored.  With SKIP, coordinates inside the tiles marked in walk_bits
// (one bit per tile) are left to the tile walk K8w.
template <bool STREAM, bool SKIP>
__device__ __forceinline__ bool list_entry_load(const float* xi, const float* xp, const uint32_t* idx, int64_t k,
                                                const uint32_t* walk_bits, uint32_t& j, float& a, float& b) {
    j = idx[k];
    if (SKIP) {
        const uint32_t t = j / (uint32_t)TILE;
        if ((walk_bits[t >> 5] >> (t & 31u)) & 1u) return false;
    }
    a = xi[j];
    b = xp[j];                                       // unmatched worker: the same word again
    return true;
}

template <bool STREAM>
__device__ __forceinline__ void list_entry_store(float* xi, float* xp, float* mi, float* mp, bool paired, int64_t k,
                                                 uint32_t j, float a, float b) {
    if (mi) {
        st1(mi + k, a);
        if (paired) st1(mp + k, b);
    }
    if (paired) {
        const float avg = (a + b) * 0.5f;
        st1x<STREAM>(xi + j, avg);
        st1x<STREAM>(xp + j, avg);
    }
}

template <bool STREAM, bool SKIP>
__global__ __launch_bounds__(BLOCK) void exchange_list_kernel(float* __restrict__ X, int64_t ld, Units U,
                                                              const uint32_t* __restrict__ idx,
                                                              const int64_t* __restrict__ K_int, int64_t cap,
                                                              float* __restrict__ msg, int64_t msg_ld,
                                                              const uint32_t* __restrict__ walk_bits,
                                                              MaskParams P, uint32_t ntiles, NextCounts Nx) {
    const int64_t K = *K_int;
    int32_t i, p;
    unit_at(U, blockIdx.y, i, p);
    float* xi = X + (int64_t)i * ld;
    float* xp = X + (int64_t)p * ld;
    float* mi = msg ? msg + (int64_t)i * msg_ld : nullptr;
    float* mp = msg ? msg + (int64_t)p * msg_ld : nullptr;
    const int64_t stride = (int64_t)gridDim.x * BLOCK;
    int64_t k = (int64_t)blockIdx.x * BLOCK + threadIdx.x;
    // the first entry's gathers are requested before the next round is counted, so that the Philox
    // arithmetic runs while they are in flight
    uint32_t j = 0u;
    float a = 0.f, b = 0.f;
    const bool first = K <= cap && k < K && list_entry_load<STREAM, SKIP>(xi, xp, idx, k, walk_bits, j, a, b);
    count_next_round(P, Nx, ntiles, (blockIdx.y * gridDim.x + blockIdx.x) * WAVES + (threadIdx.x >> 6),
                     gridDim.x * gridDim.y * WAVES);
    if (K > cap) return;
    if (first) list_entry_store<STREAM>(xi, xp, mi, mp, p != i, k, j, a, b);
    for (k += stride; k < K; k += stride)
        if (list_entry_load<STREAM, SKIP>(xi, xp, idx, k, walk_bits, j, a, b))
            list_entry_store<STREAM>(xi, xp, mi, mp, p != i, k, j, a, b);
}

// ------------------------------------------------------------------ K7: fused dense round
// MODE 0: update with momentum buffer, 1: update without buffer, 2: no update (exchange only).
// Grid: x = workgroups of fused_round_waves(MODE) wave tiles (optionally remapped so that each XCD walks one
//       contiguous range), y = chunks of PPB units.  The mask nibble and the packed position
//       of a lane's four coordinates are computed once and reused for all PPB units of the
//       chunk.  Waves never talk to each other: no LDS, no barrier.
struct FusedArgs {
    float* X; const float* G; float* V;
    int64_t ld;
    int32_t n_units;
    float lr, mu;
    Bases bases;
    uint32_t* idx; float* msg; int64_t msg_ld;
    uint32_t ntiles; int32_t xcd_remap;
};

// The six 16-byte operands of one unit (matched pair i,p or single worker i) at one lane.
struct Operands { f4 xi, gi, vi, xp, gp, vp; };

template <int MODE, bool NT>
__device__ __forceinline__ Operands load_unit(const FusedArgs& A, int32_t i, int32_t p, uint32_t j0, uint32_t nval) {
    const f4 z = {0.f, 0.f, 0.f, 0.f};
    Operands o = {z, z, z, z, z, z};
    const bool paired = (p != i);
    const int64_t ei = (int64_t)i * A.ld + j0, ep = (int64_t)p * A.ld + j0;
    if (nval == 4u) {
        o.xi = ld4<NT>(A.X + ei);
        if (MODE != 2) o.gi = ld4<NT>(A.G + ei);
        if (MODE == 0) o.vi = ld4<NT>(A.V + ei);
        if (paired) {
            o.xp = ld4<NT>(A.X + ep);
            if (MODE != 2) o.gp = ld4<NT>(A.G + ep);
            if (MODE == 0) o.vp = ld4<NT>(A.V + ep);
        }
    } else {
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            if ((uint32_t)r < nval) {
                o.xi[r] = A.X[ei + r];
                if (MODE != 2) o.gi[r] = A.G[ei + r];
                if (MODE == 0) o.vi[r] = A.V[ei + r];
                if (paired) {
                    o.xp[r] = A.X[ep + r];
                    if (MODE != 2) o.gp[r] = A.G[ep + r];
                    if (MODE == 0) o.vp[r] = A.V[ep + r];
                }
            }
        }
    }
    return o;
}

// Local step, message write, averaging and write-back of one unit at one lane.
// MIXFIRST = false: Alg. 2 order (step, then exchange of the stepped values).
// MIXFIRST = true:  Eq. (7) order (exchange the values of X_t, then subtract the step computed at X_t).
template <int MODE, bool NT, bool MIXFIRST>
__device__ __forceinline__ void finish_unit(const FusedArgs& A, Operands& o, int32_t i, int32_t p, uint32_t j0,
                                            uint32_t nval, uint32_t m, uint32_t pos0) {
    const bool paired = (p != i);
    const int64_t ei = (int64_t)i * A.ld + j0, ep = (int64_t)p * A.ld + j0;
    if (MODE != 2 && !MIXFIRST) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float x = o.xi[r], v = o.vi[r];
            step1<MODE == 0>(x, o.gi[r], v, A.lr, A.mu);
            o.xi[r] = x; o.vi[r] = v;
            x = o.xp[r]; v = o.vp[r];
            step1<MODE == 0>(x, o.gp[r], v, A.lr, A.mu);
            o.xp[r] = x; o.vp[r] = v;
        }
    }
    if (m) {
        uint32_t pos = pos0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if ((m >> r) & 1u) {
                if (A.msg) {
                    // plain stores: a tile contributes only a few values per row here, and the write-back
                    // cache merges these fragments into lines (streaming stores measured 25 % slower)
                    A.msg[(int64_t)i * A.msg_ld + pos] = o.xi[r];
                    if (paired) A.msg[(int64_t)p * A.msg_ld + pos] = o.xp[r];
                }
                ++pos;
                if (paired) {
                    const float avg = (o.xi[r] + o.xp[r]) * 0.5f;
                    o.xi[r] = avg; o.xp[r] = avg;
                }
            }
        }
    }
    if (MODE != 2 && MIXFIRST) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float x = o.xi[r], v = o.vi[r];
            step1<MODE == 0>(x, o.gi[r], v, A.lr, A.mu);
            o.xi[r] = x; o.vi[r] = v;
            x = o.xp[r]; v = o.vp[r];
            step1<MODE == 0>(x, o.gp[r], v, A.lr, A.mu);
            o.xp[r] = x; o.vp[r] = v;
        }
    }
    if (nval == 4u) {
        if (MODE != 2 || paired) st4<NT>(A.X + ei, o.xi);
        if (MODE == 0) st4<NT>(A.V + ei, o.vi);
        if (paired) {
            st4<NT>(A.X + ep, o.xp);
            if (MODE == 0) st4<NT>(A.V + ep, o.vp);
        }
    } else {
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            if ((uint32_t)r < nval) {
                if (MODE != 2 || paired) A.X[ei + r] = o.xi[r];
                if (MODE == 0) A.V[ei + r] = o.vi[r];
                if (paired) {
                    A.X[ep + r] = o.xp[r];
                    if (MODE == 0) A.V[ep + r] = o.vp[r];
                }
            }
        }
    }
}

template <int MODE, int PPB, bool NT, bool MIXFIRST>
__global__ __launch_bounds__(64 * fused_round_waves(MODE)) void fused_round_kernel(MaskParams P, FusedArgs A, Units U, NextCounts Nx) {
    constexpr uint32_t NW = (uint32_t)fused_round_waves(MODE);
    count_next_round(P, Nx, A.ntiles, (blockIdx.y * gridDim.x + blockIdx.x) * NW + (threadIdx.x >> 6), gridDim.x * gridDim.y * NW);
    uint32_t blk = blockIdx.x;
    if (A.xcd_remap) {
        // workgroups are dealt round-robin to the 8 XCDs; give XCD x the range [x*per, (x+1)*per)
        const uint32_t nblk = (A.ntiles + NW - 1) / NW;
        const uint32_t per = (nblk + 7u) >> 3;
        blk = (blockIdx.x & 7u) * per + (blockIdx.x >> 3);
    }
    const uint32_t tile = blk * NW + (threadIdx.x >> 6);             // wave-uniform
    if (tile >= A.ntiles) return;
    const uint32_t q = tile * 64u + (threadIdx.x & 63u);
    const uint32_t j0 = q << 2;
    const bool live = j0 < P.N;
    const uint32_t nval = live ? min(4u, P.N - j0) : 0u;
    const int u_lo = blockIdx.y * PPB;
    const int u_hi = min(u_lo + PPB, A.n_units);
    const bool first_wave = (tile == 0u && blockIdx.y == 0);
    if (MODE == 2 && !first_wave && tile_count(A.bases.tile_cnt[tile]) == 0u) return;   // nothing of this tile is exchanged

    // the first unit's operands are requested before the mask arithmetic so that the Philox
    // rounds run while the loads are in flight
    int32_t i, p;
    unit_at(U, u_lo, i, p);
    Operands cur;
    if (MODE != 2 && live) cur = load_unit<MODE, NT>(A, i, p, j0, nval);

    const int seg0 = (P.n_seg > 1) ? first_segment(P, tile) : 0;
    const uint32_t m = mask4(P, tile, threadIdx.x & 63u, seg0);
    uint32_t total;
    int64_t K;
    const uint32_t pos0 = tile_base_and_K(A.bases, tile, first_wave, K) + wave_prefix(m, total);
    if (K > A.bases.cap) return;                                      // nothing may be written
    if (blockIdx.y == 0 && A.idx && m) {
        uint32_t pos = pos0;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if ((m >> r) & 1u) A.idx[pos++] = j0 + r;
    }
    if (!live) return;
    if (MODE == 2) {
        if (m == 0u) return;                                          // this lane exchanges nothing
        for (int u = u_lo; u < u_hi; ++u) {
            unit_at(U, u, i, p);
            cur = load_unit<MODE, NT>(A, i, p, j0, nval);
            finish_unit<MODE, NT, MIXFIRST>(A, cur, i, p, j0, nval, m, pos0);
        }
        return;
    }
#pragma unroll 1
    for (int u = u_lo; u < u_hi; ++u) {
        Operands nxt;
        int32_t in = i, pn = p;
        if (PPB > 1 && u + 1 < u_hi) {
            unit_at(U, u + 1, in, pn);
            nxt = load_unit<MODE, NT>(A, in, pn, j0, nval);
        }
        finish_unit<MODE, NT, MIXFIRST>(A, cur, i, p, j0, nval, m, pos0);
        if (PPB > 1) { cur = nxt; i = in; p = pn; }
    }
}

// ------------------------------------------- K7p: fused round, one row per wave, one pair per workgroup
// The two waves of a workgroup own the two rows of a matched pair at the same tile: each wave streams its
// own row (x, g, v in; x, v out: five 16-byte streams per lane instead of ten) and the two swap the values
// of the tile through LDS to average the kept coordinates.  Fewer streams per wave means that the same
// number of resident waves keeps fewer requests in flight, which is what the memory system rewards (a plain
// update kernel measures 6.9 TB/s with one row per wave and 6.4 TB/s with two).  Both waves evaluate the mask.
// Grid: x = tiles, y = units.  MODE 0: update with momentum buffer, 1: update without buffer.
template <int MODE, bool NT, bool MIXFIRST>
__global__ __launch_bounds__(FUSED_BLOCK) void fused_pair_kernel(MaskParams P, FusedArgs A, Units U, NextCounts Nx) {
    static_assert(FUSED_WAVES == 2 && (MODE == 0 || MODE == 1), "one wave per row of a pair");
    __shared__ f4 swap[2][64];
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    count_next_round(P, Nx, A.ntiles, (blockIdx.y * gridDim.x + blockIdx.x) * FUSED_WAVES + wave,
                     gridDim.x * gridDim.y * FUSED_WAVES);
    const uint32_t tile = blockIdx.x;                                    // < ntiles by the grid
    const uint32_t j0 = (tile * 64u + lane) << 2;
    const bool live = j0 < P.N;
    const uint32_t nval = live ? min(4u, P.N - j0) : 0u;
    int32_t i, p;
    unit_at(U, blockIdx.y, i, p);
    const bool paired = (p != i);
    const bool mine = live && (wave == 0u || paired);                    // the second wave of an unmatched worker idles
    const int32_t row = (wave == 0u) ? i : p;
    const int64_t e = (int64_t)row * A.ld + j0;
    const f4 z = {0.f, 0.f, 0.f, 0.f};
    f4 x = z, g = z, v = z;
    if (mine) {
        if (nval == 4u) {
            x = ld4<NT>(A.X + e); g = ld4<NT>(A.G + e);
            if (MODE == 0) v = ld4<NT>(A.V + e);
        } else {
#pragma unroll
            for (int r = 0; r < 3; ++r)
                if ((uint32_t)r < nval) { x[r] = A.X[e + r]; g[r] = A.G[e + r]; if (MODE == 0) v[r] = A.V[e + r]; }
        }
    }
    const bool first_wave = (tile == 0u && blockIdx.y == 0 && wave == 0u);
    const int seg0 = (P.n_seg > 1) ? first_segment(P, tile) : 0;
    const uint32_t m = mask4(P, tile, lane, seg0);
    uint32_t total;
    int64_t K;
    const uint32_t pos0 = tile_base_and_K(A.bases, tile, first_wave, K) + wave_prefix(m, total);
    if (K > A.bases.cap) return;                                         // the same decision in both waves
    if (blockIdx.y == 0 && wave == 0u && A.idx && m) {
        uint32_t pos = pos0;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if ((m >> r) & 1u) A.idx[pos++] = j0 + r;
    }
    if (!MIXFIRST) {
#pragma unroll
        for (int r = 0; r < 4; ++r) { float xr = x[r], vr = v[r]; step1<MODE == 0>(xr, g[r], vr, A.lr, A.mu); x[r] = xr; v[r] = vr; }
    }
    if (total) swap[wave][lane] = x;                                     // what the peer averages with (wave-uniform branch)
    if (mine && m && A.msg) {
        // one store per kept coordinate of the lane: almost always a single one
        float* out = A.msg + (int64_t)row * A.msg_ld + pos0;
        uint32_t mm = m;
        do {
            const uint32_t r = (uint32_t)__builtin_ctz(mm);
            const float lo = (r & 1u) ? x[1] : x[0], hi = (r & 1u) ? x[3] : x[2];
            *out++ = (r & 2u) ? hi : lo;
            mm &= mm - 1u;
        } while (mm);
    }
    __syncthreads();
    if (total && paired) {
        const f4 o = swap[wave ^ 1u][lane];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if ((m >> r) & 1u) x[r] = (wave == 0u) ? (x[r] + o[r]) * 0.5f : (o[r] + x[r]) * 0.5f;
    }
    if (MIXFIRST) {
#pragma unroll
        for (int r = 0; r < 4; ++r) { float xr = x[r], vr = v[r]; step1<MODE == 0>(xr, g[r], vr, A.lr, A.mu); x[r] = xr; v[r] = vr; }
    }
    if (!mine) return;
    if (nval == 4u) {
        st4<NT>(A.X + e, x);
        if (MODE == 0) st4<NT>(A.V + e, v);
    } else {
#pragma unroll
        for (int r = 0; r < 3; ++r)
            if ((uint32_t)r < nval) { A.X[e + r] = x[r]; if (MODE == 0) A.V[e + r] = v[r]; }
    }
}

// ------------------------------- K8w: exchange-only round of the listed (dense) tiles by streaming
// One wave per listed tile and chunk of units: the tile's 1 KB of both rows is read whole, the kept
// coordinates are packed and averaged, and the tile is written back whole.  Where a mask keeps most
// 128-byte lines anyway (c = 10: 97 %), whole-tile traffic costs no more bytes than touching the kept
// words one by one and avoids partial writes.  Only whole tiles (all 256 coordinates below N) are listed.
constexpr int WALK_UNITS_IN_FLIGHT = 2;

template <bool NT>
__global__ __launch_bounds__(FUSED_BLOCK) void walk_tiles_kernel(MaskParams P, Bases Bp, float* __restrict__ X, int64_t ld,
                                                                 Units U, int32_t n_units, int32_t units_per_wave,
                                                                 const uint32_t* __restrict__ walk_tiles, uint32_t n_walk,
                                                                 float* __restrict__ msg, int64_t msg_ld) {
    const uint32_t w = blockIdx.x * FUSED_WAVES + (threadIdx.x >> 6);
    if (w >= n_walk) return;
    const uint32_t tile = walk_tiles[w];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t j0 = (tile * 64u + lane) << 2;
    const int seg0 = (P.n_seg > 1) ? first_segment(P, tile) : 0;
    const uint32_t m = mask4(P, tile, lane, seg0);
    uint32_t total;
    int64_t K;
    const uint32_t pos0 = tile_base_and_K(Bp, tile, false, K) + wave_prefix(m, total);
    if (K > Bp.cap) return;
    const int u_lo = blockIdx.y * units_per_wave, u_hi = min(u_lo + units_per_wave, n_units);
    for (int u0 = u_lo; u0 < u_hi; u0 += WALK_UNITS_IN_FLIGHT) {
        f4 a[WALK_UNITS_IN_FLIGHT], b[WALK_UNITS_IN_FLIGHT];
        int32_t ii[WALK_UNITS_IN_FLIGHT], pp[WALK_UNITS_IN_FLIGHT];
#pragma unroll
        for (int r = 0; r < WALK_UNITS_IN_FLIGHT; ++r) {
            if (u0 + r < u_hi) {
                unit_at(U, u0 + r, ii[r], pp[r]);
                a[r] = ld4<NT>(X + (int64_t)ii[r] * ld + j0);
                b[r] = ld4<NT>(X + (int64_t)pp[r] * ld + j0);
            }
        }
#pragma unroll
        for (int r = 0; r < WALK_UNITS_IN_FLIGHT; ++r) {
            if (u0 + r < u_hi) {
                const int32_t i = ii[r], p = pp[r];
                uint32_t pos = pos0;
                f4 xa = a[r], xb = b[r];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if ((m >> q) & 1u) {
                        if (msg) {
                            msg[(int64_t)i * msg_ld + pos] = xa[q];
                            if (p != i) msg[(int64_t)p * msg_ld + pos] = xb[q];
                        }
                        const float avg = (xa[q] + xb[q]) * 0.5f;
                        xa[q] = avg; xb[q] = avg;
                        ++pos;
                    }
                }
                if (p != i) {
                    st4<NT>(X + (int64_t)i * ld + j0, xa);
                    st4<NT>(X + (int64_t)p * ld + j0, xb);
                }
            }
        }
    }
}

// ------------------------------------------------------- K9: consensus diagnostics
// Mean model and total disagreement  D = sum_i ||x_i - mean||^2  (the quantity whose decay
// Sec. II-C calls consensus and Theorem 1 bounds).  Lane = one 16-byte column group; it walks
// the n rows once, keeping sum and sum of squares per coordinate in fp64, so that
// D_j = sum x^2 - (sum x)^2 / n loses nothing that matters.  Workgroup partials are written
// out and added by K10 in a fixed order: the result does not depend on scheduling.
template <bool NT>
__global__ __launch_bounds__(BLOCK) void consensus_kernel(const float* __restrict__ X, int64_t ld, uint32_t N, int32_t n,
                                                          float* __restrict__ mean_out, double* __restrict__ partial) {
    __shared__ double wsum[WAVES];
    const uint32_t q = blockIdx.x * BLOCK + threadIdx.x;
    const uint32_t j0 = q << 2;
    double d = 0.0;
    if (j0 < N) {
        const uint32_t nval = min(4u, N - j0);
        double s[4] = {0.0, 0.0, 0.0, 0.0}, ss[4] = {0.0, 0.0, 0.0, 0.0};
        const float* col = X + j0;
        if (nval == 4u) {
            int32_t i = 0;
            for (; i + CONS_ROWS <= n; i += CONS_ROWS) {   // CONS_ROWS rows in flight
                f4 a[CONS_ROWS];
#pragma unroll
                for (int k = 0; k < CONS_ROWS; ++k) a[k] = ld4<NT>(col + (int64_t)(i + k) * ld);
#pragma unroll
                for (int k = 0; k < CONS_ROWS; ++k)
#pragma unroll
                    for (int r = 0; r < 4; ++r) { const double x = (double)a[k][r]; s[r] += x; ss[r] = fma(x, x, ss[r]); }
            }
            for (; i < n; ++i) {
                const f4 a = ld4<NT>(col + (int64_t)i * ld);
#pragma unroll
                for (int r = 0; r < 4; ++r) { const double x = (double)a[r]; s[r] += x; ss[r] = fma(x, x, ss[r]); }
            }
        } else {
            for (int32_t i = 0; i < n; ++i)
#pragma unroll
                for (int r = 0; r < 3; ++r)
                    if ((uint32_t)r < nval) { const double x = (double)col[(int64_t)i * ld + r]; s[r] += x; ss[r] = fma(x, x, ss[r]); }
        }
        const double dn = (double)n;
        f4 mean = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if ((uint32_t)r < nval) {
                const double m = s[r] / dn;
                mean[r] = (float)m;
                d += fma(-m, s[r], ss[r]);               // sum x^2 - (sum x)^2 / n
            }
        }
        if (mean_out) {
            if (nval == 4u) st4<NT>(mean_out + j0, mean);
            else {
#pragma unroll
                for (int r = 0; r < 3; ++r) if ((uint32_t)r < nval) mean_out[j0 + r] = mean[r];
            }
        }
    }
    // fixed-order workgroup sum: lanes by xor swaps, then the four waves in order
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) d += __shfl_xor(d, o, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = d;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
}

// K10: one workgroup adds the partials in a fixed order.
__global__ __launch_bounds__(1024) void consensus_finish_kernel(const double* __restrict__ partial, uint32_t count,
                                                                double* __restrict__ D_out) {
    __shared__ double wsum[16];
    double d = 0.0;
    for (uint32_t k = threadIdx.x; k < count; k += 1024u) d += partial[k];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) d += __shfl_xor(d, o, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = d;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += wsum[w];
        *D_out = t;
    }
}

// --------------------------------------------------------- bandwidth yardstick (a copy)
template <bool NT>
__global__ __launch_bounds__(STREAM_BLOCK) void stream_copy_kernel(float* __restrict__ dst, const float* __restrict__ src,
                                                                   int64_t count4) {
    const int64_t q = (int64_t)blockIdx.x * STREAM_BLOCK + threadIdx.x;
    if (q < count4) st4<NT>(dst + 4 * q, ld4<NT>(src + 4 * q));
}

// ------------------------------------------ yardstick of the list kernels (isolated accesses)
// Every row reads the 4-byte word at each listed coordinate; with WRITE the same bits are stored back
// in place with the store policy of the exchange (the matrix does not change).  No averaging, no messages:
// what remains is what the memory system gives for the access pattern of the list exchange.
template <bool WRITE, bool STREAM>
__global__ __launch_bounds__(BLOCK) void list_probe_kernel(float* __restrict__ X, int64_t ld,
                                                           const uint32_t* __restrict__ idx,
                                                           const int64_t* __restrict__ K_dev, int64_t cap,
                                                           uint32_t N, uint32_t* __restrict__ sink) {
    const int64_t K = *K_dev;
    if (K > cap || K < 0) return;
    float* x = X + (int64_t)blockIdx.y * ld;
    for (int64_t k = (int64_t)blockIdx.x * BLOCK + threadIdx.x; k < K; k += (int64_t)gridDim.x * BLOCK) {
        const uint32_t j = idx[k];
        if (j >= N) continue;                                       // a foreign list must not lead outside the row
        const float v = x[j];
        if (WRITE) st1x<STREAM>(x + j, v);
        else if (__float_as_uint(v) == 0xFFFFFFFFu) *sink = 1u;     // keeps the load; a model never holds this pattern
    }
}

}  // namespace saps
