// Host side of the C ABI declared in include/saps.h: argument checks, the private scratch
// of a context, and the launch sequences of the SAPS-PSGD round (Alg. 2 lines 5-10).
#include "saps_device.hpp"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/saps.h"

using namespace saps;

namespace {

constexpr int RING = 4;                 // pinned staging slots for the matching
constexpr int64_t MAX_N = 0xFFFF0000ll;
constexpr int32_t MAX_WORKERS = 65535;
constexpr uint32_t LIST_GRID_X_MAX = 1024;

struct Slot {
    int32_t* host = nullptr;            // pinned: units[2n]
    hipEvent_t done = nullptr;
    bool used = false;
};

// Scratch of saps_round_static(), the entry point for callers that cannot allocate: tile and group
// counts, K, the capacity flag and an index list, in one file-scope device array instead of a context's
// hipMalloc'd buffers.  Every GPU the library runs on holds its own copy (about 3.1 MiB) until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress(): the address
// that kernels and copies may use is the one that call returns, kept per device in g_static_ptr.
constexpr int64_t STATIC_MAX_N = 1ll << 26;                                   // 67,108,864 coordinates
constexpr uint32_t STATIC_MAX_TILES = (uint32_t)(STATIC_MAX_N / TILE);
constexpr uint32_t STATIC_MAX_GROUPS = STATIC_MAX_TILES / GROUP;
constexpr int64_t STATIC_MAX_LIST = 1ll << 19;                                // entries of the internal index list
constexpr size_t ST_OFF_K = 0, ST_OFF_FLAG = 64;
constexpr size_t ST_OFF_TILE = 256;
constexpr size_t ST_OFF_GRP = ST_OFF_TILE + sizeof(uint32_t) * ((size_t)STATIC_MAX_TILES + 64);
constexpr size_t ST_OFF_IDX = ST_OFF_GRP + sizeof(uint32_t) * ((size_t)STATIC_MAX_GROUPS + 64);
constexpr size_t ST_BYTES = ST_OFF_IDX + sizeof(uint32_t) * (size_t)STATIC_MAX_LIST;
static_assert(ST_OFF_GRP % 256 == 0 && ST_OFF_IDX % 256 == 0, "scratch parts stay 256-byte aligned");
static __device__ __align__(256) unsigned char scratch[ST_BYTES];

constexpr int STATIC_MAX_DEVICES = 64;
std::mutex g_static_mu;
unsigned char* g_static_ptr[STATIC_MAX_DEVICES] = {};
thread_local std::string g_static_err;

}  // namespace

struct saps_ctx {
    int32_t n = 0;
    int64_t N = 0, ld = 0, msg_ld = 0;
    hipStream_t stream = nullptr;
    int device = 0;                     // the device that was current at creation; all scratch lives there
    uint32_t ntiles = 0;
    // mask description (segments with equal thresholds merged, empty ones dropped)
    int32_t n_seg = 1;
    uint64_t T0 = 0;
    double density = 0.0;               // expected K / N
    bool stream_scatter = true;         // scattered averages: streaming stores (true) or write-back stores (false)
    uint32_t* d_seg_end = nullptr;
    uint64_t* d_seg_T = nullptr;
    uint32_t* d_grp_seg = nullptr;      // first segment intersecting each group of 16 tiles
    uint32_t* d_walk_tiles = nullptr;   // whole tiles dense enough to be exchanged by streaming (hybrid path)
    uint32_t* d_walk_bits = nullptr;    // the same set as one bit per tile
    uint32_t n_walk = 0;
    // scratch
    uint32_t ngroups = 0;
    // Count buffers: [0] and [1] serve eager calls (a round's kernels count the next round into the one
    // that the round itself does not read), [2] serves calls made under stream capture, so that replays
    // of a graph never touch what eager calls have prepared.
    uint32_t* d_tile[3] = {nullptr, nullptr, nullptr};   // ntiles kept counts, one per wave tile
    uint32_t* d_grp[3] = {nullptr, nullptr, nullptr};    // ngroups counts, then exclusive bases after the scan
    bool prep_valid = false;            // d_tile/d_grp[prep_buf] hold the counts of (prep_seed, prep_round)
    uint64_t prep_seed = 0, prep_round = 0;
    int prep_buf = 0;
    int64_t* d_K = nullptr;             // K of the most recent mask generation
    int32_t* d_flag = nullptr;          // sticky capacity flag
    double* d_partial = nullptr;        // one fp64 partial per workgroup of the consensus kernel
    uint32_t* d_idx = nullptr;          // msg_ld entries, used when the caller passes idx == NULL
    int32_t* d_match = nullptr;         // units[2n], only used when the list is too long for the kernel arguments
    Slot ring[RING];
    uint64_t calls = 0;
    // launch-shape knobs
    int32_t ppb = 1, xcd_remap = 0, nontemporal = 1, exchange_path = 0, blocks_per_cu = -1, prepare_next = 1, row_per_wave = 1;
    // optional event pairs around the dominant kernel of a call
    bool profiling = false;
    std::vector<hipEvent_t> ev_pool;    // 2 events per record, created on demand
    size_t ev_used = 0;
    std::string err;
};

namespace {

saps_status fail(saps_ctx* c, saps_status s, const char* what) {
    if (c) c->err = what;
    return s;
}

saps_status hip_fail(saps_ctx* c, hipError_t e, const char* where) {
    if (c) {
        c->err = std::string(where) + ": " + hipGetErrorString(e);
    }
    return SAPS_EHIP;
}

#define SAPS_HIP(ctx, call)                                        \
    do {                                                           \
        hipError_t e__ = (call);                                   \
        if (e__ != hipSuccess) return hip_fail((ctx), e__, #call); \
    } while (0)

// Every entry point must be called with the context's device current (its scratch and stream are there).
saps_status check_device(saps_ctx* c) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != c->device)
        return fail(c, SAPS_EINVAL, "the context was created on another device than the current one");
    return SAPS_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

MaskParams mask_params(const saps_ctx* c, uint64_t seed, uint64_t round) {
    MaskParams P;
    P.key0 = (uint32_t)seed; P.key1 = (uint32_t)(seed >> 32);
    P.rnd0 = (uint32_t)round; P.rnd1 = (uint32_t)(round >> 32);
    P.N = (uint32_t)c->N;
    P.n_seg = c->n_seg;
    P.T0 = c->T0;
    P.seg_end = c->d_seg_end;
    P.seg_T = c->d_seg_T;
    P.grp_seg = c->d_grp_seg;
    return P;
}

// peer[] must be an involution of [0, n).
bool matching_ok(int32_t n, const int32_t* peer) {
    for (int32_t i = 0; i < n; ++i) {
        const int32_t p = peer[i];
        if (p < 0 || p >= n) return false;
        if (peer[p] != i) return false;
    }
    return true;
}

// Builds the unit list of a matching (pairs i < p, singles i == p).  Up to MAX_INLINE_UNITS
// units ride in the kernel arguments; longer lists are staged through a pinned slot and
// uploaded on the stream.
saps_status make_units(saps_ctx* c, const int32_t* peer, Units* U, int32_t* n_units) {
    int32_t u = 0;
    for (int32_t i = 0; i < c->n; ++i) u += (peer[i] >= i);
    *n_units = u;
    if (u <= MAX_INLINE_UNITS) {
        U->dev = nullptr;
        int32_t k = 0;
        for (int32_t i = 0; i < c->n; ++i)
            if (peer[i] >= i) U->packed[k++] = (uint32_t)i | ((uint32_t)peer[i] << 16);
        for (; k < MAX_INLINE_UNITS; ++k) U->packed[k] = 0u;
        return SAPS_OK;
    }
    // The staging ring waits on an event and uploads from pinned memory: neither can be recorded into a
    // graph (the copy would bake one stale staging slot into every replay).
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    SAPS_HIP(c, hipStreamIsCapturing(c->stream, &cap));
    if (cap != hipStreamCaptureStatusNone)
        return fail(c, SAPS_EINVAL, "the stream is capturing and the matching has more than 128 units: "
                                    "only matchings that fit the kernel arguments can be captured in a graph");
    if (!c->ring[0].host) return fail(c, SAPS_EINVAL, "the matching has more than 128 units");
    Slot& s = c->ring[c->calls++ % RING];
    if (s.used) SAPS_HIP(c, hipEventSynchronize(s.done));
    int32_t* units = s.host;
    int32_t k = 0;
    for (int32_t i = 0; i < c->n; ++i) {
        if (peer[i] >= i) { units[2 * k] = i; units[2 * k + 1] = peer[i]; ++k; }
    }
    SAPS_HIP(c, hipMemcpyAsync(c->d_match, units, sizeof(int32_t) * 2 * (size_t)u, hipMemcpyHostToDevice, c->stream));
    SAPS_HIP(c, hipEventRecord(s.done, c->stream));
    s.used = true;
    U->dev = c->d_match;
    return SAPS_OK;
}

void launch_idx_scatter(saps_ctx* c, const MaskParams& P, const Bases& Bp, uint32_t* list);

// Scattered 4-byte stores of the list kernels: write-back stores while the 128-byte lines that one round
// touches in all n rows fit the L2 caches (8 x 4 MB), streaming stores beyond.
constexpr double SCATTER_WRITEBACK_MAX_BYTES = 32e6;
bool stream_scatter_for(int32_t n, double expected_lines) { return (double)n * expected_lines * 128.0 > SCATTER_WRITEBACK_MAX_BYTES; }

// The streaming kernels run fastest with a moderate number of resident waves per compute unit (more requests in
// flight than the DRAM interface has credits for only queue up in front of it).  Residency is capped by giving
// each workgroup a slice of the 160 KB LDS that it never touches.  LDS is handed out in granules of 1280 bytes
// (128 per compute unit), so a slice of floor(128 / blocks) granules admits floor(128 / granules) workgroups:
// exactly `blocks` for 1..12, 14, 16, 18, 21, 25, 32, the next such value otherwise.
uint32_t residency_lds_bytes(int32_t blocks_per_cu) {
    return blocks_per_cu > 0 ? (uint32_t)(128 / blocks_per_cu) * 1280u : 0u;
}

// Compute units of a device, asked once per device.
int32_t compute_units(int device) {
    static std::mutex mu;
    static int32_t cache[STATIC_MAX_DEVICES] = {};
    if (device < 0 || device >= STATIC_MAX_DEVICES) return 256;
    std::lock_guard<std::mutex> g(mu);
    if (!cache[device]) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || v <= 0) v = 256;
        cache[device] = v;
    }
    return cache[device];
}

// Workgroups per compute unit of a streaming kernel: the caller's knob, else the kernel's built-in cap, but only
// for grids that turn the resident set over at least 32 times: a short grid loses more in its last, partly filled
// turn than the cap gains (fused round with buffer, 32 x 1.0 M: 0.111 ms capped, 0.105 uncapped; 32 x 3.0 M: 0.290
// against 0.294; 2 x 11.2 M: 0.081 against 0.079; 8 x 11.2 M: 0.280 against 0.283).
int32_t residency_for(const saps_ctx* c, int32_t builtin, uint64_t workgroups) {
    if (c->blocks_per_cu >= 0) return c->blocks_per_cu;
    return workgroups >= 32ull * (uint64_t)compute_units(c->device) * (uint64_t)builtin ? builtin : 0;
}

constexpr size_t MAX_PROFILE_RECORDS = 4096;

// Records an event on the stream if profiling is on; `second` closes the pair opened before.
void profile_mark(saps_ctx* c, bool second) {
    if (!c->profiling) return;
    if (!second) {
        if (c->ev_used / 2 >= MAX_PROFILE_RECORDS) return;
        if (c->ev_pool.size() < c->ev_used + 2) {
            hipEvent_t a = nullptr, b = nullptr;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
            c->ev_pool.push_back(a); c->ev_pool.push_back(b);
        }
        (void)hipEventRecord(c->ev_pool[c->ev_used], c->stream);
        c->ev_used += 1;
    } else if (c->ev_used & 1) {
        (void)hipEventRecord(c->ev_pool[c->ev_used], c->stream);
        c->ev_used += 1;
    }
}

// Small models skip the scan launch: the kernels that need packed positions add up the (at most
// 256) group counts themselves.
bool direct_bases(const saps_ctx* c) { return c->ngroups > 0 && c->ngroups <= DIRECT_MAX_GROUPS; }

// K1 (+ K2 unless the model is small): per-tile and per-group counts, exclusive group bases, K and
// the capacity flag.  Returns what the position-consuming kernels need.
// `with_next`: the caller launches a kernel that can count the next round on the side (the fused round
// kernel or the list exchange kernel); *Nx then says where, or holds nulls when there is nothing to prepare.
saps_status enqueue_count_scan(saps_ctx* c, const MaskParams& P, uint64_t seed, uint64_t round, int64_t* K_user,
                               Bases* Bp, bool with_next, NextCounts* Nx) {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (c->d_tile[2]) SAPS_HIP(c, hipStreamIsCapturing(c->stream, &cap));
    const bool capturing = cap != hipStreamCaptureStatusNone;
    int buf = 0;
    bool counted = false;                                  // the counts of (seed, round) are already there
    if (capturing) {
        buf = 2;
    } else {
        if (c->prep_valid && c->prep_seed == seed && c->prep_round == round) { buf = c->prep_buf; counted = true; }
        c->prep_valid = false;
    }
    Bp->grp = c->d_grp[buf]; Bp->tile_cnt = c->d_tile[buf]; Bp->K_int = c->d_K; Bp->K_user = K_user; Bp->flag = c->d_flag;
    Bp->cap = c->msg_ld; Bp->ngroups = c->ngroups; Bp->direct = direct_bases(c) ? 1 : 0;
    if (c->ngroups > 0 && !counted)
        hipLaunchKernelGGL(mask_count_kernel, dim3(c->ngroups), dim3(64 * GROUP), 0, c->stream, P, c->ntiles, c->d_tile[buf], c->d_grp[buf]);
    if (!Bp->direct)
        hipLaunchKernelGGL(group_scan_kernel, dim3(1), dim3(1024), 0, c->stream, c->d_grp[buf], c->ngroups, c->msg_ld,
                           c->d_K, K_user, c->d_flag);
    SAPS_HIP(c, hipGetLastError());
    if (Nx) {
        Nx->tile_cnt = nullptr; Nx->grp_cnt = nullptr; Nx->rnd0 = Nx->rnd1 = 0u; Nx->ngroups = c->ngroups;
        if (with_next && !capturing && c->prepare_next && c->d_tile[1] && c->ngroups > 0) {
            const int nb = buf == 0 ? 1 : 0;
            const uint64_t next = round + 1;
            Nx->tile_cnt = c->d_tile[nb]; Nx->grp_cnt = c->d_grp[nb];
            Nx->rnd0 = (uint32_t)next; Nx->rnd1 = (uint32_t)(next >> 32);
            c->prep_valid = true; c->prep_seed = seed; c->prep_round = next; c->prep_buf = nb;
        }
    }
    return SAPS_OK;
}

// K3 with one wave per tile, or one wave per group of 16 tiles when most tiles keep nothing
// (fewer than half a coordinate expected per tile of 256).
void launch_idx_scatter(saps_ctx* c, const MaskParams& P, const Bases& Bp, uint32_t* list) {
    if (c->density * TILE < 0.5) {
        const uint32_t waves = c->ngroups;
        hipLaunchKernelGGL(idx_scatter_kernel<GROUP>, dim3((waves + WAVES - 1) / WAVES), dim3(BLOCK), 0, c->stream, P, c->ntiles, Bp, list);
    } else {
        hipLaunchKernelGGL(idx_scatter_kernel<1>, dim3((c->ntiles + WAVES - 1) / WAVES), dim3(BLOCK), 0, c->stream, P, c->ntiles, Bp, list);
    }
}

uint32_t list_grid_x(const saps_ctx* c) {
    const int64_t b = (c->msg_ld + BLOCK - 1) / BLOCK;
    return (uint32_t)std::max<int64_t>(1, std::min<int64_t>(b, LIST_GRID_X_MAX));
}

template <int MODE, int PPB>
void launch_fused_nt(saps_ctx* c, const MaskParams& P, const FusedArgs& A, const Units& U, const NextCounts& Nx, dim3 grid, bool mix_first) {
    // measured best: 5 two-wave workgroups per compute unit when the momentum buffer is streamed too (ten 16-byte
    // streams per lane; 32 x 11.2 M: 1.100 ms against 1.110 at 6, 1.165 at 4), 16 one-wave workgroups without it
    // (six streams per lane; 32 x 6.65 M: 0.382 ms against 0.419 at 12, 0.392 at 14, 0.386 at 18, 0.390 at 21, 0.405 uncapped)
    const int32_t bpc = residency_for(c, MODE == 0 ? 5 : 16, (uint64_t)grid.x * grid.y);
    const uint32_t lds = (MODE == 2) ? 0u : residency_lds_bytes(bpc);
    const dim3 block(64 * fused_round_waves(MODE));
    if (MODE != 2 && mix_first) {
        if (c->nontemporal)
            hipLaunchKernelGGL((fused_round_kernel<MODE, PPB, true, MODE != 2>), grid, block, lds, c->stream, P, A, U, Nx);
        else
            hipLaunchKernelGGL((fused_round_kernel<MODE, PPB, false, MODE != 2>), grid, block, lds, c->stream, P, A, U, Nx);
    } else {
        if (c->nontemporal)
            hipLaunchKernelGGL((fused_round_kernel<MODE, PPB, true, false>), grid, block, lds, c->stream, P, A, U, Nx);
        else
            hipLaunchKernelGGL((fused_round_kernel<MODE, PPB, false, false>), grid, block, lds, c->stream, P, A, U, Nx);
    }
}

// K7p: one row per wave, one pair per workgroup (update rounds only).
template <int MODE>
void launch_fused_pair(saps_ctx* c, const MaskParams& P, const FusedArgs& A, const Units& U, const NextCounts& Nx, bool mix_first) {
    // measured on 32 x 11.2 M (rows 1 KB aligned, kernel trace on one box): 1.065 ms at 9 two-wave workgroups per compute unit,
    // 1.067 at 10, 1.074 at 11, 1.086 at 12 and uncapped, 1.107 at 8; 9 is also the best on 128 x 11.2 M, 32 x 25.6 M,
    // 32 x 100 M and 64 x 6.65 M (by 0.5-1 % over 10)
    const int32_t bpc = residency_for(c, 9, (uint64_t)c->ntiles * (uint64_t)A.n_units);
    uint32_t lds = residency_lds_bytes(bpc);
    if (lds > 2048u) lds -= 2048u;                     // the kernel's own 2 KB of LDS count towards the slice
    const dim3 grid(c->ntiles, (uint32_t)A.n_units);
    if (mix_first) {
        if (c->nontemporal) hipLaunchKernelGGL((fused_pair_kernel<MODE, true, true>), grid, dim3(FUSED_BLOCK), lds, c->stream, P, A, U, Nx);
        else hipLaunchKernelGGL((fused_pair_kernel<MODE, false, true>), grid, dim3(FUSED_BLOCK), lds, c->stream, P, A, U, Nx);
    } else {
        if (c->nontemporal) hipLaunchKernelGGL((fused_pair_kernel<MODE, true, false>), grid, dim3(FUSED_BLOCK), lds, c->stream, P, A, U, Nx);
        else hipLaunchKernelGGL((fused_pair_kernel<MODE, false, false>), grid, dim3(FUSED_BLOCK), lds, c->stream, P, A, U, Nx);
    }
}

template <int MODE>
void launch_fused(saps_ctx* c, const MaskParams& P, FusedArgs& A, const Units& U, const NextCounts& Nx, bool mix_first = false) {
    int ppb = c->ppb;
    constexpr uint32_t NW = (uint32_t)fused_round_waves(MODE);
    const uint32_t nblk = (c->ntiles + NW - 1) / NW;
    const uint32_t gx = c->xcd_remap ? 8u * ((nblk + 7u) / 8u) : nblk;
    A.xcd_remap = c->xcd_remap;
    const dim3 grid(gx, (uint32_t)((A.n_units + ppb - 1) / ppb));
    switch (ppb) {
        case 1: launch_fused_nt<MODE, 1>(c, P, A, U, Nx, grid, mix_first); break;
        case 2: launch_fused_nt<MODE, 2>(c, P, A, U, Nx, grid, mix_first); break;
        case 4: launch_fused_nt<MODE, 4>(c, P, A, U, Nx, grid, mix_first); break;
        default: launch_fused_nt<MODE, 8>(c, P, A, U, Nx, grid, mix_first); break;
    }
}

// Argument checks and launch sequence of one round; `c` is a created context or the stack-built
// description that saps_round_static() fills from its arguments.
saps_status round_impl(saps_ctx* c, float* X, const float* G, float* V, float lr, float mu,
                       uint64_t seed, uint64_t round, const int32_t* peer,
                       uint32_t* idx, float* msg, int64_t* K_dev, uint32_t flags) {
    if (flags & ~(uint32_t)SAPS_ROUND_MIX_THEN_STEP) return fail(c, SAPS_EINVAL, "unknown flag");
    const bool mix_first = (flags & SAPS_ROUND_MIX_THEN_STEP) != 0;
    if (!X || !peer) return fail(c, SAPS_EINVAL, "null pointer");
    if (!aligned16(X) || !aligned16(G) || !aligned16(V) || !aligned16(idx) || !aligned16(msg) ||
        (reinterpret_cast<uintptr_t>(K_dev) & 7u))
        return fail(c, SAPS_EINVAL, "misaligned pointer");
    if (G && !V && mu != 0.0f) return fail(c, SAPS_EINVAL, "momentum needs V");
    if (!matching_ok(c->n, peer)) return fail(c, SAPS_EMATCH, "peer[] is not an involution of [0, n)");
    int32_t n_units = 0;
    Units U;
    saps_status s = make_units(c, peer, &U, &n_units);
    if (s) return s;
    const MaskParams P = mask_params(c, seed, round);
    Bases Bp;
    NextCounts Nx;
    s = enqueue_count_scan(c, P, seed, round, K_dev, &Bp, true, &Nx);
    if (s) return s;
    if (c->ntiles == 0) return SAPS_OK;

    FusedArgs A;
    A.X = X; A.G = G; A.V = V; A.ld = c->ld;
    A.n_units = n_units;
    A.lr = lr; A.mu = mu;
    A.bases = Bp;
    A.idx = idx; A.msg = msg; A.msg_ld = c->msg_ld;
    A.ntiles = c->ntiles; A.xcd_remap = 0;

    if (G) {
        profile_mark(c, false);
        // with a momentum buffer the row-per-wave shape is faster (1.10 against 1.12 ms on 32 x 11.2 M); without one,
        // with three streams per wave, it is slower (0.49 against 0.41 ms on 32 x 6.65 M), so plain SGD needs the knob set to 2
        if (((c->row_per_wave == 1 && V) || c->row_per_wave == 2) && c->ppb == 1 && !c->xcd_remap && n_units <= 65535) {
            if (V) launch_fused_pair<0>(c, P, A, U, Nx, mix_first); else launch_fused_pair<1>(c, P, A, U, Nx, mix_first);
        } else {
            if (V) launch_fused<0>(c, P, A, U, Nx, mix_first); else launch_fused<1>(c, P, A, U, Nx, mix_first);
        }
        profile_mark(c, true);
    } else if (c->exchange_path == 2 || (c->exchange_path == 0 && c->density >= 1.0 / 12.0 && c->density < 0.2)) {
        // measured on 32 x 11.2 M: the walk wins around c = 8 (0.62 vs 0.72 ms); for denser masks its
        // per-lane message stores cost more than the list's coalesced ones (c = 2, 4: 0.82-0.86 vs 0.73 ms)
        profile_mark(c, false);
        launch_fused<2>(c, P, A, U, Nx);               // dense masks: walk the tiles
        profile_mark(c, true);
    } else {
        // sparse masks: go through the index list; path 3 streams the dense tiles of a mixed layout instead
        // (measured slower than the list alone on the 128 x 11.2 M mixed-ratio workload, so never the default)
        const bool hybrid = c->exchange_path == 3 && c->n_walk > 0 && c->d_walk_tiles;
        uint32_t* list = idx ? idx : c->d_idx;
        launch_idx_scatter(c, P, Bp, list);
        profile_mark(c, false);
        if (hybrid) {
            const int32_t upw = 2;
            const dim3 wgrid((c->n_walk + FUSED_WAVES - 1) / FUSED_WAVES, (uint32_t)((n_units + upw - 1) / upw));
            hipLaunchKernelGGL(walk_tiles_kernel<true>, wgrid, dim3(FUSED_BLOCK), 0, c->stream, P, Bp, X, c->ld, U, n_units, upw,
                               c->d_walk_tiles, c->n_walk, msg, c->msg_ld);
        }
        const dim3 lgrid(list_grid_x(c), (uint32_t)n_units);
        // long grids only: 4 four-wave workgroups per compute unit (128 x 11.2 M, mixed ratios: 0.505 against 0.511 ms uncapped,
        // 0.508 at 3, 0.511 at 6); the short grid of 32 x 25.6 M at c = 1000 loses 4 % under any cap and falls under the rule
        const uint32_t llds = residency_lds_bytes(residency_for(c, 4, (uint64_t)lgrid.x * lgrid.y));
        if (hybrid) {
            if (c->stream_scatter)
                hipLaunchKernelGGL((exchange_list_kernel<true, true>), lgrid, dim3(BLOCK), llds, c->stream, X, c->ld, U, list, c->d_K, c->msg_ld, msg, c->msg_ld, c->d_walk_bits, P, c->ntiles, Nx);
            else
                hipLaunchKernelGGL((exchange_list_kernel<false, true>), lgrid, dim3(BLOCK), llds, c->stream, X, c->ld, U, list, c->d_K, c->msg_ld, msg, c->msg_ld, c->d_walk_bits, P, c->ntiles, Nx);
        } else {
            if (c->stream_scatter)
                hipLaunchKernelGGL((exchange_list_kernel<true, false>), lgrid, dim3(BLOCK), llds, c->stream, X, c->ld, U, list, c->d_K, c->msg_ld, msg, c->msg_ld, c->d_walk_bits, P, c->ntiles, Nx);
            else
                hipLaunchKernelGGL((exchange_list_kernel<false, false>), lgrid, dim3(BLOCK), llds, c->stream, X, c->ld, U, list, c->d_K, c->msg_ld, msg, c->msg_ld, c->d_walk_bits, P, c->ntiles, Nx);
        }
        profile_mark(c, true);
    }
    if (hipError_t e = hipGetLastError(); e != hipSuccess) {
        c->prep_valid = false;                          // whatever was to count the next round may not have run
        return hip_fail(c, e, "kernel launch");
    }
    return SAPS_OK;
}

}  // namespace

extern "C" {

int32_t saps_abi_version(void) { return 4; }

// ctx == NULL: the calling thread's last saps_round_static() error
const char* saps_last_error(const saps_ctx* ctx) { return ctx ? ctx->err.c_str() : g_static_err.c_str(); }

saps_status saps_create(saps_ctx** out, const saps_layout* L, int64_t msg_ld, void* hip_stream) {
    if (!out) return SAPS_EINVAL;
    *out = nullptr;
    if (!L || !L->seg_off || !L->seg_c) return SAPS_EINVAL;
    if (L->n < 1 || L->n > MAX_WORKERS || L->N < 0 || L->N > MAX_N || L->ld < L->N || (L->ld & 3) || L->n_seg < 1)
        return SAPS_EINVAL;
    if (msg_ld < 0 || (msg_ld & 3)) return SAPS_EINVAL;
    if (L->seg_off[0] != 0 || L->seg_off[L->n_seg] != L->N) return SAPS_EINVAL;
    std::vector<uint32_t> seg_end;
    std::vector<uint64_t> seg_T;
    double expK = 0.0, expLines = 0.0;       // expected kept coordinates and touched 128-byte lines per row
    for (int32_t s = 0; s < L->n_seg; ++s) {
        const int64_t a = L->seg_off[s], b = L->seg_off[s + 1];
        const double cs = L->seg_c[s];
        if (b < a || !(cs >= 1.0)) return SAPS_EINVAL;          // also rejects NaN
        if (b == a) continue;
        const uint64_t T = (uint64_t)std::floor(4294967296.0 / cs);
        expK += (double)(b - a) * ((double)T / 4294967296.0);
        expLines += (double)(b - a) / 32.0 * (1.0 - std::pow(1.0 - (double)T / 4294967296.0, 32.0));
        if (!seg_T.empty() && seg_T.back() == T) seg_end.back() = (uint32_t)b;
        else { seg_end.push_back((uint32_t)b); seg_T.push_back(T); }
    }
    if (seg_T.empty()) { seg_end.push_back((uint32_t)L->N); seg_T.push_back(0); }

    saps_ctx* c = new (std::nothrow) saps_ctx;
    if (!c) return SAPS_EINVAL;
    c->n = L->n; c->N = L->N; c->ld = L->ld; c->msg_ld = msg_ld;
    c->stream = (hipStream_t)hip_stream;
    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return SAPS_EHIP; }
    c->ntiles = (uint32_t)((L->N + TILE - 1) / TILE);
    c->ngroups = (c->ntiles + GROUP - 1) / GROUP;
    c->n_seg = (int32_t)seg_T.size();
    c->T0 = seg_T[0];
    c->density = L->N > 0 ? expK / (double)L->N : 0.0;
    c->stream_scatter = stream_scatter_for(c->n, expLines);

    hipError_t e = hipSuccess;
    auto chk = [&](hipError_t r) { if (e == hipSuccess && r != hipSuccess) e = r; };
    chk(hipMalloc(&c->d_seg_end, sizeof(uint32_t) * seg_end.size()));
    chk(hipMalloc(&c->d_seg_T, sizeof(uint64_t) * seg_T.size()));
    // first segment that reaches into each group of GROUP tiles (GROUP * TILE coordinates)
    std::vector<uint32_t> grp_seg((size_t)c->ngroups + 1, 0u);
    {
        uint32_t sidx = 0;
        for (uint32_t g = 0; g < c->ngroups; ++g) {
            const uint64_t start = (uint64_t)g * GROUP * TILE;
            while (sidx + 1 < seg_end.size() && (uint64_t)seg_end[sidx] <= start) ++sidx;
            grp_seg[g] = sidx;
        }
    }
    chk(hipMalloc(&c->d_grp_seg, sizeof(uint32_t) * grp_seg.size()));
    // dense tiles of the hybrid exchange: whole tiles that are expected to keep at least every 12th coordinate
    std::vector<uint32_t> walk_tiles, walk_bits((size_t)c->ntiles / 32 + 1, 0u);
    {
        size_t si = 0;
        for (uint32_t t = 0; t < c->ntiles; ++t) {
            const uint64_t a = (uint64_t)t * TILE, b = a + TILE;
            if (b > (uint64_t)L->N) break;
            while (si + 1 < seg_end.size() && (uint64_t)seg_end[si] <= a) ++si;
            double e = 0.0;
            size_t s2 = si;
            for (uint64_t x = a; x < b;) {
                const uint64_t y = std::min<uint64_t>(b, seg_end[s2]);
                e += (double)(y - x) * ((double)seg_T[s2] / 4294967296.0);
                x = y;
                if (x < b) ++s2;
            }
            if (e >= (double)TILE / 12.0) { walk_tiles.push_back(t); walk_bits[t >> 5] |= 1u << (t & 31u); }
        }
    }
    c->n_walk = (uint32_t)walk_tiles.size();
    chk(hipMalloc(&c->d_walk_tiles, sizeof(uint32_t) * (walk_tiles.size() + 1)));
    chk(hipMalloc(&c->d_walk_bits, sizeof(uint32_t) * walk_bits.size()));
    if (e == hipSuccess && !walk_tiles.empty())
        chk(hipMemcpy(c->d_walk_tiles, walk_tiles.data(), sizeof(uint32_t) * walk_tiles.size(), hipMemcpyHostToDevice));
    if (e == hipSuccess) chk(hipMemcpy(c->d_walk_bits, walk_bits.data(), sizeof(uint32_t) * walk_bits.size(), hipMemcpyHostToDevice));
    if (e == hipSuccess) chk(hipMemcpy(c->d_grp_seg, grp_seg.data(), sizeof(uint32_t) * grp_seg.size(), hipMemcpyHostToDevice));
    for (int b = 0; b < 3; ++b) {
        chk(hipMalloc(&c->d_tile[b], sizeof(uint32_t) * ((size_t)c->ntiles + 1)));
        chk(hipMalloc(&c->d_grp[b], sizeof(uint32_t) * ((size_t)c->ngroups + 1)));
    }
    chk(hipMalloc(&c->d_K, sizeof(int64_t)));
    chk(hipMalloc(&c->d_partial, sizeof(double) * ((size_t)((L->N + 4 * BLOCK - 1) / (4 * BLOCK)) + 1)));
    chk(hipMalloc(&c->d_flag, sizeof(int32_t)));
    chk(hipMalloc(&c->d_idx, sizeof(uint32_t) * (size_t)std::max<int64_t>(msg_ld, 4)));
    chk(hipMalloc(&c->d_match, sizeof(int32_t) * 2 * (size_t)c->n));
    for (int r = 0; r < RING; ++r) {
        chk(hipHostMalloc(&c->ring[r].host, sizeof(int32_t) * 2 * (size_t)c->n, hipHostMallocDefault));
        chk(hipEventCreateWithFlags(&c->ring[r].done, hipEventDisableTiming));
    }
    if (e == hipSuccess) chk(hipMemcpy(c->d_seg_end, seg_end.data(), sizeof(uint32_t) * seg_end.size(), hipMemcpyHostToDevice));
    if (e == hipSuccess) chk(hipMemcpy(c->d_seg_T, seg_T.data(), sizeof(uint64_t) * seg_T.size(), hipMemcpyHostToDevice));
    if (e == hipSuccess) chk(hipMemset(c->d_K, 0, sizeof(int64_t)));
    if (e == hipSuccess) chk(hipMemset(c->d_flag, 0, sizeof(int32_t)));
    if (e != hipSuccess) {
        std::fprintf(stderr, "saps_create: %s\n", hipGetErrorString(e));
        saps_destroy(c);
        return SAPS_EHIP;
    }
    *out = c;
    return SAPS_OK;
}

saps_status saps_destroy(saps_ctx* c) {
    if (!c) return SAPS_EINVAL;
    (void)hipStreamSynchronize(c->stream);
    (void)hipFree(c->d_seg_end); (void)hipFree(c->d_seg_T); (void)hipFree(c->d_grp_seg); (void)hipFree(c->d_walk_tiles); (void)hipFree(c->d_walk_bits); for (int b = 0; b < 3; ++b) { (void)hipFree(c->d_tile[b]); (void)hipFree(c->d_grp[b]); } (void)hipFree(c->d_K); (void)hipFree(c->d_partial);
    (void)hipFree(c->d_flag); (void)hipFree(c->d_idx); (void)hipFree(c->d_match);
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    for (int r = 0; r < RING; ++r) {
        if (c->ring[r].host) (void)hipHostFree(c->ring[r].host);
        if (c->ring[r].done) (void)hipEventDestroy(c->ring[r].done);
    }
    delete c;
    return SAPS_OK;
}

saps_status saps_set_tuning(saps_ctx* c, int32_t knob, int32_t value) {
    if (!c) return SAPS_EINVAL;
    switch (knob) {
        case SAPS_TUNE_PAIRS_PER_BLOCK:
            if (value != 1 && value != 2 && value != 4 && value != 8) return fail(c, SAPS_EINVAL, "pairs per block");
            c->ppb = value; return SAPS_OK;
        case SAPS_TUNE_XCD_REMAP:
            if (value != 0 && value != 1) return fail(c, SAPS_EINVAL, "xcd remap");
            c->xcd_remap = value; return SAPS_OK;
        case SAPS_TUNE_NONTEMPORAL:
            if (value != 0 && value != 1) return fail(c, SAPS_EINVAL, "nontemporal");
            c->nontemporal = value; return SAPS_OK;
        case SAPS_TUNE_BLOCKS_PER_CU:
            if (value != -1 && value != 0 && (value < 3 || value > 32)) return fail(c, SAPS_EINVAL, "blocks per CU");
            c->blocks_per_cu = value; return SAPS_OK;
        case SAPS_TUNE_EXCHANGE_PATH:
            if (value < 0 || value > 3) return fail(c, SAPS_EINVAL, "exchange path");
            c->exchange_path = value; return SAPS_OK;
        case SAPS_TUNE_ROW_PER_WAVE:
            if (value < 0 || value > 2) return fail(c, SAPS_EINVAL, "row per wave");
            c->row_per_wave = value; return SAPS_OK;
        case SAPS_TUNE_PREPARE_NEXT:
            if (value != 0 && value != 1) return fail(c, SAPS_EINVAL, "prepare next");
            c->prepare_next = value; c->prep_valid = false; return SAPS_OK;
        default: return fail(c, SAPS_EINVAL, "unknown knob");
    }
}

saps_status saps_sgd_step(saps_ctx* c, float* X, const float* G, float* V, float lr, float mu) {
    if (!c) return SAPS_EINVAL;
    if (saps_status ds = check_device(c)) return ds;
    if (!X || !G || !aligned16(X) || !aligned16(G) || !aligned16(V)) return fail(c, SAPS_EINVAL, "X/G/V null or misaligned");
    if (!V && mu != 0.0f) return fail(c, SAPS_EINVAL, "momentum needs V");
    if (c->N == 0) return SAPS_OK;
    const uint32_t gx = (uint32_t)(((c->N + 3) / 4 + STREAM_BLOCK - 1) / STREAM_BLOCK);
    const dim3 grid(gx, (uint32_t)c->n);
    const uint32_t N = (uint32_t)c->N;
    // resident one-wave workgroups per compute unit: 10 with the momentum buffer (five 16-byte streams per lane), 16 without
    // (three streams), i.e. about fifty 1 KB requests in flight per compute unit.  Measured on 32 x 11.2 M: with the
    // buffer 6.77 TB/s at 10, 6.62 at 8, 6.49 at 16, 6.21 uncapped; without it 6.76 at 16, 6.14 at 12, 6.66 uncapped
    const uint32_t SGD_LDS = residency_lds_bytes(residency_for(c, V ? 10 : 16, (uint64_t)gx * (uint64_t)c->n));
    profile_mark(c, false);
    if (V) {
        if (c->nontemporal) hipLaunchKernelGGL((sgd_kernel<true, true>), grid, dim3(STREAM_BLOCK), SGD_LDS, c->stream, X, G, V, c->ld, N, lr, mu);
        else hipLaunchKernelGGL((sgd_kernel<true, false>), grid, dim3(STREAM_BLOCK), SGD_LDS, c->stream, X, G, V, c->ld, N, lr, mu);
    } else {
        if (c->nontemporal) hipLaunchKernelGGL((sgd_kernel<false, true>), grid, dim3(STREAM_BLOCK), SGD_LDS, c->stream, X, G, V, c->ld, N, lr, mu);
        else hipLaunchKernelGGL((sgd_kernel<false, false>), grid, dim3(STREAM_BLOCK), SGD_LDS, c->stream, X, G, V, c->ld, N, lr, mu);
    }
    profile_mark(c, true);
    SAPS_HIP(c, hipGetLastError());
    return SAPS_OK;
}

saps_status saps_mask_compact(saps_ctx* c, const float* X, uint64_t seed, uint64_t round,
                              uint32_t* idx, float* msg, int64_t* K_dev) {
    if (!c) return SAPS_EINVAL;
    if (saps_status ds = check_device(c)) return ds;
    if (!X || !idx || !msg || !K_dev) return fail(c, SAPS_EINVAL, "null pointer");
    if (!aligned16(X) || !aligned16(idx) || !aligned16(msg) || (reinterpret_cast<uintptr_t>(K_dev) & 7u))
        return fail(c, SAPS_EINVAL, "misaligned pointer");
    const MaskParams P = mask_params(c, seed, round);
    Bases Bp;
    saps_status s = enqueue_count_scan(c, P, seed, round, K_dev, &Bp, false, nullptr);
    if (s) return s;
    if (c->ntiles == 0) return SAPS_OK;
    launch_idx_scatter(c, P, Bp, idx);
    hipLaunchKernelGGL(compact_values_kernel, dim3(list_grid_x(c), (uint32_t)c->n), dim3(BLOCK), 0, c->stream,
                       X, c->ld, idx, c->d_K, c->msg_ld, msg, c->msg_ld);
    SAPS_HIP(c, hipGetLastError());
    return SAPS_OK;
}

saps_status saps_merge(saps_ctx* c, float* X, const int32_t* peer, const uint32_t* idx, const float* msg,
                       const int64_t* K_dev) {
    if (!c) return SAPS_EINVAL;
    if (saps_status ds = check_device(c)) return ds;
    if (!X || !peer || !idx || !msg || !K_dev) return fail(c, SAPS_EINVAL, "null pointer");
    if (!aligned16(X) || !aligned16(idx) || !aligned16(msg) || (reinterpret_cast<uintptr_t>(K_dev) & 7u))
        return fail(c, SAPS_EINVAL, "misaligned pointer");
    if (!matching_ok(c->n, peer)) return fail(c, SAPS_EMATCH, "peer[] is not an involution of [0, n)");
    int32_t n_units = 0;
    Units U;
    saps_status s = make_units(c, peer, &U, &n_units);
    if (s) return s;
    if (c->N == 0) return SAPS_OK;
    if (c->stream_scatter)
        hipLaunchKernelGGL(merge_kernel<true>, dim3(list_grid_x(c), (uint32_t)n_units), dim3(BLOCK), 0, c->stream,
                           X, c->ld, U, idx, msg, c->msg_ld, K_dev, c->msg_ld);
    else
        hipLaunchKernelGGL(merge_kernel<false>, dim3(list_grid_x(c), (uint32_t)n_units), dim3(BLOCK), 0, c->stream,
                           X, c->ld, U, idx, msg, c->msg_ld, K_dev, c->msg_ld);
    SAPS_HIP(c, hipGetLastError());
    return SAPS_OK;
}

saps_status saps_round(saps_ctx* c, float* X, const float* G, float* V, float lr, float mu,
                       uint64_t seed, uint64_t round, const int32_t* peer,
                       uint32_t* idx, float* msg, int64_t* K_dev) {
    return saps_round_ex(c, X, G, V, lr, mu, seed, round, peer, idx, msg, K_dev, 0u);
}

saps_status saps_round_ex(saps_ctx* c, float* X, const float* G, float* V, float lr, float mu,
                          uint64_t seed, uint64_t round, const int32_t* peer,
                          uint32_t* idx, float* msg, int64_t* K_dev, uint32_t flags) {
    if (!c) return SAPS_EINVAL;
    if (saps_status ds = check_device(c)) return ds;
    return round_impl(c, X, G, V, lr, mu, seed, round, peer, idx, msg, K_dev, flags);
}

saps_status saps_round_static(int32_t n, int64_t N, int64_t ld, double c_ratio, int64_t msg_ld, void* hip_stream,
                              float* X, const float* G, float* V, float lr, float mu,
                              uint64_t seed, uint64_t round, const int32_t* peer,
                              uint32_t* idx, float* msg, int64_t* K_dev) {
    auto bad = [](const char* what) { g_static_err = what; return SAPS_EINVAL; };
    if (n < 1 || n > MAX_WORKERS || N < 0 || ld < N || (ld & 3) || msg_ld < 0 || (msg_ld & 3)) return bad("bad n, N, ld or msg_ld");
    if (N > STATIC_MAX_N) return bad("N exceeds the static scratch (at most 67,108,864 coordinates)");
    if (!(c_ratio >= 1.0)) return bad("compression ratio below 1");
    if (!K_dev) return bad("K_dev is required: it is how the caller sees that K > msg_ld skipped the round");
    if (!idx && msg_ld > STATIC_MAX_LIST) return bad("idx == NULL needs msg_ld <= 524,288 (the internal index list)");
    if (!peer) return bad("null pointer");
    int32_t units = 0;
    for (int32_t i = 0; i < n; ++i) units += (peer[i] >= i);
    if (units > MAX_INLINE_UNITS) return bad("the matching has more than 128 units (pairs plus unmatched workers)");

    // the device's own copy of the scratch array: resolved once per device, with that device current
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) { g_static_err = "hipGetDevice"; return SAPS_EHIP; }
    unsigned char* base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_static_mu);
        if (!g_static_ptr[dev]) {
            void* ptr = nullptr;
            const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !ptr) {
                g_static_err = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e);
                return SAPS_EHIP;
            }
            g_static_ptr[dev] = static_cast<unsigned char*>(ptr);
        }
        base = g_static_ptr[dev];
    }

    // a context on the stack that points into the scratch; nothing is allocated and nothing outlives the call
    saps_ctx t;
    t.n = n; t.N = N; t.ld = ld; t.msg_ld = msg_ld;
    t.stream = (hipStream_t)hip_stream;
    t.device = dev;
    t.ntiles = (uint32_t)((N + TILE - 1) / TILE);
    t.ngroups = (t.ntiles + GROUP - 1) / GROUP;
    t.n_seg = 1;
    t.T0 = (uint64_t)std::floor(4294967296.0 / c_ratio);
    t.density = (double)t.T0 / 4294967296.0;
    t.stream_scatter = stream_scatter_for(n, (double)N / 32.0 * (1.0 - std::pow(1.0 - t.density, 32.0)));
    t.d_K = reinterpret_cast<int64_t*>(base + ST_OFF_K);
    t.d_flag = reinterpret_cast<int32_t*>(base + ST_OFF_FLAG);
    t.d_tile[0] = reinterpret_cast<uint32_t*>(base + ST_OFF_TILE);       // one buffer: every call counts for itself
    t.d_grp[0] = reinterpret_cast<uint32_t*>(base + ST_OFF_GRP);
    t.d_idx = reinterpret_cast<uint32_t*>(base + ST_OFF_IDX);
    const saps_status st = round_impl(&t, X, G, V, lr, mu, seed, round, peer, idx, msg, K_dev, 0u);
    if (st != SAPS_OK) g_static_err = t.err;
    return st;
}

saps_status saps_consensus(saps_ctx* c, const float* X, float* mean_out, double* D_dev) {
    if (!c) return SAPS_EINVAL;
    if (saps_status ds = check_device(c)) return ds;
    if (!X || !D_dev || !aligned16(X) || !aligned16(mean_out) || (reinterpret_cast<uintptr_t>(D_dev) & 7u))
        return fail(c, SAPS_EINVAL, "X/mean/D null or misaligned");
    const uint32_t blocks = (uint32_t)((c->N + 4 * BLOCK - 1) / (4 * BLOCK));
    if (blocks > 0) {
        // 8 rows in flight per lane.  When the mean is written too, 3 four-wave workgroups per compute unit are 2-3 % faster
        // than no cap (32 x 11.2 M: 0.240-0.245 against 0.247-0.251 ms over eight row strides); without it no cap is as fast
        // or faster (0.210-0.214 against 0.213-0.221 ms)
        const uint32_t clds = residency_lds_bytes(c->blocks_per_cu >= 0 ? c->blocks_per_cu : (mean_out ? 3 : 0));
        profile_mark(c, false);
        if (c->nontemporal) hipLaunchKernelGGL(consensus_kernel<true>, dim3(blocks), dim3(BLOCK), clds, c->stream, X, c->ld, (uint32_t)c->N, c->n, mean_out, c->d_partial);
        else hipLaunchKernelGGL(consensus_kernel<false>, dim3(blocks), dim3(BLOCK), clds, c->stream, X, c->ld, (uint32_t)c->N, c->n, mean_out, c->d_partial);
        profile_mark(c, true);
    }
    hipLaunchKernelGGL(consensus_finish_kernel, dim3(1), dim3(1024), 0, c->stream, c->d_partial, blocks, D_dev);
    SAPS_HIP(c, hipGetLastError());
    return SAPS_OK;
}

saps_status saps_poll_status(saps_ctx* c, int64_t* K_host) {
    if (!c) return SAPS_EINVAL;
    SAPS_HIP(c, hipStreamSynchronize(c->stream));
    int32_t flag = 0;
    SAPS_HIP(c, hipMemcpy(&flag, c->d_flag, sizeof(flag), hipMemcpyDeviceToHost));
    if (K_host) SAPS_HIP(c, hipMemcpy(K_host, c->d_K, sizeof(int64_t), hipMemcpyDeviceToHost));
    if (flag) {
        SAPS_HIP(c, hipMemset(c->d_flag, 0, sizeof(int32_t)));
        return fail(c, SAPS_ECAPACITY, "K exceeded the message capacity; the round was skipped");
    }
    return SAPS_OK;
}

saps_status saps_profile_enable(saps_ctx* c, int32_t on) {
    if (!c) return SAPS_EINVAL;
    c->profiling = on != 0;
    return SAPS_OK;
}

saps_status saps_profile_read(saps_ctx* c, int32_t* launches, double* total_ms) {
    if (!c || !launches || !total_ms) return SAPS_EINVAL;
    SAPS_HIP(c, hipStreamSynchronize(c->stream));
    double sum = 0.0;
    int32_t cnt = 0;
    for (size_t k = 0; k + 1 < c->ev_used; k += 2) {
        float ms = 0.f;
        SAPS_HIP(c, hipEventElapsedTime(&ms, c->ev_pool[k], c->ev_pool[k + 1]));
        sum += ms; ++cnt;
    }
    c->ev_used = 0;
    *launches = cnt; *total_ms = sum;
    return SAPS_OK;
}

saps_status saps_stream_copy(saps_ctx* c, float* dst, const float* src, int64_t count) {
    if (!c) return SAPS_EINVAL;
    if (saps_status ds = check_device(c)) return ds;
    if (!dst || !src || count < 0 || (count & 3) || !aligned16(dst) || !aligned16(src)) return fail(c, SAPS_EINVAL, "copy arguments");
    if (count == 0) return SAPS_OK;
    const int64_t c4 = count / 4;
    const int64_t blocks = (c4 + STREAM_BLOCK - 1) / STREAM_BLOCK;
    if (blocks > 0x7FFFFFFFll) return fail(c, SAPS_EINVAL, "copy too large");
    profile_mark(c, false);
    if (c->nontemporal) hipLaunchKernelGGL(stream_copy_kernel<true>, dim3((uint32_t)blocks), dim3(STREAM_BLOCK), 0, c->stream, dst, src, c4);
    else hipLaunchKernelGGL(stream_copy_kernel<false>, dim3((uint32_t)blocks), dim3(STREAM_BLOCK), 0, c->stream, dst, src, c4);
    profile_mark(c, true);
    SAPS_HIP(c, hipGetLastError());
    return SAPS_OK;
}

saps_status saps_list_probe(saps_ctx* c, float* X, const uint32_t* idx, const int64_t* K_dev, int32_t write_back) {
    if (!c) return SAPS_EINVAL;
    if (saps_status ds = check_device(c)) return ds;
    if (!X || !idx || !K_dev || !aligned16(X) || !aligned16(idx) || (reinterpret_cast<uintptr_t>(K_dev) & 7u))
        return fail(c, SAPS_EINVAL, "X/idx/K null or misaligned");
    if (c->N == 0) return SAPS_OK;
    const dim3 grid(list_grid_x(c), (uint32_t)c->n);
    uint32_t* sink = reinterpret_cast<uint32_t*>(c->d_partial);
    // the in-place variant runs at the residency of the exchange kernel whose yardstick it is
    const uint32_t lds = write_back ? residency_lds_bytes(residency_for(c, 4, (uint64_t)grid.x * grid.y)) : 0u;
    profile_mark(c, false);
    if (!write_back)
        hipLaunchKernelGGL((list_probe_kernel<false, false>), grid, dim3(BLOCK), 0, c->stream, X, c->ld, idx, K_dev, c->msg_ld, (uint32_t)c->N, sink);
    else if (c->stream_scatter)
        hipLaunchKernelGGL((list_probe_kernel<true, true>), grid, dim3(BLOCK), lds, c->stream, X, c->ld, idx, K_dev, c->msg_ld, (uint32_t)c->N, sink);
    else
        hipLaunchKernelGGL((list_probe_kernel<true, false>), grid, dim3(BLOCK), lds, c->stream, X, c->ld, idx, K_dev, c->msg_ld, (uint32_t)c->N, sink);
    profile_mark(c, true);
    SAPS_HIP(c, hipGetLastError());
    return SAPS_OK;
}

}  // extern "C"
