/* saps.h — C ABI of the MI355X (gfx950) library for one SAPS-PSGD round.
 *
 * The library holds the models of all n workers as one n x ld fp32 matrix in the HBM
 * of one GPU (row i = worker i, the paper's column x^(i) of X, Sec. III) and performs
 * the per-round numeric work of Alg. 2 (worker side) on all rows at once:
 *
 *   local step      Alg. 2 line 5 / procedure SGD:  x <- x - gamma * grad
 *                   (with an optional heavy-ball momentum buffer v, which the paper
 *                   does not have: v <- mu*v + g ; x <- x - lr*v)
 *   random mask     Sec. II-B, Eq. (3): m[j] = 1 with probability 1/c, the same on all
 *                   workers because every worker derives it from the round's seed
 *   sparsify        Eq. (2): x~ = x o m; only the non-zeros travel (packed, ascending j)
 *   exchange+merge  Alg. 2 lines 8-10 with GenerateW's weights (1/2, 1/2): masked
 *                   coordinates of two matched workers become the mean of the two,
 *                   all other coordinates keep their value (Eq. (7))
 *
 * Entry points of the method: saps_sgd_step, saps_mask_compact, saps_merge, saps_round (saps_round_ex,
 * saps_round_static are variants of the last), saps_consensus.  Everything after saps_last_error() in this
 * header (tuning knobs, event brackets, the two bandwidth yardsticks) is measurement tooling.
 *
 * The mask is never stored.  Coordinate j of round t is kept iff
 *     Philox4x32-10(key = (lo32 seed, hi32 seed),
 *                   ctr = (lo32(j>>2), hi32(j>>2), lo32 t, hi32 t))[j & 3]  <  floor(2^32 / c_s)
 * where s is the segment that contains j (64-bit compare; c_s = 1 keeps everything).
 *
 * Conventions
 *   - X, G, V, msg, idx, K_dev are DEVICE pointers owned by the caller, 16-byte aligned;
 *     the library keeps none of them after a call returns.  peer, seg_off, seg_c are HOST
 *     pointers, copied during the call.
 *   - X, G, V share the row stride ld (floats), ld >= N, ld % 4 == 0.  Columns [N, ld) are
 *     never read or written.  A stride that is a multiple of 64 floats (rows 256-byte aligned) is
 *     recommended: the fused round measured 12 % slower with rows that are only 16-byte aligned.  msg has row stride msg_ld (the capacity given at creation).
 *   - All work is enqueued on the HIP stream given to saps_create(); calls return without
 *     waiting for the GPU.  Calls on one context must not overlap from several threads.
 *   - K (number of kept coordinates of the round) is known only on the device.  If K exceeds
 *     the capacity msg_ld the round's kernels write NOTHING to X, V, msg, idx (K_dev is
 *     still written) and a sticky flag is raised that saps_poll_status() reports.
 *   - A context belongs to the device that was current in saps_create(); calling an entry point
 *     with another device current returns SAPS_EINVAL.
 *   - Host-detectable errors are returned immediately and nothing is enqueued.
 *   - X, G, V, msg, idx must not alias.
 *   - Limits: 1 <= n <= 65535, 0 <= N <= 0xFFFF0000, n_seg >= 1.
 */
#ifndef SAPS_H
#define SAPS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct saps_ctx saps_ctx; /* opaque; owns private device scratch only */

typedef enum {
    SAPS_OK = 0,
    SAPS_EINVAL = 1,    /* null / misaligned pointer, bad size, ld < N, ld % 4, bad segments, c < 1 */
    SAPS_EMATCH = 2,    /* peer[] out of range or not an involution                              */
    SAPS_ECAPACITY = 3, /* K > msg_ld: the round was skipped on the device (see saps_poll_status) */
    SAPS_EHIP = 4       /* a HIP runtime call failed; text in saps_last_error()                   */
} saps_status;

/* Shape of the model matrix and of the per-segment compression ratios (Sec. II-B uses one
 * c for the whole model: n_seg = 1).  seg_off has n_seg+1 non-decreasing entries with
 * seg_off[0] = 0 and seg_off[n_seg] = N; seg_c[s] >= 1 is the ratio c of segment s. */
typedef struct {
    int32_t n;             /* workers (rows)                         */
    int64_t N;             /* coordinates per model                  */
    int64_t ld;            /* row stride of X, G, V in floats        */
    int32_t n_seg;         /* number of segments                     */
    const int64_t* seg_off; /* HOST, n_seg + 1 entries               */
    const double* seg_c;    /* HOST, n_seg entries                   */
} saps_layout;

/* Creates a context for one layout.  msg_ld = capacity of a packed message row (floats,
 * multiple of 4, >= 0).  hip_stream = hipStream_t to enqueue on (NULL = default stream).
 * Allocates the private scratch (about 20 bytes per 256 coordinates: three sets of tile and group counts and
 * the list of dense tiles; plus 4*msg_ld and 16*n bytes). */
saps_status saps_create(saps_ctx** out, const saps_layout* layout, int64_t msg_ld, void* hip_stream);
saps_status saps_destroy(saps_ctx* ctx);

/* Local step of Alg. 2 line 5 on every row:  v = fma(mu, v, g); x = fma(-lr, v, x)
 * (two correctly rounded fp32 fused multiply-adds).  V == NULL is allowed iff mu == 0 and
 * gives the paper's plain x = fma(-lr, g, x).  X and V are updated in place. */
saps_status saps_sgd_step(saps_ctx* ctx, float* X, const float* G, float* V, float lr, float mu);

/* Eq. (3) + Eq. (2): generates the round's mask, writes the ascending list of kept
 * coordinates idx[0..K), the packed rows msg[i*msg_ld + k] = X[i*ld + idx[k]] and *K_dev = K.
 * X is read only.  K_dev is a device int64. */
saps_status saps_mask_compact(saps_ctx* ctx, const float* X, uint64_t seed, uint64_t round,
                              uint32_t* idx, float* msg, int64_t* K_dev);

/* Alg. 2 line 10 (averaging) for the matching peer[] (HOST, n entries, peer[peer[i]] == i;
 * peer[i] == i leaves row i untouched):  X[i*ld + idx[k]] = (msg[i][k] + msg[peer[i]][k]) * 0.5f
 * for k < *K_dev.  idx, msg, K_dev as written by saps_mask_compact. */
saps_status saps_merge(saps_ctx* ctx, float* X, const int32_t* peer, const uint32_t* idx,
                       const float* msg, const int64_t* K_dev);

/* One whole round in Alg. 2 order, bit-identical to
 *   saps_sgd_step; saps_mask_compact; saps_merge
 * but with every element of X, G, V read once and X, V written once.  G == NULL skips the
 * local step (exchange-only round; V, lr, mu ignored).  idx, msg, K_dev may each be NULL
 * when the caller does not need that output; the capacity rule (K > msg_ld skips the round)
 * holds all the same, so msg_ld must cover K even then.
 * Rounds are normally called with round = 1, 2, 3, ... and one seed: the kernels of a call therefore also count
 * the kept coordinates of (seed, round + 1) on the side, and a next call with exactly that pair starts without
 * the counting launch.  Any other pair simply counts for itself; results never depend on this.  Calls made
 * under stream capture neither use nor produce such counts (a replay cannot know what ran before it). */
saps_status saps_round(saps_ctx* ctx, float* X, const float* G, float* V, float lr, float mu,
                       uint64_t seed, uint64_t round, const int32_t* peer,
                       uint32_t* idx, float* msg, int64_t* K_dev);

/* saps_round with options.  flags = 0 is saps_round.  SAPS_ROUND_MIX_THEN_STEP selects the order of
 * Eq. (7): X_{t+1} = X_t o notM + (X_t o M) W - gamma G(X_t), i.e. the models of the start of the
 * round are packed and averaged and the local step computed from G is subtracted afterwards
 * (bit-identical to saps_mask_compact; saps_merge; saps_sgd_step).  The packed messages then carry
 * the values before the step.  Without gradients (G == NULL) both orders coincide. */
enum { SAPS_ROUND_MIX_THEN_STEP = 1u };
/* Several local steps between exchanges (communication period tau > 1): a step without exchange is a
 * round with W_t = I, for which Alg. 2 and Eq. (7) both reduce to the local step.  Per period call
 * saps_sgd_step() tau - 1 times (fresh gradients each time), then saps_round() - or saps_round_ex() with
 * SAPS_ROUND_MIX_THEN_STEP - with the gradients of the period's last step.  The momentum buffer V runs
 * through local steps and rounds alike.  Only the exchanging call consumes a (seed, round) pair. */
saps_status saps_round_ex(saps_ctx* ctx, float* X, const float* G, float* V, float lr, float mu,
                          uint64_t seed, uint64_t round, const int32_t* peer,
                          uint32_t* idx, float* msg, int64_t* K_dev, uint32_t flags);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  saps_round() without a context, for a model with ONE compression
 * ratio c (the paper's case, n_seg = 1): the private scratch that saps_create() would allocate (tile and
 * group counts, K, an index list) lives in a fixed device array inside the library instead, about 3.1 MiB
 * per GPU the library runs on, held until the process ends.  Calls no hipMalloc / hipFree and nothing
 * that allocates; only kernels are enqueued on hip_stream (no memset, no copy, no event), so a call can
 * be recorded into a graph.  The first call on a device looks up that device's copy of the array
 * (hipGetSymbolAddress): make one call outside a capture first.
 *   Arguments as saps_round(); n, N, ld, c, msg_ld as in saps_layout / saps_create().
 *   Limits (SAPS_EINVAL beyond them): N <= 67,108,864; at most 128 units in the matching (pairs plus
 *   unmatched workers, i.e. n <= 256 when everyone is matched); K_dev must not be NULL (there is no context
 *   to poll: *K_dev > msg_ld tells the caller that the round was skipped and nothing was written);
 *   idx == NULL needs msg_ld <= 524,288.
 *   All calls on one GPU share the one scratch array: calls that overlap on a GPU (two streams, two
 *   threads) race.  Results are bit-identical to saps_round() on a context of the same layout.
 *   Error text: saps_last_error(NULL) (per thread). */
saps_status saps_round_static(int32_t n, int64_t N, int64_t ld, double c, int64_t msg_ld, void* hip_stream,
                              float* X, const float* G, float* V, float lr, float mu,
                              uint64_t seed, uint64_t round, const int32_t* peer,
                              uint32_t* idx, float* msg, int64_t* K_dev);

/* Consensus diagnostics (Sec. II-C: consensus means that the workers' distance to the average
 * model goes to zero; Theorem 1 bounds sum_i ||mean - x_i||^2).  Writes the average model
 * mean_out[j] = (1/n) sum_i X[i][j] (device, N floats, may be NULL) and the total disagreement
 * *D_dev = sum_i sum_j (X[i][j] - mean[j])^2 (device double, 8-byte aligned), accumulated in fp64
 * in a fixed order, so repeated calls give identical bits.  X is read once and not modified. */
saps_status saps_consensus(saps_ctx* ctx, const float* X, float* mean_out, double* D_dev);

/* Waits for the context's stream, returns SAPS_ECAPACITY if any call since the last poll
 * was skipped for K > msg_ld (and clears that flag), else SAPS_OK.  If K_host != NULL it
 * receives the K of the most recent mask generation. */
saps_status saps_poll_status(saps_ctx* ctx, int64_t* K_host);

/* Text of the last host-side error on this context (never NULL); ctx == NULL gives the calling
 * thread's last saps_round_static() error. */
const char* saps_last_error(const saps_ctx* ctx);

/* Launch-shape knobs for measurement sweeps; results never depend on them.
 * Unknown knob or out-of-range value: SAPS_EINVAL. */
enum {
    SAPS_TUNE_PAIRS_PER_BLOCK = 0, /* fused round: matched pairs handled per workgroup: 1, 2, 4, 8 */
    SAPS_TUNE_XCD_REMAP = 1,       /* fused round: 0 = tiles in launch order, 1 = contiguous tile range per XCD */
    SAPS_TUNE_NONTEMPORAL = 2,     /* fused round and local step: 0 = plain, 1 = non-temporal loads/stores */
    SAPS_TUNE_EXCHANGE_PATH = 3,   /* exchange-only round: 0 = built-in choice by expected density, 1 = index list, 2 = tile walk,
                                      3 = index list, but whole tiles that keep at least every 12th coordinate are streamed */
    SAPS_TUNE_BLOCKS_PER_CU = 4,   /* fused round, list exchange, local step, consensus: resident workgroups per compute unit, 3..32 (rounded up to the next
                                      count that the LDS granules admit: 1..12, 14, 16, 18, 21, 25, 32), 0 = no limit, -1 = built-in
                                      choice (a measured cap per kernel for long grids, no limit for short ones) */
    SAPS_TUNE_PREPARE_NEXT = 5,    /* saps_round: 1 (default) = the kernels of round t also count the kept coordinates of round t + 1, 0 = never */
    SAPS_TUNE_ROW_PER_WAVE = 6     /* fused round with update: a workgroup's two waves take one row of the pair each (1, default: when there is a
                                      momentum buffer; 2: always) or every wave takes both rows (0) */
};
saps_status saps_set_tuning(saps_ctx* ctx, int32_t knob, int32_t value);

/* Per-kernel timing for benchmarks.  saps_profile_enable(ctx, 1) makes every following
 * saps_round / saps_sgd_step / saps_consensus / saps_stream_copy / saps_list_probe bracket its dominant kernel (the fused
 * round kernel, the list exchange kernel, the update kernel, the consensus kernel, the copy kernel) with a pair of
 * HIP events on the context's stream (at most 4096 pairs are kept; later launches are not
 * recorded).  saps_profile_read waits for the stream, returns the number of recorded
 * launches and the sum of their durations in milliseconds, and forgets them. */
saps_status saps_profile_enable(saps_ctx* ctx, int32_t on);
saps_status saps_profile_read(saps_ctx* ctx, int32_t* launches, double* total_ms);

/* Plain device-to-device streaming copy of `count` floats (16-byte aligned, count % 4 == 0)
 * with the same access shape as the round kernels: the bandwidth yardstick of the
 * benchmark and the scale reference for profiler byte counters.  Not part of the method. */
saps_status saps_stream_copy(saps_ctx* ctx, float* dst, const float* src, int64_t count);

/* Yardstick of the index-list kernels, the counterpart of saps_stream_copy() for isolated accesses: every
 * one of the n rows reads the 4-byte word at each of the coordinates idx[0..*K_dev) (as written by
 * saps_mask_compact / saps_round); with write_back != 0 the same bits are stored back in place with the
 * store policy the exchange uses for this layout, so X is unchanged either way.  No averaging and no
 * messages: the time of this call is what the memory system needs for the exchange's access pattern.
 * Entries >= N are skipped; *K_dev > msg_ld does nothing.  Not part of the method. */
saps_status saps_list_probe(saps_ctx* ctx, float* X, const uint32_t* idx, const int64_t* K_dev, int32_t write_back);

/* Library ABI version (bumped when a signature changes). */
int32_t saps_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SAPS_H */
