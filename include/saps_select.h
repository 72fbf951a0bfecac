/* saps_select.h — adaptive peer selection of SAPS-PSGD on the host (coordinator side).
 *
 * Implements Alg. 1 line 2 (GetNewConnectedGraph) and Alg. 3 (GenerateGossipMatrix) of the
 * paper: from a bandwidth matrix B, a threshold B_thres and a window T_thres, every round
 * produces a perfect matching of the workers that prefers links with B_ij >= B_thres while
 * keeping the graph of "recently connected" edges (used within the last T_thres rounds)
 * connected.  The result is returned as the permutation peer[] that saps_round() consumes
 * (GenerateW: W_ij = W_ji = 1/2 for matched i, j; W is never materialised).
 *
 * Everything here is HOST code and HOST memory; no GPU is touched.
 *
 * Readings where the paper is silent:
 *   - B is symmetrised as B_ij = B_ji = min(B_ij, B_ji) (Sec. II-C); the diagonal is ignored.
 *   - R (timestamp matrix) starts at "never" for every pair; after each round the matched
 *     pairs get R_ij = R_ji = t.  Edge (i,j) is recently connected at round t iff R_ij > t - T_thres.
 *   - RandomlyMaxMatch = maximum-cardinality matching (Edmonds' blossom algorithm) with the
 *     root order and the neighbour order shuffled by a generator seeded with (seed, t, pass).
 *   - Second pass (GetUnmatch): complete graph on the still unmatched workers.
 *   - Odd n: exactly one worker stays unmatched (peer[i] == i).
 */
#ifndef SAPS_SELECT_H
#define SAPS_SELECT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct saps_selector saps_selector;

/* What a call to saps_selector_next decided (all counts are numbers of pairs). */
typedef struct {
    int32_t rc_connected;     /* 1: recently-connected graph was connected, E = B* (Alg. 3 line 2)      */
    int32_t rc_components;    /* connected components of the recently-connected graph                    */
    int32_t first_pairs;      /* pairs found by the first RandomlyMaxMatch (Alg. 3 line 6)               */
    int32_t second_pairs;     /* pairs added by the second pass over unmatched workers (lines 7-9)      */
    double min_bandwidth;     /* smallest B_ij over the matched pairs: the round's bottleneck link        */
    double mean_bandwidth;    /* mean B_ij over the matched pairs                                         */
} saps_select_info;

/* B: HOST n x n row-major link speeds (any unit).  Returns 0 on success, 1 on bad arguments
 * (null, n < 1, T_thres < 1, NaN in B). */
int32_t saps_selector_create(saps_selector** out, int32_t n, const double* B, double B_thres,
                             int64_t T_thres, uint64_t seed);
int32_t saps_selector_destroy(saps_selector* sel);

/* Alg. 3 for round t (t must increase from call to call).  peer_out: HOST n ints, receives an
 * involution of [0, n).  info may be NULL.  Returns 0, or 1 on bad arguments. */
int32_t saps_selector_next(saps_selector* sel, int64_t t, int32_t* peer_out, saps_select_info* info);

/* Copies the timestamp matrix R (HOST n x n int64, INT64_MIN = never). */
int32_t saps_selector_get_R(const saps_selector* sel, int64_t* R_out);

/* Maximum-cardinality matching of an undirected graph given as a HOST n x n 0/1 matrix E
 * (symmetric use: an edge exists if E_ij or E_ji is non-zero; diagonal ignored), with the
 * search order shuffled from `seed`.  peer_out receives the matching as an involution
 * (unmatched: peer[i] == i).  Returns the number of matched pairs, or -1 on bad arguments. */
int32_t saps_max_matching(int32_t n, const uint8_t* E, uint64_t seed, int32_t* peer_out);

#ifdef __cplusplus
}
#endif
#endif /* SAPS_SELECT_H */
