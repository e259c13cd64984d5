/*
 * saber_measure.h - measurement aids of the MI355X LDA sampler library (not part of the sampling path).
 *
 * Same conventions as saber.h: host pointers unless stated, caller-owned buffers, a negative saber_status on
 * failure with the message in saber_last_error().
 */
#ifndef SABER_MEASURE_H
#define SABER_MEASURE_H

#include "saber.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement aid for the choice between the alias table and the tree (Sec. 3.2.3): builds an alias table (Vose's
 * construction, one thread per row) from the current Bhat row of every word that keeps a dense row, and reports
 * the device time of that build in *ms_build and the number of rows in *rows_built (may be null); the sampler
 * does not use the tables.  For the m words listed (host array; each must keep a dense row, see
 * light_word_tokens) the table is returned in prob[m][K] and alias[m][K] (host): bucket k yields topic k with
 * probability prob, else topic alias.  All memory the call needs is allocated and freed inside it (20 bytes per
 * row and topic; more than 64 GB is refused with SABER_ERANGE). */
int saber_alias_build_probe(saber_ctx *ctx, const int32_t *words, int32_t m, float *prob, int32_t *alias,
                            double *ms_build, int32_t *rows_built);

/* The alias tables of the variant saber_options.ablation bit 2 (Sec. 3.2.3: the alias table as the per-word structure
 * for the dense term instead of the tree), for the m words listed (host array): prob[m][K] and alias[m][K] (host):
 * bucket k yields topic k with probability prob, else topic alias; a dense-branch token with uniform u1 takes bucket
 * floor(u1 K) and keeps the bucket's own topic if the fraction of u1 K is below prob.  The tables are rebuilt after
 * every M-step by one workgroup per word (prefix sums and binary searches instead of Vose's pairing chain).
 * Errors: ESTATE (the context was not created with ablation bit 2), EINVAL, ENOMEM, EDEVICE. */
int saber_get_alias(saber_ctx *ctx, const int32_t *words, int32_t m, float *prob, int32_t *alias);

/* Measurement aid, independent of any context: copies `bytes` bytes device-to-device `reps` times with a
 * plain streaming kernel and reports read+write bandwidth in GB/s (the achievable-HBM yardstick, and the
 * kernel the profiler's FETCH_SIZE / WRITE_SIZE counters are calibrated against). */
int saber_bandwidth_probe(int64_t bytes, int32_t reps, double *gb_per_s);

#ifdef __cplusplus
}
#endif
#endif /* SABER_MEASURE_H */
