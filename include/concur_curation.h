/*
 * concur_curation.h -- the paper's metrics and data-curation rules as a small host-only C ABI
 * (no GPU work; part of libgqa_decode.so).  All pointers are HOST pointers.
 *
 * One record = one generation (a kernel with its reasoning trace) for one task.
 */
#ifndef CONCUR_CURATION_H
#define CONCUR_CURATION_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Equation 1: speedup[i] = t_torch[i] / t_kernel[i] if correct[i], else 0.  Returns 0, or -1 on a
 * null pointer / negative n / a correct record with t_kernel <= 0. */
int concur_speedup(int64_t n, const double* t_torch, const double* t_kernel, const uint8_t* correct,
                   double* speedup);

/* Equation 2: fast_p = (1/N) * #{ i : speedup[i] > p } over N tasks (one speedup per task).
 * Returns NaN for n <= 0 or a null pointer. */
double concur_fast_p(int64_t n_tasks, const double* speedup, double p);

/* Section 4.2: pass@k per task = 1 if at least one of its k trials is correct (Exec), or has
 * speedup > 1 (fast_1).  flags[t*k + j] / speedup[t*k + j].  Returns the fraction of tasks passing. */
double concur_exec_pass_at_k(int64_t n_tasks, int32_t k, const uint8_t* correct);
double concur_fast1_pass_at_k(int64_t n_tasks, int32_t k, const double* speedup);

/* Equation 3: ARL = (1 / (N M)) * sum_i sum_j L[i*M + j].  NaN for empty input. */
double concur_arl(int64_t n_tasks, int32_t m, const int32_t* lengths);

/* Section 6: difficulty bin of a task from its average reasoning length:
 * 0 = easy (ARL < lo), 1 = medium (lo <= ARL <= hi), 2 = hard (ARL > hi); the paper uses 4000 / 8500. */
int concur_difficulty_bins(int64_t n_tasks, const double* task_arl, double lo, double hi, int32_t* bin);

/*
 * Section 3.5, the three parts of the curated set.  Records of one task need not be adjacent.
 *   (a) per task: the generation with the shortest reasoning (ties: lowest index) is taken iff it is
 *       correct (speedup > 0) and no other generation of the task has a larger speedup;
 *   (b) every record with speedup > speedup_threshold (the paper: 5);
 *   (c) up to single_op_quota further records (the paper: 544) that are correct single-operator
 *       samples not taken by (a) or (b), shortest reasoning first (ties: lowest index).
 * The paper does not say how the (c) samples are chosen; shortest-first follows its preference for
 * concise traces.  selected[i] receives a bit mask: 1 = rule (a), 2 = rule (b), 4 = rule (c)
 * (a record can carry bits 1 and 2).  counts[3] receives the number of records with bit 1, with
 * bit 2 but not bit 1, and with bit 4.  Returns the total number selected, or -1 on bad arguments.
 */
int64_t concur_select(int64_t n, const int64_t* task_id, const double* speedup, const int32_t* reasoning_len,
                      const uint8_t* single_op, double speedup_threshold, int64_t single_op_quota,
                      uint8_t* selected, int64_t counts[3]);

#ifdef __cplusplus
}
#endif
#endif
