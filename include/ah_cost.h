/*
 * ah_cost.h — host-side arithmetic of the paper's cost model over the numbers
 * that ah_stage_profile measures (C ABI, part of libahstage.so; no GPU calls).
 *
 * All arrays are host memory owned by the caller; every function returns an
 * ah_status_t (see ah_stage.h): AH_EINVAL for NULL pointers or sizes out of
 * range, AH_EUNSUPPORTED when no assignment satisfies the constraints.
 */
#ifndef AH_COST_H
#define AH_COST_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Section III-D, Eq. 5: time of n layers estimated from the times profiled for 1, 2, 4, ... layers:
 * T(n) = sum over the set bits i of n of t_pow2[i], with k = floor(log2 n) < n_pow2. */
int ah_cost_layers_time(int n, const double* t_pow2, int n_pow2, double* out);

/* Section III-A, Eq. 1 for one data-parallel group under the 1F1B schedule: sum of the P stage
 * times (one micro-batch, forward + backward) plus (K - 1) times the slowest stage. */
int ah_cost_pipeline_time(const double* t_stage, int P, int K, double* out);

/* Eq. 1: iteration time = max over the groups of ah_cost_pipeline_time, plus t_sync.
 * t_stage holds the groups' stage times back to back; stages[j] is group j's stage count. */
int ah_cost_iteration_time(const double* t_stage, const int* stages, int n_groups, int K, double t_sync, double* out);

/* Idle share of every stage of one group (Section II-D's toy example): stage i is busy K * t_i of
 * the group's pipeline time.  idle[P] and *mean_idle are outputs (mean_idle may be NULL). */
int ah_cost_idle_fractions(const double* t_stage, int P, int K, double* idle, double* mean_idle);

/* Section III-C, Eq. 4, read as balancing time: choose l_i >= 1 layers per stage with sum l_i =
 * n_layers minimising max_i l_i * t_layer[i] (t_layer[i] = time of one layer on stage i's GPU, i.e.
 * the reciprocal of its computing power) subject to the memory constraint of Eq. 4c,
 *   l_i * (fixed_bytes_per_layer + act_bytes_per_layer * in_flight[i]) <= mem_bytes[i].
 * Among optimal assignments the one returned gives surplus layers to earlier stages first.
 * l_out[P] and *bottleneck (the minimised maximum) are outputs. */
int ah_cost_partition_layers(int P, int n_layers, const double* t_layer, const double* mem_bytes,
                             double fixed_bytes_per_layer, double act_bytes_per_layer, const int* in_flight,
                             int* l_out, double* bottleneck);

#ifdef __cplusplus
}
#endif
#endif /* AH_COST_H */
