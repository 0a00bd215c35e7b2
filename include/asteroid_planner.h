/*
 * asteroid_planner.h -- C ABI of the parallelism planner (Sec. 3.3 "Parallelism Planning").
 *
 * The planner takes the profiler's tables -- per layer l the output size a_l, the weight
 * size w_l and the FP / BP time t_f^{d,l}(beta), t_b^{d,l}(beta) on every device d for every
 * batch size beta, plus device memory budgets u_d and device-to-device bandwidths b_{d,d'}
 * (Sec. 3.3 "DNN Model and Asteroid Profiler", Table 3) -- and returns the hybrid pipeline
 * configuration with the smallest estimated HPP-Round latency: model partition points, device
 * groups and the split of a micro-batch inside every group.
 *
 * Everything here is host code on host memory: every pointer is HOST memory owned by the
 * caller, read (const) or written during the call only; nothing is kept after a call returns.
 * No entry point touches a GPU.  Every function returns an ast_status (asteroid.h); on
 * failure asteroid_last_error() holds a message.  Times are in the unit of the tables, sizes
 * in bytes, bandwidths in bytes per time unit.
 */
#ifndef ASTEROID_PLANNER_H
#define ASTEROID_PLANNER_H

#include <stdint.h>

#include "asteroid.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Planner input (notation of Table 3).
 *   L layers, N devices, micro-batches of B samples, M micro-batches per HPP-Round.
 *   host_tf, host_tb  [N][L][B+1]  time of layer l on device d at batch size beta; entry
 *                                  beta = 0 must be 0.  Not assumed proportional to beta.
 *   host_a    [L]     bytes per sample of the layer's output (what crosses a stage boundary)
 *   host_act  [L]     bytes per sample of activation memory the layer keeps for its backward
 *                     (equal to a_l when a "layer" is a single tensor-producing module)
 *   host_w    [L]     bytes of the layer's parameters
 *   host_u    [N]     memory budget of each device
 *   host_fixed [L]    bytes the layer needs whatever K and beta are (workspace, derived weight copies);
 *                     Eq. (3) has no such term: NULL = none, and the paper's formula is what is evaluated
 *   host_bw   [N][N]  bandwidth between devices (diagonal ignored)
 *   mod_factor, opt_factor: Mem^MOD = mod_factor * sum w_l (2: parameters + accumulated
 *                     gradients), Mem^OPT = opt_factor * sum w_l (1: momentum)   (Eq. (3))
 *   block             samples moved per iteration of the offloading phase of Alg. 1 (>= 1)
 */
typedef struct {
  int32_t L, N, B, M;
  int32_t block;
  double mod_factor, opt_factor;
  const double* host_tf;
  const double* host_tb;
  const double* host_a;
  const double* host_act;
  const double* host_w;
  const double* host_u;
  const double* host_bw;
  const double* host_fixed;
} ast_plan_problem;

/* Eq. (3): footprint in bytes of the stage of layers [lo, hi) with K resident micro-batches of
 * beta samples: mod_factor*W + opt_factor*W + K * beta * sum(act_l) (+ sum(fixed_l) when host_fixed is given).
 * AST_EINVAL on a bad range, K < 1 or beta outside 0..B. */
int32_t asteroid_plan_stage_memory(const ast_plan_problem* pr, int32_t lo, int32_t hi, int32_t K, int32_t beta,
                                   double* bytes);

/* Alg. 1: split the B samples of a micro-batch over the g devices host_group[0..g) (distinct
 * device ids) that replicate layers [lo, hi) with K resident micro-batches.
 * Phase 1 (MemoryAwareBalancing) hands out whole-sample shares in proportion to the capacities
 * v_d of Eq. (9), capped by what fits each budget, re-sharing the remainder among devices with
 * room; phase 2 (StragglerWorkloadOffloading) moves `block` samples at a time from the slowest
 * device to the fastest one with room while that makes the slowest device faster.
 * Writes host_y[0..g) (samples per device, in the order of host_group) and the step's
 * E_f, E_b of Eq. (8).  *feasible = 0 (and nothing else written) when the micro-batch does not
 * fit, or a member cannot hold the replica -- the "Exit with Fail" of Alg. 1. */
int32_t asteroid_plan_allocate(const ast_plan_problem* pr, int32_t lo, int32_t hi, const int32_t* host_group,
                               int32_t g, int32_t K, int32_t* host_y, double* Ef, double* Eb, int32_t* feasible);

/* Eq. (4)-(6): HPP-Round latency of a pipeline given per step (first stage first, execution
 * and communication steps alternating, S odd) E_f^s, E_b^s and T_a^s (0 for communication
 * steps), with M micro-batches.  *dm receives the dominant step: the first step with the
 * largest M*(E_f+E_b) + sum_{i<s}(E_f^i+E_b^i)  (Eq. (11)). */
int32_t asteroid_plan_round_latency(int32_t S, const double* host_Ef, const double* host_Eb, const double* host_Ta,
                                    int32_t M, double* latency, int32_t* dm);

/* Alg. 2: dynamic programme over Q(l, n, p) (Eq. (10)), dominant step by Eq. (11).
 * Devices are ordered by memory budget, largest first (ties keep their order); stage k takes
 * the next host_stage_ndev[k] devices of that order.  Outputs:
 *   *P                     number of stages (0 when no configuration fits: *latency = +inf)
 *   host_stage_lo  [N+1]   first layer of each stage; host_stage_lo[*P] = L
 *   host_stage_ndev[N]     devices per stage
 *   host_dev_order [N]     device ids in memory order
 *   host_y         [N]     samples of a micro-batch per device, indexed by device id
 *   *latency               estimated HPP-Round latency, Eq. (4)
 * The head stage of a sub-pipeline of p stages is planned with K = 2p - 1 resident
 * micro-batches (Sec. 3.2).  Cost: O(min(L,N) * N^2 * L^2) stage evaluations. */
int32_t asteroid_plan_hpp(const ast_plan_problem* pr, int32_t* P, int32_t* host_stage_lo, int32_t* host_stage_ndev,
                          int32_t* host_dev_order, int32_t* host_y, double* latency);

#ifdef __cplusplus
}
#endif
#endif
