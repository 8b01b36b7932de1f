/*
 * plora_plan.h - C ABI of the packing planner: which LoRA configurations to train together, on how many
 * GPUs, and in which order (paper section 3.2; appendices A, B, D).  Host only: every pointer here is HOST
 * memory, no call touches a device.  The calls are pure functions of their arguments (no state, thread-safe).
 *
 * Notation of the paper: K the set of configurations, r_k the rank of configuration k, M_lora,k its memory,
 * M_base the base model's, M_gpu a GPU's capacity and C the load factor, G the GPUs, d_j the parallel degree of
 * job j (a power of two), T() the duration of a job as a cost model estimates it.
 *
 * The cost model is the caller's, in the form the packed execution has (the base model's share of an iteration
 * grows with the packed tokens, every adapter adds its own low-rank work): for degree d = 2^i and a set H,
 *     T(H, d) = t_base[i] + sum_{k in H} t_config[i][k].
 * bench.py shows how to fill it from measured kernel times.
 */
#ifndef PLORA_PLAN_H
#define PLORA_PLAN_H

#include <stddef.h>
#include <stdint.h>

#include "plora.h"

#ifdef __cplusplus
extern "C" {
#endif

#define PLORA_PLAN_MAX_CONFIGS 4096
#define PLORA_PLAN_MAX_DEGREES 8          /* degrees 1, 2, 4, .. 128 */

/* ---- memory model (appendix B) -------------------------------------------------------------------------- */

/* The seven projections that can carry an adapter, in the bit order of plora_plan_lora.targets. */
enum { PLORA_PROJ_Q = 0, PLORA_PROJ_K, PLORA_PROJ_V, PLORA_PROJ_O, PLORA_PROJ_UP, PLORA_PROJ_GATE, PLORA_PROJ_DOWN };

typedef struct {
    int32_t n_layers;
    int64_t hidden;               /* model width: h_in of q, k, v, o, up, gate; h_out of q, o, down      */
    int64_t kv_hidden;            /* h_out of k and v (grouped-query attention)                           */
    int64_t inter;                /* MLP width: h_out of up and gate, h_in of down                        */
    double c_prec;                /* bytes per parameter                                                  */
    double c_grad;                /* gradient-sized buffers per parameter (3 for AdamW: gradient, momentum,
                                     velocity)                                                            */
} plora_plan_model;

typedef struct {
    int32_t rank, batch, seq;     /* r, b, s                                                              */
    uint32_t targets;             /* bit i set: projection i carries an adapter                           */
} plora_plan_lora;

typedef struct {
    int32_t zero_level;           /* 0: nothing sharded by FSDP; 1, 2, 3: the ZeRO levels                  */
    int32_t d_tp, d_pp, d_fsdp;   /* tensor-, pipeline-, FSDP-parallel degrees, each >= 1                  */
} plora_plan_sharding;

/*
 * M_lora,k on one device (appendix B): parameters n_layers (h_in r + h_out r) c_prec over the targeted projections,
 * divided by d_tp d_pp; c_grad gradient-sized buffers (one gradient, c_grad - 1 of optimizer state), sharded by
 * d_fsdp as the ZeRO level says; activations b s r c_prec per layer and targeted projection.  sharding NULL: one
 * device.  Returns a negative number for invalid arguments.
 */
double plora_plan_lora_bytes(const plora_plan_model *model, const plora_plan_lora *cfg, const plora_plan_sharding *sharding);

/* ---- packing and scheduling (section 3.2) ----------------------------------------------------------------- */

typedef struct {
    int32_t n_configs;            /* |K|, 1 .. PLORA_PLAN_MAX_CONFIGS                                      */
    int32_t n_degrees;            /* degrees 2^0 .. 2^(n_degrees - 1), 1 .. PLORA_PLAN_MAX_DEGREES         */
    const int32_t *rank;          /* [n_configs] r_k >= 1                                                  */
    const double *mem;            /* [n_configs] M_lora,k >= 0                                             */
    double mem_base;              /* M_base >= 0                                                           */
    double mem_gpu;               /* M_gpu > 0                                                             */
    double load;                  /* C in (0, 1]                                                           */
    const double *t_base;         /* [n_degrees] >= 0                                                      */
    const double *t_config;       /* [n_degrees][n_configs] > 0                                            */
} plora_plan_problem;

/* One packed job.  Its configurations are configs_out[first .. first + count) of the call that returned it. */
typedef struct {
    int32_t first, count;
    int32_t gpus;                 /* d_j                                                                   */
    int32_t proved;               /* 1: the packing is proved optimal; 0: the search hit its node limit and this is the
                                     best packing found                                                    */
    double value;                 /* its F: sum of ranks / duration                                        */
    double start, end;            /* plora_plan_schedule only                                              */
} plora_plan_job;

/*
 * F(D, K) with the degree fixed (section 3.2): among the non-empty subsets H of the available configurations with
 * M_base + sum M_lora,k <= C M_gpu D, one that maximises sum_k H_k r_k / T(H, D).  Solved exactly (a fractional
 * 0-1 programme: parametric search over the ratio, each step a 0-1 knapsack by branch and bound), up to a node
 * limit of 2^26 per knapsack.
 *   avail        [n_configs] nonzero: the configuration is still to be scheduled; NULL: all are
 *   configs_out  [n_configs] receives the chosen configurations in increasing order
 *   job_out      first = 0, count, gpus = 2^degree_index, value, proved; count = 0 if nothing fits
 * Errors: PLORA_ERR_NULL, PLORA_ERR_SHAPE (sizes or values outside the ranges above, degree_index out of range).
 */
plora_status plora_plan_pack(const plora_plan_problem *p, int32_t degree_index, const uint8_t *avail,
                             int32_t *configs_out, plora_plan_job *job_out);

/*
 * Decomposed throughput maximisation (Alg. 1) on `gpus` free GPUs: the recursion over the degrees g' = 2^floor(log2 g),
 * g'/2, .., 1 (capped by n_degrees), each step packing one job with F and recursing on what is left; of the
 * candidate sets of concurrent jobs, the one with the largest total throughput sum_j F_j (the first in the order
 * of the recursion wins a tie).  A degree at which nothing fits packs no job.
 *   jobs_out [jobs_cap], configs_out [n_configs], *n_jobs_out: the jobs in the order they were packed.
 * Errors as above; PLORA_ERR_WORKSPACE if jobs_cap is too small (gpus jobs always suffice).
 */
plora_status plora_plan_dtm(const plora_plan_problem *p, int32_t gpus, const uint8_t *avail, plora_plan_job *jobs_out,
                            int32_t jobs_cap, int32_t *n_jobs_out, int32_t *configs_out);

typedef struct {
    double makespan;              /* F of appendix D: the latest end                                       */
    double gpu_work;              /* W = sum_j d_j T_j; makespan >= W / G                                   */
    double tail_bound;            /* appendix D: F / (F - T_last (G - D) / G) for the job that ends last    */
    int32_t n_jobs;
    int32_t n_unscheduled;        /* configurations that fit no degree: configs_out[n_configs - n_unscheduled ..) */
    int32_t all_proved;           /* 1: every packing in the schedule is proved optimal                     */
} plora_plan_summary;

/*
 * The job planner (Alg. 2): whenever GPUs are free, DTM on the free GPUs and the remaining configurations; the jobs
 * start at once; time then moves to the next completion (jobs that end together free their GPUs together).
 *   jobs_out [jobs_cap] in starting order with start and end; n_configs jobs always suffice.
 * Errors as above.
 */
plora_status plora_plan_schedule(const plora_plan_problem *p, int32_t gpus, plora_plan_job *jobs_out, int32_t jobs_cap,
                                 int32_t *configs_out, plora_plan_summary *summary_out);

#ifdef __cplusplus
}
#endif
#endif /* PLORA_PLAN_H */
