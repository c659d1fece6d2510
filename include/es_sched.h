/*
 * libes - scheduler-side planning: the analytical performance model of the
 * intra-job scheduler's companion module (paper §3.4, Eq. 1a-1d) and the search
 * for EST-to-GPU mapping configurations under it.
 *
 * HOST-only arithmetic: no call in this header touches a device, none needs a
 * handle, all pointers are HOST pointers owned by the caller, nothing is kept
 * between calls, and every call is safe from any thread.  Status codes are
 * those of es.h (ES_OK, ES_EINVAL, ES_ENOMEM).
 *
 * Model (§3.4).  A job may use N[i] GPUs of type i; one GPU of type i runs C[i]
 * mini-batches per second of this workload and is given at most A[i] ESTs (one
 * mini-batch per EST per global step); the developer fixed the number of
 * logical workers at maxP.
 *
 *   Eq. 1a  nEST       = sum_i N[i] * A[i],            nEST >= maxP
 *   Eq. 1b  f_overload = max over used types of A[i] / C[i]   (seconds per global
 *                        step: training is synchronous, the most loaded type
 *                        holds every GPU back)
 *   Eq. 1c  waste      = sum over used types of idle capability
 *                        + (nEST - maxP) / f_overload
 *   Eq. 1d  throughput = sum_i N[i] * C[i] - waste
 *
 * Reading of Eq. 1c.  The printed sum has the term C[i] - A[i]/f_overload once
 * per TYPE although Eq. 1a and 1d count every GPU.  ES_SCHED_WASTE_PER_GPU
 * weights the term by N[i]; the model is then consistent with itself (the
 * estimate equals maxP / f_overload: the useful mini-batches of a global step
 * over its duration).  ES_SCHED_WASTE_AS_PRINTED evaluates the sum as printed;
 * with several GPUs of an under-loaded type it estimates more than
 * nEST / f_overload, which no plan can deliver.  The searches below rank by
 * f_overload and therefore do not depend on the reading; the figures they
 * report use ES_SCHED_WASTE_PER_GPU.
 *
 * All arithmetic is IEEE double; quotients A[i]/C[i] are single divisions, so
 * equal ratios compare equal.
 */
#ifndef ES_SCHED_H
#define ES_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ES_SCHED_MAX_TYPES 8        /* GPU types per job */
#define ES_SCHED_MAX_P     4096     /* largest maxP the searches accept */

enum {
    ES_SCHED_WASTE_PER_GPU    = 0,
    ES_SCHED_WASTE_AS_PRINTED = 1
};

/* One plan of the plan database (§3.4: quantity of GPUs, mapping, estimate). */
typedef struct es_sched_plan {
    uint32_t n_used[ES_SCHED_MAX_TYPES];        /* N[i]; entries >= n_types are 0 */
    uint32_t est_per_gpu[ES_SCHED_MAX_TYPES];   /* A[i]; 0 where N[i] = 0 */
    uint32_t n_gpus;                            /* sum_i N[i] */
    uint32_t n_est;                             /* Eq. 1a */
    double   f_overload;                        /* Eq. 1b */
    double   waste;                             /* Eq. 1c */
    double   throughput;                        /* Eq. 1d, mini-batches per second */
} es_sched_plan;

/*
 * Eq. 1a-1d for one given configuration.
 *   n_types       1 .. ES_SCHED_MAX_TYPES
 *   capability    C[i], finite and > 0, n_types entries
 *   n_used        N[i] <= 65535, at least one > 0
 *   est_per_gpu   A[i] in 1 .. 65535 where N[i] > 0 (ignored elsewhere)
 *   max_p         1 .. 65535; nEST < max_p is ES_EINVAL (Eq. 1a's constraint)
 *   waste_reading ES_SCHED_WASTE_PER_GPU or ES_SCHED_WASTE_AS_PRINTED
 * *out is written only on ES_OK.
 */
int es_sched_evaluate(uint32_t n_types, const double* capability, const uint32_t* n_used,
                      const uint32_t* est_per_gpu, uint32_t max_p, int waste_reading,
                      es_sched_plan* out);

/*
 * The best allocation A for fixed GPU counts (the scheduler's role 1, §3.4: under
 * the current resources apply the configuration with the highest estimate).
 * Among all integer A[i] >= 1 on the used types with nEST >= max_p: the smallest
 * f_overload (= the highest estimate), then the smallest nEST (least
 * over-provisioning), then the lexicographically smallest A.
 *   max_p   1 .. ES_SCHED_MAX_P
 * ES_EINVAL also when no GPU is used or the GPUs outnumber the ESTs (a GPU
 * without an EST is no part of a plan).
 */
int es_sched_best_mapping(uint32_t n_types, const double* capability, const uint32_t* n_used,
                          uint32_t max_p, es_sched_plan* out);

/*
 * The plan database (§3.4): for every choice of GPU counts 0 <= N[i] <=
 * available[i] with 1 <= sum N[i] <= max_p its best mapping, ranked by
 * f_overload ascending (highest estimate first), then fewer GPUs, then smaller
 * nEST, then lexicographically smaller N, then A.  The first min(top_k, number
 * of plans) are written to out; *n_out receives how many.
 *   available  n_types entries; the product of (available[i] + 1) must not
 *              exceed 2^20, and that product times max_p must not exceed 2^27
 *              (ES_EINVAL otherwise).  Cost: one best-mapping search per count
 *              vector, each on the order of n_types * max_p steps; measured on one
 *              host core 0.4 s for 70,784 vectors at max_p = 1024, so the bound
 *              keeps a call to a few seconds.  A scheduler that needs a larger space
 *              enumerates it in slices (fix the count of one type per call).
 *   top_k      >= 1; out must hold top_k entries
 */
int es_sched_enumerate(uint32_t n_types, const double* capability, const uint32_t* available,
                       uint32_t max_p, uint32_t top_k, es_sched_plan* out, uint32_t* n_out);

/*
 * The EST-to-worker mapping of a plan, in the form es_set_grouping takes.
 * Workers are the plan's GPUs in type order, each with a quota of A[type] ESTs;
 * the nEST - max_p over-provisioned places are given back one at a time, going
 * over the GPUs from the last to the first again and again, never emptying
 * one; virtual ranks 0 .. max_p-1 are then dealt out contiguously.
 *   plan           n_used and est_per_gpu are read (the other fields are not)
 *   worker_of_est, slot_of_est   max_p entries each, written on ES_OK
 *   n_workers      receives sum N[i]
 * ES_EINVAL if the plan holds fewer than max_p places or more GPUs than ESTs.
 */
int es_sched_grouping(uint32_t n_types, const es_sched_plan* plan, uint32_t max_p,
                      uint32_t* worker_of_est, uint32_t* slot_of_est, uint32_t* n_workers);

#ifdef __cplusplus
}
#endif
#endif /* ES_SCHED_H */
