/*
 * Cache provisioning of the LoRA Server for the tail-TTFT target (Sec. 4.2).  Host code only:
 * every pointer below is ordinary process memory, nothing touches a GPU.
 *
 * Sec. 4.2 reduces the P95 TTFT target to an Immediate Admissibility Rate: a request is
 * admitted at once if its adapter is resident or a free slot exists.  With invocation
 * probabilities p_i (i = 1..N), global batch size LB = L * B and cache capacity M:
 *   lambda_i = LB * p_i;
 *   q_i = Pr[Poisson(lambda_i) > tau*]                                   (Eq. 2)
 *   tau* such that sum_i q_i = M                                          (Eq. 3)
 *   IAR(M) = sum_i p_i [ q_i + (1 - q_i) P_free(i) ]                      (Eq. 4)
 *   P_free(i) = Pr[at most M - 1 of the adapters j != i are resident], each independently
 *               with probability q_j;
 *   M* = min { M in 1..N : IAR(M) >= alpha }                              (Eq. 1, Algorithm 1)
 * The Poisson tail is continued to real tau >= -1 by the regularized incomplete gamma
 * function (equal to Eq. 2 at the integers), so that Eq. 3 has a solution for every M below
 * the number of adapters with p_i > 0; from that number on every such adapter is resident.
 *
 * All functions return LORA_PROVISION_OK or a negative code and write nothing on error.
 */
#ifndef LORA_PROVISION_H
#define LORA_PROVISION_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    LORA_PROVISION_OK = 0,
    LORA_PROVISION_ERR_INVALID_ARG = -1,         /* NULL, N < 1, LB <= 0, M or alpha out of range,
                                                    a negative or non-finite probability */
    LORA_PROVISION_ERR_NOT_A_DISTRIBUTION = -2   /* the p_i do not sum to 1 within 1e-6 */
};

/*
 * IAR(M) of Eq. 4.  p: host, [N], non-negative, summing to 1.  1 <= M <= N.
 * iar: result.  tau (may be NULL): the threshold tau* of Eq. 3 (-1 when all adapters with
 * p_i > 0 fit).  q (may be NULL): host, [N], receives the residency probabilities of Eq. 2.
 */
int lora_provision_iar(const double *p, int N, double LB, int M, double *iar, double *tau,
                       double *q);

/*
 * M* of Eq. 1 / Algorithm 1: candidates M = 1, 2, ... in turn, the first whose IAR reaches
 * alpha (0 < alpha <= 1).  iar_at_M (may be NULL) receives IAR(M*).
 */
int lora_provision_min_cache(const double *p, int N, double LB, double alpha, int *M_star,
                             double *iar_at_M);

/* Minimum pool memory M * Mem_LoRA (Sec. 4.2, last step); adapter_bytes is the footprint of one
 * adapter, e.g. lora_pool_bytes of a one-adapter pool.  -1 on a negative argument. */
int64_t lora_provision_memory_bytes(int M, int64_t adapter_bytes);

#ifdef __cplusplus
}
#endif
#endif /* LORA_PROVISION_H */
