/*
 * kvl_sched -- the paper's request scheduling rules and its bottleneck-free
 * P/D range, as plain host functions (no GPU is touched).  They decide which of
 * the two load paths a request's cache takes; the data movement itself is kvl.h.
 *
 * All functions return 0 or a negative KVL_E* code from kvl.h.  Arrays are host
 * memory owned by the caller.  Ties are broken towards the lowest index.
 */
#ifndef KVL_SCHED_H
#define KVL_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Bottleneck-free analysis, Section 4.2, eqs. (3), (5), (7), (8), (9):
 *   s/(g-s) <= P/D <= min{ (g-2s)/s, (g-s)/(2s), (M/Bs - 3)/2 }
 * g GPUs per node, storage bandwidth per node = s x B (B = one compute NIC),
 * M = memory bandwidth per node, storage_bw = B*s, same unit as M. */
typedef struct {
    double lo;            /* s/(g-s): prefill-engine NIC write direction, eq. (3) */
    double hi;            /* the minimum of the three upper bounds, eq. (9) */
    double hi_de_read;    /* (g-2s)/s, eq. (5) */
    double hi_de_write;   /* (g-s)/(2s), eq. (7) */
    double hi_dram;       /* (M/Bs-3)/2, eq. (8) */
    int feasible;         /* lo <= hi */
} kvl_pd_range_t;
int kvl_pd_range(double g, double s, double mem_bw, double storage_bw, kvl_pd_range_t *out);

/* Inter-engine prefill scheduling, Section 6.1, Algorithm 1.  One fetch of a
 * prefill-engine group.  An engine is overloaded while tok > beta and then gets
 * nothing; of the others, those on nodes with a short reading queue
 * (read_q <= alpha) are served before those with a long one.  The waiting queue is
 * taken in FIFO order: each request goes to the engine with the smallest tok among
 * the short-queue engines if any is left, else among the long-queue engines, and
 * tok of the chosen engine grows by the request's tokens -- which may make it
 * overloaded for the rest of the fetch (the categories follow tok as it is updated).
 * When no engine is left the fetch ends and the remaining requests stay in the
 * queue.  An engine at exactly beta still takes one request.
 * tok[], read_q[]: n_engines entries, tok is updated in place.
 * assign[]: n_req entries, engine index or -1 for requests left in the queue
 * (always a tail of the queue); *n_assigned (may be NULL): how many were placed. */
int kvl_sched_pe_fetch(uint64_t *tok, const uint64_t *read_q, uint32_t n_engines,
                       const uint64_t *req_tokens, uint32_t n_req,
                       uint64_t alpha, uint64_t beta, int32_t *assign, uint32_t *n_assigned);

/* Decode scheduling phase 1, Section 6.1: every request of the global queue goes
 * to the group whose total tok is smallest; that total grows by the request's
 * length.  group_tok[] is updated in place. */
int kvl_sched_de_groups(uint64_t *group_tok, uint32_t n_groups,
                        const uint64_t *req_len, uint32_t n_req, int32_t *assign_group);

/* Decode scheduling phase 2, Section 6.1, within one group.  R = the longest
 * head of the private queue whose total length fits the group's total free HBM;
 * Z = 1.05 * (sum_{r in R} len_r + sum_e tok_e) / |E|.  Requests are popped from
 * the head; among engines with free_hbm >= len, those with tok + len <= Z are
 * preferred and the one with the smallest seq is taken, else the one with the
 * smallest tok; the fetch ends at the first request no engine can hold.
 * tok[], seq[], free_hbm[] (all in tokens) are updated in place; *z_out (may be
 * NULL) receives Z; assign[]: engine index or -1. */
int kvl_sched_de_fetch(uint64_t *tok, uint64_t *seq, uint64_t *free_hbm, uint32_t n_engines,
                       const uint64_t *req_len, uint32_t n_req, int32_t *assign,
                       uint32_t *n_assigned, double *z_out);

/* Read-path choice, Section 6.1: read on the side with the shorter reading
 * queue.  Returns 0 for the prefill side (also on a tie), 1 for the decode side. */
int kvl_sched_read_side(uint64_t read_q_pe_node, uint64_t read_q_de_node);

#ifdef __cplusplus
}
#endif
#endif /* KVL_SCHED_H */
