// Host-only scheduling rules of the paper's Section 6.1 and the range of eq. (9).
#include <cmath>
#include <limits>
#include <vector>

#include "kvl.h"
#include "kvl_sched.h"

extern "C" {

int kvl_pd_range(double g, double s, double mem_bw, double storage_bw, kvl_pd_range_t *out) {
    if (!out || !(g > 0) || !(s > 0) || !(mem_bw > 0) || !(storage_bw > 0)) return KVL_EINVAL;
    if (s >= g) return KVL_EINVAL;          // the analysis assumes s <= g; s = g leaves no lower bound
    kvl_pd_range_t r;
    r.lo = s / (g - s);
    r.hi_de_read = (g - 2 * s) / s;
    r.hi_de_write = (g - s) / (2 * s);
    r.hi_dram = (mem_bw / storage_bw - 3) / 2;
    r.hi = std::fmin(r.hi_de_read, std::fmin(r.hi_de_write, r.hi_dram));
    r.feasible = r.lo <= r.hi ? 1 : 0;
    *out = r;
    return KVL_OK;
}

int kvl_sched_pe_fetch(uint64_t *tok, const uint64_t *read_q, uint32_t n_engines,
                       const uint64_t *req_tokens, uint32_t n_req, uint64_t alpha, uint64_t beta,
                       int32_t *assign, uint32_t *n_assigned) {
    if ((n_engines && (!tok || !read_q)) || (n_req && (!req_tokens || !assign))) return KVL_EINVAL;
    for (uint32_t r = 0; r < n_req; ++r) assign[r] = -1;
    uint32_t done = 0;
    for (uint32_t r = 0; r < n_req; ++r) {
        // one pass finds the emptiest engine of each class among those not over the limit;
        // membership follows tok as it stands now, so an engine filled by this fetch drops out
        int64_t best_short = -1, best_long = -1;
        for (uint32_t e = 0; e < n_engines; ++e) {
            if (tok[e] > beta) continue;                       // overloaded: gets nothing
            int64_t &best = read_q[e] <= alpha ? best_short : best_long;
            if (best < 0 || tok[e] < tok[best]) best = e;
        }
        const int64_t pick = best_short >= 0 ? best_short : best_long;
        if (pick < 0) break;                                   // no engine left: the fetch ends here
        assign[r] = (int32_t)pick;
        tok[pick] += req_tokens[r];
        ++done;
    }
    if (n_assigned) *n_assigned = done;
    return KVL_OK;
}

int kvl_sched_de_groups(uint64_t *group_tok, uint32_t n_groups, const uint64_t *req_len, uint32_t n_req,
                        int32_t *assign_group) {
    if (n_groups == 0 || !group_tok || (n_req && (!req_len || !assign_group))) return KVL_EINVAL;
    for (uint32_t r = 0; r < n_req; ++r) {
        uint32_t best = 0;
        for (uint32_t g = 1; g < n_groups; ++g)
            if (group_tok[g] < group_tok[best]) best = g;
        assign_group[r] = (int32_t)best;
        group_tok[best] += req_len[r];
    }
    return KVL_OK;
}

int kvl_sched_de_fetch(uint64_t *tok, uint64_t *seq, uint64_t *free_hbm, uint32_t n_engines,
                       const uint64_t *req_len, uint32_t n_req, int32_t *assign, uint32_t *n_assigned,
                       double *z_out) {
    if (n_engines == 0 || !tok || !seq || !free_hbm || (n_req && (!req_len || !assign))) return KVL_EINVAL;
    uint64_t total_free = 0, total_tok = 0;
    for (uint32_t e = 0; e < n_engines; ++e) {
        total_free += free_hbm[e];
        total_tok += tok[e];
    }
    // R: the head of the queue that fits the group's free HBM if it were one piece
    uint64_t len_R = 0;
    for (uint32_t r = 0; r < n_req; ++r) {
        if (len_R + req_len[r] > total_free) break;
        len_R += req_len[r];
    }
    const double Z = 1.05 * (double)(len_R + total_tok) / (double)n_engines;
    if (z_out) *z_out = Z;
    for (uint32_t r = 0; r < n_req; ++r) assign[r] = -1;
    uint32_t done = 0;
    for (uint32_t r = 0; r < n_req; ++r) {
        const uint64_t len = req_len[r];
        int64_t low = -1, high = -1;        // best engine under / over the threshold
        for (uint32_t e = 0; e < n_engines; ++e) {
            if (free_hbm[e] < len) continue;
            if ((double)(tok[e] + len) > Z) {
                if (high < 0 || tok[e] < tok[high]) high = e;
            } else {
                if (low < 0 || seq[e] < seq[low]) low = e;
            }
        }
        const int64_t pick = low >= 0 ? low : high;
        if (pick < 0) break;                 // no engine has the HBM: the fetch ends
        assign[r] = (int32_t)pick;
        tok[pick] += len;
        seq[pick] += 1;
        free_hbm[pick] -= len;
        ++done;
    }
    if (n_assigned) *n_assigned = done;
    return KVL_OK;
}

int kvl_sched_read_side(uint64_t read_q_pe_node, uint64_t read_q_de_node) {
    return read_q_de_node < read_q_pe_node ? 1 : 0;
}

}  // extern "C"
