// Host arithmetic of the offloading scheduler (Sec. 3.4) and of the choice of a pre-recorded
// graph (Sec. 3.2.2).  No device code: it lives in this library so that a proxy written in any
// language can take its decisions from the same place the kernels come from.
#include "../../include/adr.h"

#include <cmath>

extern "C" {

// Eq. 1: the executors' share of memory capacity and of memory bandwidth, each summed over the
// n prefill instances and taken relative to the decode instance; the smaller ratio bounds.
double adr_offload_bound_mem(const double *hbm_prefill, const double *bw_prefill, int n, double hbm_decode,
                             double bw_decode)
{
    if (n < 0 || (n > 0 && (!hbm_prefill || !bw_prefill)) || !(hbm_decode > 0.0) || !(bw_decode > 0.0))
        return NAN;
    double hbm = 0.0, bw = 0.0;
    for (int i = 0; i < n; ++i) {
        hbm += hbm_prefill[i];
        bw += bw_prefill[i];
    }
    return std::fmin(hbm / hbm_decode, bw / bw_decode);
}

// Eq. 2: how far the decode batch may grow before the non-attention kernels stop being
// memory-bound (B_max), relative to the batch the TPOT target allows without offloading.
double adr_offload_bound_comp(double b_max, double b_tpot)
{
    if (!(b_tpot > 0.0))
        return NAN;
    return (b_max - b_tpot) / b_tpot;
}

// Eq. 3
double adr_offload_bound(double ob_mem, double ob_comp) { return std::fmin(ob_mem, ob_comp); }

// Algorithm 1.  C1: the offloaded requests' current tokens plus the new request at its maximal
// length stay below the local requests' current tokens times the bound.  C2: the same with the
// new request's current length, and the offloaded batch, one larger, stays below the local
// batch times the bound.  Both comparisons are strict.
int adr_need_offload(const adr_request_tokens *req, const adr_request_tokens *local, int n_local,
                     const adr_request_tokens *offloaded, int n_offloaded, double bound)
{
    if (!req || n_local < 0 || n_offloaded < 0 || (n_local > 0 && !local) || (n_offloaded > 0 && !offloaded))
        return -ADR_ERR_NULL;
    double attn_used = 0.0, decode_used = 0.0;
    for (int i = 0; i < n_offloaded; ++i)
        attn_used += (double)offloaded[i].used_token;
    for (int i = 0; i < n_local; ++i)
        decode_used += (double)local[i].used_token;
    const double budget = decode_used * bound;
    if (attn_used + (double)req->max_token < budget)
        return 1; // C1
    if (attn_used + (double)req->used_token < budget && (double)(n_offloaded + 1) < (double)n_local * bound)
        return 1; // C2
    return 0;
}

// Sec. 3.2.2: graphs are recorded for capacities at a configurable interval; a batch of n rows
// runs the smallest recorded capacity that holds it (the remaining rows are padded rows).
int adr_graph_capacity(int n, int interval, int max_capacity)
{
    if (n < 0 || interval <= 0 || max_capacity < interval)
        return -1;
    const int steps = n == 0 ? 1 : (n + interval - 1) / interval;
    const int capacity = steps * interval;
    return capacity <= max_capacity ? capacity : -1;
}

} // extern "C"
