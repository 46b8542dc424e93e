// okt_balance_plan: the communication scheme of the data-balancing step that
// precedes the allgatherv of the global top-k values (Sec. 3.1.2: from the
// gathered buffer sizes every worker derives which chunk goes to which worker),
// and the rule for when the step is worth taking (Sec. 5.3: when the largest
// buffer is more than four times the average).  Host arithmetic only.
//
// The P buffers, in worker order, form one list of T entries (it ascends in the
// index, since worker i holds region i).  Balancing re-cuts that list into P
// consecutive pieces of floor or ceil T / P entries: worker j ends up with the
// list positions [floor(j T / P), floor((j+1) T / P)).  A chunk of the plan is a
// non-empty overlap of an old buffer with a new one; both sequences of cut points
// ascend, so one merge over them lists all chunks, at most 2 P - 1.
#include "okt.h"

extern "C" int okt_balance_plan(const uint64_t* h_sizes, uint32_t P, okt_chunk* h_plan_out,
                                uint32_t plan_capacity, uint32_t* h_plan_len_out,
                                int* h_triggered_out) {
    if (!h_sizes || P == 0 || !h_plan_len_out || !h_triggered_out) return OKT_ERR_INVALID_ARG;
    uint64_t total = 0, largest = 0;
    for (uint32_t i = 0; i < P; ++i) {
        if (h_sizes[i] > 0xffffffffull) return OKT_ERR_INVALID_ARG;
        total += h_sizes[i];
        if (h_sizes[i] > largest) largest = h_sizes[i];
    }
    *h_plan_len_out = 0;
    // largest > 4 * (total / P), in integers
    *h_triggered_out = largest * (uint64_t)P > 4 * total ? 1 : 0;
    if (!*h_triggered_out) return OKT_OK;
    if (!h_plan_out) return OKT_ERR_INVALID_ARG;

    uint32_t src = 0, dst = 0, n = 0;
    uint64_t src_first = 0;                       // list position of the first entry of buffer src
    uint64_t at = 0;                              // list position of the next entry to place
    while (at < total) {
        while (src_first + h_sizes[src] <= at) src_first += h_sizes[src++];
        // worker dst owns [dst_first, dst_end); 128-bit products: T and P are below 2^32 * 2^32
        uint64_t dst_first = (uint64_t)(((unsigned __int128)dst * total) / P);
        uint64_t dst_end = (uint64_t)(((unsigned __int128)(dst + 1) * total) / P);
        while (dst_end <= at) {
            ++dst;
            dst_first = dst_end;
            dst_end = (uint64_t)(((unsigned __int128)(dst + 1) * total) / P);
        }
        const uint64_t src_end = src_first + h_sizes[src];
        const uint64_t stop = src_end < dst_end ? src_end : dst_end;
        if (n == plan_capacity) return OKT_ERR_INVALID_ARG;
        h_plan_out[n].src = src;
        h_plan_out[n].dst = dst;
        h_plan_out[n].src_offset = at - src_first;
        h_plan_out[n].dst_offset = at - dst_first;
        h_plan_out[n].count = stop - at;
        ++n;
        at = stop;
    }
    *h_plan_len_out = n;
    return OKT_OK;
}
