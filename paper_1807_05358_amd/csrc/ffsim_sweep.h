// Small kernels around the trial-mutation kernel: the list of a strategy's neighbours, the
// reduction over their times, and a counter reset.  Included by the host file only (the
// kernels here are not templates: one definition in the library).
#pragma once
#include "ffsim_device.h"

namespace ffsim {

// ---- neighbour sweep (Section 8: is a strategy locally optimal?) --------------------------
//
// The neighbours of a strategy differ from it in the configuration of one op.  Neighbour k of
// the enumeration: ops op_begin..op_end-1 in order; per op every degree tuple of its list, in
// list order; per tuple every device offset 0..n_dev-1; stride 1.  first[o - op_begin] is the
// index of the first neighbour of op o.  Writes the same mutation for every chain ([M][C]).
// status: null, or one word that is nonzero if `first` could not be built (see k_neighbour_first): every
// mutation then names an op outside the graph, which the trial kernel answers with "invalid".
__global__ __launch_bounds__(WAVE) void k_neighbour_list(const uint32_t* __restrict__ tuple_ptr, const uint32_t* __restrict__ tuples,
                                                         const uint32_t* __restrict__ first, uint32_t op_begin, uint32_t op_end,
                                                         uint32_t n_dev, uint32_t M, uint32_t C, uint32_t* __restrict__ muts,
                                                         const uint32_t* __restrict__ status) {
    const uint32_t k = blockIdx.x * WAVE + threadIdx.x;
    if (k >= M) return;
    if (status && *status) {
        for (uint32_t c = 0; c < C; c++) {
            uint32_t* mu = muts + ((size_t)k * C + c) * 3;
            mu[0] = 0xffffffffu; mu[1] = 0; mu[2] = 0;
        }
        return;
    }
    // binary search for the op whose range holds k
    uint32_t lo = 0, hi = op_end - op_begin;       // first[lo] <= k < first[hi]
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) / 2;
        if (first[mid] <= k) lo = mid; else hi = mid;
    }
    const uint32_t op = op_begin + lo;
    const uint32_t r = k - first[lo];
    const uint32_t deg = tuples[tuple_ptr[op] + r / n_dev];
    const uint32_t off = r % n_dev;
    for (uint32_t c = 0; c < C; c++) {
        uint32_t* mu = muts + ((size_t)k * C + c) * 3;
        mu[0] = op; mu[1] = deg; mu[2] = off | (1u << 16);
    }
}

// The index of every op's first neighbour, built on the device (one wavefront): first[o - op_begin]
// for o = op_begin..op_end (the last entry is the total).  *status = 0 if every range of tuple_ptr is
// well formed (ascending, inside the list of n_tuples entries), the total fits 32 bits and equals the
// M the caller sized its buffers for; 1 otherwise.  Writes op_end - op_begin + 1 entries of first.
__global__ __launch_bounds__(WAVE) void k_neighbour_first(const uint32_t* __restrict__ tuple_ptr, uint32_t n_tuples, uint32_t op_begin,
                                                          uint32_t op_end, uint32_t n_dev, uint32_t M, uint32_t* __restrict__ first,
                                                          uint32_t* __restrict__ status) {
    const int lane = lane_id();
    u64 carry = 0;
    bool bad = false;
    for (uint32_t base = op_begin; base < op_end; base += WAVE) {
        const uint32_t o = base + lane;
        u64 n = 0;
        if (o < op_end) {
            const uint32_t a = tuple_ptr[o], b = tuple_ptr[o + 1];
            if (a > b || b > n_tuples) bad = true; else n = (u64)(b - a) * n_dev;
        }
        // inclusive prefix sum over the lanes
        u64 incl = n;
#pragma unroll
        for (int sft = 1; sft < WAVE; sft <<= 1) {
            const uint32_t lo = __shfl_up((uint32_t)incl, sft), hi = __shfl_up((uint32_t)(incl >> 32), sft);
            if (lane >= sft) incl += ((u64)hi << 32) | lo;
        }
        const u64 excl = carry + incl - n;
        if (o < op_end) {
            if (excl > 0xffffffffull) bad = true;
            first[o - op_begin] = (uint32_t)excl;
        }
        carry += readlane_u64(incl, WAVE - 1);
    }
    if (carry > 0xffffffffull || carry != M) bad = true;
    const bool any_bad = ballot(bad) != 0;
    if (lane == 0) {
        first[op_end - op_begin] = (uint32_t)carry;
        *status = any_bad ? 1u : 0u;
    }
}

// per chain: the smallest time among its M results ([M][C]) and the lowest index that has it;
// one wavefront per chain
__global__ __launch_bounds__(WAVE) void k_best_of(const u64* __restrict__ ns, uint32_t M, uint32_t C, u64* __restrict__ best_ns,
                                                  uint32_t* __restrict__ best_idx) {
    const uint32_t c = blockIdx.x;
    if (c >= C) return;
    u64 b = ~0ull;
    uint32_t bi = 0xffffffffu;
    for (uint32_t k = lane_id(); k < M; k += WAVE) {
        const u64 v = ns[(size_t)k * C + c];
        if (v < b) { b = v; bi = k; }        // ascending k: the first index wins inside a lane
    }
    const u64 m = wave_min_u64(b);
    const uint32_t mi = wave_min_u32(b == m ? bi : 0xffffffffu);
    if (lane_id() == 0) { best_ns[c] = m; best_idx[c] = mi; }
}

// clears the work counter of k_sim_chain_try (a kernel, so that a captured stream sees a node)
// the proposals of the steps done[c] .. done[c] + n_ahead - 1 of every chain, as mutation records
// [n_ahead][C] {op, cfg.x, cfg.y}; op = all ones where there is none (no list, or beyond the call's steps)
__global__ void k_search_ahead_proposals(SearchDev search, uint32_t n_ops, uint32_t n_dev, uint32_t C, uint32_t n_steps, uint32_t* muts) {
    const uint32_t idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= search.n_ahead * C) return;
    const uint32_t j = idx / C, c = idx % C;
    const uint32_t s = search.done[c] + j;
    uint32_t op = 0xffffffffu;
    uint2 cfg = make_uint2(0, 0);
    if (s < n_steps) {
        uint32_t o;
        if (search_proposal(search, n_ops, n_dev, c, search.first_step + s, o, cfg)) op = o;
    }
    muts[(size_t)idx * 3 + 0] = op;
    muts[(size_t)idx * 3 + 1] = cfg.x;
    muts[(size_t)idx * 3 + 2] = cfg.y;
}

__global__ void k_zero_u32(uint32_t* p) { if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0; }
__global__ void k_zero_words(uint32_t* p, uint32_t n) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

}  // namespace ffsim
