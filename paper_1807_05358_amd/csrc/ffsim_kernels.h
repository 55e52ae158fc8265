// Kernels of the batched execution simulator: one candidate strategy per wavefront.
//
// Task-graph construction (Section 5.1) and Algorithm 1 are fused: the task graph is never
// written out.  A compute task is (op, part); its id is op*64 + part, which is
// order-isomorphic to the dense construction-order id.  Communication tasks are never
// stored: the transfers that start when a producer part finishes are enumerated at that
// moment, one consumer part per lane, and queued on their link rows in
// (edge, producer part, consumer part) order, which is their id order.
//
// The priority queue of Algorithm 1 is a 64-ary min-tree over one 64-bit word per compute
// task (encoding: ffsim_device.h).  Level 0 (the words) lives in HBM, or in LDS for small
// graphs; level 1 (one minimum per op) lives in LDS, or in a register for graphs of up to 64 ops;
// level 2 (one per 64 ops, large graphs only) in a register.  Popping the
// minimum word and taking the lowest index among equal words reproduces the
// (readyTime, id) order: at equal times, finished producers release their transfers (kind
// 0) before READY compute tasks are dequeued (kind 1); the two kinds never share a device
// row, so only the order inside each kind matters.  All parts of one op that hold the
// minimum word are handled in one step, serialised per device row in lane (= id) order.
//
// Files: ffsim_device.h (word encoding, wavefront primitives), ffsim_strategy.h (configurations,
// geometry, kept per-edge set-up, validity), ffsim_events.h (FIFO, recording, initial state, event
// loop), this file (the batch kernel), ffsim_chain.h (delta simulation, search), ffsim_sweep.h
// (neighbour list and reduction), ffsim_select.h + ffsim_k_*.hip (the instantiations, compiled
// side by side), ffsim.hip (host side of the C boundary).
#pragma once
#include "ffsim_events.h"

namespace ffsim {

// One candidate: build + simulate.  Returns the makespan or one of the RESULT_* codes.
// WIDE selects 64-bit element counts (tensors of 2^32 bytes or more).
template <bool WIDE, bool RECORD, bool STATS, int Q, bool CACHE, class SimX>
__device__ u64 simulate_candidate(SimX& m, Counters& cnt, Recorder& rec) {
#ifdef FFSIM_PROFILE
    const u64 prof_t0 = __builtin_readcyclecounter();
#endif
    const StrategyClass cls = validate_strategy(m);
    if (cls == STRATEGY_INVALID) return RESULT_INVALID;
    m.want_sort = cls != STRATEGY_REGULAR;
    init_state(m, cnt);
#ifdef FFSIM_PROFILE
    cnt.exit_code = __builtin_readcyclecounter() - prof_t0;   // reported as section 0
#endif
    const u64 rc = cls == STRATEGY_REGULAR ? run_events<WIDE, RECORD, true, STATS, Q, CACHE>(m, cnt, rec)
                                            : run_events<WIDE, RECORD, false, STATS, Q, CACHE>(m, cnt, rec);
    if (rc) return rc;
    if (STATS) {   // diagnostics: tasks that never ran (0 in a correct run)
        for (uint32_t j = 0; j < m.S.n_ops; j++) cnt.n_stuck += __popcll(ballot(m.words[j * WAVE + lane_id()] != W_NONE));
    }
    return makespan(m);
}

__device__ __forceinline__ void store_counters(Counters c, Counters* out) {
    u64 s = c.sum_comm_ns;   // accumulated per lane
#pragma unroll
    for (int k = 1; k < WAVE; k <<= 1) s += shfl_xor_u64(s, k);
    c.sum_comm_ns = s;
    if (lane_id() == 0) *out = c;
}

// LDSW: the task words and per-op exeTimes of the candidate live in LDS (small graphs).
// CACHE: the per-edge set-up is kept (after the task words: in LDS if LDSW, else in the slot).
// EXT: with the link table and / or explicit devices (devmaps, else null and never read).
// GPN: compiled for machines with this many GPUs per node (0 = any).
template <bool WIDE, bool LDSW, bool STATS, int Q, bool CACHE, int EXT, int GPN>
__global__ __launch_bounds__(WAVE) void k_sim_batch(SimDev S, const DOp* __restrict__ ops, const DEdge* __restrict__ edges,
                                                    const DEdge* __restrict__ in_edges, const uint32_t* __restrict__ cost,
                                                    const uint32_t* __restrict__ magic, const uint2* __restrict__ strategies,
                                                    uint32_t B, u64* __restrict__ out_ns, Counters* __restrict__ stats,
                                                    unsigned char* __restrict__ ws, size_t slot_stride,
                                                    const uint16_t* __restrict__ devmaps) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const Tables T{ops, edges, in_edges, cost};
    u64* words;
    uint32_t* exe_of;
    uint32_t* ecache = nullptr;
    unsigned char* lds_rest = lds_raw;
    const size_t state_bytes = (slot_bytes(S.n_ops, S.n_ops_pad) + 15) & ~(size_t)15;
    if (LDSW) {
        words = (u64*)lds_raw;
        exe_of = (uint32_t*)(lds_raw + (size_t)S.n_ops * WAVE * 8);
        lds_rest = lds_raw + state_bytes;
        if (CACHE) { ecache = (uint32_t*)lds_rest; lds_rest += ecache_bytes(S.n_edges); }
    } else {
        unsigned char* slot = ws + (size_t)blockIdx.x * slot_stride;
        words = (u64*)slot;
        exe_of = (uint32_t*)(slot + (size_t)S.n_ops * WAVE * 8);
        if (CACHE) ecache = (uint32_t*)(slot + state_bytes);
    }
    const WaveLds L = carve_lds(lds_rest, S);
    const uint32_t magic_v = load_magic(magic);
    Recorder none = {};
    for (uint32_t b = blockIdx.x; b < B; b += gridDim.x) {
        Counters cnt = {};
        SimT<false, EXT, GPN> m{S, T, strategies + (size_t)b * S.n_ops, words, exe_of, L, magic_v, 0, false, NO_OVERRIDE, make_uint2(0, 0), ecache, true};
        if (EXT) {
            m.links = (const uint4*)(magic + LINK_TABLE_AT);
            m.node_links = m.links + (size_t)S.gpus_per_node * S.gpus_per_node;
            if (EXT >= 2 && S.ties) m.tie = magic + tie_table_at(S.gpus_per_node, S.n_nodes);
            if (devmaps) m.devmap = devmaps + (size_t)b * S.n_ops * WAVE;
        }
        const u64 mk = simulate_candidate<WIDE, false, STATS, Q, CACHE>(m, cnt, none);
        if (lane_id() == 0) out_ns[b] = mk;
        if (STATS) store_counters(cnt, stats + b);
        wave_sync();
    }
}

}  // namespace ffsim

#include "ffsim_chain.h"
