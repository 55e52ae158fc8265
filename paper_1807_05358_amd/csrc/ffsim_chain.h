// Chains of strategies: delta simulation (Section 5.3), trial proposals, the search loop
// (Section 6) and the neighbour sweep (Section 8.4).
#pragma once
#include "ffsim_events.h"

namespace ffsim {

// ---- delta simulation (Section 5.3) ---------------------------------------------------
//
// A chain keeps, in HBM, its current strategy, the endTime of every task of the simulation of
// that strategy (the accepted timeline) and up to n_snaps snapshots of the simulation state
// taken whenever the event time crossed a multiple of `step`.  When the configuration of one
// op changes, nothing can differ before the first producer of that op finishes (its transfers
// are the first tasks that depend on the op's configuration), so the simulation is resumed
// from the last snapshot before that time: the op's own tasks are rebuilt, the input counts of
// its consumers are corrected, and Algorithm 1 continues from there.  The resulting timeline is
// the one a full simulation produces.  Every such run is recorded beside the accepted timeline
// (see Recorder) and becomes the accepted one only when it is committed, so a search proposal
// costs one resumed simulation whether it is accepted or not.
struct ChainMeta {
    u64 step;           // event-word distance between snapshots (2 * time)
    uint32_t n_valid;   // snapshots 1..n_valid-1 are usable (0 = none; index 0 is the initial state)
    uint32_t stale;     // the stored timeline does not belong to the current strategy
    // telemetry (ff_sim_chains_get_stats)
    u64 n_steps;        // mutations applied
    u64 n_resumed;      // of those, resumed from a snapshot instead of simulated from time 0
    u64 n_events;       // queue pops spent in mutation steps
    u64 n_events_full;  // queue pops of the last simulation from time 0 (one full simulation)
    u64 cur_ns;         // simulated time of the chain's current strategy (result code if it has none)
    u64 idle_steps;     // search steps since the chain's best time last improved
    u64 n_converged;    // committed steps whose run stopped early because it re-joined the accepted timeline
    uint32_t loc;       // bit k: which of its two places holds snapshot k of the accepted timeline
    uint32_t tag;       // tag of the last recorded run (1..0xffff; 0 marks entries never written)
};

struct ChainMem {       // all pointers are per chain
    uint2* cfgs;
    u64* words;
    uint32_t* exe_of;
    u64* end_of;        // accepted timeline
    u64* end_try;       // tag<<48 | endTime, written by recorded runs
    u64* snap_words;    // [2][n_snaps][n_ops*64]
    u64* snap_l1;       // [2][n_snaps][n_ops_pad]
    u64* snap_free;     // [2][n_snaps][n_rows, padded to even]
    uint32_t* ecache;   // kept per-edge set-up of the chain's current strategy (see EdgeLane)
    ChainMeta* meta;
};

// byte offset of the ChainMeta record inside a chain block (it comes last)
__host__ __device__ inline size_t chain_meta_offset(uint32_t n_ops, uint32_t n_ops_pad, uint32_t n_rows, uint32_t n_snaps,
                                                    uint32_t n_edges) {
    size_t b = (size_t)n_ops_pad * 8;                       // cfgs
    b += ecache_bytes(n_edges);
    b += (size_t)n_ops * WAVE * 8 * 3;                      // words, end_of, end_try
    b += 2 * (size_t)n_snaps * ((size_t)n_ops * WAVE * 8 + (size_t)n_ops_pad * 8 + (size_t)((n_rows + 1) & ~1u) * 8);
    b += (size_t)n_ops_pad * 4;                             // exe_of
    return b;
}
__host__ __device__ inline size_t chain_bytes(uint32_t n_ops, uint32_t n_ops_pad, uint32_t n_rows, uint32_t n_snaps, uint32_t n_edges) {
    return (chain_meta_offset(n_ops, n_ops_pad, n_rows, n_snaps, n_edges) + sizeof(ChainMeta) + 255) & ~(size_t)255;
}

__device__ __forceinline__ ChainMem carve_chain(unsigned char* base, const SimDev& S, uint32_t n_snaps) {
    ChainMem c;
    const size_t nw = (size_t)S.n_ops * WAVE;
    c.cfgs = (uint2*)base; base += (size_t)S.n_ops_pad * 8;
    c.ecache = (uint32_t*)base; base += ecache_bytes(S.n_edges);
    c.words = (u64*)base; base += nw * 8;
    c.end_of = (u64*)base; base += nw * 8;
    c.end_try = (u64*)base; base += nw * 8;
    c.snap_words = (u64*)base; base += 2 * (size_t)n_snaps * nw * 8;
    c.snap_l1 = (u64*)base; base += 2 * (size_t)n_snaps * S.n_ops_pad * 8;
    c.snap_free = (u64*)base; base += 2 * (size_t)n_snaps * ((S.n_rows + 1) & ~1u) * 8;
    c.exe_of = (uint32_t*)base; base += (size_t)S.n_ops_pad * 4;
    c.meta = (ChainMeta*)base;
    return c;
}

// Where may a simulation start after op `mo` went from configuration `ocfg` to the one now
// in m.cfgs?  Nothing can differ before the first task of a producer of op mo finishes (the
// transfers released then are the first tasks that depend on op mo's configuration); time 0
// if op mo has no producer or has a part without inputs.  Returns the index of the last
// snapshot at or before that time (0 = start from time 0) and, in pend_new, the number of
// inputs every part of op mo waits for under the new configuration.
template <class SimX>
__device__ __forceinline__ uint32_t resume_point(const SimX& m, const u64* end_of, const ChainMeta& meta, uint32_t mo, uint2 ocfg,
                                                 uint32_t& pend_new) {
    const int lane = lane_id();
    const OpCfg cn = m.cfg(mo);
    const OpCfg co = unpack_cfg(ocfg);
    const uint32_t in_begin = m.T.ops[mo].in_begin, in_end = m.T.ops[mo].in_end;
    u64 tau = in_end > in_begin ? W_NONE : 0;
    for (uint32_t q = in_begin; q < in_end; q++) {
        const uint32_t p = m.T.in_edges[q].src;
        const OpCfg cp = m.cfg(p);
        const u64 t = wave_min_u64((uint32_t)lane < cp.parts ? end_of[p * WAVE + lane] : W_NONE);
        tau = t < tau ? t : tau;
    }
    pend_new = count_pending(m, mo, cn);
    uint32_t pend_old = 0;
    {
        const uint32_t digits = part_digits(co, lane, m.magic_v);
        for (uint32_t q = in_begin; q < in_end; q++) {
            const DEdge e = m.T.in_edges[q];
            pend_old += count_inputs<SimX::kTrain>(e, m.cfg(e.src), co.x, digits, m.magic_v);
        }
    }
    if (ballot(((uint32_t)lane < cn.parts && pend_new == 0) || ((uint32_t)lane < co.parts && pend_old == 0))) tau = 0;
    if (SimX::kTrain) {
        // Which consumer parts a part of op mo contributes to depends on how op mo is cut (a coarser part also
        // covers what lies between the ranges of finer ones), unlike which consumer parts READ op mo at all.  A
        // consumer part that takes a contribution from op mo under one of the two configurations and none
        // under the other may be dequeued at any time in one of the two timelines: start from time 0.
        const uint32_t ob = m.T.ops[mo].out_begin, oe = m.T.ops[mo].out_end;
        for (uint32_t ei = ob; ei < oe; ei++) {
            const DEdge e = m.T.edges[ei];
            if (!e.kind) continue;
            const OpCfg cj = m.cfg(e.dst);
            const uint32_t digits = part_digits(cj, lane, m.magic_v);
            const uint32_t was = count_inputs<true>(e, co, cj.x, digits, m.magic_v);
            const uint32_t is = count_inputs<true>(e, cn, cj.x, digits, m.magic_v);
            if (ballot((uint32_t)lane < cj.parts && (was == 0) != (is == 0))) tau = 0;
        }
    }
    u64 k64 = (2 * tau) / meta.step;
    if (k64 > meta.n_valid - 1) k64 = meta.n_valid - 1;
    return (uint32_t)k64;
}

// A simulation state taken before anything depended on op mo's configuration holds two static
// things about it: the op's own tasks (all still waiting for all their inputs) and, in its
// consumers' waiting tasks, how many inputs come from op mo.  Rewrites both for the new
// configuration.  words / l1: the state to patch (a stored snapshot, or live state).
template <class SimX>
__device__ __forceinline__ void patch_state_for_op(const SimX& m, u64* words, u64* l1, uint32_t mo, uint2 ocfg, uint32_t pend_new) {
    const int lane = lane_id();
    const OpCfg cn = m.cfg(mo);
    const OpCfg co = unpack_cfg(ocfg);
    const u64 w_own = (uint32_t)lane >= cn.parts ? W_NONE : (W_WAIT | ((u64)pend_new << 48));
    words[mo * WAVE + lane] = w_own;
    const u64 w_own_min = wave_min_u64(w_own);
    if (lane == 0) l1[mo] = w_own_min;
    const uint32_t ob = m.T.ops[mo].out_begin, oe = m.T.ops[mo].out_end;
    for (uint32_t ei = ob; ei < oe; ei++) {
        const DEdge e = m.T.edges[ei];
        const uint32_t j = e.dst;
        const OpCfg cj = m.cfg(j);
        const uint32_t digits = part_digits(cj, lane, m.magic_v);
        const uint32_t was = count_inputs<SimX::kTrain>(e, co, cj.x, digits, m.magic_v);
        const uint32_t is = count_inputs<SimX::kTrain>(e, cn, cj.x, digits, m.magic_v);
        if (!ballot((uint32_t)lane < cj.parts && was != is)) continue;
        const u64 w = words[j * WAVE + lane];
        // a part of op j that reads op mo at all is still waiting in such a state
        const bool waiting = (uint32_t)lane < cj.parts && (w >> 63) && w != W_NONE;
        if (waiting && was != is) {
            const uint32_t pending = ((uint32_t)(w >> 48) & PENDING_LIMIT) - was + is;
            words[j * WAVE + lane] = W_WAIT | ((u64)pending << 48) | (w & (TIME_LIMIT - 1));
        }
        // level 1 of op j is unaffected: waiting words are not events
    }
}

// ---- search (Section 6): proposals and Metropolis acceptance, all in integers ------------
//
// Counter-based draws: SplitMix64's finaliser chained over (seed, purpose, chain, step), the
// same generator the input generators use, so a host reference can reproduce every decision.
__device__ __forceinline__ u64 mix64(u64 x) {
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}
__device__ __forceinline__ u64 draw64(u64 seed, u64 purpose, u64 chain, u64 step) {
    const u64 K = 0xD6E8FEB86659FD93ull;
    u64 h = mix64(seed);
    h = mix64(h ^ (purpose * K));
    h = mix64(h ^ (chain * K));
    h = mix64(h ^ (step * K));
    return h;
}

// what ff_sim_search hands to the kernel (device pointers)
struct SearchDev {
    u64 seed;
    u64 first_step;              // draws use first_step + s, so that consecutive calls continue one sequence
    u64 bucket_ns;               // width of an acceptance bucket
    const uint32_t* accept;      // [n_buckets] acceptance probability * 2^32 for a proposal worse by that bucket
    const uint32_t* tuple_ptr;   // [n_ops+1] ranges into tuples[]
    const uint32_t* tuples;      // degree tuples (four bytes each) a proposal may pick for each op
    uint32_t n_buckets;
    uint32_t enabled;
    uint32_t n_tuples;           // entries of tuples[]
    u64 patience;                // a chain stops proposing after this many steps without a new best (0 = never)
    u64* best_ns;                // [C] best simulated time seen (in/out)
    uint2* best_cfgs;            // [C][n_ops] the strategy that achieved it (in/out)
    // ff_sim_search_ahead: every chain has its own position in the call's steps, and a launch takes it at most
    // n_ahead steps further.
    // Look-ahead (ahead_ns given).  The proposal of a step does not depend on the chain's strategy, and a
    // rejected proposal leaves it unchanged: the proposals of the next n_ahead steps of every chain have been
    // simulated beforehand, each against the chain's current strategy (ahead_ns[j][c] for step done[c] + j), and
    // are valid for as long as everything before them is rejected.  A chain walks through them without
    // simulating, and stops for this launch after the first one it accepts.
    const u64* ahead_ns;         // [n_ahead][C] or null (every proposal is simulated in its turn)
    uint32_t* done;              // [C] steps of the call that the chain has finished (in/out), or null (all chains in step)
    uint32_t* n_accepted;        // [C] proposals taken so far (in/out; with done)
    uint32_t n_ahead;
    // without look-ahead: a launch may also end by the clock (ticks of the constant-rate counter, 0 = no limit): every
    // chain then stops after the step during which the time ran out, wherever it is, and no chain waits for a slower one
    u64 time_limit;
};

// The proposal of step st of chain c (Section 6.2): a random op, one of its listed degree tuples, a random
// device offset, stride 1.  false if the op has no list.  The same draws whoever asks.
__device__ __forceinline__ bool search_proposal(const SearchDev& search, uint32_t n_ops, uint32_t n_dev, uint32_t c, u64 st,
                                                uint32_t& op, uint2& cfg) {
    op = (uint32_t)(draw64(search.seed, 10, c, st) % n_ops);
    // (the host has checked the ranges; the clamp keeps the read inside the list even if the
    // caller changed them afterwards)
    const uint32_t t0 = search.tuple_ptr[op];
    const uint32_t t1r = search.tuple_ptr[op + 1];
    const uint32_t t1 = t1r < search.n_tuples ? t1r : search.n_tuples;
    if (t1 <= t0) return false;
    const uint32_t deg = search.tuples[t0 + (uint32_t)(draw64(search.seed, 11, c, st) % (t1 - t0))];
    const uint32_t off = (uint32_t)(draw64(search.seed, 12, c, st) % n_dev);
    cfg = make_uint2(deg, off | (1u << 16));   // stride 1
    return true;
}

// Section 6.1 with tabulated probabilities: is a proposal with simulated time mk taken by a chain whose
// strategy takes cur?  (mk: a time, or one of the RESULT_* codes, which are never taken)
__device__ __forceinline__ bool search_accepts(const SearchDev& search, uint32_t c, u64 st, u64 mk, u64 cur) {
    if (mk >= RESULT_OVERFLOW) return false;
    if (mk <= cur) return true;
    u64 b = (mk - cur) / search.bucket_ns;
    if (b >= search.n_buckets) b = search.n_buckets - 1;
    const uint32_t u = (uint32_t)(draw64(search.seed, 13, c, st) >> 32);
    return u < search.accept[b];
}

// the kept set-up of op j's in-edges follows its configuration
template <class SimX>
__device__ __forceinline__ void refresh_ecache_for_op(const SimX& m, uint32_t j) {
    const OpCfg cj = m.cfg(j);
    const uint32_t in_begin = m.T.ops[j].in_begin, in_end = m.T.ops[j].in_end;
    for (uint32_t q = in_begin; q < in_end; q++) {
        const DEdge e = m.T.in_edges[q];
        ecache_store(m.ecache, m.S.n_edges, e.eid, edge_lane(m, e, cj));
    }
    __threadfence_block();
    wave_sync();
}

// the same for every op that takes the configuration of op `lead` (tied configurations)
template <class SimX>
__device__ __forceinline__ void refresh_ecache_for_group(const SimX& m, uint32_t lead) {
    if (!(SimX::kTrain && m.tie)) { refresh_ecache_for_op(m, lead); return; }
    for (uint32_t j = 0; j < m.S.n_ops; j++)
        if (first_u32(m.tie[j]) == lead) refresh_ecache_for_op(m, j);
}

// Makes a recorded run the chain's accepted timeline: the snapshots it wrote (first..next-1)
// take the place of the old ones, the endTimes it wrote are copied over the old ones.
// converged: the run stopped where it re-joined the accepted timeline, whose later snapshots and
// endTimes stay.
__device__ __forceinline__ void commit_run(const ChainMem& cm, ChainMeta& meta, const Recorder& rec, uint32_t first, uint32_t n_words,
                                           bool converged) {
    const uint32_t written = rec.next > first ? (uint32_t)(((1ull << rec.next) - 1) & ~((1ull << first) - 1)) : 0u;
    meta.loc ^= written;
    if (!converged) meta.n_valid = rec.next;
    const u64 tag = rec.tag;
    for (uint32_t t = lane_id(); t < n_words; t += WAVE) {
        const u64 v = cm.end_try[t];
        if ((v & ~(TIME_LIMIT - 1)) == tag) cm.end_of[t] = v & (TIME_LIMIT - 1);
    }
    __threadfence_block();
    wave_sync();
}

// One kernel drives a chain through a sequence of steps.  Three sources of steps:
//   muts == nullptr and no search: simulate the chain's starting strategy (n_steps is 1);
//   muts: forced mutations, [n_steps][C] records {op, cfg.x, cfg.y}, always committed;
//   search: per step one proposal (random op, random configuration from its list, random
//           device offset), committed if it is not slower, else with the tabulated probability.
// A step is one recorded simulation (resumed from the last snapshot before the change can
// matter), then either commit_run or nothing.  Every simulation goes through the single
// run_events call site below, including the pass that only finds the makespan when no
// snapshot spacing is set yet.
// A forced mutation that names an op outside the graph poisons the chain: this and all
// later results are RESULT_INVALID.  out_ns[s][c] is the time of the chain's strategy after
// step s.
// CACHE: the chain keeps the per-edge set-up of its current strategy (all extents fit 16 bits).
// EXT: 0 plain, 1 with the refinements of the inputs, 2 also training-iteration graphs.  GPN: compiled for this many GPUs per node (0 = any).
template <bool WIDE, bool TREE, bool CACHE, int EXT, int GPN>
__global__ __launch_bounds__(WAVE) void k_sim_chain_steps(SimDev S, const DOp* __restrict__ ops, const DEdge* __restrict__ edges,
                                                          const DEdge* __restrict__ in_edges, const uint32_t* __restrict__ cost,
                                                          const uint32_t* __restrict__ magic, unsigned char* chain_mem,
                                                          size_t chain_stride, uint32_t n_snaps, uint32_t C,
                                                          const uint32_t* __restrict__ muts, uint32_t n_steps,
                                                          u64* __restrict__ out_ns, uint32_t* chain_flags, SearchDev search) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const Tables T{ops, edges, in_edges, cost};
    // the chain's strategy is worked on in LDS (and written through to HBM), so that the many
    // uniform configuration look-ups do not queue behind the wavefront's stores to HBM
    uint2* cfg_lds = (uint2*)lds_raw;
    const WaveLds L = carve_lds(lds_raw + (size_t)S.n_ops_pad * 8, S);
    const uint32_t c = blockIdx.x;
    if (c >= C) return;
    const int lane = lane_id();
    const ChainMem cm = carve_chain(chain_mem + (size_t)c * chain_stride, S, n_snaps);
    const uint32_t magic_v = load_magic(magic);
    const uint32_t n_words = S.n_ops * WAVE;
    for (uint32_t i = lane; i < S.n_ops; i += WAVE) cfg_lds[i] = cm.cfgs[i];
    wave_sync();
    bool poisoned = first_u32(chain_flags[c]) != 0;
    ChainMeta meta = *cm.meta;
    meta.step = first_u64(meta.step);
    meta.n_valid = first_u32(meta.n_valid);
    meta.stale = first_u32(meta.stale);
    meta.n_steps = first_u64(meta.n_steps);
    meta.n_resumed = first_u64(meta.n_resumed);
    meta.n_events = first_u64(meta.n_events);
    meta.n_events_full = first_u64(meta.n_events_full);
    meta.cur_ns = first_u64(meta.cur_ns);
    meta.idle_steps = first_u64(meta.idle_steps);
    meta.n_converged = first_u64(meta.n_converged);
    meta.loc = first_u32(meta.loc);
    meta.tag = first_u32(meta.tag);
    Recorder rec{cm.end_try, cm.snap_words, cm.snap_l1, cm.snap_free, meta.step, 0, meta.loc, n_snaps, 1, 0, 0};
    SimT<false, EXT, GPN> m{S, T, cfg_lds, cm.words, cm.exe_of, L, magic_v, 0, false, NO_OVERRIDE, make_uint2(0, 0), CACHE ? cm.ecache : nullptr, true};
    if (EXT) { m.links = (const uint4*)(magic + LINK_TABLE_AT); m.node_links = m.links + (size_t)S.gpus_per_node * S.gpus_per_node; }
    if (EXT >= 2 && S.ties) m.tie = magic + tie_table_at(S.gpus_per_node, S.n_nodes);
    // With tied configurations a mutation changes several ops at once: such steps are simulated from time 0.
    const bool tied = EXT >= 2 && S.ties;
    m.want_sort = true;          // a later step may make the strategy a general one: the kept set-up is always complete
    u64 best = search.enabled ? first_u64(search.best_ns[c]) : 0;
    if (search.enabled && !poisoned && !meta.stale && meta.cur_ns < best) {
        // the strategy the search starts from counts as seen
        best = meta.cur_ns;
        for (uint32_t i = lane; i < S.n_ops; i += WAVE) search.best_cfgs[(size_t)c * S.n_ops + i] = cfg_lds[i];
    }

    // look-ahead: this launch takes the chain from step done[c] up to its first accepted proposal, at most n_ahead steps
    const bool own_position = search.enabled && search.done != nullptr;
    const bool ahead = own_position && search.ahead_ns != nullptr;
    uint32_t s_begin = 0, s_end = n_steps, n_taken = 0;
    if (own_position) {
        s_begin = first_u32(search.done[c]);
        s_begin = s_begin < n_steps ? s_begin : n_steps;
        s_end = n_steps - s_begin < search.n_ahead ? n_steps : s_begin + search.n_ahead;
    }
    const u64 clock_begin = (own_position && search.time_limit) ? wall_clock64() : 0;
    uint32_t s = s_begin;
    for (; s < s_end; s++) {
        Counters cnt = {};
        bool proposal = false, valid = true;
        bool known_rejected = false;     // look-ahead: simulated beforehand and not taken
        uint32_t op = 0;
        uint2 ocfg = make_uint2(0, 0);
        if (search.enabled) {
            if (!poisoned && !meta.stale && !(search.patience && meta.idle_steps >= search.patience)) {
                const u64 st = search.first_step + s;
                uint2 ncfg;
                if (search_proposal(search, S.n_ops, S.n_dev, c, st, op, ncfg)) {   // an op without a list gets no proposals
                    op = first_u32(op);
                    if (ahead && !search_accepts(search, c, st, first_u64(search.ahead_ns[(size_t)(s - s_begin) * C + c]), meta.cur_ns)) {
                        known_rejected = true;
                    } else {
                        ocfg = cfg_lds[op];
                        wave_sync();
                        if (lane == 0) cfg_lds[op] = make_uint2(first_u32(ncfg.x), first_u32(ncfg.y));
                        wave_sync();
                        proposal = true;
                    }
                }
            }
        } else if (muts) {
            const uint32_t* mu = muts + ((size_t)s * C + c) * 3;
            op = first_u32(mu[0]);
            if (op >= S.n_ops) poisoned = true;
            if (!poisoned) {
                ocfg = cfg_lds[op];
                wave_sync();
                if (lane == 0) {
                    const uint2 ncfg = make_uint2(mu[1], mu[2]);
                    cfg_lds[op] = ncfg;
                    cm.cfgs[op] = ncfg;
                }
                wave_sync();
            }
        }
        u64 mk = RESULT_INVALID;
        StrategyClass cls = STRATEGY_INVALID;
        // (a proposal known to be rejected changes nothing: the strategy in force was validated when it was taken)
        if (!poisoned && !known_rejected) cls = validate_strategy(m);
        valid = known_rejected || cls != STRATEGY_INVALID;
        if (!poisoned && !valid && !proposal) { meta.stale = 1; meta.cur_ns = RESULT_INVALID; }
        const bool changed = muts != nullptr || proposal;
        if ((changed || known_rejected) && !poisoned) meta.n_steps++;
        bool accepted = false;

        if (search.enabled && !proposal && !poisoned && !meta.stale) {
            mk = meta.cur_ns;   // no proposal this step: nothing to simulate
        } else if (!poisoned && valid) {
            // where the simulation may start (0 = time 0)
            uint32_t k = 0, pend_new = 0;
            if (changed && !meta.stale && meta.n_valid > 1 && meta.step != 0 && !tied) k = resume_point(m, cm.end_of, meta, op, ocfg, pend_new);
            const uint32_t capacity = n_snaps;
            // phase 1: makespan only, to fix the snapshot spacing (no snapshots yet);
            // phase 2: the recorded simulation
            int phase = (k == 0 && meta.step == 0) ? 1 : 2;
            u64 rc = 0;
            bool converged = false;
            while (phase < 3) {
                const bool record = phase == 2;
                const u64 before = cnt.n_events;
                if (record) {
                    meta.tag = meta.tag >= 0xffffu ? 0u : meta.tag;
                    if (meta.tag == 0) {
                        // tags start over: forget what earlier runs wrote
                        for (uint32_t t = lane; t < n_words; t += WAVE) cm.end_try[t] = 0;
                        __threadfence_block();
                        wave_sync();
                    }
                    meta.tag++;
                }
                rec.step = meta.step;
                rec.tag = (u64)meta.tag << 48;
                rec.loc = meta.loc;
                rec.n_snaps = record ? capacity : 0;
                rec.end_try = record ? cm.end_try : nullptr;
                rec.next = k + 1;
                // a resumed run of a changed strategy may re-join the accepted timeline
                rec.check_below = (record && k > 0 && changed) ? meta.n_valid : 0u;
                rec.check_op = op;
                if (k == 0) {
                    init_state(m, cnt);
                } else {
                    if (CACHE && record) refresh_ecache_for_op(m, op);
                    load_snapshot(m, rec, k);
                    // the loaded state still describes the op under its old configuration
                    patch_state_for_op(m, m.words, L.l1, op, ocfg, pend_new);
                    wave_sync();
                    rebuild_l2(m);
                }
                rc = cls == STRATEGY_REGULAR ? run_events<WIDE, true, true, false, TREE ? Q_TREE : Q_FLAT, CACHE>(m, cnt, rec)
                                             : run_events<WIDE, true, false, false, TREE ? Q_TREE : Q_FLAT, CACHE>(m, cnt, rec);
                if (rc == RUN_CONVERGED) { converged = true; rc = 0; mk = meta.cur_ns; break; }
                mk = rc ? rc : makespan(m);
                if (rc) break;
                if (phase == 1) { meta.step = (2 * mk) / capacity + 1; phase = 2; continue; }
                if (k == 0) meta.n_events_full = cnt.n_events - before;
                break;
            }
            if (changed) meta.n_events += cnt.n_events;
            // the decision: forced mutations and the starting strategy are always taken; a proposal
            // by the Metropolis rule (Section 6.1) with tabulated probabilities
            if (!rc) accepted = proposal ? search_accepts(search, c, search.first_step + s, mk, meta.cur_ns) : true;
            if (accepted) {
                if (proposal && lane == 0) cm.cfgs[op] = cfg_lds[op];
                if (k > 0) {
                    meta.n_resumed++;
                    // what the snapshots that stay hold about the op is rewritten for its new configuration
                    for (uint32_t sn = 1; sn <= k; sn++) {
                        const size_t at = (size_t)(((meta.loc >> sn) & 1u) * n_snaps + sn);
                        patch_state_for_op(m, cm.snap_words + at * n_words, cm.snap_l1 + at * S.n_ops_pad, op, ocfg, pend_new);
                    }
                }
                commit_run(cm, meta, rec, k + 1, n_words, converged);
                if (converged) meta.n_converged++;
                meta.stale = 0;
                meta.cur_ns = mk;
                // the spacing was fixed by an earlier makespan; if the timeline has become more than
                // twice shorter or longer, re-space: the snapshots are dropped and the next simulation
                // starts from time 0 with the new spacing
                const u64 ideal = (2 * mk) / capacity + 1;
                if (ideal * 2 < meta.step || ideal > meta.step * 2) { meta.step = ideal; meta.n_valid = 1; }
            } else if (proposal) {
                wave_sync();
                if (lane == 0) cfg_lds[op] = ocfg;
                wave_sync();
                if (CACHE) refresh_ecache_for_group(m, op);
                mk = meta.cur_ns;
            } else {
                // a forced step whose simulation failed (overflow): no timeline for this strategy
                meta.stale = 1;
                meta.n_valid = 0;
                meta.cur_ns = mk;
            }
        } else if (proposal && !valid) {
            // an invalid proposal is rejected
            wave_sync();
            if (lane == 0) cfg_lds[op] = ocfg;
            wave_sync();
            mk = meta.cur_ns;
        }
        if (search.enabled) meta.idle_steps++;
        if (search.enabled && !poisoned && mk < RESULT_OVERFLOW && mk < best) {
            best = mk;
            meta.idle_steps = 0;
            for (uint32_t i = lane; i < S.n_ops; i += WAVE) search.best_cfgs[(size_t)c * S.n_ops + i] = cfg_lds[i];
        }
        if (lane == 0) out_ns[(size_t)s * C + c] = mk;
        wave_sync();
        // what was simulated ahead for the later steps assumed the strategy this step has just replaced
        if (proposal && accepted) n_taken++;
        if (ahead && proposal && accepted) { s++; break; }
        if (own_position && search.time_limit && first_u64(wall_clock64() - clock_begin) >= search.time_limit) { s++; break; }
    }
    if (lane == 0) {
        chain_flags[c] = poisoned ? 1u : 0u;
        *cm.meta = meta;
        if (search.enabled) search.best_ns[c] = best;
        if (own_position) { search.done[c] = s; search.n_accepted[c] += n_taken; }
    }
}

// Trial mutations (the proposals of Section 6.2 before acceptance): evaluates M alternative
// single-op mutations per chain, each against the chain's current strategy and stored
// timeline, without changing the chain.  One wavefront per (proposal, chain); its task words
// live in a private workspace slot, the chain's snapshots are only read.
template <bool WIDE, bool TREE, bool CACHE, int EXT, int GPN>
__global__ __launch_bounds__(WAVE) void k_sim_chain_try(SimDev S, const DOp* __restrict__ ops, const DEdge* __restrict__ edges,
                                                        const DEdge* __restrict__ in_edges, const uint32_t* __restrict__ cost,
                                                        const uint32_t* __restrict__ magic, const unsigned char* __restrict__ chain_mem,
                                                        size_t chain_stride, uint32_t n_snaps, uint32_t C,
                                                        const uint32_t* __restrict__ muts, uint32_t M, u64* __restrict__ out_ns,
                                                        const uint32_t* __restrict__ chain_flags, uint32_t* __restrict__ next_item,
                                                        unsigned char* __restrict__ ws, size_t slot_stride) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const Tables T{ops, edges, in_edges, cost};
    const WaveLds L = carve_lds(lds_raw, S);
    const uint32_t magic_v = load_magic(magic);
    unsigned char* slot = ws + (size_t)blockIdx.x * slot_stride;
    u64* words = (u64*)slot;
    uint32_t* exe_of = (uint32_t*)(slot + (size_t)S.n_ops * WAVE * 8);
    const uint32_t total = M * C;
    // proposals differ a lot in cost (how much of the timeline they keep): wavefronts draw the
    // next one from a counter instead of striding
    for (;;) {
        uint32_t id = 0;
        if (lane_id() == 0) id = atomicAdd(next_item, 1u);
        id = first_u32(id);
        if (id >= total) break;
        const uint32_t c = id % C;
        // the chain is only read here
        const ChainMem cm = carve_chain(const_cast<unsigned char*>(chain_mem) + (size_t)c * chain_stride, S, n_snaps);
        ChainMeta meta = *cm.meta;
        meta.step = first_u64(meta.step);
        meta.n_valid = first_u32(meta.n_valid);
        meta.stale = first_u32(meta.stale);
        const uint32_t* mu = muts + (size_t)id * 3;     // [M][C] records {op, cfg.x, cfg.y}
        const uint32_t op = first_u32(mu[0]);
        u64 mk = RESULT_INVALID;
        if (op < S.n_ops && first_u32(chain_flags[c]) == 0) {
            const uint2 ocfg = cm.cfgs[op];
            SimT<true, EXT, GPN> m{S, T, cm.cfgs, words, exe_of, L, magic_v, 0, false, op, make_uint2(first_u32(mu[1]), first_u32(mu[2])),
                              CACHE ? cm.ecache : nullptr, false};
            if (EXT) { m.links = (const uint4*)(magic + LINK_TABLE_AT); m.node_links = m.links + (size_t)S.gpus_per_node * S.gpus_per_node; }
            if (EXT >= 2 && S.ties) m.tie = magic + tie_table_at(S.gpus_per_node, S.n_nodes);
            m.want_sort = true;
            const StrategyClass cls = validate_strategy(m);
            if (cls != STRATEGY_INVALID) {
                Counters cnt = {};
                Recorder rec{nullptr, cm.snap_words, cm.snap_l1, cm.snap_free, meta.step, 0, first_u32(meta.loc), n_snaps, 1, 0, 0};
                uint32_t k = 0, pend_new = 0;
                if (!meta.stale && meta.n_valid > 1 && meta.step != 0 && !(EXT >= 2 && S.ties)) k = resume_point(m, cm.end_of, meta, op, ocfg, pend_new);
                if (k == 0) {
                    init_state(m, cnt);
                } else {
                    load_snapshot(m, rec, k);
                    patch_state_for_op(m, m.words, L.l1, op, ocfg, pend_new);
                    wave_sync();
                    rebuild_l2(m);
                }
                const u64 rc = cls == STRATEGY_REGULAR ? run_events<WIDE, false, true, false, TREE ? Q_TREE : Q_FLAT, CACHE>(m, cnt, rec)
                                                       : run_events<WIDE, false, false, false, TREE ? Q_TREE : Q_FLAT, CACHE>(m, cnt, rec);
                mk = rc ? rc : makespan(m);
            }
        }
        if (lane_id() == 0) out_ns[id] = mk;
        wave_sync();
    }
}

}  // namespace ffsim
