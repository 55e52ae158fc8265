// Algorithm 1 on the device: the per-row FIFO, the recording of a run (endTimes, snapshots), the
// initial state and the event loop.
#pragma once
#include "ffsim_strategy.h"

namespace ffsim {

// Serialise tasks that become ready at the same time r on device rows, in lane order
// (= id order): end = max(r, row free time) + running sum of exeTimes on that row.
// One LDS round trip: every lane writes its lane id to a one-byte tag of its row, then reads
// the tag back together with the row's free time.  A lane that reads another lane's id
// shares its row; the lanes of such rows are grouped and ranked with ballots (never through
// memory), everybody else is done at once.  The last lane of every row writes the new free
// time.  `may_share` = false promises distinct rows and skips the tags.
__device__ __forceinline__ u64 fifo_commit(bool act, uint32_t row, u64 exe, u64 r, bool may_share, const WaveLds& L) {
    const int lane = lane_id();
    u64 f = 0;
    bool lost = false;
    if (may_share) {
        if (act) L.tag[row] = (uint8_t)lane;
        wave_sync();
        if (act) { lost = L.tag[row] != (uint8_t)lane; f = L.free_at[row]; }
    } else if (act) {
        f = L.free_at[row];
    }
    const u64 base = f > r ? f : r;         // identical for all lanes of one row
    u64 end = base + exe;
    bool last = act;
    u64 todo = ballot(lost);
    while (todo) {
        const int l = __builtin_ctzll(todo);
        const uint32_t lrow = readlane_u32(row, l);
        const bool peer = act && row == lrow;   // includes the lane whose tag survived
        const u64 peers = ballot(peer);
        todo &= ~peers;
        const int first = __builtin_ctzll(peers);
        const u64 exe_l = readlane_u64(exe, first);
        if (!ballot(peer && exe != exe_l)) {
            // equal exeTimes (symmetric parts): the position in the group is enough
            const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(peers >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)peers, 0u)) + 1;
            if (peer) end = base + (u64)rank * exe;
        } else {
            u64 t = 0;
            u64 pm = peers;
            while (pm) {
                const int p = __builtin_ctzll(pm);
                pm &= pm - 1;
                t += readlane_u64(exe, p);
                if (lane == p) end = base + t;
            }
        }
        if (peer) last = lane == 63 - __builtin_clzll(peers);
    }
    if (last) L.free_at[row] = end;
    wave_sync();
    return end;
}

// Optional recording for delta simulation: endTime of every task, and snapshots of the
// simulation state whenever the event time crosses a multiple of `step`.
//
// Every snapshot index has two storage places (set 0 and set 1).  Bit k of `loc` says which of
// them holds snapshot k of the chain's ACCEPTED timeline; a recorded run writes snapshot k into
// the other place, and endTimes into their own array, marked with the run's tag.  Nothing of
// the accepted timeline is touched until the run is committed (the bits of the snapshots it
// wrote are flipped, its endTimes are copied over); a run that is not committed leaves no trace.
struct Recorder {
    u64* end_try;            // [n_ops*64] tag<<48 | endTime of the tasks the run committed (null: not recorded)
    u64* snap_words;         // [2][n_snaps][n_ops*64]
    u64* snap_l1;            // [2][n_snaps][n_ops_pad]
    u64* snap_free;          // [2][n_snaps][n_rows]
    u64 step;                // snapshot k holds the state before the first event with word >= k*step
    u64 tag;                 // this run's tag, already shifted (tag << 48)
    uint32_t loc;            // see above
    uint32_t n_snaps;        // capacity (snapshot 0 is the initial state and is never stored)
    uint32_t next;           // next snapshot index to write
    // Re-convergence: a run that resumed after a change of op check_op compares every state it
    // snapshots (index < check_below) with the accepted timeline's snapshot of the same index.
    // Once they agree (and check_op has no task left), the rest of the two timelines is the same
    // and the run stops.  check_below = 0: no comparison.
    uint32_t check_below;
    uint32_t check_op;
};
constexpr uint32_t MAX_SNAPSHOTS = 32;   // bits of loc
constexpr u64 RUN_CONVERGED = 1;         // run_events: stopped because the timeline re-joined the accepted one

template <class SimX>
__device__ __forceinline__ void rebuild_l2(const SimX& m) {
    if (m.S.n_groups > FLAT_GROUPS) {
        for (uint32_t g = 0; g < m.S.n_groups; g++) {
            const u64 wmin = wave_min_u64(m.L.l1[g * WAVE + lane_id()]);
            if (lane_id() == 0) m.L.l2[g] = wmin;
        }
        wave_sync();
    }
}

// count_inputs (ffsim_strategy.h) from ranges that are already known
template <bool TRAIN = false>
__device__ __forceinline__ uint32_t count_inputs_of(const DEdge& e, const OpCfg& cp, const EdgeLane& el, uint32_t magic_v) {
    if (TRAIN && e.kind) return count_contributors(e, cp, el.nlo, el.nhi, magic_v);   // (the kept ranges are the part's own box)
    uint32_t n = 1;
#pragma unroll
    for (int d = 0; d < 4; d++) {
        if ((uint32_t)d < e.src_ndim) {
            uint32_t c;
            if (cp.deg[d] == 1) {
                c = el.nhi[d] > el.nlo[d] ? 1u : 0u;           // the producer does not split this dim (uniform)
            } else if (e.map[d].src_dim < 0) {
                c = cp.deg[d];                                   // the whole extent is read: every part (uniform)
            } else {
                c = 0;
                if (el.nhi[d] > el.nlo[d])
                    c = owner_part((uint32_t)el.nhi[d] - 1, e.src_extent[d], cp.deg[d]) - owner_part((uint32_t)el.nlo[d], e.src_extent[d], cp.deg[d]) + 1;
            }
            n *= c;
        }
    }
    return n;
}

// Section 5.1 step 1 and the start of Algorithm 1: the tasks, how many inputs each waits
// for, the initial READY set, idle devices.
template <class SimX>
__device__ __forceinline__ void init_state(SimX& m, Counters& cnt) {
    const int lane = lane_id();
    for (uint32_t r = lane; r < m.S.n_rows; r += WAVE) m.L.free_at[r] = 0;
    for (uint32_t j = 0; j < m.S.n_ops; j++) {
        const OpCfg cj = m.cfg(j);
        uint32_t pending = 0;
        if (m.ecache && m.ecache_fill) {
            // what every later release of an in-edge needs about this op's parts is computed here, once
            const uint32_t in_begin = m.T.ops[j].in_begin, in_end = m.T.ops[j].in_end;
            for (uint32_t q = in_begin; q < in_end; q++) {
                const DEdge e = m.T.in_edges[q];
                const EdgeLane el = edge_lane(m, e, cj);
                ecache_store(m.ecache, m.S.n_edges, e.eid, el);
                pending += count_inputs_of<SimX::kTrain>(e, m.cfg(e.src), el, m.magic_v);
            }
        } else {
            pending = count_pending(m, j, cj);
        }
        // pending < PENDING_LIMIT is guaranteed by ff_sim_create (at most 511 in-edges per op)
        const u64 w = (uint32_t)lane >= cj.parts ? W_NONE : (pending == 0 ? 1ull : (W_WAIT | ((u64)pending << 48)));
        m.words[j * WAVE + lane] = w;
        // level 1 only has to order pending events: at the start an op has one (READY at time 0) or none
        const u64 any_ready = ballot(w == 1ull);
        if (lane == 0) m.L.l1[j] = any_ready ? 1ull : W_NONE;
        cnt.n_compute += cj.parts;
    }
    for (uint32_t j = m.S.n_ops + lane; j < m.S.n_ops_pad; j += WAVE) m.L.l1[j] = W_NONE;
    wave_sync();
    rebuild_l2(m);
    m.last_key = 0;
    m.overflow = false;
}

// wavefront-wide copy of n 64-bit words between 16-byte aligned HBM buffers, n a multiple of
// 64: 16 bytes per lane and eight loads in flight before the first store
__device__ __forceinline__ void copy_words(u64* __restrict__ dst, const u64* __restrict__ src, uint32_t n) {
    const uint4* __restrict__ s4 = (const uint4*)src;
    uint4* __restrict__ d4 = (uint4*)dst;
    const uint32_t n4 = n / 2;          // multiple of 32
    uint32_t t = lane_id();
    for (; t + 7 * WAVE < n4; t += 8 * WAVE) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = s4[t + u * WAVE];
#pragma unroll
        for (int u = 0; u < 8; u++) d4[t + u * WAVE] = v[u];
    }
    for (; t < n4; t += WAVE) d4[t] = s4[t];
}

// the same copy, and: does src differ from old anywhere?  (per lane; combine with a ballot)
__device__ __forceinline__ bool copy_words_compare(u64* __restrict__ dst, const u64* __restrict__ src, const u64* __restrict__ old,
                                                   uint32_t n) {
    const uint4* __restrict__ s4 = (const uint4*)src;
    const uint4* __restrict__ o4 = (const uint4*)old;
    uint4* __restrict__ d4 = (uint4*)dst;
    const uint32_t n4 = n / 2;
    uint32_t diff = 0;
    uint32_t t = lane_id();
    for (; t + 3 * WAVE < n4; t += 4 * WAVE) {
        uint4 v[4], o[4];
#pragma unroll
        for (int u = 0; u < 4; u++) { v[u] = s4[t + u * WAVE]; o[u] = o4[t + u * WAVE]; }
#pragma unroll
        for (int u = 0; u < 4; u++) {
            d4[t + u * WAVE] = v[u];
            diff |= (v[u].x ^ o[u].x) | (v[u].y ^ o[u].y) | (v[u].z ^ o[u].z) | (v[u].w ^ o[u].w);
        }
    }
    for (; t < n4; t += WAVE) {
        const uint4 v = s4[t], o = o4[t];
        d4[t] = v;
        diff |= (v.x ^ o.x) | (v.y ^ o.y) | (v.z ^ o.z) | (v.w ^ o.w);
    }
    return diff != 0;
}

// Writes the next snapshot.  Returns true if the comparison is on and the state equals the
// accepted timeline's snapshot of the same index for everything that can still matter: all task
// words, and the free time of every device row, where rows that are idle at the snapshot's
// time count as equal (any later task is ready at or after that time).
template <class SimX>
__device__ __forceinline__ bool save_snapshot(const SimX& m, Recorder& rec) {
    const int lane = lane_id();
    const uint32_t idx = rec.next;
    const size_t k = (size_t)((((rec.loc >> idx) & 1u) ^ 1u) * rec.n_snaps + idx);   // the place the accepted timeline does not use
    const bool check = idx < rec.check_below;
    bool differs = false;
    const size_t nw = (size_t)m.S.n_ops * WAVE;
    if (check) {
        const size_t old = (size_t)(((rec.loc >> idx) & 1u) * rec.n_snaps + idx);
        differs = copy_words_compare(rec.snap_words + k * nw, m.words, rec.snap_words + old * nw, m.S.n_ops * WAVE);
        const u64 t_snap = ((u64)idx * rec.step) >> 1;
        const u64* ofr = rec.snap_free + old * (size_t)m.S.n_rows;
        for (uint32_t t = lane; t < m.S.n_rows; t += WAVE) {
            const u64 a = m.L.free_at[t], b = ofr[t];
            differs = differs || (a > t_snap ? a : t_snap) != (b > t_snap ? b : t_snap);
        }
        // a task of the changed op still pending would make equal words mean different things
        differs = differs || m.words[(size_t)rec.check_op * WAVE + lane] != W_NONE;
    } else {
        copy_words(rec.snap_words + k * nw, m.words, m.S.n_ops * WAVE);
    }
    u64* l1 = rec.snap_l1 + k * (size_t)m.S.n_ops_pad;
    for (uint32_t t = lane; t < m.S.n_ops_pad; t += WAVE) l1[t] = m.L.l1[t];
    u64* fr = rec.snap_free + k * (size_t)m.S.n_rows;
    for (uint32_t t = lane; t < m.S.n_rows; t += WAVE) fr[t] = m.L.free_at[t];
    rec.next++;
    return check && !ballot(differs);
}

// snapshot k of the accepted timeline
template <class SimX>
__device__ __forceinline__ void load_snapshot(SimX& m, const Recorder& rec, uint32_t k) {
    const int lane = lane_id();
    const size_t at = (size_t)(((rec.loc >> k) & 1u) * rec.n_snaps + k);
    copy_words(m.words, rec.snap_words + at * m.S.n_ops * WAVE, m.S.n_ops * WAVE);
    const u64* l1 = rec.snap_l1 + at * m.S.n_ops_pad;
    for (uint32_t t = lane; t < m.S.n_ops_pad; t += WAVE) m.L.l1[t] = l1[t];
    const u64* fr = rec.snap_free + at * m.S.n_rows;
    for (uint32_t t = lane; t < m.S.n_rows; t += WAVE) m.L.free_at[t] = fr[t];
    wave_sync();
    m.last_key = (u64)k * rec.step;
    m.overflow = false;
}

// Algorithm 1, main loop, from the current state to the end.  RECORD: keep endTimes and
// snapshots for delta simulation.  Returns 0 or a RESULT_* code.
// REG: the strategy is STRATEGY_REGULAR.  STATS: also count pairs and transfers (the optional
// per-candidate record); a compile-time switch so that the counters cost the timed path nothing.
// CACHE: the per-edge set-up was stored by init_state (m.ecache).
// Q: shape of the queue above the task words.
//   Q_ONE   at most 64 ops: level 1 (one minimum per op) sits in a register, lane = op; nothing of
//           the queue is in LDS while the loop runs (batch kernels only: level 1 is not written back);
//   Q_ONE16 the same for at most 16 ops of at most 16 parts each (16 columns in the cost table): every
//           reduction over ops or over parts ends in the first row of 16 lanes;
//   Q_FLAT  up to FLAT_GROUPS groups of 64 ops: level 1 in LDS, every lane scans its column;
//   Q_TREE  more groups: level 1 in LDS, level 2 (one minimum per group) in a register, lane = group.
enum QueueShape : int { Q_ONE = 0, Q_FLAT = 1, Q_TREE = 2, Q_ONE16 = 3 };
template <bool WIDE, bool RECORD, bool REG, bool STATS, int Q, bool CACHE, class SimX>
__device__ u64 run_events(SimX& m, Counters& cnt, Recorder& rec) {
    constexpr bool TREE = Q == Q_TREE;
    constexpr bool ONE = Q == Q_ONE || Q == Q_ONE16, ROW0 = Q == Q_ONE16;
    // runs of events (below) are formed where looking for them pays: graphs of more than 64 ops
#if defined(FFSIM_NO_RUNS)
    constexpr bool RUNS = false;
#elif defined(FFSIM_RUNS_ALL)
    constexpr bool RUNS = true;
#else
    constexpr bool RUNS = !ONE;
#endif
    const int lane = lane_id();
    PROF_DECL
    const SimDev& S = m.S;
    const WaveLds& L = m.L;
    const DOp* __restrict__ ops = m.T.ops;
    const DEdge* __restrict__ edges = m.T.edges;
    u64* words = m.words;
    const uint32_t magic_v = m.magic_v;
    u64 last_key = m.last_key;
    bool overflow = m.overflow;
    // the register-resident level of the queue (see QueueShape)
    u64 qreg = W_NONE;
    if (ONE) qreg = L.l1[lane];
    if (Q == Q_TREE) qreg = (uint32_t)lane < S.n_groups ? L.l2[lane] : W_NONE;
    // Values chosen per lane between two of these (same node or not) must sit in registers: a
    // select between two fields of the argument block is otherwise turned into a per-lane load
    // from that block, a vector memory round trip for every producer part.
    // They are kept in vector registers for the whole loop: a select then is one instruction (it can
    // read only one scalar operand, the lane mask), and six scalar registers stay free.
    const uint32_t bw_intra = vector_copy(S.bw_intra), bw_inter = vector_copy(S.bw_inter);
    const uint32_t m_bw_intra = vector_copy(S.m_bw_intra), m_bw_inter = vector_copy(S.m_bw_inter);
    const uint32_t lat_intra = vector_copy(S.lat_intra), lat_inter = vector_copy(S.lat_inter);
    const u64 max_events = 2ull * S.n_ops * WAVE + 8;   // every task is popped at most twice
    for (u64 ev = 0; ev < max_events; ev++) {
        u64 kmin;
        uint32_t i;
        // what the search for the popped op leaves behind for `others_min` below
        u64 row_rest = W_NONE;      // TREE: smallest key of the other ops of the popped op's group
        u64 k1 = W_NONE;            // FLAT: this lane's column minimum of level 1
        uint32_t gbest = 0, col = 0;
        if (ONE) {
            kmin = wave_min_from<ROW0>(qreg, last_key);
            if (kmin >> 63) break;
            const u64 m1 = ballot(qreg == kmin);
            if (!m1) { cnt.exit_code = 1; return RESULT_INTERNAL; }
            i = __builtin_ctzll(m1);                 // lowest op index among equal keys
        } else if (TREE) {
            const u64 k2 = qreg;
            kmin = wave_min_from(k2, last_key);
            if (kmin >> 63) break;
            const uint32_t g = __builtin_ctzll(ballot(k2 == kmin));
            const u64 row = L.l1[g * WAVE + lane];
            const u64 m1 = ballot(row == kmin);
            if (!m1) { cnt.exit_code = 1; return RESULT_INTERNAL; }   // tree inconsistent: give up, never spin
            col = __builtin_ctzll(m1);
            i = g * WAVE + col;
            // the group's minimum once the popped op is set aside: the end of the event needs it for
            // level 2 (no second pass over the row), and a run of events may extend up to it
            row_rest = wave_min_from((uint32_t)lane == col ? W_NONE : row, last_key);
        } else {
            // few ops: every lane scans its column of level 1, no level 2
            k1 = L.l1[lane];
            for (uint32_t g = 1; g < S.n_groups; g++) {
                const u64 k = L.l1[g * WAVE + lane];
                if (k < k1) { k1 = k; gbest = g; }
            }
            kmin = wave_min_from(k1, last_key);
            if (kmin >> 63) break;
            // lowest op index among equal keys: smallest group first, then lowest lane
            u64 m1 = ballot(k1 == kmin);
            if (!m1) { cnt.exit_code = 1; return RESULT_INTERNAL; }
            if (m1 & (m1 - 1)) {    // several columns hold the minimum: smallest group wins
                const uint32_t gmin = wave_min_u32(k1 == kmin ? gbest : 0xffffffffu);
                m1 = ballot(k1 == kmin && gbest == gmin);
            }
            col = __builtin_ctzll(m1);
            i = readlane_u32(gbest, col) * WAVE + col;
        }
        static_assert(!(RECORD && ONE), "snapshots read level 1 from LDS");
        if (RECORD) {
            // the state before the first event at or after a multiple of `step` is a snapshot
            while (rec.next < rec.n_snaps && kmin >= (u64)rec.next * rec.step) {
                if (save_snapshot(m, rec)) { m.last_key = last_key; return RUN_CONVERGED; }
            }
        }
        last_key = kmin;
        PROF_MARK(1)
        // everything that depends only on i is requested together
        u64 k0 = words[i * WAVE + lane];
        const DOp* __restrict__ opi_p = ops + i;
        const uint32_t out_begin = opi_p->out_begin, out_end = opi_p->out_end;
        const OpCfg ci = m.cfg(i);
        const u64 exe = m.exe_of[i];
        const uint32_t dev_p = m.template device_of<REG>(i, ci);   // (with explicit devices a load: requested with the words)
        PROF_MARK(1)
        PROF_VMWAIT(2)
        const u64 mask_same = ballot(k0 == kmin);       // parts of op i that hold the minimum
        if (!mask_same) { cnt.exit_code = 2; return RESULT_INTERNAL; }
        cnt.n_events++;
        const u64 now = kmin >> 1;
        const u64 k_own = k0;                            // the event words of op i as loaded
        // A RUN of events.  The events of Algorithm 1's queue that follow the popped one in
        // (time, kind, op, part) order and belong to the same op and kind can be handled in the same step, each
        // at its own time, as long as no event of another op, no event of the other kind of this op and
        // (RECORD) no snapshot boundary lies before them: they are consecutive in the order, so handling
        // them together IS handling them in order.  The events a run creates must not fall inside it:
        // a dequeued task is released exeTime after its readyTime or later; a release makes consumer
        // tasks READY, whose dequeuing touches nothing a release touches (compute device rows and their
        // own words against link rows and waiting words), but whose own releases come exeTime later.
        // READY tasks only in the regular form (the parts of an op sit on distinct devices); releases only
        // if the op has one out-edge (transfers of several edges interleave by time on shared links)
        // and no parameter traffic (queued per replica after the op's transfers).
        u64 mask = mask_same;
        bool mixed = false;                              // the step holds events of different times
        if (RUNS && ((kmin & 1) ? REG : (out_end - out_begin == 1 && !(SimX::kExt && S.sync)))) {
            const bool same_kind = !(k0 >> 63) && (((uint32_t)k0 ^ (uint32_t)kmin) & 1u) == 0;
            const u64 kind_m = ballot(same_kind);
            if (kind_m != mask_same) {
                // smallest key among the other ops
                u64 bound;
                if (ONE) {
                    bound = wave_min_from<ROW0>((uint32_t)lane == i ? W_NONE : qreg, last_key);
                } else if (TREE) {
                    bound = wave_min_from((uint32_t)lane == (i >> 6) ? row_rest : qreg, last_key);
                } else {
                    // the other columns' minima, and the popped op's column in the other groups
                    u64 v = (uint32_t)lane == col ? W_NONE : k1;
                    if ((uint32_t)lane < S.n_groups && (uint32_t)lane != (i >> 6)) {
                        const u64 c = L.l1[lane * WAVE + col];
                        v = c < v ? c : v;
                    }
                    bound = wave_min_from(v, last_key);
                }
                // the op's own events of the other kind end the run as well
                const bool other_kind = !(k0 >> 63) && (((uint32_t)k0 ^ (uint32_t)kmin) & 1u) != 0;
                if (ballot(other_kind)) {
                    const u64 r0 = wave_min_from<ROW0>(other_kind ? k0 : W_NONE, last_key);
                    bound = r0 < bound ? r0 : bound;
                }
                // what the run itself brings about must come after it: the releases of the tasks it
                // dequeues (a task ends exeTime after its start or later), or the releases of the consumer
                // tasks it makes READY (dequeued at or after the release that completed their inputs)
                const u64 next_exe = (kmin & 1) ? exe : (u64)m.exe_of[opi_p->first.dst];
                const u64 first_new = kmin + 2 * next_exe;
                bound = first_new < bound ? first_new : bound;
                if (RECORD) {
                    if (rec.next < rec.n_snaps) {
                        const u64 edge = (u64)rec.next * rec.step;
                        bound = edge < bound ? edge : bound;
                    }
                }
                const u64 far = kmin + 0xfffffff0ull;    // times inside a step are told apart by 32-bit distances
                bound = far < bound ? far : bound;
                mask = mask_same | ballot(same_kind && k0 < bound);
                mixed = mask != mask_same;
            }
        }
        const bool in_mask = lanes_of(mask);

        if (kmin & 1) {
            // dequeue READY compute tasks: start = max(readyTime, device free), end = start + exeTime
            const bool may_share = REG ? false : ((SimX::kExt && m.devmap != nullptr) || !(ci.stride == 1 && ci.parts <= S.n_dev));
            // (a run of READY tasks: every task at its own readyTime; their devices are distinct)
            const u64 end = fifo_commit(in_mask, dev_p, exe, (REG && mixed) ? (k_own >> 1) : now, may_share, L);
            overflow = overflow || (in_mask && end >= TIME_LIMIT);
            // a finished task is looked at again only if it has something to release
            const bool releases = out_end > out_begin || (SimX::kExt && S.sync && opi_p->param_bytes != 0);
            if (in_mask) k0 = releases ? end << 1 : W_NONE;
            if (RECORD) { if (in_mask && rec.end_try) rec.end_try[i * WAVE + lane] = rec.tag | end; }
            PROF_MARK(3)
        } else {
            // the parts in `mask` finished at `now`: release their successors edge by edge
            DEdge e = opi_p->first;
            // the box of every part of the producer (what a reading edge intersects), from the op's own shape
            // (a contributing edge brings its own ranges, below)
            Box pb = {};
            bool pb_is_own = false;
            if (!(SimX::kTrain && e.kind)) {
                pb = part_box(e.src_extent, ci, lane, magic_v);
                pb_is_own = true;
            }
            const uint32_t node_p = m.node_of(dev_p);
            for (uint32_t ei = out_begin; ei < out_end; ei++) {
                if (ei != out_begin) e = edges[ei];
                const uint32_t j = e.dst;
                // a contributing edge intersects, instead, the range of the consumer's tensor that every producer part
                // contributes to (the range that follows the part's box through the edge's maps)
                if (SimX::kTrain && e.kind) {
                    const uint32_t digits_p = part_digits(ci, lane, magic_v);
#pragma unroll
                    for (int d = 0; d < 4; d++) {
                        int32_t lo = 0, hi = 1;
                        if ((uint32_t)d < e.src_ndim) needed_range(e.map[d], e.src_extent[d], ci.x, digits_p, magic_v, lo, hi);
                        pb.lo[d] = (uint32_t)lo; pb.hi[d] = (uint32_t)hi;
                    }
                    pb_is_own = false;
                } else if (SimX::kTrain && !pb_is_own) {
                    pb = part_box(e.src_extent, ci, lane, magic_v);      // (a reading edge after a contributing one)
                    pb_is_own = true;
                }
                u64 w = words[j * WAVE + lane];
                // REG: consumer parts sit on consecutive, distinct devices, so the transfers from
                // one producer part can share a link row only when their consumers sit on the
                // same remote node, and those consumers are a run of consecutive lanes (the node
                // of lane 0 may come back once more at the end, after the device numbers wrapped
                // around).  The FIFO order on every shared row is then a running sum along the
                // run, and no search for lanes with equal rows is needed.
                // (the op of a trial mutation differs from what the chain's kept set-up describes)
                const EdgeLane el = (CACHE && !m.overridden(j)) ? ecache_load(m.ecache, ei) : edge_lane(m, e, m.cfg(j));
                const bool mine = el.mine;
                int32_t nlo[4], nhi[4];
#pragma unroll
                for (int d = 0; d < 4; d++) { nlo[d] = el.nlo[d]; nhi[d] = el.nhi[d]; }
                const uint32_t dev_c = el.dev_c, node_c = el.node_c;
                const uint32_t local_c = m.local_of(dev_c, node_c);
                const uint32_t G = m.gpn();
                const uint32_t pos = el.pos, first_len = el.first_len, last_run_mask = el.last_run_mask;
                const bool wrapped = el.wrapped;
                const u64 run_end_m = REG ? ballot(el.run_end) : 0;
                // (general form: the consumer's parts in (node, part) order, and which of them share a GPU)
                const uint32_t sortw = (REG || WIDE) ? 0u : ((CACHE && !m.overridden(j)) ? ecache_sort_word(m.ecache, S.n_edges, ei) : el.sortw);
                const u64 dup_m = (REG || WIDE) ? 0 : ballot((sortw >> 23) & 1u);
                u64 ready = w & (TIME_LIMIT - 1);
                uint32_t pending = (uint32_t)(w >> 48) & PENDING_LIMIT;
                // Which lanes take part is kept as 64-bit lane masks and combined with scalar
                // instructions; a per-lane condition is made from a mask only where a lane acts on it.
                const u64 mine_m = ballot(mine);
                u64 touched_m = 0;
                u64 todo = mask;
                PROF_MARK(4)
                PROF_VMWAIT(5)
                while (todo) {
                    // next producer part: by part index; in a run of releases by (time, part index)
                    int kp = __builtin_ctzll(todo);
                    u64 now_kp = now;
                    if (mixed) {
                        const uint32_t dist = lanes_of(todo) ? (uint32_t)(k_own - kmin) : 0xffffffffu;
                        const uint32_t dmin = wave_min_u32(dist);
                        kp = __builtin_ctzll(ballot(dist == dmin));
                        now_kp = (kmin + dmin) >> 1;
                    }
                    todo &= ~(1ull << kp);
                    u64 hit_m = mine_m;
                    u64 elems = 1;
                    // (the number of dims stays one scalar that is compared here: taken out of the loop, the
                    // four comparisons would each occupy a pair of scalar registers as a lane mask)
                    uint32_t n_dims = first_u32(e.src_ndim);
                    asm volatile("" : "+s"(n_dims));
#pragma unroll
                    for (int d = 0; d < 4; d++) {
                        if ((uint32_t)d < n_dims) {
                            const int32_t plo = (int32_t)readlane_u32(pb.lo[d], kp), phi = (int32_t)readlane_u32(pb.hi[d], kp);
                            const int32_t lo = nlo[d] > plo ? nlo[d] : plo;
                            const int32_t hi = nhi[d] < phi ? nhi[d] : phi;
                            hit_m &= ballot(hi > lo);
                            // (a lane that misses in some dim carries a meaningless product: it is
                            // only used by lanes that hit in all dims)
                            if (WIDE) elems *= (u64)(uint32_t)(hi - lo);
                            else elems = (uint32_t)elems * (uint32_t)(hi - lo);
                        }
                    }
                    if (!hit_m) continue;
                    const uint32_t dev_a = readlane_u32(dev_p, kp);
                    const uint32_t node_a = readlane_u32(node_p, kp);
                    const u64 comm_mask = hit_m & ballot(dev_c != dev_a);
                    const bool comm = lanes_of(comm_mask);
                    u64 arrive = now_kp;
                    if (comm_mask) {
                        const u64 same_m = ballot(node_c == node_a);
                        const bool same_node = lanes_of(same_m);
                        // Section 5.1: the link device between the two devices.  The producer's share of
                        // the row index is scalar; per lane one select between two sums.
                        // (node * G * G + local * G = device * G)
                        const uint32_t row_intra = S.n_dev + dev_a * G;
                        const uint32_t row_inter = S.n_dev + S.n_nodes * G * G + node_a * S.n_nodes;
                        const uint32_t to_intra = row_intra + local_c, to_inter = row_inter + node_c;
                        const uint32_t row = same_node ? to_intra : to_inter;
                        // assumption A2: transfer time = size / bandwidth (rounded up) + latency
                        uint32_t bw = same_node ? bw_intra : bw_inter;
                        uint32_t m_bw = same_node ? m_bw_intra : m_bw_inter;
                        uint32_t lat = same_node ? lat_intra : lat_inter;
                        if (SimX::kExt && S.link_table) {
                            // links inside a node that are not all alike: the pair's own figures
                            if (comm && same_node) {
                                const uint4 t = m.links[m.local_of(dev_a, node_a) * G + local_c];
                                bw = t.x; m_bw = t.y; lat = t.z;
                            }
                        }
                        if (SimX::kExt && S.node_table) {
                            // network links that are not all alike: the node pair's own figures
                            if (comm && !same_node) {
                                const uint4 t = m.node_links[node_a * S.n_nodes + node_c];
                                bw = t.x; m_bw = t.y; lat = t.z;
                            }
                        }
                        u64 ns;
                        if (WIDE) {
                            const u64 bytes = elems * S.elem_bytes;
                            ns = (bytes + bw - 1) / bw;
                        } else {
                            const uint32_t bytes = (uint32_t)elems * S.elem_bytes;
                            ns = ceil_div_u32(comm ? bytes : 1u, bw, m_bw);
                        }
                        ns += lat;
                        u64 end;
                        if (REG) {
                            const u64 f = L.free_at[row];                  // in range for every lane
                            const u64 base = f > now_kp ? f : now_kp;            // the same for all lanes of a row
                            const bool chained = lanes_of(comm_mask & ~same_m);   // rows between GPUs of one node are private
                            u64 incl;
                            if (!WIDE) {
                                // a row's running sum of transfer times cannot reach 2^32 (the host
                                // selects the WIDE kernels otherwise)
                                uint32_t acc = chained ? (uint32_t)ns : 0u, t = acc;
                                for (uint32_t sft = 1; sft < G; sft++) {
                                    t = wave_shr1_u32(t);
                                    if (pos < sft) t = 0;
                                    acc += t;
                                }
                                if (wrapped) acc += readlane_u32(acc, (int)first_len - 1) & last_run_mask;
                                incl = acc;
                            } else {
                                u64 t = incl = chained ? ns : 0;
                                for (uint32_t sft = 1; sft < G; sft++) {
                                    t = wave_shr1_u64(t);
                                    if (pos < sft) t = 0;
                                    incl += t;
                                }
                                if (wrapped) {
                                    const u64 first_total = readlane_u64(incl, (int)first_len - 1);
                                    if (last_run_mask) incl += first_total;
                                }
                            }
                            end = base + (same_node ? ns : incl);
                            const u64 write_m = (comm_mask & same_m) | (run_end_m & ~same_m & ballot(incl != 0));
                            if (lanes_of(write_m)) L.free_at[row] = end;
                            wave_sync();
                        } else if (!WIDE) {
                            // General strategies.  Transfers to another node queue on the link row of the node pair
                            // in consumer-part order: a running sum along the consumer's parts taken in (node, part)
                            // order (kept with the edge's set-up), cut where the node changes; every lane of a row
                            // reads the same free time and the row keeps the largest end.
                            const bool inter = lanes_of(comm_mask & ~same_m);
                            const uint32_t at_pos = gather_u32(inter ? (uint32_t)ns : 0u, sortw & 63u);
                            const uint32_t sum_pos = seg_running_sum(at_pos, (sortw >> 22) & 1u);
                            const uint32_t incl = gather_u32(sum_pos, (sortw >> 6) & 63u);
                            u64 f = 0;
                            if (inter) f = L.free_at[row];
                            end = (f > now_kp ? f : now_kp) + incl;
                            if (inter) __hip_atomic_fetch_max(&L.free_at[row], end, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                            wave_sync();
                            // Transfers inside the producer's node have a row per GPU pair: they only meet if two
                            // consumer parts sit on one GPU.
                            const u64 near_m = comm_mask & same_m;
                            if (near_m) {
                                const bool near = lanes_of(near_m);
                                const u64 end_near = fifo_commit(near, row, ns, now_kp, (near_m & dup_m) != 0, L);
                                if (near) end = end_near;
                            }
                        } else {
                            end = fifo_commit(comm, row, ns, now_kp, true, L);
                        }
                        if (comm) arrive = end;
                        if (STATS) {
                            cnt.n_comm += __popcll(comm_mask);
                            if (comm) cnt.sum_comm_ns += ns;   // per-lane partial sums, reduced by the caller
                        }
                    }
                    if (lanes_of(hit_m)) {
                        ready = arrive > ready ? arrive : ready;
                        pending -= 1;
                    }
                    touched_m |= hit_m;
                    if (STATS) cnt.n_pairs += __popcll(hit_m);
                }
                PROF_MARK(6)
                const bool touched = lanes_of(touched_m);
                overflow = overflow || (touched && ready >= TIME_LIMIT);
                const bool now_ready = touched && pending == 0;
                if (touched) {
                    w = now_ready ? ((ready << 1) | 1) : (W_WAIT | ((u64)pending << 48) | (ready & (TIME_LIMIT - 1)));
                    words[j * WAVE + lane] = w;
                }
                if (ballot(now_ready)) {
                    const u64 nmin = wave_min_from<ROW0>(now_ready ? w : W_NONE, last_key);
                    if (ONE) {
                        if ((uint32_t)lane == j && nmin < qreg) qreg = nmin;
                    } else {
                        if (lane == 0 && nmin < L.l1[j]) L.l1[j] = nmin;
                        if (TREE && (uint32_t)lane == (j >> 6) && nmin < qreg) qreg = nmin;
                        if (TREE && (j >> 6) == (i >> 6) && nmin < row_rest) row_rest = nmin;
                    }
                }
                PROF_MARK(7)
            }
            if (SimX::kExt && S.sync) {
                // Parameter synchronisation (a refinement of the inputs; Section 8 discusses the traffic,
                // Section 5.1 has no construction for it).  The op's parameters are cut into one shard per
                // index along the dims that index them; parts that differ only in the other dims are
                // replicas of a shard, and the replica with index 0 in those dims owns it.  A replica
                // that has finished sends its gradient of the shard to the owner's device: a transfer
                // with no successor, queued on its link row after the op's transfers to consumers.
                const uint32_t pbytes = opi_p->param_bytes;
                if (pbytes) {
                    const uint32_t pdims = opi_p->param_dims;
                    const uint32_t digits = part_digits(ci, lane, magic_v);
                    uint32_t owner = 0, shards = 1;
#pragma unroll
                    for (int d = 0; d < 4; d++) {
                        const bool indexes = (pdims >> d) & 1u;         // uniform
                        owner = owner * ci.deg[d] + (indexes ? (digits >> (8 * d)) & 0xffu : 0u);
                        if (indexes) shards *= ci.deg[d];
                    }
                    const uint32_t shard_bytes = (pbytes - 1) / shards + 1;       // ceil, pbytes >= 1
                    const uint32_t dev_o = m.template device_of_part<REG>(i, ci, in_mask ? owner : 0u);
                    const bool act = in_mask && owner != (uint32_t)lane && dev_o != dev_p;
                    if (ballot(act)) {
                        const uint32_t G = m.gpn();
                        const uint32_t node_o = m.node_of(dev_o);
                        const uint32_t local_o = m.local_of(dev_o, node_o);
                        const bool same_node = node_o == node_p;
                        const uint32_t row = same_node ? S.n_dev + dev_p * G + local_o
                                                       : S.n_dev + S.n_nodes * G * G + node_p * S.n_nodes + node_o;
                        uint32_t bw = same_node ? bw_intra : bw_inter;
                        uint32_t m_bw = same_node ? m_bw_intra : m_bw_inter;
                        uint32_t lat = same_node ? lat_intra : lat_inter;
                        if (S.link_table) {
                            if (act && same_node) {
                                const uint4 t = m.links[m.local_of(dev_p, node_p) * G + local_o];
                                bw = t.x; m_bw = t.y; lat = t.z;
                            }
                        }
                        if (S.node_table) {
                            if (act && !same_node) {
                                const uint4 t = m.node_links[node_p * S.n_nodes + node_o];
                                bw = t.x; m_bw = t.y; lat = t.z;
                            }
                        }
                        const u64 ns = (WIDE ? ((u64)shard_bytes + bw - 1) / bw : (u64)ceil_div_u32(shard_bytes, bw, m_bw)) + lat;
                        const u64 end = fifo_commit(act, act ? row : 0u, ns, now, true, L);
                        overflow = overflow || (act && end >= TIME_LIMIT);
                        if (STATS) {
                            cnt.n_comm += __popcll(ballot(act));
                            if (act) cnt.sum_comm_ns += ns;
                        }
                    }
                }
            }
            if (in_mask) k0 = W_NONE;
        }
        if (in_mask) words[i * WAVE + lane] = k0;
        const u64 new_l1 = wave_min_from<ROW0>(k0, last_key);
        if (ONE) {
            if ((uint32_t)lane == i) qreg = new_l1;
            wave_sync();
        } else {
            wave_sync();
            if (lane == 0) L.l1[i] = new_l1;
            wave_sync();
        }
        if (TREE) {
            // level 2 of the group: the popped op's new minimum against the rest of its row
            const u64 new_l2 = new_l1 < row_rest ? new_l1 : row_rest;
            if ((uint32_t)lane == (i >> 6)) qreg = new_l2;
        }
        PROF_MARK(7)
    }
    m.last_key = last_key;
    PROF_STORE(cnt)
    if (ballot(overflow)) return RESULT_OVERFLOW;
    return 0;
}

// Algorithm 1, result (largest endTime): every transfer feeds a compute task that ends
// later, so the makespan is the largest free time over the compute device rows.
template <class SimX>
__device__ __forceinline__ u64 makespan(const SimX& m) {
    // (parameter-synchronisation transfers feed nothing: with them the link rows count as well)
    const uint32_t n = (SimX::kExt && m.S.sync) ? m.S.n_rows : m.S.n_dev;
    u64 mk = 0;
    for (uint32_t d = lane_id(); d < n; d += WAVE) mk = m.L.free_at[d] > mk ? m.L.free_at[d] : mk;
    return wave_max_u64(mk);
}

}  // namespace ffsim
