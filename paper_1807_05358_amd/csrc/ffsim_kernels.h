// Kernels of the batched execution simulator: one candidate strategy per wavefront.
//
// Task-graph construction (Section 5.1) and Algorithm 1 are fused: the task graph is never
// written out.  A compute task is (op, part); its id is op*64 + part, which is
// order-isomorphic to the dense construction-order id.  Communication tasks are never
// stored: the transfers that start when a producer part finishes are enumerated at that
// moment, one consumer part per lane, and queued on their link rows in
// (edge, producer part, consumer part) order, which is their id order.
//
// The priority queue of Algorithm 1 is a 64-ary min-tree over one key per compute task:
//   key = time*2 + 1  while the task is READY and waits to be dequeued (time = readyTime),
//   key = time*2      after it was dequeued and until its successors were released
//                     (time = endTime; the transfers it feeds have readyTime = endTime),
//   key = KEY_NONE    otherwise.
// Level 0 (one key per task) lives in HBM, level 1 (one per op) and level 2 (one per 64 ops)
// in LDS.  Popping the minimum key and taking the lowest index among equal keys reproduces
// the (readyTime, id) order: at equal times, finished producers release their transfers
// (even keys) before READY compute tasks are dequeued (odd keys); the two kinds never share
// a device row, so only the order inside each kind matters.
#pragma once
#include "ffsim_device.h"

namespace ffsim {

struct Counters { u64 n_compute, n_pairs, n_comm, sum_comm_ns, n_events, exit_code, n_stuck, want_check; };

// LDS layout of one wavefront
struct WaveLds {
    u64* free_at;     // [n_rows]   endTime of the last task on every device / link row
    u64* l1;          // [n_ops_pad] min key per op
    u64* l2;          // [64]       min key per group of 64 ops
    uint8_t* tag;     // [n_rows]   scratch for conflict detection between lanes
};

__host__ __device__ inline size_t lds_bytes(uint32_t n_rows, uint32_t n_ops_pad) {
    return (size_t)n_rows * 8 + (size_t)n_ops_pad * 8 + 64 * 8 + ((n_rows + 15) & ~15u);
}

__device__ __forceinline__ WaveLds carve_lds(unsigned char* base, const SimDev& S) {
    WaveLds L;
    L.free_at = (u64*)base;
    L.l1 = L.free_at + S.n_rows;
    L.l2 = L.l1 + S.n_ops_pad;
    L.tag = (uint8_t*)(L.l2 + 64);
    return L;
}

struct OpCfg { uint32_t deg[4]; uint32_t off, stride, parts; };

__device__ __forceinline__ OpCfg load_cfg(const uint2* cfgs, uint32_t i) {
    uint2 c = cfgs[i];
    OpCfg o;
    o.deg[0] = c.x & 0xff; o.deg[1] = (c.x >> 8) & 0xff; o.deg[2] = (c.x >> 16) & 0xff; o.deg[3] = c.x >> 24;
    o.off = c.y & 0xffff; o.stride = c.y >> 16;
    o.parts = o.deg[0] * o.deg[1] * o.deg[2] * o.deg[3];
    return o;
}

// Section 4: validity of a configuration for its op
__device__ __forceinline__ bool cfg_ok(const DOp& op, const OpCfg& c, const SimDev& S) {
    bool ok = true;
#pragma unroll
    for (int d = 0; d < 4; d++) {
        bool par = (uint32_t)d < op.ndim && ((op.par_mask >> d) & 1);
        ok = ok && c.deg[d] >= 1 && (par ? c.deg[d] <= op.extent[d] : c.deg[d] == 1);
    }
    // each degree <= 255, so the product cannot wrap
    return ok && c.parts <= S.max_parts && c.off < S.n_dev;
}

// output box of part k of an op: [lo[d], hi[d]) (equal-size partitions, Section 4)
struct Box { uint32_t lo[4], hi[4]; };

__device__ __forceinline__ Box part_box(const DOp& op, const OpCfg& c, uint32_t k, const uint32_t* magic) {
    Box b;
    uint32_t rem = k;
#pragma unroll
    for (int d = 3; d >= 0; d--) {
        uint32_t q = div_small(rem, c.deg[d], magic);
        uint32_t idx = rem - q * c.deg[d];
        rem = q;
        b.lo[d] = div_small(idx * op.extent[d], c.deg[d], magic);
        b.hi[d] = div_small((idx + 1) * op.extent[d], c.deg[d], magic);
    }
    return b;
}

__device__ __forceinline__ uint32_t part_device(const OpCfg& c, uint32_t k, const SimDev& S) {
    uint32_t n = c.off + k * c.stride;
    return n - div_magic(n, S.n_dev, S.magic_dev) * S.n_dev;
}

// range of the producer's dim d read by a consumer part with output box cb
__device__ __forceinline__ void needed_range(const DMap& m, uint32_t extent, const Box& cb, int32_t& lo, int32_t& hi) {
    if (m.src_dim < 0) { lo = 0; hi = (int32_t)extent; return; }
    // extents <= 2^20, stride <= 65535 and |a|,|b| < 2^31: do the affine map in 64 bits
    const int c = m.src_dim;   // select without indexing a register array by a run-time value
    const uint32_t clo = c == 0 ? cb.lo[0] : c == 1 ? cb.lo[1] : c == 2 ? cb.lo[2] : cb.lo[3];
    const uint32_t chi = c == 0 ? cb.hi[0] : c == 1 ? cb.hi[1] : c == 2 ? cb.hi[2] : cb.hi[3];
    long long l = (long long)clo * m.stride + m.a;
    long long h = ((long long)chi - 1) * m.stride + m.b + 1;
    const long long E = (long long)extent;
    l = l < 0 ? 0 : (l > E ? E : l);
    h = h < 0 ? 0 : (h > E ? E : h);
    lo = (int32_t)l;
    hi = (int32_t)(h < l ? l : h);
}

// index of the producer part (along one dim) that owns coordinate x: the largest p with
// floor(p*E/deg) <= x
__device__ __forceinline__ uint32_t owner_part(uint32_t x, uint32_t E, uint32_t deg) {
    return ((x + 1) * deg - 1) / E;
}

// Serialise tasks that become ready at the same time r on device rows, in lane order
// (= id order): end = max(r, row free time) + running sum of exeTimes on that row.
// Lanes whose row is used by no other lane go in one parallel step.
__device__ __forceinline__ u64 fifo_commit(bool act, uint32_t row, u64 exe, u64 r, const WaveLds& L) {
    const int lane = lane_id();
    u64 end = 0;
    if (act) L.tag[row] = (uint8_t)lane;
    wave_sync();
    bool lost = act && L.tag[row] != (uint8_t)lane;
    u64 lost_mask = __ballot(lost);
    bool slow = false;
    if (lost_mask) {
        if (lost) L.tag[row] = 0xff;
        wave_sync();
        slow = act && L.tag[row] == 0xff;
    }
    if (act && !slow) {
        u64 f = L.free_at[row];
        end = (f > r ? f : r) + exe;
        L.free_at[row] = end;
    }
    u64 todo = __ballot(slow);
    while (todo) {
        int l = __builtin_ctzll(todo);
        todo &= todo - 1;
        wave_sync();
        if (lane == l) {
            u64 f = L.free_at[row];
            end = (f > r ? f : r) + exe;
            L.free_at[row] = end;
        }
    }
    wave_sync();
    return end;
}

// One candidate: build + simulate.  cfgs = its n_ops configurations; keys / state = this
// wavefront's HBM slot ([n_ops*64] each).  Returns the makespan, or KEY_NONE for an
// invalid strategy and KEY_INTERNAL if the event tree is found inconsistent (a bug; the loop
// never spins).  cfgs is deliberately not __restrict__: the chain kernel rewrites it between
// calls, and loads from it must not be treated as invariant.  WIDE selects 64-bit element counts (tensors of 2^32 bytes or more).
template <bool WIDE>
__device__ u64 simulate_candidate(const SimDev& S, const uint2* cfgs, u64* __restrict__ keys,
                                  TaskState* __restrict__ state, const WaveLds& L, Counters& cnt) {
    const int lane = lane_id();
    const uint32_t* __restrict__ magic = S.magic;

    // ---- validate the strategy (lanes over ops) ----
    uint32_t bad = 0;
    for (uint32_t i = lane; i < S.n_ops; i += WAVE) {
        OpCfg c = load_cfg(cfgs, i);
        if (!cfg_ok(S.ops[i], c, S)) bad = 1;
    }
    if (__ballot(bad != 0)) return KEY_NONE;

    // ---- Section 5.1 step 1 + the start of Algorithm 1: tasks, their number of inputs, initial READY set ----
    for (uint32_t r = lane; r < S.n_rows; r += WAVE) L.free_at[r] = 0;
    for (uint32_t j = 0; j < S.n_ops; j++) {
        const DOp opj = S.ops[j];
        const OpCfg cj = load_cfg(cfgs, j);
        const bool mine = (uint32_t)lane < cj.parts;
        const Box cb = part_box(opj, cj, mine ? lane : 0, magic);
        uint32_t pending = 0;
        for (uint32_t q = opj.in_begin; q < opj.in_end; q++) {
            const DEdge e = S.edges[S.in_list[q]];
            const DOp opi = S.ops[e.src];
            const OpCfg ci = load_cfg(cfgs, e.src);
            uint32_t n = 1;
#pragma unroll
            for (int d = 0; d < 4; d++) {
                if ((uint32_t)d < opi.ndim) {
                    int32_t lo, hi;
                    needed_range(e.map[d], opi.extent[d], cb, lo, hi);
                    uint32_t c = 0;
                    if (hi > lo) c = owner_part(hi - 1, opi.extent[d], ci.deg[d]) - owner_part(lo, opi.extent[d], ci.deg[d]) + 1;
                    n *= c;
                }
            }
            pending += n;
        }
        u64 key = (mine && pending == 0) ? 1ull : KEY_NONE;   // READY at time 0
        keys[j * WAVE + lane] = key;
        TaskState st; st.ready = 0; st.pending = pending; st.pad = 0;
        state[j * WAVE + lane] = st;
        u64 kmin = wave_min_u64(key);
        if (lane == 0) L.l1[j] = kmin;
        cnt.n_compute += cj.parts;
    }
    for (uint32_t j = S.n_ops + lane; j < S.n_ops_pad; j += WAVE) L.l1[j] = KEY_NONE;
    wave_sync();
    for (uint32_t g = 0; g < S.n_groups; g++) {
        u64 kmin = wave_min_u64(L.l1[g * WAVE + lane]);
        if (lane == 0) L.l2[g] = kmin;
    }
    wave_sync();

    // ---- Algorithm 1, main loop ----
    const u64 max_events = 2ull * S.n_ops * WAVE + 8;   // every task is popped at most twice
    for (u64 ev = 0; ev < max_events; ev++) {
        u64 k2 = (uint32_t)lane < S.n_groups ? L.l2[lane] : KEY_NONE;
        const u64 kmin = wave_min_u64(k2);
        if (kmin == KEY_NONE) break;
        const uint32_t g = __builtin_ctzll(__ballot(k2 == kmin));
        u64 k1 = L.l1[g * WAVE + lane];
        u64 m1 = __ballot(k1 == kmin);
        if (!m1) { cnt.exit_code = 1; return KEY_INTERNAL; }   // tree inconsistent: give up, never spin
        const uint32_t i = g * WAVE + __builtin_ctzll(m1);
        u64 k0 = keys[i * WAVE + lane];
        const u64 mask = __ballot(k0 == kmin);            // parts of op i with this key
        if (!mask) { cnt.exit_code = 2; return KEY_INTERNAL; }
        cnt.n_events++;
        const u64 now = kmin >> 1;
        const DOp opi = S.ops[i];
        const OpCfg ci = load_cfg(cfgs, i);
        const bool in_mask = (mask >> lane) & 1;
        const uint32_t dev_p = part_device(ci, lane, S);

        if (kmin & 1) {
            // dequeue READY compute tasks: start = max(readyTime, device free), end = start + exeTime
            const u64 exe = S.cost[(size_t)i * S.n_cols + (ci.parts - 1)];
            u64 end = fifo_commit(in_mask, dev_p, exe, now, L);
            if (in_mask) k0 = opi.out_end > opi.out_begin ? end << 1 : KEY_NONE;
        } else {
            // the parts in `mask` finished at `now`: release their successors edge by edge
            const Box pb = part_box(opi, ci, lane, magic);
            const uint32_t node_p = div_magic(dev_p, S.gpus_per_node, S.magic_gpn);
            for (uint32_t ei = opi.out_begin; ei < opi.out_end; ei++) {
                const DEdge e = S.edges[ei];
                const uint32_t j = e.dst;
                const DOp opj = S.ops[j];
                const OpCfg cj = load_cfg(cfgs, j);
                const bool mine = (uint32_t)lane < cj.parts;
                const Box cb = part_box(opj, cj, mine ? lane : 0, magic);
                int32_t nlo[4], nhi[4];
#pragma unroll
                for (int d = 0; d < 4; d++) needed_range(e.map[d], opi.extent[d], cb, nlo[d], nhi[d]);
                const uint32_t dev_c = part_device(cj, lane, S);
                const uint32_t node_c = div_magic(dev_c, S.gpus_per_node, S.magic_gpn);
                TaskState st = state[j * WAVE + lane];
                const uint32_t pending_before = st.pending;
                u64 todo = mask;
                while (todo) {
                    const int kp = __builtin_ctzll(todo);
                    todo &= todo - 1;
                    bool hit = mine;
                    u64 elems = 1;
#pragma unroll
                    for (int d = 0; d < 4; d++) {
                        if ((uint32_t)d < opi.ndim) {
                            int32_t plo = (int32_t)readlane_u32(pb.lo[d], kp), phi = (int32_t)readlane_u32(pb.hi[d], kp);
                            int32_t lo = nlo[d] > plo ? nlo[d] : plo;
                            int32_t hi = nhi[d] < phi ? nhi[d] : phi;
                            hit = hit && hi > lo;
                            if (WIDE) elems *= (u64)(uint32_t)(hi > lo ? hi - lo : 0);
                            else elems = (uint32_t)elems * (uint32_t)(hi > lo ? hi - lo : 0);
                        }
                    }
                    const uint32_t dev_a = readlane_u32(dev_p, kp);
                    const uint32_t node_a = readlane_u32(node_p, kp);
                    const bool comm = hit && dev_c != dev_a;
                    const bool same_node = node_c == node_a;
                    // Section 5.1: the link device between the two devices
                    const uint32_t G = S.gpus_per_node;
                    uint32_t row = same_node
                        ? S.n_dev + node_a * G * G + (dev_a - node_a * G) * G + (dev_c - node_c * G)
                        : S.n_dev + S.n_nodes * G * G + node_a * S.n_nodes + node_c;
                    // assumption A2: transfer time = size / bandwidth (rounded up) + latency
                    const uint32_t bw = same_node ? S.bw_intra : S.bw_inter;
                    u64 ns;
                    if (WIDE) {
                        u64 bytes = elems * S.elem_bytes;
                        ns = (bytes + bw - 1) / bw;
                    } else {
                        uint32_t bytes = (uint32_t)elems * S.elem_bytes;
                        ns = ceil_div_u32(comm ? bytes : 1u, bw, same_node ? S.m_bw_intra : S.m_bw_inter);
                    }
                    ns += same_node ? S.lat_intra : S.lat_inter;
                    const u64 comm_mask = __ballot(comm);
                    u64 arrive = now;
                    if (comm_mask) {
                        u64 end = fifo_commit(comm, row, ns, now, L);
                        if (comm) arrive = end;
                    }
                    if (hit) {
                        st.ready = arrive > st.ready ? arrive : st.ready;
                        st.pending -= 1;
                    }
                    cnt.n_pairs += __popcll(__ballot(hit));
                    cnt.n_comm += __popcll(comm_mask);
                    if (comm) cnt.sum_comm_ns += ns;   // per-lane partial sums, reduced by the caller
                }
                const bool now_ready = mine && pending_before != 0 && st.pending == 0;
                if (mine) state[j * WAVE + lane] = st;
                const u64 nk = now_ready ? (st.ready << 1) | 1 : KEY_NONE;
                if (now_ready) keys[j * WAVE + lane] = nk;
                const u64 nmin = wave_min_u64(nk);
                if (nmin != KEY_NONE && lane == 0) {
                    if (nmin < L.l1[j]) L.l1[j] = nmin;
                    if (nmin < L.l2[j >> 6]) L.l2[j >> 6] = nmin;
                }
            }
            if (in_mask) k0 = KEY_NONE;
        }
        if (in_mask) keys[i * WAVE + lane] = k0;
        const u64 new_l1 = wave_min_u64(k0);
        wave_sync();
        if (lane == 0) L.l1[i] = new_l1;
        wave_sync();
        const u64 new_l2 = wave_min_u64(L.l1[g * WAVE + lane]);
        if (lane == 0) L.l2[g] = new_l2;
        wave_sync();
    }

    // Algorithm 1, result (largest endTime): every transfer feeds a compute task that ends later, so the
    // makespan is the largest free time over the compute device rows.
    if (cnt.want_check) {   // diagnostics: tasks that never ran (0 in a correct run)
        for (uint32_t j = 0; j < S.n_ops; j++) {
            const OpCfg cj = load_cfg(cfgs, j);
            const bool stuck = (uint32_t)lane < cj.parts && (state[j * WAVE + lane].pending != 0 || keys[j * WAVE + lane] != KEY_NONE);
            cnt.n_stuck += __popcll(__ballot(stuck));
        }
    }
    u64 mk = 0;
    for (uint32_t d = lane; d < S.n_dev; d += WAVE) mk = L.free_at[d] > mk ? L.free_at[d] : mk;
    return wave_max_u64(mk);
}

__device__ __forceinline__ void store_counters(Counters c, Counters* out) {
    // sum_comm_ns was accumulated per lane
    u64 s = c.sum_comm_ns;
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) s += shfl_xor_u64(s, m);
    c.sum_comm_ns = s;
    if (lane_id() == 0) *out = c;
}

template <bool WIDE>
__global__ __launch_bounds__(WAVE) void k_sim_batch(SimDev S, const uint2* __restrict__ strategies, uint32_t B,
                                                    u64* __restrict__ out_ns, Counters* __restrict__ stats,
                                                    unsigned char* __restrict__ ws, size_t slot_bytes) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const WaveLds L = carve_lds(lds_raw, S);
    unsigned char* slot = ws + (size_t)blockIdx.x * slot_bytes;
    TaskState* state = (TaskState*)slot;
    u64* keys = (u64*)(slot + (size_t)S.n_ops * WAVE * sizeof(TaskState));
    for (uint32_t b = blockIdx.x; b < B; b += gridDim.x) {
        Counters cnt = {};
        cnt.want_check = stats != nullptr;
        u64 mk = simulate_candidate<WIDE>(S, strategies + (size_t)b * S.n_ops, keys, state, L, cnt);
        if (lane_id() == 0) out_ns[b] = mk;
        if (stats) store_counters(cnt, stats + b);
        wave_sync();
    }
}

// Delta entry, first form: every step applies the mutation to the chain's strategy and
// re-runs build + Algorithm 1 (the definition of the delta result, Section 5.3).
template <bool WIDE>
__global__ __launch_bounds__(WAVE) void k_sim_chain_steps(SimDev S, uint2* __restrict__ chain_cfgs, uint32_t C,
                                                          const uint32_t* __restrict__ muts, uint32_t n_steps,
                                                          u64* __restrict__ out_ns, unsigned char* __restrict__ ws,
                                                          size_t slot_bytes) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const WaveLds L = carve_lds(lds_raw, S);
    const uint32_t c = blockIdx.x;
    if (c >= C) return;
    unsigned char* slot = ws + (size_t)c * slot_bytes;
    TaskState* state = (TaskState*)slot;
    u64* keys = (u64*)(slot + (size_t)S.n_ops * WAVE * sizeof(TaskState));
    uint2* cfgs = chain_cfgs + (size_t)c * S.n_ops;
    for (uint32_t s = 0; s < n_steps; s++) {
        if (muts) {   // muts: [n_steps][C] records of {op, cfg.x, cfg.y}
            const uint32_t* m = muts + ((size_t)s * C + c) * 3;
            uint32_t op = m[0];
            if (lane_id() == 0 && op < S.n_ops) cfgs[op] = make_uint2(m[1], m[2]);
            __threadfence_block();
            wave_sync();
        }
        Counters cnt = {};
        u64 mk = simulate_candidate<WIDE>(S, cfgs, keys, state, L, cnt);
        if (lane_id() == 0) out_ns[(size_t)s * C + c] = mk;
        wave_sync();
    }
}

}  // namespace ffsim
