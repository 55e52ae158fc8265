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
// graphs; level 1 (one minimum per op) and level 2 (one per 64 ops) live in LDS.  Popping the
// minimum word and taking the lowest index among equal words reproduces the
// (readyTime, id) order: at equal times, finished producers release their transfers (kind
// 0) before READY compute tasks are dequeued (kind 1); the two kinds never share a device
// row, so only the order inside each kind matters.  All parts of one op that hold the
// minimum word are handled in one step, serialised per device row in lane (= id) order.
#pragma once
#include "ffsim_device.h"

namespace ffsim {

// up to this many groups of 64 ops the queue has no level 2: lanes scan level 1 directly
constexpr uint32_t FLAT_GROUPS = 8;

// Section timing for development builds (-DFFSIM_PROFILE): shader-clock ticks per section are
// accumulated in a register array and reported through the stats record instead of the
// usual counters.  Compiled out otherwise.
#ifdef FFSIM_PROFILE
#define PROF_DECL u64 prof_t[8] = {0, 0, 0, 0, 0, 0, 0, 0}; u64 prof_last = __builtin_readcyclecounter();
#define PROF_MARK(k) { const u64 prof_now = __builtin_readcyclecounter(); prof_t[k] += prof_now - prof_last; prof_last = prof_now; }
#define PROF_STORE(c) { c.n_compute = prof_t[0]; c.n_pairs = prof_t[1]; c.n_comm = prof_t[2]; c.sum_comm_ns = lane_id() == 0 ? prof_t[3] : 0; \
                        c.exit_code = prof_t[4]; c.n_stuck = prof_t[5]; c.want_check = prof_t[6]; }
#else
#define PROF_DECL
#define PROF_MARK(k)
#define PROF_STORE(c)
#endif

struct Counters { u64 n_compute, n_pairs, n_comm, sum_comm_ns, n_events, exit_code, n_stuck, want_check; };

// read-only tables shared by all candidates (pointers come from __restrict__ kernel
// arguments, so loads through them can use the scalar unit)
struct Tables {
    const DOp* ops;
    const DEdge* edges;       // sorted by (producer, consumer)
    const DEdge* in_edges;    // the same records sorted by (consumer, edge id)
    const uint32_t* cost;     // [n_ops][n_cols]
};

// LDS of one wavefront
struct WaveLds {
    u64* free_at;     // [n_rows]    endTime of the last task on every device / link row
    u64* l1;          // [n_ops_pad] min word per op
    u64* l2;          // [64]        min word per group of 64 ops
    uint8_t* tag;     // [n_rows]    scratch for conflict detection between lanes
};

__host__ __device__ inline size_t lds_common_bytes(uint32_t n_rows, uint32_t n_ops_pad) {
    return (size_t)n_rows * 8 + (size_t)n_ops_pad * 8 + 64 * 8 + ((n_rows + 15) & ~15u);
}
// per-candidate task words + per-op exeTime: in LDS for small graphs, else in an HBM slot
__host__ __device__ inline size_t slot_bytes(uint32_t n_ops, uint32_t n_ops_pad) {
    return (size_t)n_ops * WAVE * 8 + (size_t)n_ops_pad * 4;
}

__device__ __forceinline__ WaveLds carve_lds(unsigned char* base, const SimDev& S) {
    WaveLds L;
    L.free_at = (u64*)base;
    L.l1 = L.free_at + S.n_rows;
    L.l2 = L.l1 + S.n_ops_pad;
    L.tag = (uint8_t*)(L.l2 + 64);
    return L;
}

struct OpCfg { uint32_t deg[4]; uint32_t off, stride, parts, x; };   // x = the four degrees, one byte each

// a configuration is the same for all lanes: keep it on the scalar unit
__device__ __forceinline__ OpCfg unpack_cfg(uint2 c) {
    OpCfg o;
    c.x = first_u32(c.x);
    c.y = first_u32(c.y);
    o.deg[0] = c.x & 0xff; o.deg[1] = (c.x >> 8) & 0xff; o.deg[2] = (c.x >> 16) & 0xff; o.deg[3] = c.x >> 24;
    o.off = c.y & 0xffff; o.stride = c.y >> 16; o.x = c.x;
    o.parts = o.deg[0] * o.deg[1] * o.deg[2] * o.deg[3];
    return o;
}

// per-lane variant (each lane looks at a different op)
__device__ __forceinline__ OpCfg unpack_cfg_lane(uint2 c) {
    OpCfg o;
    o.deg[0] = c.x & 0xff; o.deg[1] = (c.x >> 8) & 0xff; o.deg[2] = (c.x >> 16) & 0xff; o.deg[3] = c.x >> 24;
    o.off = c.y & 0xffff; o.stride = c.y >> 16; o.x = c.x;
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

// floor(n / d), d uniform in 1..64, n <= 2^26, without branches.  Lane d-1 of magic_v holds
// floor(2^32/d)+1 for d >= 2 and 0 for d = 1 (where the quotient is n itself), so the
// constant comes from a register instead of memory.
struct Divisor { uint32_t d, m, pass; };   // pass = all ones iff d == 1
__device__ __forceinline__ Divisor divisor(uint32_t d, uint32_t magic_v) {
    Divisor v;
    v.d = d;
    v.m = readlane_u32(magic_v, (int)((d - 1) & 63));
    v.pass = d == 1 ? 0xffffffffu : 0u;
    return v;
}
__device__ __forceinline__ uint32_t div_by(uint32_t n, const Divisor& v) { return __umulhi(n, v.m) + (n & v.pass); }

// output box of part k of an op: [lo[d], hi[d]) (equal-size partitions, Section 4)
struct Box { uint32_t lo[4], hi[4]; };

__device__ __forceinline__ Box part_box(const uint32_t extent[4], const OpCfg& c, uint32_t k, uint32_t magic_v) {
    Box b;
    uint32_t rem = k;
#pragma unroll
    for (int d = 3; d >= 0; d--) {
        if (c.deg[d] == 1) {          // uniform: most dims are not split
            b.lo[d] = 0;
            b.hi[d] = extent[d];
        } else {
            const Divisor dv = divisor(c.deg[d], magic_v);
            uint32_t q = div_by(rem, dv);
            uint32_t idx = rem - q * c.deg[d];
            rem = q;
            b.lo[d] = div_by(idx * extent[d], dv);
            b.hi[d] = div_by((idx + 1) * extent[d], dv);
        }
    }
    return b;
}

__device__ __forceinline__ uint32_t part_device(const OpCfg& c, uint32_t k, const SimDev& S) {
    uint32_t n = c.off + k * c.stride;
    return n - div_magic(n, S.magic_dev, S.pass_dev) * S.n_dev;
}

// index of part k along each dim (mixed radix over the degree tuple, dim 0 slowest), packed
// one byte per dim
__device__ __forceinline__ uint32_t part_digits(const OpCfg& c, uint32_t k, uint32_t magic_v) {
    uint32_t rem = k, packed = 0;
#pragma unroll
    for (int d = 3; d >= 0; d--) {
        if (c.deg[d] != 1) {          // uniform
            const Divisor dv = divisor(c.deg[d], magic_v);
            const uint32_t q = div_by(rem, dv);
            packed |= (rem - q * c.deg[d]) << (8 * d);
            rem = q;
        }
    }
    return packed;
}

// Range of the producer's dim read by a consumer part (Section 4: the input sub-tensor
// follows from the output sub-tensor).  m: the map of that producer dim; extent: the
// producer's extent; cfg_x: the consumer's four degrees (one byte each); digits: the consumer
// part's index per dim (part_digits).  All values fit 32 bits: extents <= 2^20, stride <= 1024,
// |a|,|b| <= 2^29.  No branch on the lane's data.
__device__ __forceinline__ void needed_range(const DMap& m, uint32_t extent, uint32_t cfg_x, uint32_t digits,
                                             uint32_t magic_v, int32_t& lo, int32_t& hi) {
    if (m.src_dim < 0) { lo = 0; hi = (int32_t)extent; return; }   // uniform
    const uint32_t sh = 8u * (uint32_t)m.src_dim;
    const Divisor dv = divisor((cfg_x >> sh) & 0xff, magic_v);
    const uint32_t idx = (digits >> sh) & 0xff;
    const int32_t clo = (int32_t)div_by(idx * m.cext, dv);
    const int32_t chi = (int32_t)div_by((idx + 1) * m.cext, dv);
    int32_t l = clo * (int32_t)m.stride + m.a;
    int32_t h = (chi - 1) * (int32_t)m.stride + m.b + 1;
    const int32_t E = (int32_t)extent;
    l = l < 0 ? 0 : (l > E ? E : l);
    h = h < 0 ? 0 : (h > E ? E : h);
    lo = l;
    hi = h < l ? l : h;
}

// index of the producer part (along one dim) that owns coordinate x: the largest p with
// floor(p*E/deg) <= x
__device__ __forceinline__ uint32_t owner_part(uint32_t x, uint32_t E, uint32_t deg) {
    return ((x + 1) * deg - 1) / E;
}

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
    u64 todo = __ballot(lost);
    while (todo) {
        const int l = __builtin_ctzll(todo);
        const uint32_t lrow = readlane_u32(row, l);
        const bool peer = act && row == lrow;   // includes the lane whose tag survived
        const u64 peers = __ballot(peer);
        todo &= ~peers;
        const int first = __builtin_ctzll(peers);
        const u64 exe_l = readlane_u64(exe, first);
        if (!__ballot(peer && exe != exe_l)) {
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

// One candidate: build + simulate.  cfgs = its n_ops configurations; words / exe_of = this
// wavefront's task words [n_ops*64] and per-op exeTime [n_ops] (LDS or HBM).  Returns the
// makespan or one of the RESULT_* codes.  cfgs is deliberately not __restrict__: the chain
// kernel rewrites it between calls, so loads from it must not be treated as invariant.
// WIDE selects 64-bit element counts (tensors of 2^32 bytes or more).
template <bool WIDE>
__device__ u64 simulate_candidate(const SimDev& S, const Tables& T, const uint2* cfgs, u64* words, uint32_t* exe_of,
                                  const WaveLds& L, uint32_t magic_v, Counters& cnt) {
    const int lane = lane_id();
    PROF_DECL
    const DOp* __restrict__ ops = T.ops;
    const DEdge* __restrict__ edges = T.edges;
    const DEdge* __restrict__ in_edges = T.in_edges;
    const uint32_t* __restrict__ cost = T.cost;

    // ---- validate the strategy (lanes over ops) ----
    bool bad = false;
    for (uint32_t i = lane; i < S.n_ops; i += WAVE) {
        OpCfg c = unpack_cfg_lane(cfgs[i]);
        if (!cfg_ok(ops[i], c, S)) bad = true;
        else exe_of[i] = cost[(size_t)i * S.n_cols + (c.parts - 1)];
    }
    if (__ballot(bad)) return RESULT_INVALID;

    // ---- Section 5.1 step 1 and the start of Algorithm 1: the tasks, how many inputs each
    //      waits for (in closed form per in-edge), and the initial READY set ----
    for (uint32_t r = lane; r < S.n_rows; r += WAVE) L.free_at[r] = 0;
    for (uint32_t j = 0; j < S.n_ops; j++) {
        const uint32_t in_begin = ops[j].in_begin, in_end = ops[j].in_end;
        const OpCfg cj = unpack_cfg(cfgs[j]);
        const bool mine = (uint32_t)lane < cj.parts;
        const uint32_t digits = part_digits(cj, lane, magic_v);
        uint32_t pending = 0;
        for (uint32_t q = in_begin; q < in_end; q++) {
            const DEdge e = in_edges[q];
            const OpCfg ci = unpack_cfg(cfgs[e.src]);
            uint32_t n = 1;
#pragma unroll
            for (int d = 0; d < 4; d++) {
                if ((uint32_t)d < e.src_ndim) {
                    if (e.map[d].src_dim < 0) {
                        n *= ci.deg[d];
                    } else {
                        int32_t lo, hi;
                        needed_range(e.map[d], e.src_extent[d], cj.x, digits, magic_v, lo, hi);
                        uint32_t c = 0;
                        if (hi > lo) c = owner_part(hi - 1, e.src_extent[d], ci.deg[d]) - owner_part(lo, e.src_extent[d], ci.deg[d]) + 1;
                        n *= c;
                    }
                }
            }
            pending += n;
        }
        // pending < PENDING_LIMIT is guaranteed by ff_sim_create (at most 511 in-edges per op)
        const u64 w = !mine ? W_NONE : (pending == 0 ? 1ull : (W_WAIT | ((u64)pending << 48)));
        words[j * WAVE + lane] = w;
        const u64 wmin = wave_min_u64(w);
        if (lane == 0) L.l1[j] = wmin;
        cnt.n_compute += cj.parts;
    }
    for (uint32_t j = S.n_ops + lane; j < S.n_ops_pad; j += WAVE) L.l1[j] = W_NONE;
    wave_sync();
    if (S.n_groups > FLAT_GROUPS) {
        for (uint32_t g = 0; g < S.n_groups; g++) {
            const u64 wmin = wave_min_u64(L.l1[g * WAVE + lane]);
            if (lane == 0) L.l2[g] = wmin;
        }
        wave_sync();
    }

    PROF_MARK(0)
    // ---- Algorithm 1, main loop ----
    bool overflow = false;
    u64 last_key = 0;
    const u64 max_events = 2ull * S.n_ops * WAVE + 8;   // every task is popped at most twice
    for (u64 ev = 0; ev < max_events; ev++) {
        u64 kmin;
        uint32_t i;
        if (S.n_groups > FLAT_GROUPS) {
            const u64 k2 = (uint32_t)lane < S.n_groups ? L.l2[lane] : W_NONE;
            kmin = wave_min_from(k2, last_key);
            if (kmin >> 63) break;
            const uint32_t g = __builtin_ctzll(__ballot(k2 == kmin));
            const u64 k1 = L.l1[g * WAVE + lane];
            const u64 m1 = __ballot(k1 == kmin);
            if (!m1) { cnt.exit_code = 1; return RESULT_INTERNAL; }   // tree inconsistent: give up, never spin
            i = g * WAVE + __builtin_ctzll(m1);
        } else {
            // few ops: every lane scans its column of level 1, no level 2
            u64 k1 = L.l1[lane];
            uint32_t gbest = 0;
            for (uint32_t g = 1; g < S.n_groups; g++) {
                const u64 k = L.l1[g * WAVE + lane];
                if (k < k1) { k1 = k; gbest = g; }
            }
            kmin = wave_min_from(k1, last_key);
            if (kmin >> 63) break;
            // lowest op index among equal keys: smallest group first, then lowest lane
            u64 m1 = __ballot(k1 == kmin);
            if (!m1) { cnt.exit_code = 1; return RESULT_INTERNAL; }
            if (m1 & (m1 - 1)) {    // several columns hold the minimum: smallest group wins
                const uint32_t gmin = wave_min_u32(k1 == kmin ? gbest : 0xffffffffu);
                m1 = __ballot(k1 == kmin && gbest == gmin);
            }
            const int col = __builtin_ctzll(m1);
            i = readlane_u32(gbest, col) * WAVE + col;
        }
        last_key = kmin;
        PROF_MARK(1)
        // everything that depends only on i is requested together
        u64 k0 = words[i * WAVE + lane];
        const DOp* __restrict__ opi_p = ops + i;
        const uint32_t out_begin = opi_p->out_begin, out_end = opi_p->out_end;
        const OpCfg ci = unpack_cfg(cfgs[i]);
        const u64 exe = exe_of[i];
        const u64 mask = __ballot(k0 == kmin);            // parts of op i that hold the minimum
        if (!mask) { cnt.exit_code = 2; return RESULT_INTERNAL; }
        cnt.n_events++;
        const u64 now = kmin >> 1;
        const bool in_mask = (mask >> lane) & 1;
        const uint32_t dev_p = part_device(ci, lane, S);

        if (kmin & 1) {
            // dequeue READY compute tasks: start = max(readyTime, device free), end = start + exeTime
            const bool may_share = !(ci.stride == 1 && ci.parts <= S.n_dev);
            const u64 end = fifo_commit(in_mask, dev_p, exe, now, may_share, L);
            overflow = overflow || end >= TIME_LIMIT;
            if (in_mask) k0 = out_end > out_begin ? end << 1 : W_NONE;
            PROF_MARK(2)
        } else {
            // the parts in `mask` finished at `now`: release their successors edge by edge
            DEdge e = opi_p->first;
            const Box pb = part_box(e.src_extent, ci, lane, magic_v);
            const uint32_t node_p = div_magic(dev_p, S.magic_gpn, S.pass_gpn);
            for (uint32_t ei = out_begin; ei < out_end; ei++) {
                if (ei != out_begin) e = edges[ei];
                const uint32_t j = e.dst;
                u64 w = words[j * WAVE + lane];
                const OpCfg cj = unpack_cfg(cfgs[j]);
                const bool mine = (uint32_t)lane < cj.parts;
                const uint32_t digits = part_digits(cj, lane, magic_v);
                int32_t nlo[4], nhi[4];
#pragma unroll
                for (int d = 0; d < 4; d++) {
                    nlo[d] = 0; nhi[d] = 1;
                    if ((uint32_t)d < e.src_ndim) needed_range(e.map[d], e.src_extent[d], cj.x, digits, magic_v, nlo[d], nhi[d]);
                }
                const uint32_t dev_c = part_device(cj, lane, S);
                const uint32_t node_c = div_magic(dev_c, S.magic_gpn, S.pass_gpn);
                u64 ready = w & (TIME_LIMIT - 1);
                uint32_t pending = (uint32_t)(w >> 48) & PENDING_LIMIT;
                bool touched = false;
                u64 todo = mask;
                PROF_MARK(3)
                while (todo) {
                    const int kp = __builtin_ctzll(todo);
                    todo &= todo - 1;
                    bool hit = mine;
                    u64 elems = 1;
#pragma unroll
                    for (int d = 0; d < 4; d++) {
                        if ((uint32_t)d < e.src_ndim) {
                            const int32_t plo = (int32_t)readlane_u32(pb.lo[d], kp), phi = (int32_t)readlane_u32(pb.hi[d], kp);
                            const int32_t lo = nlo[d] > plo ? nlo[d] : plo;
                            const int32_t hi = nhi[d] < phi ? nhi[d] : phi;
                            hit = hit && hi > lo;
                            if (WIDE) elems *= (u64)(uint32_t)(hi > lo ? hi - lo : 0);
                            else elems = (uint32_t)elems * (uint32_t)(hi > lo ? hi - lo : 0);
                        }
                    }
                    const u64 hit_mask = __ballot(hit);
                    if (!hit_mask) continue;
                    const uint32_t dev_a = readlane_u32(dev_p, kp);
                    const uint32_t node_a = readlane_u32(node_p, kp);
                    const bool comm = hit && dev_c != dev_a;
                    const u64 comm_mask = __ballot(comm);
                    u64 arrive = now;
                    if (comm_mask) {
                        const bool same_node = node_c == node_a;
                        // Section 5.1: the link device between the two devices
                        const uint32_t G = S.gpus_per_node;
                        const uint32_t row = same_node
                            ? S.n_dev + node_a * G * G + (dev_a - node_a * G) * G + (dev_c - node_c * G)
                            : S.n_dev + S.n_nodes * G * G + node_a * S.n_nodes + node_c;
                        // assumption A2: transfer time = size / bandwidth (rounded up) + latency
                        const uint32_t bw = same_node ? S.bw_intra : S.bw_inter;
                        u64 ns;
                        if (WIDE) {
                            const u64 bytes = elems * S.elem_bytes;
                            ns = (bytes + bw - 1) / bw;
                        } else {
                            const uint32_t bytes = (uint32_t)elems * S.elem_bytes;
                            ns = ceil_div_u32(comm ? bytes : 1u, bw, same_node ? S.m_bw_intra : S.m_bw_inter);
                        }
                        ns += same_node ? S.lat_intra : S.lat_inter;
                        const u64 end = fifo_commit(comm, row, ns, now, true, L);
                        if (comm) arrive = end;
                        if (cnt.want_check) {
                            cnt.n_comm += __popcll(comm_mask);
                            if (comm) cnt.sum_comm_ns += ns;   // per-lane partial sums, reduced by the caller
                        }
                    }
                    if (hit) {
                        ready = arrive > ready ? arrive : ready;
                        pending -= 1;
                        touched = true;
                    }
                    if (cnt.want_check) cnt.n_pairs += __popcll(hit_mask);
                }
                PROF_MARK(4)
                overflow = overflow || (touched && ready >= TIME_LIMIT);
                const bool now_ready = touched && pending == 0;
                if (touched) {
                    w = now_ready ? ((ready << 1) | 1) : (W_WAIT | ((u64)pending << 48) | (ready & (TIME_LIMIT - 1)));
                    words[j * WAVE + lane] = w;
                }
                if (__ballot(now_ready)) {
                    const u64 nmin = wave_min_from(now_ready ? w : W_NONE, last_key);
                    if (lane == 0) {
                        if (nmin < L.l1[j]) L.l1[j] = nmin;
                        if (S.n_groups > FLAT_GROUPS && nmin < L.l2[j >> 6]) L.l2[j >> 6] = nmin;
                    }
                }
                PROF_MARK(5)
            }
            if (in_mask) k0 = W_NONE;
        }
        if (in_mask) words[i * WAVE + lane] = k0;
        const u64 new_l1 = wave_min_from(k0, last_key);
        wave_sync();
        if (lane == 0) L.l1[i] = new_l1;
        wave_sync();
        if (S.n_groups > FLAT_GROUPS) {
            const uint32_t g = i >> 6;
            const u64 new_l2 = wave_min_from(L.l1[g * WAVE + lane], last_key);
            if (lane == 0) L.l2[g] = new_l2;
            wave_sync();
        }
        PROF_MARK(6)
    }
    if (__ballot(overflow)) return RESULT_OVERFLOW;

    if (cnt.want_check) {   // diagnostics: tasks that never ran (0 in a correct run)
        for (uint32_t j = 0; j < S.n_ops; j++) cnt.n_stuck += __popcll(__ballot(words[j * WAVE + lane] != W_NONE));
    }
    // Algorithm 1, result (largest endTime): every transfer feeds a compute task that ends
    // later, so the makespan is the largest free time over the compute device rows.
    u64 mk = 0;
    for (uint32_t d = lane; d < S.n_dev; d += WAVE) mk = L.free_at[d] > mk ? L.free_at[d] : mk;
    PROF_STORE(cnt)
    return wave_max_u64(mk);
}

__device__ __forceinline__ void store_counters(Counters c, Counters* out) {
    u64 s = c.sum_comm_ns;   // accumulated per lane
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) s += shfl_xor_u64(s, m);
    c.sum_comm_ns = s;
    if (lane_id() == 0) *out = c;
}

// lane l gets the multiply-high constant of the divisor l+1
__device__ __forceinline__ uint32_t load_magic(const uint32_t* __restrict__ magic) { return magic[lane_id() + 1]; }

// LDSW: the task words and per-op exeTimes of the candidate live in LDS (small graphs).
// CFGL: the candidate's configurations are copied to LDS first (graphs of moderate size), so
// that the many uniform look-ups of a configuration do not go to memory.
template <bool WIDE, bool LDSW, bool CFGL>
__global__ __launch_bounds__(WAVE) void k_sim_batch(SimDev S, const DOp* __restrict__ ops, const DEdge* __restrict__ edges,
                                                    const DEdge* __restrict__ in_edges, const uint32_t* __restrict__ cost,
                                                    const uint32_t* __restrict__ magic, const uint2* __restrict__ strategies,
                                                    uint32_t B, u64* __restrict__ out_ns, Counters* __restrict__ stats,
                                                    unsigned char* __restrict__ ws, size_t slot_stride) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const Tables T{ops, edges, in_edges, cost};
    u64* words;
    uint32_t* exe_of;
    unsigned char* lds_rest = lds_raw;
    if (LDSW) {
        words = (u64*)lds_raw;
        exe_of = (uint32_t*)(lds_raw + (size_t)S.n_ops * WAVE * 8);
        lds_rest = lds_raw + ((slot_bytes(S.n_ops, S.n_ops_pad) + 15) & ~(size_t)15);
    } else {
        unsigned char* slot = ws + (size_t)blockIdx.x * slot_stride;
        words = (u64*)slot;
        exe_of = (uint32_t*)(slot + (size_t)S.n_ops * WAVE * 8);
    }
    uint2* cfg_lds = (uint2*)lds_rest;
    if (CFGL) lds_rest += (size_t)S.n_ops_pad * 8;
    const WaveLds L = carve_lds(lds_rest, S);
    const uint32_t magic_v = load_magic(magic);
    for (uint32_t b = blockIdx.x; b < B; b += gridDim.x) {
        Counters cnt = {};
        cnt.want_check = stats != nullptr;
        const uint2* cfgs = strategies + (size_t)b * S.n_ops;
        u64 mk;
        if (CFGL) {
            for (uint32_t i = lane_id(); i < S.n_ops; i += WAVE) cfg_lds[i] = cfgs[i];
            wave_sync();
            mk = simulate_candidate<WIDE>(S, T, cfg_lds, words, exe_of, L, magic_v, cnt);
        } else {
            mk = simulate_candidate<WIDE>(S, T, cfgs, words, exe_of, L, magic_v, cnt);
        }
        if (lane_id() == 0) out_ns[b] = mk;
        if (stats) store_counters(cnt, stats + b);
        wave_sync();
    }
}

// Delta entry, first form: every step applies the mutation to the chain's strategy and
// re-runs build + Algorithm 1 (the definition of the delta result, Section 5.3).  A
// mutation that names an op outside the graph makes this and all later results of the
// chain RESULT_INVALID.
template <bool WIDE>
__global__ __launch_bounds__(WAVE) void k_sim_chain_steps(SimDev S, const DOp* __restrict__ ops, const DEdge* __restrict__ edges,
                                                          const DEdge* __restrict__ in_edges, const uint32_t* __restrict__ cost,
                                                          const uint32_t* __restrict__ magic, uint2* chain_cfgs, uint32_t C,
                                                          const uint32_t* __restrict__ muts, uint32_t n_steps,
                                                          u64* __restrict__ out_ns, uint32_t* chain_flags,
                                                          unsigned char* __restrict__ ws, size_t slot_stride) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const Tables T{ops, edges, in_edges, cost};
    const WaveLds L = carve_lds(lds_raw, S);
    const uint32_t c = blockIdx.x;
    if (c >= C) return;
    unsigned char* slot = ws + (size_t)c * slot_stride;
    u64* words = (u64*)slot;
    uint32_t* exe_of = (uint32_t*)(slot + (size_t)S.n_ops * WAVE * 8);
    uint2* cfgs = chain_cfgs + (size_t)c * S.n_ops;
    const uint32_t magic_v = load_magic(magic);
    bool poisoned = first_u32(chain_flags[c]) != 0;
    for (uint32_t s = 0; s < n_steps; s++) {
        if (muts) {   // muts: [n_steps][C] records of {op, cfg.x, cfg.y}
            const uint32_t* m = muts + ((size_t)s * C + c) * 3;
            const uint32_t op = first_u32(m[0]);
            if (op < S.n_ops) {
                if (lane_id() == 0) cfgs[op] = make_uint2(m[1], m[2]);
            } else {
                poisoned = true;
            }
            __threadfence_block();
            wave_sync();
        }
        Counters cnt = {};
        u64 mk = RESULT_INVALID;
        if (!poisoned) mk = simulate_candidate<WIDE>(S, T, cfgs, words, exe_of, L, magic_v, cnt);
        if (lane_id() == 0) out_ns[(size_t)s * C + c] = mk;
        wave_sync();
    }
    if (lane_id() == 0) chain_flags[c] = poisoned ? 1u : 0u;
}

}  // namespace ffsim
