// Device-side tables and wavefront primitives of the batched execution simulator (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ffsim {

typedef unsigned long long u64;
typedef uint32_t u32;

constexpr int WAVE = 64;

// ---- one 64-bit word per compute task (index op*64 + part) -----------------------------
//   bit 63 clear: a pending event of the task, word = time*2 + kind
//       kind 1: the task is READY and waits to be dequeued, time = readyTime
//       kind 0: the task was dequeued, time = endTime; its successors are released then
//   bit 63 set:  no pending event
//       W_NONE                       unused lane, or the task is complete
//       W_WAIT | pending<<48 | ready the task still waits for `pending` inputs; `ready` is
//                                    the largest endTime among the inputs seen so far
// Words with bit 63 set compare greater than every event, so a plain unsigned minimum over
// words finds the next event.
constexpr u64 W_NONE = ~0ull;
constexpr u64 W_WAIT = 1ull << 63;
constexpr u64 TIME_LIMIT = 1ull << 48;      // times must stay below this (about 78 hours)
constexpr u32 PENDING_LIMIT = 0x7fff;       // a task may wait for fewer than this many inputs

// results that are not times
constexpr u64 RESULT_INVALID = ~0ull;        // invalid strategy
constexpr u64 RESULT_INTERNAL = ~0ull - 1;   // internal consistency check failed (a bug)
constexpr u64 RESULT_OVERFLOW = ~0ull - 2;   // a simulated time reached TIME_LIMIT

// cext = extent of the consumer's dim src_dim (1 if src_dim < 0)
struct DMap { int32_t src_dim; uint32_t stride; int32_t a, b; uint32_t cext; };
// a tensor edge with the shapes of both ends inlined, so that releasing the successors of
// a finished producer needs no second table lookup
// A READING edge (kind 0): map[d] belongs to dim d of the producer's tensor, src_dim names a consumer dim,
// src_ndim / src_extent are the producer's.  A CONTRIBUTING edge (kind 1, a gradient flowing back along a forward
// edge): the roles are exchanged -- map[d] belongs to dim d of the CONSUMER's tensor, src_dim names a producer
// dim (cext = the producer's extent there), and src_ndim / src_extent hold the consumer's shape: they always
// describe the tensor in which the ranges of the two parts are intersected.
struct DEdge {
    uint32_t src, dst, src_ndim, eid;   // eid: index of the record in the producer-sorted array
    uint32_t src_extent[4];
    uint32_t kind;               // 0 reading, 1 contributing
    uint32_t unused[3];
    DMap map[4];
};
struct DOp {
    uint32_t extent[4];          // 1 beyond ndim
    uint32_t ndim, par_mask;
    uint32_t out_begin, out_end; // range in edges[] (edges are sorted by producer)
    uint32_t in_begin, in_end;   // range in in_list[]
    uint32_t param_bytes;        // parameters the op holds (0: none) and the output dims that index them (bit d);
    uint32_t param_dims;         // used when SimDev::sync is set
    DEdge first;                 // copy of edges[out_begin] (most ops have one consumer): one
                                 // scalar burst brings the op and its first out-edge
};

// scalars describing (G, D, cost table); passed by value
struct SimDev {
    uint32_t n_ops, n_edges, n_cols, max_parts;
    uint32_t n_nodes, gpus_per_node, n_dev, n_rows;
    uint32_t bw_intra, bw_inter, lat_intra, lat_inter, elem_bytes;
    uint32_t m_bw_intra, m_bw_inter;   // floor(2^32 / bw) (2^32-1 for bw = 1)
    uint32_t magic_dev, magic_gpn;     // floor(2^32/d)+1 for d = n_dev, gpus_per_node (0 if d = 1)
    uint32_t pass_dev, pass_gpn;       // all ones iff the divisor is 1
    uint32_t n_ops_pad;                // n_ops rounded up to a multiple of 64
    uint32_t n_groups;                 // n_ops_pad / 64  (<= 64)
    uint32_t link_table;               // 1: links inside a node differ per ordered GPU pair (see LINK_TABLE_AT)
    uint32_t sync;                     // 1: parameter synchronisation transfers are simulated (DOp::param_bytes)
    uint32_t node_table;               // 1: links between nodes differ per ordered node pair (table behind the one above)
    uint32_t ties;                     // 1: op i takes the configuration of op tie[i] (table behind the link tables)
};
// The constants buffer every kernel receives: words 0..64 are division constants
// (floor(2^32/d)+1 for d = 2..64); if SimDev::link_table is set, four words per ordered pair of
// local GPUs (from * gpus_per_node + to) follow at word LINK_TABLE_AT: bandwidth (B/ns),
// floor(2^32 / bandwidth), latency (ns), 0.  Behind that area (always gpus_per_node^2 entries long), if
// SimDev::node_table is set, the same four words per ordered pair of nodes (from * n_nodes + to; always
// n_nodes^2 entries).  Behind that, if SimDev::ties is set, one word per op: the op whose configuration it takes.
constexpr uint32_t LINK_TABLE_AT = 128;
__host__ __device__ inline uint32_t tie_table_at(uint32_t gpus_per_node, uint32_t n_nodes) {
    return LINK_TABLE_AT + 4u * (gpus_per_node * gpus_per_node + n_nodes * n_nodes);
}

// the per-lane condition "my bit of this lane mask is set" (the mask is used as it is)
__device__ __forceinline__ bool lanes_of(u64 mask) { return __builtin_amdgcn_inverse_ballot_w64(mask); }

// a uniform value placed in a vector register, opaque to the compiler (which would otherwise copy
// it from its scalar register again at every use)
__device__ __forceinline__ uint32_t vector_copy(uint32_t uniform) {
    uint32_t v;
    asm volatile("v_mov_b32 %0, %1" : "=v"(v) : "s"(uniform));
    return v;
}

__device__ __forceinline__ int lane_id() { return (int)threadIdx.x & (WAVE - 1); }

// Orders LDS traffic between the lanes of the (single-wavefront) workgroup.  LDS operations
// of one wavefront execute in program order, so no wait and no s_barrier is needed; the
// fence only keeps the compiler from forwarding or reordering LDS accesses across it.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// mask of the lanes where p holds.  (The toolkit's __ballot takes an int: a bool costs a
// select and a compare before the mask exists.)
__device__ __forceinline__ u64 ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// the readlane / readfirstlane builtins return int: go through uint32_t before widening
__device__ __forceinline__ uint32_t first_u32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ u64 first_u64(u64 v) { return (u64)first_u32((uint32_t)v) | ((u64)first_u32((uint32_t)(v >> 32)) << 32); }
__device__ __forceinline__ uint32_t readlane_u32(uint32_t v, int l) { return (uint32_t)__builtin_amdgcn_readlane((int)v, l); }
__device__ __forceinline__ u64 readlane_u64(u64 v, int l) {
    return (u64)readlane_u32((uint32_t)v, l) | ((u64)readlane_u32((uint32_t)(v >> 32), l) << 32);
}

__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int m) {
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    lo = __shfl_xor(lo, m);
    hi = __shfl_xor(hi, m);
    return ((u64)hi << 32) | lo;
}

// lane i of every row of 16 lanes reads lane perm(i) of the same row (DPP controls:
// quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E, row_half_mirror = 0x141,
// row_mirror = 0x140); all of them are permutations, so every lane reads a valid lane.
// Call only with all 64 lanes active.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    // old = 0 with bound_ctrl lets the compiler fold the move into the consuming instruction
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}

// lane l reads lane l-1 of the whole wavefront, lane 0 reads 0 (DPP wave_shr:1).  Call only
// with all 64 lanes active.
__device__ __forceinline__ uint32_t wave_shr1_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x138, 0xf, 0xf, true);
}
__device__ __forceinline__ u64 wave_shr1_u64(u64 v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, 0x138, 0xf, 0xf, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), 0x138, 0xf, 0xf, true);
    return ((u64)hi << 32) | lo;
}

// lane l reads v of lane src (any permutation or gather; through the LDS crossbar, no LDS memory).  Call only
// with all 64 lanes active.
__device__ __forceinline__ uint32_t gather_u32(uint32_t v, uint32_t src) {
    return (uint32_t)__builtin_amdgcn_ds_bpermute((int)(src << 2), (int)v);
}
// lane l hands v to lane dst (dst must be a permutation of the lanes).  All 64 lanes active.
__device__ __forceinline__ uint32_t scatter_u32(uint32_t v, uint32_t dst) {
    return (uint32_t)__builtin_amdgcn_ds_permute((int)(dst << 2), (int)v);
}

// Segmented inclusive running sum along the 64 lanes: lane l gets the sum of v over the lanes from the
// last lane <= l whose `head` is set up to l (lane 0 counts as a head).  Six DPP steps on the pair
// (head seen so far, sum): shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of
// rows 0 / 2 into rows 1 / 3 and lane 31 into rows 2 and 3.  Lanes that a step gives no source keep
// their value (old = 0 is the identity of both components).  All 64 lanes active.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void seg_step(uint32_t& f, uint32_t& v) {
    const uint32_t tv = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
    const uint32_t tf = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)f, CTRL, ROW_MASK, 0xf, false);
    v += f ? 0u : tv;
    f |= tf;
}
__device__ __forceinline__ uint32_t seg_running_sum(uint32_t v, bool head) {
    uint32_t f = head ? 1u : 0u;
    seg_step<0x111, 0xf>(f, v);      // row_shr:1
    seg_step<0x112, 0xf>(f, v);      // row_shr:2
    seg_step<0x114, 0xf>(f, v);      // row_shr:4
    seg_step<0x118, 0xf>(f, v);      // row_shr:8
    seg_step<0x142, 0xa>(f, v);      // row_bcast:15 into rows 1 and 3
    seg_step<0x143, 0xc>(f, v);      // row_bcast:31 into rows 2 and 3
    return v;
}

// wavefront-wide min of a 32-bit value, uniform result: butterfly inside each row of 16
// lanes with DPP, then the four row results are combined on the scalar unit
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    uint32_t t;
    t = dpp_u32<0xB1>(v); v = t < v ? t : v;
    t = dpp_u32<0x4E>(v); v = t < v ? t : v;
    t = dpp_u32<0x141>(v); v = t < v ? t : v;
    t = dpp_u32<0x140>(v); v = t < v ? t : v;
    uint32_t a = readlane_u32(v, 0), b = readlane_u32(v, 16), c = readlane_u32(v, 32), d = readlane_u32(v, 48);
    a = a < b ? a : b;
    c = c < d ? c : d;
    return a < c ? a : c;
}

// minimum over the wavefront, uniform result: high words first, then the low words of the
// lanes that hold the minimal high word
__device__ __forceinline__ u64 wave_min_u64(u64 v) {
    const uint32_t hi = (uint32_t)(v >> 32), lo = (uint32_t)v;
    const uint32_t mhi = wave_min_u32(hi);
    const uint32_t mlo = wave_min_u32(hi == mhi ? lo : 0xffffffffu);
    return ((u64)mhi << 32) | mlo;
}
__device__ __forceinline__ u64 wave_max_u64(u64 v) { return ~wave_min_u64(~v); }

// Same minimum for words that are all >= base (pending events never lie before the event
// popped last): one 32-bit reduction over the saturated distance to base; the 64-bit
// reduction only runs if every distance is 2^32-1 or more (no event, or a far one).
// ROW0: the caller knows at compile time that lanes 16..63 hold words with bit 63 set (no event
// there): the butterfly inside the first row of 16 lanes is then the whole reduction.
__device__ __forceinline__ uint32_t row0_min_u32(uint32_t v) {
    uint32_t t;
    t = dpp_u32<0xB1>(v); v = t < v ? t : v;
    t = dpp_u32<0x4E>(v); v = t < v ? t : v;
    t = dpp_u32<0x141>(v); v = t < v ? t : v;
    t = dpp_u32<0x140>(v); v = t < v ? t : v;
    return readlane_u32(v, 0);
}
template <bool ROW0 = false>
__device__ __forceinline__ u64 wave_min_from(u64 v, u64 base) {
    const u64 d = v - base;
    const uint32_t sat = (uint32_t)(d >> 32) ? 0xffffffffu : (uint32_t)d;
    const uint32_t m = ROW0 ? row0_min_u32(sat) : wave_min_u32(sat);
    if (m != 0xffffffffu) return base + m;
    return wave_min_u64(v);
}

// floor(n / d) with magic = floor(2^32/d)+1 (0 if d = 1) and pass = all ones iff d = 1;
// exact while n*d < 2^32; no branch
__device__ __forceinline__ uint32_t div_magic(uint32_t n, uint32_t magic, uint32_t pass) {
    return __umulhi(n, magic) + (n & pass);
}
// ceil(n / d) for any 32-bit n >= 1, m = floor(2^32/d) (one fix-up step)
__device__ __forceinline__ uint32_t ceil_div_u32(uint32_t n, uint32_t d, uint32_t m) {
    uint32_t x = n - 1;
    uint32_t q = __umulhi(x, m);
    uint32_t r = x - q * d;
    q += (r >= d) ? 1u : 0u;
    return q + 1;
}

}  // namespace ffsim
