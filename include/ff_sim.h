/* ff_sim.h -- C boundary of the batched execution simulator for gfx950 (MI355X).
 *
 * The library predicts the per-iteration execution time of an operator graph G on a
 * simulated device topology D under a parallelization strategy S (FlexFlow, Section 5: the
 * simulator's inputs are G, D and S, its output is the predicted time).  It does so for many
 * candidate strategies at once, one candidate per wavefront.
 *
 * All times are unsigned 64-bit integer nanoseconds.  Results are bit-exact: the value
 * returned for a strategy is the makespan of Algorithm 1 (full simulation) run on the task
 * graph of Section 5.1, with tasks leaving the queue in (readyTime, task id) order, where
 * task ids follow construction order: compute tasks by (op, part index), then
 * communication tasks by (tensor edge, producer part, consumer part).
 *
 * Pointers named d_* are DEVICE pointers (e.g. a torch tensor's data_ptr()); all other
 * pointers are HOST pointers.  The caller owns every buffer it passes.  Device buffers
 * must stay valid until the work queued on the stream has finished.  Handles are not
 * thread-safe; distinct handles are independent.  No function throws or aborts; every
 * int-returning function returns FF_OK (0) or a negative FF_E* code.
 */
#ifndef FF_SIM_H
#define FF_SIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    FF_OK = 0,
    FF_EINVAL = -1,     /* malformed argument (null pointer, unsorted edges, bad field) */
    FF_ENOMEM = -2,     /* host or device allocation failed */
    FF_EWORKSPACE = -3, /* no workspace set, or too small for this call */
    FF_ERANGE = -4,     /* a documented size limit is exceeded */
    FF_EHIP = -5        /* a HIP runtime call failed */
};

#define FF_MAX_DIMS 4
#define FF_MAX_PARTS 64          /* largest |c_i|: one wavefront lane per part */
#define FF_MAX_OPS 4096
#define FF_MAX_EXTENT (1u << 20)
#define FF_MAX_DEVICES 1024
/* Graph and machine together must also fit one workgroup's LDS (160 KB on gfx950), else
 * ff_sim_create returns FF_ERANGE: 16 * ceil(n_ops / 64) * 64 + 9 * R + 1040 bytes, where
 * R = n_devices + n_nodes * gpus_per_node^2 + n_nodes^2 is the number of device rows (compute
 * devices, links inside nodes, links between nodes).  Examples that fit: 4096 ops on 16 x 4
 * devices; any graph of up to 1024 ops on 64 x 4 or 120 x 1 devices. */
#define FF_MAX_MAP_STRIDE 1024       /* ff_dimmap_t.stride */
#define FF_MAX_MAP_OFFSET (1 << 29)  /* |ff_dimmap_t.a|, |ff_dimmap_t.b| */
#define FF_MAX_IN_EDGES 511          /* tensor edges into one op */
#define FF_TIME_LIMIT_NS (1ull << 48) /* simulated times must stay below this */
#define FF_INVALID_NS UINT64_MAX /* result for a candidate whose strategy is invalid */
#define FF_INTERNAL_NS (UINT64_MAX - 1) /* result if an internal consistency check failed (a library bug) */
#define FF_OVERFLOW_NS (UINT64_MAX - 2) /* result if a simulated time reached FF_TIME_LIMIT_NS */

/* How a consumer part's output range along one dim selects the range it reads along one
 * PRODUCER dim (Section 4: the input tensors a task needs follow from its output tensor and
 * the type of the operation).  src_dim = consumer output dim driving this
 * producer dim, or -1 if every consumer part reads the producer's whole extent.  For a
 * consumer part covering [lo, hi) along src_dim the range read is
 * [lo*stride + a, (hi-1)*stride + b + 1), clamped to [0, extent).  stride >= 1. */
typedef struct {
    int8_t src_dim;
    uint8_t kind;   /* 0: the consumer reads (above); 1: the producer contributes (below); the same on all four maps of an edge */
    uint16_t stride;
    int32_t a, b;
} ff_dimmap_t;
/* kind = 1 marks a CONTRIBUTING edge: the gradient that flows back along a forward edge in a training
 * iteration (Sections 2 and 8 are about training iterations; Section 5.1's construction is stated for
 * tensor edges in general).  It is the forward edge with the roles exchanged: map[] is indexed by the
 * CONSUMER's dims, src_dim names a PRODUCER dim, and a producer part covering [lo, hi) along src_dim
 * contributes to [lo*stride + a, (hi-1)*stride + b + 1) of the consumer's dim, clamped to its extent.  A
 * producer part and a consumer part share the elements of that range that lie in the consumer part's
 * box.  With the backward ops cut like their forward ops, the pairs and sizes are the forward edge's,
 * transposed. */

/* One operation o_i of the operator graph (Section 3.1): the shape of its single output
 * tensor and which output dims may be partitioned (Table 1; bit d of par_mask). */
typedef struct {
    uint8_t ndim; /* 1..4 */
    uint8_t par_mask;
    uint16_t type; /* informational */
    uint32_t extent[FF_MAX_DIMS]; /* 1..FF_MAX_EXTENT for d < ndim; ignored beyond */
} ff_op_t;

/* One tensor edge (o_src, o_dst); map[] is indexed by the PRODUCER (src) dim. */
typedef struct {
    uint32_t src_op, dst_op;
    ff_dimmap_t map[FF_MAX_DIMS];
} ff_edge_t;

/* Operator graph.  Ops must be in topological order (src_op < dst_op for every edge) and
 * edges sorted by (src_op, dst_op); the position in `edges` is the edge id used in
 * communication-task ids.  n_ops <= FF_MAX_OPS. */
typedef struct {
    uint32_t n_ops, n_edges;
    const ff_op_t* ops;
    const ff_edge_t* edges;
} ff_opgraph_t;

/* Simulated machine (device topology, Section 3.1): n_nodes x gpus_per_node compute
 * devices, device id = node*gpus_per_node + local.  Every ordered GPU pair inside a node
 * has its own link (intra_* bandwidth in bytes/ns and latency); every ordered node pair
 * has one network link shared by all its GPU pairs (inter_*).  Transfer time of s bytes =
 * ceil(s / bandwidth) + latency (assumption A2 plus the edge latency label). */
typedef struct {
    uint32_t n_nodes, gpus_per_node;
    uint32_t intra_Bpns, inter_Bpns;
    uint32_t intra_lat_ns, inter_lat_ns;
    uint32_t elem_bytes;
} ff_machine_t;

/* exeTime of a compute task (Section 5.1: measured once per op type and output size, then
 * cached -- here handed in): ns[op*n_cols + (parts-1)] for an op split into `parts` tasks.
 * Every entry must be >= 1.  Configurations with more than n_cols parts are invalid. */
typedef struct {
    uint32_t n_ops, n_cols;
    const uint32_t* ns;
} ff_costtable_t;

/* Parallelization configuration c_i of one op (Section 4): a degree per output dim
 * (1 on dims that are not parallelizable or beyond ndim; deg[d] <= extent[d]; product
 * <= min(FF_MAX_PARTS, n_cols)); part k (row-major over deg, dim 0 slowest) covers
 * [floor(p*E/deg), floor((p+1)*E/deg)) in each dim and runs on device
 * (dev_offset + k*dev_stride) mod n_devices, dev_offset < n_devices. */
typedef struct {
    uint8_t deg[FF_MAX_DIMS];
    uint16_t dev_offset;
    uint16_t dev_stride;
} ff_opcfg_t;

/* A proposal of the search (Section 6.2): op's configuration is replaced by cfg. */
typedef struct {
    uint32_t op;
    ff_opcfg_t cfg;
} ff_mutation_t;

/* Per-candidate counters written by ff_sim_batch when a stats buffer is set. */
typedef struct {
    uint64_t n_compute;   /* compute tasks = sum of |c_i| */
    uint64_t n_pairs;     /* producer/consumer task pairs with a shared sub-tensor */
    uint64_t n_comm;      /* of those, pairs on different devices (communication tasks) */
    uint64_t sum_comm_ns; /* sum of communication-task exeTimes */
    uint64_t n_events;    /* queue pops of the event loop */
    uint64_t exit_code;   /* 0 = event loop ran to completion (anything else is a library bug) */
    uint64_t n_stuck;     /* compute tasks that never ran (0 in a correct run) */
    uint64_t reserved;
} ff_stats_t;

typedef struct ff_sim ff_sim_t;
typedef struct ff_chains ff_chains_t;

/* Validates and deep-copies graph, machine and cost table (HOST pointers; may be freed on
 * return) and uploads them to the current HIP device.  Section 5, inputs G and D. */
int ff_sim_create(const ff_opgraph_t* graph, const ff_machine_t* machine, const ff_costtable_t* cost,
                  ff_sim_t** out);

/* The same with the cost of an op's tasks given per DEGREE TUPLE instead of per number of parts:
 * how long a task runs depends on which dims are split, not only on how many parts there are
 * (Section 5.1 takes exeTime from measurements of the operation at the task's output size).
 * Op i's entries are tuples[tuple_ptr[i] .. tuple_ptr[i+1]) -- four degrees, one byte each,
 * deg[0] lowest, strictly ascending as integers -- with exeTime ns[] (>= 1) at the same index.
 * A configuration whose tuple is not listed has no cost: the strategy is invalid
 * (FF_INVALID_NS).  HOST pointers, deep-copied. */
typedef struct {
    uint32_t n_ops;
    const uint32_t* tuple_ptr;   /* [n_ops + 1], tuple_ptr[0] = 0 */
    const uint32_t* tuples;      /* [tuple_ptr[n_ops]] */
    const uint32_t* ns;          /* [tuple_ptr[n_ops]] */
} ff_tuplecost_t;
int ff_sim_create_tuplecost(const ff_opgraph_t* graph, const ff_machine_t* machine, const ff_tuplecost_t* costs,
                            ff_sim_t** out);
void ff_sim_destroy(ff_sim_t* sim);

/* Links inside a node that are not all alike (Section 3: the device topology's connections each
 * carry their own bandwidth and latency; Section 8.1's older cluster pairs GPUs on boards behind
 * a shared switch).  Bpns[a * gpus_per_node + b] / lat_ns[...] describe the link from local
 * GPU a to local GPU b, the same in every node; entries with a == b are not used; lat_ns may be
 * null (0 ns).  They replace machine.intra_Bpns / intra_lat_ns for every later call; links
 * between nodes keep the machine's figures.  links == NULL returns to the machine's single
 * figures.  HOST pointers, deep-copied.  Waits for the device to be idle.  Chain sets created
 * before the call hold timelines simulated with the old links: every later ff_sim_delta,
 * ff_sim_delta_try, ff_sim_search and ff_sim_neighbours on them returns FF_EINVAL (destroy them).
 * FF_EINVAL if gpus_per_node differs from the machine's or if a bandwidth is 0. */
typedef struct {
    uint32_t gpus_per_node;
    const uint32_t* Bpns;
    const uint32_t* lat_ns;
} ff_linktable_t;
int ff_sim_set_links(ff_sim_t* sim, const ff_linktable_t* links);

/* Network links between nodes that are not all alike (Section 3, as above): Bpns[a * n_nodes + b] /
 * lat_ns[...] describe the link from node a to node b; entries with a == b are not used; lat_ns may
 * be null (0 ns).  They replace machine.inter_Bpns / inter_lat_ns for every later call; each ordered
 * node pair keeps its one link, shared by all GPU pairs of the two nodes.  links == NULL returns to
 * the machine's single figures.  Independent of ff_sim_set_links; otherwise the same rules (HOST
 * pointers, deep-copied, waits for the device, invalidates chain sets created before).  FF_EINVAL if
 * n_nodes differs from the machine's or if a bandwidth is 0. */
typedef struct {
    uint32_t n_nodes;
    const uint32_t* Bpns;
    const uint32_t* lat_ns;
} ff_nodelinks_t;
int ff_sim_set_node_links(ff_sim_t* sim, const ff_nodelinks_t* links);

/* Tied configurations (Section 4 gives every OPERATION one configuration; in the graph of a training
 * iteration an operation appears as several ops: its forward and its backward computation, or the
 * unrolled steps of a recurrent layer that share parameters).  leader[i] = the op whose entry of the
 * strategy op i takes (leader[leader[i]] == leader[i], else FF_EINVAL); entries of ops that lead
 * nobody are not read; a strategy is invalid unless the configuration is valid for every op that takes
 * it.  HOST pointer [n_ops], deep-copied; NULL: every op takes its own entry.  Waits for the device;
 * invalidates chain sets created before, as ff_sim_set_links does.  With ties a mutation changes several
 * ops at once: ff_sim_delta, ff_sim_delta_try, ff_sim_search and the neighbour sweeps stay exact but
 * simulate every step from time 0 (mutations of ops that lead nobody change nothing). */
int ff_sim_set_ties(ff_sim_t* sim, const uint32_t* leader);

/* Parameter synchronisation (Section 8 compares strategies by the data they move to keep the
 * replicas of an op's parameters in step; Section 5.1 has no construction for it).  Reading
 * taken: op i holds param_bytes[i] bytes of parameters (0: none), indexed by the output dims in
 * param_dims[i] (bit d = dim d).  A configuration cuts them into one shard per index along those
 * dims (shards = product of their degrees, ceil(param_bytes / shards) bytes each); the parts that
 * differ only in the other dims are replicas of a shard, and the replica with index 0 in all
 * other dims owns it.  When a replica's task has finished it sends its gradient of the shard to
 * the owner's device: one communication task per replica that sits on another device than the
 * owner, with the replica's task as its only predecessor and no successor, created right after
 * the communication tasks of the op's out-edges (ids go op by op).  The simulated time is then
 * the largest endTime over compute and communication tasks.  The update and the way back are
 * not modelled.
 * HOST pointers [n_ops], deep-copied; param_bytes == NULL switches it off.  Waits for the
 * device to be idle; chain sets created before the call are invalidated as by ff_sim_set_links. */
int ff_sim_set_params(ff_sim_t* sim, const uint32_t* param_bytes, const uint8_t* param_dims);

/* Scratch for a batch of B candidates (per-task queue keys and readyTime / pending-input
 * counters of the resident candidates).  The workspace is caller-allocated device memory,
 * 256-byte aligned, and may be shared by successive calls on the same stream.  Small
 * graphs keep this state in LDS; then 0 bytes are needed and no workspace has to be set. */
size_t ff_sim_workspace_bytes(const ff_sim_t* sim, uint32_t B);
int ff_sim_set_workspace(ff_sim_t* sim, void* d_ws, size_t bytes);

/* Optional: d_stats[B] receives counters on every later ff_sim_batch (null to stop). */
int ff_sim_set_stats(ff_sim_t* sim, ff_stats_t* d_stats);

/* Section 5.1 + Algorithm 1 for B strategies: d_strategies is [B][n_ops] configurations,
 * d_out_ns[b] receives the simulated execution time of candidate b, or FF_INVALID_NS if
 * its strategy is invalid.  Asynchronous on hip_stream (a hipStream_t, null = default). */
int ff_sim_batch(ff_sim_t* sim, const ff_opcfg_t* d_strategies, uint32_t B, uint64_t* d_out_ns,
                 void* hip_stream);
/* ff_sim_batch, ff_sim_batch_devmaps, ff_sim_delta and ff_sim_delta_try put nothing but kernel
 * launches on the stream (no allocation, no memset, no copy): they may be recorded into a HIP
 * graph.  So may ff_sim_search from the second call with the same d_tuple_ptr / n_tuples on (the
 * first one reads the ranges back to check them; they must not change afterwards).
 * ff_sim_neighbours allocates and waits: not for capture. */

/* Which kernel instantiation ff_sim_batch launches for B candidates on this handle (measurement
 * aid: a profile of the kernel can be matched to the launch it belongs to): writes
 * "k_sim_batch<WIDE, LDSW, STATS, Q, CACHE, EXT, GPN>" with the template arguments as they appear
 * in a kernel trace into buf (HOST memory, len bytes; FF_ERANGE if it does not fit). */
int ff_sim_batch_kernel_name(const ff_sim_t* sim, uint32_t B, char* buf, size_t len);

/* The same with the device of every task given one by one (Section 4: a configuration assigns
 * each of its tasks a device) instead of dev_offset + k * dev_stride: d_devmaps is
 * [B][n_ops][FF_MAX_PARTS], entry k of an op = device of its part k (< n_devices, else the
 * strategy is invalid); entries beyond the op's number of parts have no meaning (all FF_MAX_PARTS
 * entries of an op must be readable), and the configurations' dev_offset / dev_stride are not
 * read.  Device memory, read only.  Workspace, stats and
 * results as for ff_sim_batch. */
int ff_sim_batch_devmaps(ff_sim_t* sim, const ff_opcfg_t* d_strategies, const uint16_t* d_devmaps, uint32_t B,
                         uint64_t* d_out_ns, void* hip_stream);

/* Delta simulation (Section 5.3, Algorithm 2's contract: same timeline as a full simulation
 * of the changed strategy).  A chain set holds C current strategies on the device;
 * d_out_ns0[c] receives the time of the starting strategies.  The library owns the
 * chains' state and allocates it here with hipMalloc: per chain the strategy, one word and two
 * endTimes per possible task, and two places for each of 32 snapshots of the simulation state
 * (about 67 * 512 * n_ops bytes: 80 MB for a 2321-op graph).  Destroy only after the work queued on the stream has finished. */
int ff_sim_chains_create(ff_sim_t* sim, const ff_opcfg_t* d_strategies, uint32_t C, uint64_t* d_out_ns0,
                         void* hip_stream, ff_chains_t** out);
/* Applies d_muts[s][c] (step-major, [n_steps][C]) to chain c for s = 0..n_steps-1,
 * cumulatively, and writes the simulated time after every step to d_out_ns[s][c]
 * (FF_INVALID_NS while the chain's strategy is invalid). */
int ff_sim_delta(ff_chains_t* chains, const ff_mutation_t* d_muts, uint32_t n_steps, uint64_t* d_out_ns,
                 void* hip_stream);
void ff_sim_chains_destroy(ff_chains_t* chains);

/* Trial mutations: the proposals of the search before acceptance (Section 6.2).  Evaluates M
 * alternative single-op mutations per chain -- d_muts is [M][C], proposal-major -- each against
 * the chain's current strategy and stored timeline, and writes the simulated times to
 * d_out_ns[M][C].  The chains are NOT changed (commit an accepted proposal with
 * ff_sim_delta).  Results equal a full simulation of the mutated strategy (Section 5.3).
 * Needs the handle's workspace (ff_sim_set_workspace) to hold
 * ff_sim_delta_try_workspace_bytes(chains, M) bytes.  Asynchronous on hip_stream; must not
 * overlap with ff_sim_delta on the same chains or with other users of the workspace. */
size_t ff_sim_delta_try_workspace_bytes(const ff_chains_t* chains, uint32_t M);
int ff_sim_delta_try(ff_chains_t* chains, const ff_mutation_t* d_muts, uint32_t M, uint64_t* d_out_ns,
                     void* hip_stream);

/* Neighbour sweep (Section 8.4's check that a strategy is locally optimal: compare it with all
 * of its neighbours, the strategies that differ in the configuration of one op).  For every
 * chain, simulates every neighbour of its current strategy for the ops op_begin..op_end-1:
 * neighbour index k runs over the ops in order, per op over the degree tuples of its list
 * (d_tuple_ptr / d_tuples as in ff_search_t, list order), per tuple over dev_offset
 * 0..n_devices-1, dev_stride 1 (the op's current configuration is among them).
 * ff_sim_neighbour_count gives their number M.  d_muts[M][C] receives the list itself,
 * d_out_ns[M][C] the simulated times, d_best_ns[c] / d_best_index[c] the smallest time of
 * chain c and the lowest neighbour index that reaches it.  The chains are not changed.
 * Workspace as for ff_sim_delta_try with the same M.  Both calls copy n_ops+1 integers back
 * and ff_sim_neighbours returns only when the stream has finished the work. */
int ff_sim_neighbour_count(const ff_chains_t* chains, const uint32_t* d_tuple_ptr, uint32_t n_tuples,
                           uint32_t op_begin, uint32_t op_end, uint32_t* out_count);
int ff_sim_neighbours(ff_chains_t* chains, const uint32_t* d_tuple_ptr, const uint32_t* d_tuples, uint32_t n_tuples,
                      uint32_t op_begin, uint32_t op_end, ff_mutation_t* d_muts, uint64_t* d_out_ns,
                      uint64_t* d_best_ns, uint32_t* d_best_index, void* hip_stream);

/* ff_sim_neighbours for callers that cannot allocate or wait: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs and results as
 * ff_sim_neighbours, but the call only puts kernels on the stream: it allocates nothing (host or
 * device), copies nothing back and does not synchronise.  The index of every op's first neighbour,
 * which ff_sim_neighbours builds on the host and keeps in a temporary allocation, is built by a
 * kernel in a fixed scratch array that lives in the library's device image (16.6 KB per GPU, held
 * until the process ends).  The caller passes M, the neighbour count it sized d_muts / d_out_ns for
 * (ff_sim_neighbour_count, called once outside the loop); the ranges of d_tuple_ptr are checked on
 * the device: if they are malformed or do not add up to M, every result of the call is
 * FF_INVALID_NS (d_best_ns too) and d_muts names no op.
 * Limits: op_end - op_begin <= 4096 (FF_ERANGE beyond; the library's own limit on ops), M * C < 2^32.
 * All calls on one GPU share the one scratch array: calls that overlap in time on the same GPU (other
 * streams, other chain sets, other threads) race; calls in stream order do not.  Workspace as for
 * ff_sim_delta_try with the same M. */
int ff_sim_neighbours_noalloc(ff_chains_t* chains, const uint32_t* d_tuple_ptr, const uint32_t* d_tuples, uint32_t n_tuples,
                              uint32_t op_begin, uint32_t op_end, uint32_t M, ff_mutation_t* d_muts, uint64_t* d_out_ns,
                              uint64_t* d_best_ns, uint32_t* d_best_index, void* hip_stream);

/* The search loop of Section 6 on the device, one Markov chain per chain: per step one
 * proposal (Section 6.2: a random op gets a random configuration) is simulated as a trial
 * and accepted by the Metropolis rule of Section 6.1, min(1, exp(beta*(cost - cost*))), which
 * the caller supplies in integers so that every decision is reproducible: a proposal that is
 * not slower is always accepted; one that is slower by delta ns is accepted iff
 * (draw >> 32) < d_accept[min(delta / bucket_ns, n_buckets - 1)], i.e. d_accept holds
 * probabilities scaled by 2^32.  Draws are counter based: with K = 0xD6E8FEB86659FD93 and
 * mix64 = the SplitMix64 finaliser (x += 0x9E3779B97F4A7C15; x = (x ^ x>>30) * 0xBF58476D1CE4E5B9;
 * x = (x ^ x>>27) * 0x94D049BB133111EB; x ^= x>>31),
 *   draw(purpose, chain, step) = mix64(mix64(mix64(mix64(seed) ^ purpose*K) ^ chain*K) ^ step*K),
 * step counted from first_step; op = draw(10) mod n_ops; the configuration is entry
 * draw(11) mod (number of entries) of the op's list d_tuples[d_tuple_ptr[op] .. d_tuple_ptr[op+1])
 * (four degrees, one byte each, deg[0] lowest), dev_offset = draw(12) mod n_devices,
 * dev_stride = 1; the acceptance draw is draw(13).  An invalid proposal is rejected.
 * Stopping (Section 6.2 gives two criteria): the budget is n_steps, the caller's; and a chain that
 * has gone `patience` steps without finding a new best makes no further proposals (its time
 * repeats in the trace; a caller who wants the paper's setting passes half of its step budget);
 * the count carries over between calls on the same chains.
 * d_trace_ns[s][c] receives the time of chain c's strategy after step s; d_best_ns[c] /
 * d_best[c][n_ops] are updated whenever a step ends with a better time than d_best_ns[c]
 * (initialise it to UINT64_MAX).  All d_* are device pointers.  The call copies n_ops+1
 * integers back to validate d_tuple_ptr (it synchronises the stream's device). */
typedef struct {
    uint64_t seed;
    uint64_t first_step;
    uint64_t bucket_ns;
    uint64_t patience;              /* steps without a new best after which a chain stops proposing; 0 = never */
    uint32_t n_buckets;
    uint32_t n_tuples;              /* entries in d_tuples */
    const uint32_t* d_accept;       /* [n_buckets] */
    const uint32_t* d_tuple_ptr;    /* [n_ops + 1] */
    const uint32_t* d_tuples;       /* [n_tuples] */
    uint64_t* d_best_ns;            /* [C] in/out */
    ff_opcfg_t* d_best;             /* [C][n_ops] out */
} ff_search_t;
int ff_sim_search(ff_chains_t* chains, const ff_search_t* params, uint32_t n_steps, uint64_t* d_trace_ns,
                  void* hip_stream);

/* The same search, with the same result in every respect that ff_sim_search documents (trace, best
 * times and strategies, the chains' strategies afterwards), for callers with FEWER chains than the
 * GPU has room for: one chain is one wavefront in ff_sim_search, whatever the size of the device.
 * Section 6.2's proposal for a step depends on the step's random draws alone, not on the chain's
 * strategy, and a rejected proposal leaves the strategy as it was (Section 6.1).  So the proposals of
 * the next K steps of every chain are simulated side by side, each against the chain's current
 * strategy (the trial kernel of ff_sim_delta_try); a chain then walks through them in order, takes
 * the decisions of ff_sim_search with the same draws, and stops at the first proposal it accepts,
 * which is simulated once more and committed; what was simulated for the steps after it is dropped,
 * and the next round starts from there.  A round costs about two simulations and takes a chain to
 * its first accepted proposal, so it pays when few proposals are accepted (the later, longer part
 * of a search): the call measures the share of accepted proposals as it goes, simulates ahead
 * (K about two over that share, at most max_ahead and at most what the trial kernel has wavefronts
 * for) while the share is below a quarter, and otherwise -- or when the chains alone fill the
 * device -- simulates the steps one by one in stretches: 8 steps, then stretches that end by the
 * device's clock, each four times as long as the one before, every chain stopping where it is.
 * max_ahead | FF_AHEAD_ALWAYS switches the measuring off: every round simulates ahead, with K =
 * max_ahead (or what fits), for callers who know that few proposals will be taken.
 * Needs the handle's workspace to hold ff_sim_delta_try_workspace_bytes(chains, max_ahead) bytes
 * (FF_EWORKSPACE otherwise).  NOT asynchronous: the call allocates its buffers on first use and waits
 * for hip_stream after every round (it copies C integers back to see how far the chains are), so
 * it cannot be captured into a graph.  h_stats (HOST, may be null): rounds taken, proposals
 * simulated ahead, steps made (n_steps * C when the call returns FF_OK), proposals accepted. */
#define FF_AHEAD_ALWAYS 0x80000000u
typedef struct { uint64_t rounds, proposals_simulated, steps, accepted; } ff_ahead_stats_t;
int ff_sim_search_ahead(ff_chains_t* chains, const ff_search_t* params, uint32_t n_steps, uint32_t max_ahead,
                        uint64_t* d_trace_ns, void* hip_stream, ff_ahead_stats_t* h_stats);

/* The acceptance table of ff_sim_search for the Metropolis rule of Section 6.1 with a given beta:
 * out[b] = floor(2^32 * exp(-beta_per_ns * b * bucket_ns)), capped at 2^32 - 1 -- the probability
 * of accepting a proposal that is slower by b * bucket_ns, the lower edge of bucket b (so a
 * proposal slower by delta is accepted with exp(-beta * bucket_ns * floor(delta / bucket_ns)),
 * at most a factor exp(beta * bucket_ns) above the rule's exp(-beta * delta); beyond the last
 * bucket the probability stays at that bucket's).  Double-precision arithmetic on the host, in
 * this order: ((-beta_per_ns) * b) * bucket_ns.  out: HOST array of n_buckets entries (upload it
 * as ff_search_t.d_accept).  FF_EINVAL for beta < 0 or NaN, bucket_ns = 0, n_buckets = 0. */
int ff_sim_accept_table(double beta_per_ns, uint64_t bucket_ns, uint32_t n_buckets, uint32_t* out);

/* Telemetry of the chains (HOST array of C records; synchronises the device): how many
 * mutations were applied, how many of them resumed from a stored snapshot of the timeline
 * instead of simulating from time 0, how many queue pops they took in total, how many
 * pops the last simulation from time 0 took, and how many committed steps stopped early
 * because their timeline had re-joined the previous one (Section 5.3: most of the timeline
 * does not change). */
typedef struct {
    uint64_t n_steps, n_resumed, n_events, n_events_full, n_converged;
} ff_chain_stats_t;
int ff_sim_chains_get_stats(ff_chains_t* chains, ff_chain_stats_t* h_out);

const char* ff_sim_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* FF_SIM_H */
