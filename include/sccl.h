/*
 * sccl.h -- C ABI of the MI355X schedule executor.
 *
 * The library executes a k-chunk, S-step collective schedule in the sense of
 * "Synthesizing Optimal Collective Algorithms" (SCCL) for P *virtual* ranks
 * whose buffers all live in the memory of ONE GPU.  It does not synthesize
 * schedules; it validates and runs them.
 *
 * Vocabulary (paper, section 3.2-3.3):
 *   P        number of nodes (ranks)
 *   G        global number of chunks; every rank buffer is one contiguous
 *            array of G chunks and chunk c sits at element offset
 *            c * elems_per_chunk in EVERY rank's buffer (global chunk
 *            numbering, section 3.2.2).  Collectives run in place.
 *   B        bandwidth relation: pairs (L, b), L a set of directed node
 *            pairs, b the number of chunks that may cross L per round
 *            (section 3.2.1)
 *   pre/post relations over (chunk, node) (Tables 1 and 2)
 *   (Q, T)   the schedule: Q = r_0..r_{S-1} rounds per step, T a set of sends
 *            (c, n, n', s) (section 3.3).  Steps are numbered from 0.
 *
 * All pointers in the structs below are HOST pointers, read during the call
 * and never retained.  rank_buffers[] entries are DEVICE pointers.
 * Functions return a status and never throw, abort or print.
 */
#ifndef SCCL_H
#define SCCL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SCCL_MAX_RANKS 64          /* P may not exceed this */

typedef enum {
    SCCL_OK = 0,
    SCCL_ERR_INVALID_ARG = 1,      /* null pointer, index out of range, r_s < 1, unknown op/dtype, P > SCCL_MAX_RANKS,
                                      REDUCE send in a non-combining collective */
    SCCL_ERR_TOPOLOGY = 2,         /* malformed bandwidth relation (edge out of range, negative b, self loop) */
    SCCL_ERR_SEND_NO_SOURCE = 3,   /* a send reads (c, n) that is not in V_s (section 3.3), or that was consumed */
    SCCL_ERR_SEND_NO_LINK = 4,     /* (n, n') is not a usable link: not in E of section 3.4 */
    SCCL_ERR_BANDWIDTH = 5,        /* some (L, b) sees more than b * r_s sends in step s (section 3.3) */
    SCCL_ERR_POSTCONDITION = 6,    /* post not reached after S steps */
    SCCL_ERR_HAZARD = 7,           /* a step reads and writes one (c, n), writes it twice, or counts a rank twice */
    SCCL_ERR_ALIGNMENT = 8,        /* a rank buffer is not 16-byte aligned */
    SCCL_ERR_OVERLAP = 9,          /* two rank buffers overlap */
    SCCL_ERR_NOMEM = 10,
    SCCL_ERR_DEVICE = 11,          /* a HIP call failed, execute on a host-only plan, or execute while another
                                      device than the plan's is current */
    SCCL_ERR_SCRATCH = 12          /* sccl_execute_static only: the plan's step table does not fit the library's
                                      static device array of SCCL_STATIC_SCRATCH_BYTES */
} sccl_status_t;

typedef enum {
    SCCL_I32 = 0,                  /* wrapping 32-bit sum */
    SCCL_F32 = 1,                  /* IEEE binary32 add, round to nearest even */
    SCCL_F16 = 2                   /* binary16 in memory; widened exactly to binary32, summed in binary32 and
                                      rounded to nearest even ONCE per reduce group per step */
} sccl_dtype_t;

typedef enum { SCCL_COPY = 0, SCCL_REDUCE_SUM = 1 } sccl_sendop_t;

/* One directed node pair. */
typedef struct { int32_t src, dst; } sccl_edge_t;

/* One element (L, b) of the bandwidth relation B (section 3.2.1): at most
 * chunks_per_round * r_s sends of step s may use the edges listed.  A pair is a
 * usable link iff at least one entry lists it and every entry that lists it
 * has chunks_per_round > 0. */
typedef struct {
    const sccl_edge_t* edges;
    int32_t num_edges;
    int32_t chunks_per_round;
} sccl_bw_t;

typedef struct {
    int32_t num_nodes;             /* P */
    const sccl_bw_t* bw;
    int32_t num_bw;
} sccl_topology_t;

/* A collective as a (pre, post) pair over (chunk, node), Table 2 of the paper.
 * pre and post are G x P row-major arrays of 0/1 bytes: pre[c*P + n] != 0 iff
 * (c, n) is in the relation.
 * combining == 0: chunks are only copied; pre says where chunk c is at the
 *   start, post where it must be at the end.  Regions outside pre are
 *   undefined inputs and are never read.
 * combining == 1 (section 3.5): pre says which ranks hold a *version* of
 *   chunk c, post where the sum over all P ranks' versions must be at the end
 *   (Reducescatter: pre All, post Scattered; Allreduce: pre All, post All). */
typedef struct {
    int32_t num_global_chunks;     /* G */
    const uint8_t* pre;
    const uint8_t* post;
    int32_t combining;
    sccl_dtype_t dtype;
    int64_t elems_per_chunk;       /* >= 0; chunk bytes = elems_per_chunk * sizeof(dtype) */
    /* Optional layout.  The paper numbers chunks globally (section 3.2.2) but leaves open where a node
     * keeps them.  slot == NULL: every rank keeps chunk c at chunk position c of a G-chunk buffer.
     * Otherwise slot is G x P row-major, slot[c*P + n] = chunk position of chunk c in rank n's buffer
     * of slots_per_rank chunks, or -1 if rank n never holds chunk c.  Required (else
     * SCCL_ERR_INVALID_ARG): a position for every (c, n) in pre and for the source and destination of
     * every send; positions in range; two chunks never share a position on one rank. */
    const int32_t* slot;
    int32_t slots_per_rank;
} sccl_collective_t;

/* One send (c, n, n', s) of section 3.3 plus, for combining collectives, what
 * the receiver does with it (section 4, first paragraph): SCCL_COPY replaces
 * the destination's chunk, SCCL_REDUCE_SUM adds the source's version to it. */
typedef struct { int32_t chunk, src, dst, step; int32_t op; } sccl_send_t;

/* The candidate solution (Q, T).  The ORDER of `sends` matters: all
 * SCCL_REDUCE_SUM sends of one step into the same (chunk, dst) form one group
 * and are added left to right in array order, starting from the
 * destination's own value. */
typedef struct {
    int32_t num_steps;             /* S */
    const int32_t* rounds;         /* Q: r_0 .. r_{S-1}, each >= 1 */
    const sccl_send_t* sends;
    int64_t num_sends;
} sccl_schedule_t;

/* Options of sccl_plan_create_ex; zero-initialise for the defaults. */
#define SCCL_PLAN_HOST_ONLY 1u     /* validate and compile only: touches no device; the plan cannot be executed */

/* How sccl_execute lowers the plan (paper, section 4: the same schedule admits several lowerings).
 *   SCCL_LOWER_MEMORY  every send reads and writes the rank buffers; what one step wrote the next step
 *                      reads back through the cache hierarchy.  Work is split by (chunk, element tile).
 *   SCCL_LOWER_STAGED  a workgroup takes one slice (a run of consecutive vectors) of one chunk, loads it from
 *                      every cell (rank, chunk position) of that chunk the schedule reads into the local
 *                      data share, runs all the chunk's sends there, dependency level by dependency level,
 *                      and writes the cells the schedule wrote back once.  Same operations in the same
 *                      order per element, hence the same bits; made for small buffers, where the time is
 *                      the chain of memory round trips (the latency term of the paper's cost model, section
 *                      3.6) and not the bytes.  Needs room for one slice of every cell of a chunk and fewer
 *                      than 256 dependency levels per chunk: SCCL_ERR_INVALID_ARG if asked for explicitly
 *                      and that does not hold.
 *   SCCL_LOWER_AUTO    from measured crossovers: staged when possible and either the P rank buffers together
 *                      are at most 512 KiB (launch overhead dominates; staged never loses), or staging saves at
 *                      least three memory round trips per chunk (groups of the longest chunk chain minus
 *                      sccl_stats_t.staged_levels) and the staged kernel has at most 4096 work items;
 *                      through memory otherwise. */
#define SCCL_LOWER_AUTO   0
#define SCCL_LOWER_MEMORY 1
#define SCCL_LOWER_STAGED 2

typedef struct {
    uint32_t flags;
    int32_t block_threads;         /* through-memory kernel: 0 = choose from the chunk size; else 64, 128 or 256 */
    int32_t vectors_per_thread;    /* through-memory kernel: 0 = choose; else 1, 2, 4 or 8 vectors per lane and operand */
    int32_t max_workgroups;        /* 0 = choose (through memory: one workgroup per compute unit); else the
                                      grid size of either kernel; always capped by the number of work items */
    int32_t lowering;              /* SCCL_LOWER_* */
    int32_t slice_vectors;         /* staged kernel: 0 = choose; else a power of two: vectors of every cell of a chunk
                                      a workgroup stages at a time */
    int32_t staged_threads;        /* staged kernel: 0 = one wavefront (64); else 64, 128, 256, 512 or 1024 */
    int32_t reserved;              /* must be 0 */
} sccl_options_t;

typedef struct {
    int32_t num_nodes, num_global_chunks;
    int32_t num_steps;             /* S */
    int32_t num_rounds;            /* R = sum of Q */
    int32_t k;                     /* R - S: the schedule is k-synchronous (section 3.1) */
    int64_t num_sends;
    int64_t num_copy_groups;       /* (step, chunk, src) groups */
    int64_t num_reduce_groups;     /* (step, chunk, dst) groups */
    int32_t max_fan_in, max_fan_out;
    int32_t chunks_per_node;       /* C: the most chunks any node holds in pre (section 3.2.2) */
    int64_t chunk_bytes;
    int64_t bytes_per_rank;        /* G (or slots_per_rank) * chunk_bytes */
    int64_t bytes_min;             /* sum over copy groups of (1 + k) chunks and over reduce groups of (k + 2) chunks */
    int64_t bytes_unfused;         /* 2 chunks per COPY send + 3 per REDUCE send */
    /* launch shape chosen for the kernel */
    int32_t vector_bytes;          /* 16, 8, 4 or 2: widest access that divides the chunk size */
    int32_t block_threads, vectors_per_thread;
    int64_t num_work_items;        /* G * tiles per chunk */
    int32_t grid_workgroups;       /* grid of the kernel sccl_execute launches; 0 for a host-only plan */
    /* the staged lowering: dependency structure of the schedule and what a workgroup stages */
    int32_t lowering;              /* SCCL_LOWER_MEMORY or SCCL_LOWER_STAGED: what sccl_execute runs */
    int32_t staged_available;      /* 1 if one slice of every cell of a chunk fits the local data share */
    int32_t num_cells;             /* distinct (rank, chunk position) pairs some send touches, over all chunks */
    int32_t num_cells_loaded;      /* of those, read before any send writes them */
    int32_t num_cells_stored;      /* of those, written by some send */
    int32_t num_levels;            /* length of the longest chain of dependent groups (of any one chunk) */
    int32_t staged_levels;         /* levels the staged kernel runs: copies whose source stays put are propagated at
                                      plan time (the destination is stored from the source's place in the local
                                      data share), so an Allgather has 0 and an Allreduce about half of num_levels */
    int32_t staged_tasks;          /* cell writes left after that, over all chunks */
    int32_t max_level_tasks;       /* most cell writes any one level of any one chunk performs */
    int32_t max_chunk_groups;      /* most groups any one chunk has (its chain in the through-memory kernel) */
    int32_t slice_vectors, staged_threads;
    int32_t staged_lds_bytes;      /* local data share one workgroup uses */
    int64_t num_slices;            /* staged work items: G * ceil(vectors per chunk / slice_vectors) */
    int64_t static_table_bytes;    /* bytes of the step table sccl_execute_static would place in its static array */
} sccl_stats_t;

typedef struct sccl_plan sccl_plan_t;

/*
 * Validate (Q, T) against the topology and the collective (section 3.3's run
 * and bandwidth constraint; for combining collectives the contribution-set
 * rules documented at SCCL_ERR_HAZARD) and compile it into a device step
 * table on the current HIP device.  Everything passed in is deep-copied; the
 * caller may free its arrays on return.  On error *out_plan is NULL.
 * The plan owns its device memory until sccl_plan_destroy.
 */
sccl_status_t sccl_plan_create(const sccl_topology_t* topology, const sccl_collective_t* collective,
                               const sccl_schedule_t* schedule, sccl_plan_t** out_plan);

/* As above with explicit options (may be NULL). */
sccl_status_t sccl_plan_create_ex(const sccl_topology_t* topology, const sccl_collective_t* collective,
                                  const sccl_schedule_t* schedule, const sccl_options_t* options,
                                  sccl_plan_t** out_plan);

/*
 * Execute the plan in place: all S steps of sends (section 3.3; lowered as one
 * kernel as in section 4, "single kernel") on the P device buffers
 * rank_buffers[0..P-1], each G (or slots_per_rank) * elems_per_chunk elements, 16-byte aligned and
 * pairwise disjoint (checked: SCCL_ERR_ALIGNMENT / SCCL_ERR_OVERLAP).
 * `stream` is a hipStream_t (NULL = the default stream).  Which kernel runs is
 * the plan's lowering (sccl_options_t.lowering, reported by sccl_plan_stats).
 * The call enqueues one kernel and returns; it does not synchronise and does not allocate.  The
 * pointer array is read on the host during the call.  Nothing is launched
 * when the status is not SCCL_OK.  A plan is immutable: concurrent calls with
 * one plan are allowed as long as their buffers differ.  Because the call does
 * nothing but check its arguments on the host and enqueue one kernel, it may
 * be made while `stream` is being captured into a HIP graph.
 */
sccl_status_t sccl_execute(const sccl_plan_t* plan, void* const* rank_buffers, void* stream);

/*
 * The two other lowerings the paper compares its fused kernel with (section 4, "single and multiple
 * kernels", and section 5.5): same arguments, same checks and same results as sccl_execute.
 *
 * sccl_execute_stepwise enqueues ONE kernel per step (the kernel boundary is the global
 * synchronisation between steps); each kernel fuses the copy and reduce groups of its step.
 *
 * sccl_execute_memcpy enqueues one device-to-device hipMemcpyAsync per COPY send, in step order
 * (the copy-engine lowering).  Only for plans without REDUCE sends: otherwise SCCL_ERR_INVALID_ARG.
 */
sccl_status_t sccl_execute_stepwise(const sccl_plan_t* plan, void* const* rank_buffers, void* stream);
sccl_status_t sccl_execute_memcpy(const sccl_plan_t* plan, void* const* rank_buffers, void* stream);

/*
 * sccl_execute for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same checks, same kernels and same results as
 * sccl_execute, but the step table the kernel walks is not the copy sccl_plan_create uploaded: it lives in a
 * static device array of SCCL_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU the
 * library runs on holds its own copy until the process ends).  So the plan may be a SCCL_PLAN_HOST_ONLY plan,
 * whose creation touched no device; with such a plan no call of this library ever allocates device memory.
 *
 * The call (1) returns SCCL_ERR_SCRATCH, before anything else is looked at and with nothing enqueued, when the
 * table of the plan's lowering is larger than the array (sccl_stats_t.static_table_bytes says how large it is);
 * (2) checks the buffers like sccl_execute; (3) writes the table into the array with small kernels enqueued on
 * `stream`, one per 3.5 KiB of table (the words travel as kernel arguments: no copy from host memory and no
 * staging buffer is involved) -- the array keeps whatever the last call left there, so this is skipped only
 * when the last call on this GPU was for the same plan; (4) enqueues the plan's kernel on `stream`.  It calls
 * no hipMalloc, no hipFree, no memset and no routine that allocates, and does not synchronise.  The launch
 * shape is sized for the current device.
 *
 * All calls on one GPU share the one array: calls on different streams, or from different threads, whose
 * work may overlap on the GPU race for it.  Serialise them on one stream (or with events).  Under graph
 * capture the table writes are captured too, by value, so a replay is correct whatever ran in between; and
 * because a replay rewrites the array at a time the library cannot see, from the first call on a capturing
 * stream on every call on that GPU writes its table, captured or not.
 */
#define SCCL_STATIC_SCRATCH_BYTES (256 * 1024)
sccl_status_t sccl_execute_static(const sccl_plan_t* plan, void* const* rank_buffers, void* stream);

/* S, R, k, group counts, algorithmic byte counts and the launch shape. */
sccl_status_t sccl_plan_stats(const sccl_plan_t* plan, sccl_stats_t* out_stats);

/*
 * The compiled step table of a plan as 32-bit words: exactly what the kernel of the given lowering walks (and what
 * sccl_execute_static writes into its array).  Host only; for inspection, and so that the plan compiler can be
 * checked without a GPU by interpreting the table.  Copies at most `capacity` words into `out` (NULL allowed when
 * capacity is 0); *out_words is always the table's length; info[0..3] describe it.  An operand is
 * rank | chunk position << 8.  SCCL_ERR_INVALID_ARG for an unknown lowering or a staged table the plan does not have
 * (sccl_stats_t.staged_available == 0).
 *
 * lowering == SCCL_LOWER_MEMORY.  info[0] = word at which the op lists start.  Words 0 .. G: for every chunk the
 * offset of its op list relative to info[0], and the end.  An op list is the chunk's groups in step order, each
 *     header   bit 0: 0 copy group, 1 reduce group; k << 8
 *     anchor   copy: the source operand; reduce: the destination operand
 *     k words  copy: the destination operands; reduce: the source operands in schedule order
 * A copy group stores the anchor's chunk to every destination; a reduce group adds the sources, left to right, onto
 * the destination's own value.
 *
 * lowering == SCCL_LOWER_STAGED.  info[0] = words per block (one block per chunk), info[1] = words reserved for
 * storage operands, info[2] = log2 of the slice length in vectors, info[3] = byte offset of the identity storage.
 * A workgroup keeps one slice (1 << info[2] vectors of sccl_stats_t.vector_bytes) of every "storage" of a chunk in
 * its local data share, storage i at byte i * slice bytes; below, a storage is named by that byte offset.  Block:
 *     8 words          storages, storages to load (the first ones), cells to store, levels, tasks, overflow words, 0, 0
 *     info[1] words    the operand each storage is loaded from (meaningful for the storages to load)
 *     levels + 2       index of the first task of every level, then the number of tasks, twice
 *     2 x stores       for every cell the schedule wrote: the storage holding its final value, its operand
 *     (padding to a multiple of 4 words)
 *     8 x tasks        destination storage | k << 24, overflow index, four source storages, two words of padding.
 *                      k == 0: a copy of the first source.  Otherwise the destination's own value plus the first
 *                      min(k, 4) sources in order (unused ones name the identity storage, which holds the additive
 *                      identity), plus overflow[index .. index + k - 5] for k > 4; written to the destination.
 *     overflow words   fifth and later sources
 * Tasks of one level touch no storage in conflicting ways; levels run in order; then the stores.
 */
sccl_status_t sccl_plan_table(const sccl_plan_t* plan, int32_t lowering, int32_t* out, int64_t capacity,
                              int64_t* out_words, int32_t info[4]);

/* Frees host and device memory of the plan; NULL is allowed.  The caller
 * makes sure no execute of this plan is still running. */
void sccl_plan_destroy(sccl_plan_t* plan);

const char* sccl_status_string(sccl_status_t status);

/*
 * The paper's cost model (section 3.6): with a node's L input bytes cut into C chunks, step s of r_s rounds
 * takes alpha + (r_s / C) * L * beta seconds, the plan S * alpha + (R / C) * L * beta.  Here L = C *
 * chunk_bytes of the plan.  alpha (seconds per step) and beta (seconds per byte) must be >= 0.  Host only.
 */
sccl_status_t sccl_plan_cost(const sccl_plan_t* plan, double alpha, double beta, double* out_seconds);

/*
 * Which of several plans for the same collective and input size the cost model prefers (section 5.5: the
 * latency-optimal algorithm for small inputs, the bandwidth-optimal one for large inputs): the index of the
 * plan with the lowest sccl_plan_cost, the earliest on ties.  plans is a host array of num_plans >= 1 plans.
 */
sccl_status_t sccl_select_plan(const sccl_plan_t* const* plans, int32_t num_plans, double alpha, double beta,
                               int32_t* out_best);

/*
 * Fit of the model's two constants to n >= 2 measurements t[i] of algorithms with latency cost a[i] (= S) and
 * bandwidth cost b[i] (= R / C * L, in bytes): least squares for t = a * alpha + b * beta.  Host arrays.
 * SCCL_ERR_INVALID_ARG if the samples do not determine both constants (a and b proportional).
 */
sccl_status_t sccl_cost_fit(int32_t n, const double* a, const double* b, const double* t, double* out_alpha,
                            double* out_beta);

/*
 * The same fit with a constant term: least squares for t = t0 + a * alpha + b * beta, n >= 3.  On one GPU a
 * launch costs a few microseconds whatever the schedule, which the paper's two-term model (section 3.6) has no
 * place for; with t0 taken out, alpha and beta describe what a step and a byte add.  t0 does not change which of
 * several plans sccl_select_plan prefers; the alpha and beta fitted beside it do.  `weights` (n values >= 0, or
 * NULL for all ones) scales each sample's residual: with weights 1 / t the fit minimises RELATIVE errors, so that
 * the microsecond-sized samples near the crossover count as much as the millisecond-sized ones.
 * SCCL_ERR_INVALID_ARG if the samples do not determine the three constants.
 */
sccl_status_t sccl_cost_fit_intercept(int32_t n, const double* a, const double* b, const double* t, const double* weights,
                                      double* out_t0, double* out_alpha, double* out_beta);

#ifdef __cplusplus
}
#endif
#endif /* SCCL_H */
