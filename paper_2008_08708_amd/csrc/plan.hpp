// Internal: the compiled plan shared by the host compiler (plan.cpp) and the device side (exec.hip).
#pragma once

#include <cstdint>
#include <vector>

#include "sccl.h"

// Device step table ("program"): one op list per chunk, ops in step order.
// Ops of different chunks never touch the same memory (chunk c lives at the
// same offset in every rank buffer), so the only ordering the schedule imposes
// is between the ops of ONE chunk.  An op is
//   word 0      : kind (bit 0: 0 copy group, 1 reduce group) | count << 8
//   word 1      : copy: the source operand       reduce: the destination operand
//   word 2..    : copy: `count` destination operands; reduce: `count` source operands, in schedule order
// An operand is  rank | slot << 8 : the rank whose buffer is touched and the chunk position of this
// chunk in that buffer (the chunk id itself under the default layout).
constexpr int32_t OP_KIND_REDUCE = 1;
constexpr int32_t OPERAND_RANK_BITS = 8;
constexpr int32_t OPERAND_RANK_MASK = (1 << OPERAND_RANK_BITS) - 1;
constexpr int32_t MAX_SLOTS = 1 << (31 - OPERAND_RANK_BITS);

// Tables of the staged lowering, one block per chunk (chunks never share memory, so each has its own cells,
// levels and tasks).  A *cell* is one (rank, chunk position) pair some send of the chunk touches.  Cells that need
// room in the local data share ("storages") are numbered: those a send reads before any send writes them come
// first (they are what a workgroup loads), then those a task writes first; a cell that only ever receives a
// copy of a value that stays put has no storage of its own and is stored from the storage that holds its value
// (copy propagation, plan.cpp).  A *task* is one cell write that is left after that: a reduce group, or one
// destination of a copy group.  Tasks are sorted by dependency level: a task's level is one more than the highest
// level among the earlier tasks whose storages it reads after they wrote them, or writes after they read or wrote
// them, so the tasks of one level touch no storage in conflicting ways and a workgroup barrier between levels is
// all the ordering needed.
//   table:  G blocks of one stride (the largest block), so that a workgroup can fetch what it needs first
//           (header, cell words, level table) before it knows the header.
//   block:  8 header words        storages | loaded storages | stored cells | levels | tasks | overflow sources | 0 | 0
//           cell words            operand word (rank | position << 8) of every storage; room for the most any
//                                 chunk has, rounded up to 4
//           levels + 2            first task of every level, the end, the end again
//           2 x stored cells      the cells to store at the end: the storage that holds the value, the cell's
//                                 operand word; then padding to 4 words
//           8 x tasks             per task: destination storage | k << 24 ; the index of the task's fifth source in
//                                 the overflow list ; four source storages in schedule order -- a copy (k == 0) has
//                                 its source in the first, unused ones name the identity storage (one past the last
//                                 real one; the kernel fills it with the additive identity) ; two words of padding
//           overflow sources      fifth and later sources of reduce tasks with more than four; padding
//   In the device table a storage is the BYTE offset of its slice in the workgroup's cell area (storage i starts at
//   i * slice vectors * vector bytes).  The host-side pieces the table is made from keep storage ids, and their task
//   records are: destination | k << 16 ; copy: the source, reduce: the overflow index ; the first four sources.
constexpr int32_t STAGED_HEADER_WORDS = 8;
constexpr int32_t STAGED_TASK_WORDS = 8;
constexpr int32_t STAGED_TASK_K_SHIFT = 24;               // word 0 of a task record: destination byte offset | fan-in << 24
constexpr int32_t STAGED_MAX_LEVELS = 256;                // a wavefront keeps the level table in four registers per lane
constexpr int64_t STAGED_LDS_LIMIT = 160 * 1024;          // local data share of one gfx950 compute unit
constexpr int64_t STAGED_AUTO_TINY_BYTES = 512ll << 10;   // all rank buffers together: launch overhead dominates
constexpr int32_t STAGED_AUTO_MIN_SAVING = 3;             // memory round trips per chunk the staged kernel must save to be chosen
constexpr int64_t STAGED_AUTO_MAX_ITEMS = 4096;           // work items (16 per compute unit) up to which the saving pays

struct sccl_staged {
    bool available = false;
    // totals over the chunks (statistics) and maxima over the chunks (sizes a workgroup needs)
    // n_levels: dependency levels of the schedule; staged_levels: levels left after copy propagation (what the kernel runs)
    int32_t n_cells = 0, n_in = 0, n_out = 0, n_levels = 0, staged_levels = 0, n_tasks = 0, max_level_tasks = 0;
    int32_t max_chunk_groups = 0;
    int32_t max_chunk_cells = 0, max_chunk_in = 0, max_chunk_out = 0, max_block_words = 0, cell_words_room = 0;
    // per chunk, with storage ids; the device table is made from these once the slice length is known
    struct Pieces { std::vector<int32_t> cell_word, out_cells, lev_first, tasks, extra; int32_t n_in = 0, n_levels = 0; };
    std::vector<Pieces> pieces;
    std::vector<int32_t> table;
    // launch shape
    int32_t log_slice_vectors = 0;
    int32_t threads = 0;
    int64_t slices_per_chunk = 0;
    int64_t num_slices = 0;                               // work items: G x slices per chunk
    int32_t lds_bytes = 0;
    int32_t grid = 0;
};

struct sccl_plan {
    // problem
    int32_t P = 0, G = 0, S = 0;
    sccl_dtype_t dtype = SCCL_F32;
    int32_t combining = 0;
    int64_t elems_per_chunk = 0;
    std::vector<int32_t> rounds;
    // compiled program (host copy)
    std::vector<int32_t> prog;
    std::vector<int32_t> chunk_off;     // G + 1 offsets into prog
    // the same groups in step order, for the step-per-launch lowering
    std::vector<int32_t> step_prog;
    std::vector<int32_t> group_off;     // word offset of every group in step_prog, in step order
    std::vector<int32_t> step_first;    // S + 1 indices into group_off
    // COPY sends in step order (array order inside a step), for the copy-engine lowering
    struct CopySend { int32_t src, src_slot, dst, dst_slot; };
    std::vector<CopySend> copy_sends;
    sccl_stats_t stats{};
    sccl_options_t opts{};
    // launch shape
    int32_t vector_bytes = 16;
    int32_t block_threads = 256;
    int32_t vectors_per_thread = 2;
    int64_t vecs_per_chunk = 0;
    int32_t tiles_per_chunk = 0;
    int64_t num_items = 0;
    int32_t grid = 0;
    // device side (owned)
    int device = -1;
    int num_cus = 0;
    int32_t* d_prog = nullptr;
    int32_t* d_chunk_off = nullptr;
    int32_t* d_step_prog = nullptr;
    int32_t* d_group_off = nullptr;
    // the staged lowering
    sccl_staged staged;
    int32_t lowering = SCCL_LOWER_MEMORY;
    int32_t* d_staged = nullptr;
    // what sccl_execute_static writes into the library's static device array when the plan is lowered through
    // memory: chunk_off (padded to a multiple of four words), then prog at word static_prog_off.  (A staged plan
    // places staged.table there.)
    std::vector<int32_t> static_image;
    int32_t static_prog_off = 0;
    // distinct for every plan this process creates (never reused, unlike the plan's address): names whose
    // table the static array holds
    uint64_t id = 0;
};

// Validates the schedule and fills everything except the device fields and `grid`.
// num_cus is the CU count the launch shape is sized for.
sccl_status_t sccl_compile_host(const sccl_topology_t* topo, const sccl_collective_t* coll,
                                const sccl_schedule_t* sched, const sccl_options_t* opts, int num_cus,
                                sccl_plan* plan);
