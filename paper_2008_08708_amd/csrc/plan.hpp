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
};

// Validates the schedule and fills everything except the device fields and `grid`.
// num_cus is the CU count the launch shape is sized for.
sccl_status_t sccl_compile_host(const sccl_topology_t* topo, const sccl_collective_t* coll,
                                const sccl_schedule_t* sched, const sccl_options_t* opts, int num_cus,
                                sccl_plan* plan);
