// Host side of the library: validation of a schedule and its compilation into the
// per-chunk op lists the kernel walks.  No HIP calls in this file.
//
// Validation follows the paper's definition of a valid candidate solution
// (section 3.3): the run V_0 = pre, V_{s+1} = V_s + {(c,n') : (c,n) in V_s and
// (c,n,n',s) in T}; post must be reached (read as post being a subset of V_S,
// which is what constraint C2 of section 3.4 states); and for every step s and
// every (L, b) in B the sends of step s on edges of L number at most b * r_s.
// Combining collectives (section 3.5) are checked with contribution sets: the
// set of ranks whose input is summed into the value held at (c, n).

#include "plan.hpp"

#include <algorithm>
#include <cstring>
#include <map>
#include <new>
#include <utility>

namespace {

struct Group {
    int32_t kind;                 // 0 copy, 1 reduce
    int32_t chunk;
    int32_t anchor;               // copy: source rank; reduce: destination rank
    std::vector<int32_t> others;  // copy: destinations; reduce: sources (schedule order)
};

int elem_bytes(sccl_dtype_t d) { return d == SCCL_F16 ? 2 : 4; }

// Tables of the staged lowering: one block per chunk, from the chunk's op list in step order (plan.prog).
// Returns false when some chunk has more levels than the kernel keeps in registers.
//
// Copies are propagated at plan time.  Inside the local data share a COPY moves bits from one cell to another and
// nothing else, so when the source's storage is never written again (and neither is the destination) the
// destination simply ALIASES the source's storage: no task is emitted, later reads of the destination read the
// source's storage, and the final store of the destination is made from there.  What is stored where is unchanged
// bit for bit.  An Allgather, a Broadcast, a Scatter, a Gather or an Alltoall then has no level at all (load the
// holder's slice once, store it to every cell post or a forwarding step names), and an Allreduce keeps only the
// levels of its reducing half.  A copy that does not meet the condition stays a task.
bool build_staged_tables(const sccl_plan& plan, sccl_staged* out) {
    sccl_staged& sg = *out;
    sg = sccl_staged();
    const int32_t G = plan.G;
    typedef sccl_staged::Pieces Pieces;
    std::vector<Pieces>& pieces = sg.pieces;
    pieces.assign((size_t)G, Pieces());
    for (int32_t c = 0; c < G; c++) {
        // the chunk's groups: (pointer to header word) in step order
        std::vector<const int32_t*> groups;
        for (int32_t w = plan.chunk_off[(size_t)c]; w < plan.chunk_off[(size_t)c + 1];) {
            groups.push_back(&plan.prog[(size_t)w]);
            w += 2 + (plan.prog[(size_t)w] >> 8);
        }
        const size_t n_groups = groups.size();
        // pass 1: the cells (rank, chunk position) the chunk's sends touch, which of them are read before they are
        // written, and the last group that writes each
        std::map<int32_t, int32_t> first_access;          // operand word -> 0 read first, 1 written first
        std::vector<int32_t> order;                       // operand words by first appearance
        auto touch = [&](int32_t w, int32_t how) {
            if (first_access.emplace(w, how).second) order.push_back(w);
        };
        for (const int32_t* op : groups) {
            const int32_t k = op[0] >> 8;
            const bool reduce = (op[0] & OP_KIND_REDUCE) != 0;
            touch(op[1], 0);                              // copy: the source; reduce: the destination's own value
            for (int32_t j = 0; j < k; j++) touch(op[2 + j], reduce ? 0 : 1);
        }
        std::map<int32_t, int32_t> cell;                  // operand word -> logical cell id, read-first cells first
        std::vector<int32_t> cell_word;
        int32_t n_read_first = 0;
        for (int pass = 0; pass < 2; pass++)
            for (int32_t w : order)
                if (first_access[w] == pass) { cell[w] = (int32_t)cell_word.size(); cell_word.push_back(w); n_read_first += pass == 0; }
        const int32_t n_cells = (int32_t)cell_word.size();
        std::vector<int32_t> last_write((size_t)n_cells, -1);
        std::vector<uint8_t> written((size_t)n_cells, 0);
        for (size_t g = 0; g < n_groups; g++) {
            const int32_t* op = groups[g];
            const int32_t k = op[0] >> 8;
            if (op[0] & OP_KIND_REDUCE) { last_write[(size_t)cell[op[1]]] = (int32_t)g; written[(size_t)cell[op[1]]] = 1; }
            else for (int32_t j = 0; j < k; j++) { last_write[(size_t)cell[op[2 + j]]] = (int32_t)g; written[(size_t)cell[op[2 + j]]] = 1; }
        }

        // pass 2: dependency levels of the schedule itself (statistics; the through-memory kernel's chain).
        // wl/rl: level of the last write of a cell / highest level that read it.
        int32_t sched_levels = 0;
        {
            std::vector<int32_t> wl((size_t)n_cells, 0), rl((size_t)n_cells, 0);
            for (size_t g = 0; g < n_groups; g++) {
                const int32_t* op = groups[g];
                const int32_t k = op[0] >> 8;
                const bool reduce = (op[0] & OP_KIND_REDUCE) != 0;
                const int32_t anchor = cell[op[1]];
                int32_t lv = 1;
                if (reduce) {
                    lv = std::max(lv, std::max(wl[(size_t)anchor], rl[(size_t)anchor]) + 1);
                    for (int32_t j = 0; j < k; j++) lv = std::max(lv, wl[(size_t)cell[op[2 + j]]] + 1);
                    for (int32_t j = 0; j < k; j++) { int32_t& r = rl[(size_t)cell[op[2 + j]]]; r = std::max(r, lv); }
                    wl[(size_t)anchor] = lv;
                } else {
                    lv = std::max(lv, wl[(size_t)anchor] + 1);
                    for (int32_t j = 0; j < k; j++) {
                        const int32_t d = cell[op[2 + j]];
                        lv = std::max(lv, std::max(wl[(size_t)d], rl[(size_t)d]) + 1);
                    }
                    rl[(size_t)anchor] = std::max(rl[(size_t)anchor], lv);
                    for (int32_t j = 0; j < k; j++) wl[(size_t)cell[op[2 + j]]] = lv;
                }
                sched_levels = std::max(sched_levels, lv);
            }
        }

        // pass 3: copy propagation.  alias[x] = the logical cell whose STORAGE holds x's current value.  A real
        // task reads storages and writes its destination's own storage.
        struct Task { int32_t dst; std::vector<int32_t> srcs; bool reduce; int32_t level = 0; };
        std::vector<Task> tasks_in_order;
        std::vector<int32_t> alias((size_t)n_cells);
        std::vector<uint8_t> has_storage((size_t)n_cells, 0);
        for (int32_t i = 0; i < n_cells; i++) { alias[(size_t)i] = i; has_storage[(size_t)i] = i < n_read_first; }
        for (size_t g = 0; g < n_groups; g++) {
            const int32_t* op = groups[g];
            const int32_t k = op[0] >> 8;
            if (op[0] & OP_KIND_REDUCE) {
                const int32_t d = cell[op[1]];             // alias[d] == d here: a copy into a cell that is written again is never elided
                Task t{d, {}, true};
                for (int32_t j = 0; j < k; j++) t.srcs.push_back(alias[(size_t)cell[op[2 + j]]]);
                tasks_in_order.push_back(std::move(t));
                alias[(size_t)d] = d; has_storage[(size_t)d] = 1;
            } else {
                const int32_t r = alias[(size_t)cell[op[1]]];
                for (int32_t j = 0; j < k; j++) {
                    const int32_t d = cell[op[2 + j]];
                    if (last_write[(size_t)r] <= (int32_t)g && last_write[(size_t)d] <= (int32_t)g) {
                        alias[(size_t)d] = r;              // elided: d's value lives in r's storage to the end
                    } else {
                        tasks_in_order.push_back(Task{d, {r}, false});
                        alias[(size_t)d] = d; has_storage[(size_t)d] = 1;
                    }
                }
            }
        }
        // storages: the cells to load first (read before written), then the cells real tasks write first
        std::vector<int32_t> storage((size_t)n_cells, -1), storage_word;
        for (int32_t i = 0; i < n_cells; i++)
            if (has_storage[(size_t)i]) { storage[(size_t)i] = (int32_t)storage_word.size(); storage_word.push_back(cell_word[(size_t)i]); }
        const int32_t n_storage = (int32_t)storage_word.size(), n_in = n_read_first;

        // pass 4: levels of the real tasks, by storage
        int32_t n_levels = 0;
        {
            std::vector<int32_t> wl((size_t)n_storage, 0), rl((size_t)n_storage, 0);
            for (Task& t : tasks_in_order) {
                const int32_t d = storage[(size_t)t.dst];
                int32_t lv = std::max(wl[(size_t)d], rl[(size_t)d]) + 1;      // its own read of the destination is no conflict
                for (int32_t sc : t.srcs) lv = std::max(lv, wl[(size_t)storage[(size_t)sc]] + 1);
                for (int32_t sc : t.srcs) { int32_t& r = rl[(size_t)storage[(size_t)sc]]; r = std::max(r, lv); }
                wl[(size_t)d] = lv;
                t.level = lv;
                n_levels = std::max(n_levels, lv);
            }
        }
        if (n_levels >= STAGED_MAX_LEVELS) return false;

        // pass 5: the records, level by level, tasks in step order inside a level.  A task record is eight
        // words: destination | k << 16, then for a copy (k == 0) the source, for a reduce the index of its fifth
        // source in the overflow list, then the first four sources, then padding.  All are storage ids.
        std::vector<int32_t> out_cells, lev_first((size_t)n_levels + 1, 0), tasks, extra;
        for (int32_t i = 0; i < n_cells; i++)
            if (written[(size_t)i]) { out_cells.push_back(storage[(size_t)alias[(size_t)i]]); out_cells.push_back(cell_word[(size_t)i]); }
        int32_t widest = 0;
        for (int32_t lv = 1; lv <= n_levels; lv++) {
            lev_first[(size_t)lv - 1] = (int32_t)(tasks.size() / STAGED_TASK_WORDS);
            for (const Task& t : tasks_in_order) {
                if (t.level != lv) continue;
                const int32_t k = (int32_t)t.srcs.size();
                if (t.reduce) {
                    int32_t rec[STAGED_TASK_WORDS] = {storage[(size_t)t.dst] | (k << 16), (int32_t)extra.size(), 0, 0, 0, 0, 0, 0};
                    for (int32_t j = 0; j < k; j++) {
                        if (j < 4) rec[2 + j] = storage[(size_t)t.srcs[(size_t)j]];
                        else extra.push_back(storage[(size_t)t.srcs[(size_t)j]]);
                    }
                    tasks.insert(tasks.end(), rec, rec + STAGED_TASK_WORDS);
                } else {
                    const int32_t rec[STAGED_TASK_WORDS] = {storage[(size_t)t.dst], storage[(size_t)t.srcs[0]], 0, 0, 0, 0, 0, 0};
                    tasks.insert(tasks.end(), rec, rec + STAGED_TASK_WORDS);
                }
            }
            widest = std::max(widest, (int32_t)(tasks.size() / STAGED_TASK_WORDS) - lev_first[(size_t)lv - 1]);
        }
        lev_first[(size_t)n_levels] = (int32_t)(tasks.size() / STAGED_TASK_WORDS);
        lev_first.push_back(lev_first.back());            // the kernel reads one level ahead

        const int32_t n_out = (int32_t)(out_cells.size() / 2), n_tasks = (int32_t)(tasks.size() / STAGED_TASK_WORDS);
        Pieces& pc = pieces[(size_t)c];
        pc.cell_word = storage_word; pc.out_cells = out_cells; pc.lev_first = lev_first; pc.tasks = tasks; pc.extra = extra;
        pc.n_in = n_in; pc.n_levels = n_levels;

        sg.n_cells += n_cells; sg.n_in += n_in; sg.n_out += n_out; sg.n_tasks += n_tasks;
        sg.n_levels = std::max(sg.n_levels, sched_levels);
        sg.staged_levels = std::max(sg.staged_levels, n_levels);
        sg.max_level_tasks = std::max(sg.max_level_tasks, widest);
        sg.max_chunk_groups = std::max(sg.max_chunk_groups, (int32_t)n_groups);
        sg.max_chunk_cells = std::max(sg.max_chunk_cells, n_storage);
        sg.max_chunk_in = std::max(sg.max_chunk_in, n_in);
        sg.max_chunk_out = std::max(sg.max_chunk_out, n_out);
    }
    // every block has the size of the largest (none depends on the slice length)
    sg.cell_words_room = (sg.max_chunk_cells + 3) & ~3;
    for (const Pieces& pc : pieces) {
        int32_t words = STAGED_HEADER_WORDS + sg.cell_words_room + (int32_t)pc.lev_first.size() + (int32_t)pc.out_cells.size();
        words = (words + 3) & ~3;
        words += (int32_t)pc.tasks.size() + (int32_t)pc.extra.size();
        sg.max_block_words = std::max(sg.max_block_words, (words + 3) & ~3);
    }
    return true;
}

// The device table, once the slice length is known: the blocks, all of one stride, so that a workgroup can fetch
// everything it needs first (header, cell words, level table) without knowing the header:
// header | cell words, room for the most any chunk has | level table | stored cells | (pad) task records | overflow
// sources | (pad).  Storage ids become BYTE offsets into the workgroup's cell area (storage i starts at
// i * slice vectors * vector bytes), and the unused source slots of a task point at the identity storage, one
// past the last real one, which the kernel fills with the additive identity: every lane then runs the same
// four-source code whatever the fan-in.
void emit_staged_table(sccl_staged* out, int32_t log_slice, int32_t vector_bytes) {
    sccl_staged& sg = *out;
    auto at = [&](int32_t storage) { return (int32_t)(((int64_t)storage << log_slice) * vector_bytes); };
    const int32_t identity = at(sg.max_chunk_cells);
    sg.table.clear();
    for (size_t c = 0; c < sg.pieces.size(); c++) {
        const sccl_staged::Pieces& pc = sg.pieces[c];
        std::vector<int32_t>& o = sg.table;
        const size_t before = o.size();
        const int32_t hdr[STAGED_HEADER_WORDS] = {(int32_t)pc.cell_word.size(), pc.n_in, (int32_t)(pc.out_cells.size() / 2), pc.n_levels,
                                                  (int32_t)(pc.tasks.size() / STAGED_TASK_WORDS), (int32_t)pc.extra.size(), 0, 0};
        o.insert(o.end(), hdr, hdr + STAGED_HEADER_WORDS);
        o.insert(o.end(), pc.cell_word.begin(), pc.cell_word.end());
        o.resize(before + STAGED_HEADER_WORDS + (size_t)sg.cell_words_room, 0);
        o.insert(o.end(), pc.lev_first.begin(), pc.lev_first.end());
        for (size_t i = 0; i < pc.out_cells.size(); i += 2) { o.push_back(at(pc.out_cells[i])); o.push_back(pc.out_cells[i + 1]); }
        while ((o.size() - before) % 4) o.push_back(0);               // records are read as 16-byte vectors
        for (size_t t = 0; t < pc.tasks.size(); t += STAGED_TASK_WORDS) {
            const int32_t dst = pc.tasks[t] & 0xffff, k = pc.tasks[t] >> 16;
            int32_t rec[STAGED_TASK_WORDS] = {at(dst) | (k << STAGED_TASK_K_SHIFT), pc.tasks[t + 1], identity, identity, identity, identity, 0, 0};
            if (k == 0) rec[2] = at(pc.tasks[t + 1]);                 // a copy: its source sits in the first source slot
            for (int32_t j = 0; j < k && j < 4; j++) rec[2 + j] = at(pc.tasks[t + 2 + j]);
            o.insert(o.end(), rec, rec + STAGED_TASK_WORDS);
        }
        for (int32_t e : pc.extra) o.push_back(at(e));
        o.resize((c + 1) * (size_t)sg.max_block_words, 0);
    }
}

int32_t log2_of(int32_t p) { int32_t l = 0; while ((1 << l) < p) l++; return l; }

}  // namespace

// Copy-only plans: the most tile writes a work item performs from writing a cell (inclusive) to reading it back;
// 0 when nothing that was written is read again.  1 means every forwarded chunk is read back by the very next write.
static int32_t copy_reread_distance(const sccl_plan& plan) {
    int32_t worst = 0;
    std::vector<std::pair<int32_t, int32_t>> wrote;       // (operand word, number of writes before it)
    for (int32_t c = 0; c < plan.G; c++) {
        wrote.clear();
        int32_t writes = 0;
        const int32_t* op = plan.prog.data() + plan.chunk_off[(size_t)c];
        const int32_t* end = plan.prog.data() + plan.chunk_off[(size_t)c + 1];
        while (op < end) {
            const int32_t k = op[0] >> 8;
            if (op[0] & OP_KIND_REDUCE) return 0;         // not a copy-only plan
            for (size_t i = wrote.size(); i-- > 0;)
                if (wrote[i].first == op[1]) { worst = std::max(worst, writes - wrote[i].second); break; }
            for (int32_t j = 0; j < k; j++) wrote.emplace_back(op[2 + j], writes++);
            op += 2 + k;
        }
    }
    return worst;
}

sccl_status_t sccl_compile_host(const sccl_topology_t* topo, const sccl_collective_t* coll,
                                const sccl_schedule_t* sched, const sccl_options_t* opts, int num_cus,
                                sccl_plan* plan) {
    if (!topo || !coll || !sched || !plan) return SCCL_ERR_INVALID_ARG;
    const int32_t P = topo->num_nodes;
    const int32_t G = coll->num_global_chunks;
    const int32_t S = sched->num_steps;
    if (P < 1 || P > SCCL_MAX_RANKS || G < 1 || S < 1) return SCCL_ERR_INVALID_ARG;
    if (!coll->pre || !coll->post || !sched->rounds) return SCCL_ERR_INVALID_ARG;
    if (coll->elems_per_chunk < 0) return SCCL_ERR_INVALID_ARG;
    // a caller may hand over any integer in the enum's place: look at the bits before treating it as the enum
    int32_t dtype_bits;
    static_assert(sizeof(coll->dtype) == sizeof(dtype_bits), "sccl_dtype_t is a 32-bit enum in this ABI");
    std::memcpy(&dtype_bits, &coll->dtype, sizeof(dtype_bits));
    if (dtype_bits != SCCL_I32 && dtype_bits != SCCL_F32 && dtype_bits != SCCL_F16) return SCCL_ERR_INVALID_ARG;
    const sccl_dtype_t dtype = (sccl_dtype_t)dtype_bits;
    if (sched->num_sends < 0 || (sched->num_sends > 0 && !sched->sends)) return SCCL_ERR_INVALID_ARG;
    if (topo->num_bw < 0 || (topo->num_bw > 0 && !topo->bw)) return SCCL_ERR_INVALID_ARG;
    if (opts) {
        const int32_t bt = opts->block_threads, vt = opts->vectors_per_thread;
        if (!(bt == 0 || bt == 64 || bt == 128 || bt == 256)) return SCCL_ERR_INVALID_ARG;
        if (!(vt == 0 || vt == 1 || vt == 2 || vt == 4 || vt == 8)) return SCCL_ERR_INVALID_ARG;
        if (opts->max_workgroups < 0) return SCCL_ERR_INVALID_ARG;
        if (opts->lowering != SCCL_LOWER_AUTO && opts->lowering != SCCL_LOWER_MEMORY && opts->lowering != SCCL_LOWER_STAGED)
            return SCCL_ERR_INVALID_ARG;
        const int32_t sv = opts->slice_vectors, sth = opts->staged_threads;
        if (sv < 0 || sv > (1 << 20) || (sv & (sv - 1))) return SCCL_ERR_INVALID_ARG;
        if (!(sth == 0 || sth == 64 || sth == 128 || sth == 256 || sth == 512 || sth == 1024)) return SCCL_ERR_INVALID_ARG;
        if (opts->reserved != 0) return SCCL_ERR_INVALID_ARG;
    }
    int64_t R = 0;
    for (int32_t s = 0; s < S; s++) {
        if (sched->rounds[s] < 1) return SCCL_ERR_INVALID_ARG;
        R += sched->rounds[s];
    }

    // ---- bandwidth relation: usable links, and for every edge the constraints that cover it
    std::vector<uint8_t> mentioned((size_t)P * P, 0), blocked((size_t)P * P, 0);
    std::vector<std::vector<int32_t>> covering((size_t)P * P);
    for (int32_t i = 0; i < topo->num_bw; i++) {
        const sccl_bw_t& c = topo->bw[i];
        if (c.num_edges < 0 || c.chunks_per_round < 0 || (c.num_edges > 0 && !c.edges)) return SCCL_ERR_TOPOLOGY;
        for (int32_t j = 0; j < c.num_edges; j++) {
            const int32_t a = c.edges[j].src, b = c.edges[j].dst;
            if (a < 0 || a >= P || b < 0 || b >= P || a == b) return SCCL_ERR_TOPOLOGY;
            const size_t e = (size_t)a * P + b;
            mentioned[e] = 1;
            if (c.chunks_per_round == 0) blocked[e] = 1;
            if (covering[e].empty() || covering[e].back() != i) covering[e].push_back(i);
        }
    }

    // ---- sends: ranges, ops, links
    const int64_t N = sched->num_sends;
    for (int64_t i = 0; i < N; i++) {
        const sccl_send_t& t = sched->sends[i];
        if (t.chunk < 0 || t.chunk >= G || t.src < 0 || t.src >= P || t.dst < 0 || t.dst >= P ||
            t.step < 0 || t.step >= S || t.src == t.dst)
            return SCCL_ERR_INVALID_ARG;
        if (t.op != SCCL_COPY && t.op != SCCL_REDUCE_SUM) return SCCL_ERR_INVALID_ARG;
        if (t.op == SCCL_REDUCE_SUM && !coll->combining) return SCCL_ERR_INVALID_ARG;
    }
    // ---- layout: where rank n keeps chunk c
    const int32_t slots = coll->slot ? coll->slots_per_rank : G;
    if (slots < 1 || slots > MAX_SLOTS) return SCCL_ERR_INVALID_ARG;
    auto slot_of = [&](int32_t c, int32_t n) -> int32_t { return coll->slot ? coll->slot[(size_t)c * P + n] : c; };
    if (coll->slot) {
        std::vector<uint8_t> taken((size_t)P * slots, 0);
        for (int32_t c = 0; c < G; c++)
            for (int32_t n = 0; n < P; n++) {
                const int32_t sl = coll->slot[(size_t)c * P + n];
                if (sl < -1 || sl >= slots) return SCCL_ERR_INVALID_ARG;
                if (sl < 0) {
                    if (coll->pre[(size_t)c * P + n]) return SCCL_ERR_INVALID_ARG;
                    continue;
                }
                if (taken[(size_t)n * slots + sl]) return SCCL_ERR_INVALID_ARG;
                taken[(size_t)n * slots + sl] = 1;
            }
        for (int64_t i = 0; i < N; i++) {
            const sccl_send_t& t = sched->sends[i];
            if (slot_of(t.chunk, t.src) < 0 || slot_of(t.chunk, t.dst) < 0) return SCCL_ERR_INVALID_ARG;
        }
    }
    auto operand = [&](int32_t c, int32_t n) -> int32_t { return n | (slot_of(c, n) << OPERAND_RANK_BITS); };

    for (int64_t i = 0; i < N; i++) {
        const sccl_send_t& t = sched->sends[i];
        const size_t e = (size_t)t.src * P + t.dst;
        if (!mentioned[e] || blocked[e]) return SCCL_ERR_SEND_NO_LINK;
    }

    // ---- bucket the sends by step, keeping array order inside a step
    std::vector<int64_t> first((size_t)S + 1, 0);
    for (int64_t i = 0; i < N; i++) first[(size_t)sched->sends[i].step + 1]++;
    for (int32_t s = 0; s < S; s++) first[(size_t)s + 1] += first[s];
    std::vector<int64_t> order((size_t)N);
    {
        std::vector<int64_t> fill(first.begin(), first.end() - 1);
        for (int64_t i = 0; i < N; i++) order[(size_t)fill[sched->sends[i].step]++] = i;
    }

    // ---- the run, with contribution sets.  held[c*P+n] == 0: chunk not present (or consumed).
    const uint64_t everyone = (P == 64) ? ~0ull : ((1ull << P) - 1ull);
    std::vector<uint64_t> held((size_t)G * P, 0);
    for (int32_t c = 0; c < G; c++)
        for (int32_t n = 0; n < P; n++)
            if (coll->pre[(size_t)c * P + n]) held[(size_t)c * P + n] = coll->combining ? (1ull << n) : everyone;

    std::vector<std::vector<Group>> per_chunk((size_t)G);   // op lists in step order
    std::vector<int64_t> load(topo->num_bw > 0 ? (size_t)topo->num_bw : 1);
    std::vector<uint8_t> is_read((size_t)G * P, 0), is_written((size_t)G * P, 0);   // 1 copy-written, 2 reduced into
    int64_t n_copy_groups = 0, n_reduce_groups = 0, chunks_min = 0, chunks_unfused = 0;
    int32_t max_in = 0, max_out = 0;
    plan->step_prog.clear(); plan->group_off.clear(); plan->copy_sends.clear();
    plan->step_first.assign((size_t)S + 1, 0);

    for (int32_t s = 0; s < S; s++) {
        const int64_t lo = first[s], hi = first[(size_t)s + 1];
        // bandwidth constraint of section 3.3
        std::fill(load.begin(), load.end(), 0);
        for (int64_t q = lo; q < hi; q++) {
            const sccl_send_t& t = sched->sends[order[(size_t)q]];
            for (int32_t ci : covering[(size_t)t.src * P + t.dst]) load[(size_t)ci]++;
        }
        for (int32_t i = 0; i < topo->num_bw; i++)
            if (load[(size_t)i] > (int64_t)topo->bw[i].chunks_per_round * sched->rounds[s]) return SCCL_ERR_BANDWIDTH;
        // every value read must be present at the start of the step
        for (int64_t q = lo; q < hi; q++) {
            const sccl_send_t& t = sched->sends[order[(size_t)q]];
            if (!held[(size_t)t.chunk * P + t.src]) return SCCL_ERR_SEND_NO_SOURCE;
            if (t.op == SCCL_REDUCE_SUM && !held[(size_t)t.chunk * P + t.dst]) return SCCL_ERR_SEND_NO_SOURCE;
        }
        // hazards: with none, executing the ops one after the other equals "all reads see the start of the step"
        for (int64_t q = lo; q < hi; q++) {
            const sccl_send_t& t = sched->sends[order[(size_t)q]];
            is_read[(size_t)t.chunk * P + t.src] = 1;
        }
        sccl_status_t hazard = SCCL_OK;
        for (int64_t q = lo; q < hi && hazard == SCCL_OK; q++) {
            const sccl_send_t& t = sched->sends[order[(size_t)q]];
            const size_t d = (size_t)t.chunk * P + t.dst;
            if (is_read[d]) hazard = SCCL_ERR_HAZARD;
            else if (t.op == SCCL_COPY) {
                if (is_written[d]) hazard = SCCL_ERR_HAZARD;
                is_written[d] = 1;
            } else {
                if (is_written[d] == 1) hazard = SCCL_ERR_HAZARD;
                is_written[d] = 2;
            }
        }
        for (int64_t q = lo; q < hi; q++) {
            const sccl_send_t& t = sched->sends[order[(size_t)q]];
            is_read[(size_t)t.chunk * P + t.src] = 0;
            is_written[(size_t)t.chunk * P + t.dst] = 0;
        }
        if (hazard != SCCL_OK) return hazard;

        // apply the step to the contribution sets and form the groups
        std::vector<std::pair<size_t, uint64_t>> updates;      // deferred: all reads see the start of the step
        std::vector<size_t> consumed;
        std::map<std::pair<int32_t, size_t>, size_t> index;    // (kind, c*P + anchor) -> position in `groups`
        std::vector<Group> groups;
        std::map<size_t, uint64_t> reduced;                    // running union per reduce destination
        for (int64_t q = lo; q < hi; q++) {
            const sccl_send_t& t = sched->sends[order[(size_t)q]];
            const size_t src = (size_t)t.chunk * P + t.src, dst = (size_t)t.chunk * P + t.dst;
            if (t.op == SCCL_COPY) {
                updates.emplace_back(dst, held[src]);
                auto key = std::make_pair((int32_t)0, src);
                auto it = index.find(key);
                if (it == index.end()) {
                    index[key] = groups.size();
                    groups.push_back(Group{0, t.chunk, t.src, {t.dst}});
                } else {
                    groups[it->second].others.push_back(t.dst);
                }
                chunks_unfused += 2;
            } else {
                auto r = reduced.find(dst);
                uint64_t cur = (r == reduced.end()) ? held[dst] : r->second;
                if (cur & held[src]) return SCCL_ERR_HAZARD;   // some rank would be counted twice
                reduced[dst] = cur | held[src];
                consumed.push_back(src);
                auto key = std::make_pair((int32_t)1, dst);
                auto it = index.find(key);
                if (it == index.end()) {
                    index[key] = groups.size();
                    groups.push_back(Group{1, t.chunk, t.dst, {t.src}});
                } else {
                    groups[it->second].others.push_back(t.src);
                }
                chunks_unfused += 3;
            }
        }
        for (auto& u : updates) held[u.first] = u.second;
        for (auto& r : reduced) held[r.first] = r.second;
        for (size_t c : consumed) held[c] = 0;
        plan->step_first[(size_t)s] = (int32_t)plan->group_off.size();
        for (int64_t q = lo; q < hi; q++) {
            const sccl_send_t& t = sched->sends[order[(size_t)q]];
            if (t.op == SCCL_COPY) plan->copy_sends.push_back({t.src, slot_of(t.chunk, t.src), t.dst, slot_of(t.chunk, t.dst)});
        }
        for (Group& g : groups) {
            const int32_t k = (int32_t)g.others.size();
            plan->group_off.push_back((int32_t)plan->step_prog.size());
            plan->step_prog.push_back(g.kind | (k << 8));
            plan->step_prog.push_back(operand(g.chunk, g.anchor));
            for (int32_t o : g.others) plan->step_prog.push_back(operand(g.chunk, o));
            if (g.kind == 0) { n_copy_groups++; chunks_min += 1 + k; max_out = std::max(max_out, k); }
            else             { n_reduce_groups++; chunks_min += k + 2; max_in = std::max(max_in, k); }
            per_chunk[(size_t)g.chunk].push_back(std::move(g));
        }
    }
    plan->step_first[(size_t)S] = (int32_t)plan->group_off.size();
    for (int32_t c = 0; c < G; c++)
        for (int32_t n = 0; n < P; n++)
            if (coll->post[(size_t)c * P + n] && held[(size_t)c * P + n] != everyone) return SCCL_ERR_POSTCONDITION;

    // ---- emit the program: per chunk, its groups in step order
    plan->prog.clear();
    plan->chunk_off.assign((size_t)G + 1, 0);
    for (int32_t c = 0; c < G; c++) {
        plan->chunk_off[(size_t)c] = (int32_t)plan->prog.size();
        for (const Group& g : per_chunk[(size_t)c]) {
            plan->prog.push_back(g.kind | ((int32_t)g.others.size() << 8));
            plan->prog.push_back(operand(c, g.anchor));
            for (int32_t o : g.others) plan->prog.push_back(operand(c, o));
        }
    }
    plan->chunk_off[(size_t)G] = (int32_t)plan->prog.size();

    // ---- record the problem and the statistics
    plan->P = P; plan->G = G; plan->S = S;
    plan->dtype = dtype;
    plan->combining = coll->combining;
    plan->elems_per_chunk = coll->elems_per_chunk;
    plan->rounds.assign(sched->rounds, sched->rounds + S);
    if (opts) plan->opts = *opts;
    // sizes in bytes must fit 63 bits: the chunk, a rank buffer, and the two byte counts of the statistics
    int64_t chunk_bytes, probe;
    if (__builtin_mul_overflow(coll->elems_per_chunk, (int64_t)elem_bytes(dtype), &chunk_bytes) ||
        __builtin_mul_overflow(chunk_bytes, (int64_t)slots, &probe) ||
        __builtin_mul_overflow(chunk_bytes, chunks_min, &probe) ||
        __builtin_mul_overflow(chunk_bytes, chunks_unfused, &probe))
        return SCCL_ERR_INVALID_ARG;
    sccl_stats_t& st = plan->stats;
    st.num_nodes = P; st.num_global_chunks = G;
    st.num_steps = S; st.num_rounds = (int32_t)R; st.k = (int32_t)(R - S);
    st.num_sends = N;
    st.num_copy_groups = n_copy_groups; st.num_reduce_groups = n_reduce_groups;
    st.max_fan_in = max_in; st.max_fan_out = max_out;
    st.chunks_per_node = 0;
    for (int32_t n = 0; n < P; n++) {
        int32_t have = 0;
        for (int32_t c = 0; c < G; c++) have += coll->pre[(size_t)c * P + n] != 0;
        st.chunks_per_node = std::max(st.chunks_per_node, have);
    }
    if (st.chunks_per_node == 0) st.chunks_per_node = 1;
    st.chunk_bytes = chunk_bytes;
    st.bytes_per_rank = chunk_bytes * slots;
    st.bytes_min = chunks_min * chunk_bytes;
    st.bytes_unfused = chunks_unfused * chunk_bytes;

    // ---- launch shape: how the element range of a chunk is cut into tiles (work distribution per chunk size)
    int32_t W = 16;
    while (W > elem_bytes(dtype) && chunk_bytes % W != 0) W >>= 1;
    plan->vector_bytes = W;
    plan->vecs_per_chunk = chunk_bytes / W;
    // Work distribution, chosen per chunk size and per schedule (the analogue of choosing the
    // number of thread blocks per link, paper section 4): one workgroup per CU, and each lane keeps
    // about 16-20 vector loads in flight per op: an op with fan-in k issues k + 1 loads per
    // vector, so lanes of a fan-in-4 Allreduce take 4 vectors and lanes of a ring or a copy-only
    // schedule take 8.  Small chunks shrink the tile until every CU has a work item.
    int32_t bt = (opts && opts->block_threads) ? opts->block_threads : 256;
    int32_t vt = (opts && opts->vectors_per_thread) ? opts->vectors_per_thread : 0;
    auto items_for = [&](int32_t b, int32_t v) {
        const int64_t tile = (int64_t)b * v;
        return (int64_t)G * ((plan->vecs_per_chunk + tile - 1) / tile);
    };
    const int64_t want = (num_cus > 0 ? num_cus : 256);
    if (vt == 0) {
        const int32_t loads_per_vector = max_in + 1;
        vt = 8;
        while (vt > 1 && vt * loads_per_vector > 20) vt >>= 1;
        // A copy chain (every forwarded chunk is read back right after it was written, nothing else written in
        // between): what a workgroup wrote is still in the L2 for the next hop only while the compute units of an
        // XCD have about half a MiB of fresh writes between them, i.e. 16 KiB tiles.  Measured on ring Allgathers,
        // Gathers and Alltoalls on three topologies at 16 MiB to 256 MiB per rank: 5 to 28 % faster than 32 KiB
        // tiles, whose re-reads go to memory; with longer distances, or reductions (which read the destination
        // before they write it), the larger tile wins.
        if (st.num_reduce_groups == 0 && copy_reread_distance(*plan) == 1 && vt > 4) vt = 4;
        while (vt > 1 && items_for(bt, vt) < want) vt >>= 1;
    }
    if (!(opts && opts->block_threads))
        while (bt > 64 && items_for(bt, vt) < want) bt >>= 1;
    plan->block_threads = bt;
    plan->vectors_per_thread = vt;
    const int64_t tile = (int64_t)bt * vt;
    const int64_t tiles = (plan->vecs_per_chunk + tile - 1) / tile;
    if (tiles > 0x7fffffff) return SCCL_ERR_INVALID_ARG;
    plan->tiles_per_chunk = (int32_t)tiles;
    plan->num_items = (int64_t)G * tiles;
    st.vector_bytes = W;
    st.block_threads = bt;
    st.vectors_per_thread = vt;
    st.num_work_items = plan->num_items;
    st.grid_workgroups = 0;

    // ---- the staged lowering: tables, then the slice a workgroup stages at a time
    sccl_staged& sg = plan->staged;
    const int32_t want_lowering = opts ? opts->lowering : SCCL_LOWER_AUTO;
    if (build_staged_tables(*plan, &sg) && sg.n_out > 0 && plan->vecs_per_chunk > 0) {
        const int64_t block_bytes = (int64_t)sg.max_block_words * 4;
        const int64_t room = STAGED_LDS_LIMIT - block_bytes;                  // bytes left for the cells
        const int64_t max_slice = room > 0 ? room / ((int64_t)(sg.max_chunk_cells + 1) * W) : 0;   // vectors per storage that fit (one more: the identity)
        if (max_slice >= 1) {
            int32_t sv;
            if (opts && opts->slice_vectors) {
                sv = opts->slice_vectors;
            } else {
                // Measured best over the size sweep: single-wavefront workgroups (no barriers at all) that move
                // four vectors per lane, i.e. slices of up to 16 vectors, shortened while that leaves compute
                // units without a work item.
                sv = 16;
                while (sv > 1 && ((int64_t)G * ((plan->vecs_per_chunk + sv - 1) / sv) < want || sv / 2 >= plan->vecs_per_chunk)) sv >>= 1;
                // With no level left (copies only) a work item is one load and a row of stores per cell: longer
                // slices, up to 64 vectors, keep the number of work items down (measured on the torus Allgather at
                // 4 MiB per rank: 21.3 us with 16 vectors, 19.0 us with 64; the through-memory kernel 22.4 us).
                while (sg.staged_levels == 0 && sv < 64 && (int64_t)G * ((plan->vecs_per_chunk + sv - 1) / sv) > STAGED_AUTO_MAX_ITEMS) sv <<= 1;
                while (sv > 1 && sv > max_slice) sv >>= 1;
            }
            if (sv <= max_slice) {
                sg.available = true;
                sg.log_slice_vectors = log2_of(sv);
                sg.slices_per_chunk = (plan->vecs_per_chunk + sv - 1) / sv;
                sg.num_slices = (int64_t)G * sg.slices_per_chunk;
                sg.lds_bytes = (int32_t)(block_bytes + (int64_t)(sg.max_chunk_cells + 1) * sv * W);
                emit_staged_table(&sg, sg.log_slice_vectors, W);
                int32_t th = (opts && opts->staged_threads) ? opts->staged_threads : 64;
                sg.threads = th;
            }
        }
    }
    if (want_lowering == SCCL_LOWER_STAGED && !sg.available) return SCCL_ERR_INVALID_ARG;
    // SCCL_LOWER_AUTO, from the measured crossovers (both lowerings on twelve schedules, 64 KiB to 256 MiB in all): the
    // staged kernel never loses while launch overhead dominates (tiny totals); beyond that it wins where it saves
    // memory round trips -- the through-memory kernel pays one per group of a chunk's chain, the staged kernel one
    // per level that is left after copy propagation, so the saving is their difference (12 on the torus Allgather,
    // 18 on its Allreduce, 5 on a Broadcast tree, 7 on a ring Allreduce; 2 on two-hop schedules such as Gather or
    // Alltoall, which do not pay for it) -- and only while its single-wavefront work items stay few.
    const bool tiny = (int64_t)P * st.bytes_per_rank <= STAGED_AUTO_TINY_BYTES;
    const bool saves_round_trips = sg.max_chunk_groups - sg.staged_levels >= STAGED_AUTO_MIN_SAVING;
    const bool few_items = sg.num_slices <= STAGED_AUTO_MAX_ITEMS;
    const bool automatic = sg.available && (tiny || (saves_round_trips && few_items));
    plan->lowering = (want_lowering == SCCL_LOWER_STAGED || (want_lowering == SCCL_LOWER_AUTO && automatic))
                         ? SCCL_LOWER_STAGED : SCCL_LOWER_MEMORY;
    st.lowering = plan->lowering;
    st.staged_available = sg.available ? 1 : 0;
    st.num_cells = sg.n_cells; st.num_cells_loaded = sg.n_in; st.num_cells_stored = sg.n_out;
    st.num_levels = sg.n_levels; st.staged_levels = sg.staged_levels; st.staged_tasks = sg.n_tasks; st.max_level_tasks = sg.max_level_tasks; st.max_chunk_groups = sg.max_chunk_groups;
    st.slice_vectors = sg.available ? (1 << sg.log_slice_vectors) : 0;
    st.staged_threads = sg.threads;
    st.staged_lds_bytes = sg.lds_bytes;
    st.num_slices = sg.num_slices;

    // ---- the table as sccl_execute_static places it in the static device array
    plan->static_image.assign(plan->chunk_off.begin(), plan->chunk_off.end());
    while (plan->static_image.size() % 4) plan->static_image.push_back(0);
    plan->static_prog_off = (int32_t)plan->static_image.size();
    plan->static_image.insert(plan->static_image.end(), plan->prog.begin(), plan->prog.end());
    st.static_table_bytes = 4 * (int64_t)(plan->lowering == SCCL_LOWER_STAGED ? sg.table.size() : plan->static_image.size());
    return SCCL_OK;
}


extern "C" sccl_status_t sccl_plan_table(const sccl_plan_t* plan, int32_t lowering, int32_t* out, int64_t capacity,
                                         int64_t* out_words, int32_t info[4]) {
    if (!plan || !out_words || !info || capacity < 0 || (capacity > 0 && !out)) return SCCL_ERR_INVALID_ARG;
    const std::vector<int32_t>* table;
    if (lowering == SCCL_LOWER_MEMORY) {
        table = &plan->static_image;
        info[0] = plan->static_prog_off; info[1] = info[2] = info[3] = 0;
    } else if (lowering == SCCL_LOWER_STAGED && plan->staged.available) {
        const sccl_staged& sg = plan->staged;
        table = &sg.table;
        info[0] = sg.max_block_words; info[1] = sg.cell_words_room; info[2] = sg.log_slice_vectors;
        info[3] = (int32_t)(((int64_t)sg.max_chunk_cells << sg.log_slice_vectors) * plan->vector_bytes);
    } else {
        return SCCL_ERR_INVALID_ARG;
    }
    *out_words = (int64_t)table->size();
    const int64_t n = std::min<int64_t>(capacity, (int64_t)table->size());
    if (n > 0) std::memcpy(out, table->data(), (size_t)n * sizeof(int32_t));
    return SCCL_OK;
}
