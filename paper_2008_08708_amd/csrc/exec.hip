// Device side of the library: the gfx950 executor kernel, plan upload and the C entry points.
//
// How a schedule is executed (paper, section 4: all steps fused into ONE kernel, a chunk
// being usable as soon as the send that produces it is done -- there with a flag per
// chunk and connection, no global barrier between steps):
//
//   * Every rank buffer holds chunk c at one fixed position (by default the same offset in
//     every buffer), and two chunks never share a position on a rank, so the sends of different
//     chunks touch disjoint memory, and sends of one chunk act element by element.  The
//     only order the schedule imposes is therefore, per chunk and per element, the
//     order of that chunk's sends by step.
//   * The element range of a chunk is cut into tiles; a work item is (chunk, tile).  A
//     workgroup takes a work item and walks the chunk's whole op list, step by step.
//     Lane t of the workgroup touches the SAME element positions in every op, so every
//     value a lane reads in step s+1 was written by that same lane in step s: the
//     inter-step dependency is plain program order of one thread.  No flags, no
//     barrier, no cross-workgroup visibility is needed, and the result is bit-identical
//     to the synchronous execution because each element sees the same operations in
//     the same order.
//   * One op = one copy group (load once, store to every destination) or one reduce
//     group (load destination and all sources, add left to right in fp32 / wrapping
//     int32, store once).  All loads of an op are issued before the first use.
//   * Values travel through memory between steps (L2 / memory-side cache absorb most
//     of the re-reads because a lane re-reads what it just wrote); nothing is kept in
//     registers across ops.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>

#include "plan.hpp"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int W> struct VecOf;
template <> struct VecOf<16> { typedef u32x4 type; };
template <> struct VecOf<8>  { typedef u32x2 type; };
template <> struct VecOf<4>  { typedef uint32_t type; };
template <> struct VecOf<2>  { typedef uint16_t type; };

// The step table is written once at plan creation and never by a kernel: reading it through
// the constant address space lets the compiler use scalar loads (one fetch per wavefront,
// not ordered against the data loads' counter).
typedef const int32_t __attribute__((address_space(4)))* table_ptr;

struct ExecArgs {
    const int32_t* prog;
    const int32_t* chunk_off;
    int64_t chunk_bytes;
    int64_t num_items;
    int32_t tiles_per_chunk;
    int32_t pad;
    char* bufs[SCCL_MAX_RANKS];
};

// ---- memory access through buffer descriptors.
// A descriptor covers exactly one tile of one rank's chunk (base = start of the tile, size = the
// bytes of the tile that exist), so (1) the hardware's range check drops the lanes beyond a ragged
// chunk end -- loads return 0, stores are discarded -- and no lane predicate is needed, (2) lane
// offsets are small 32-bit numbers however large the buffers are, and addresses live in scalar
// registers, which keeps the vector register count low.  All accesses use the default cache
// policy: non-temporal loads and stores for data that is touched once were measured and lose
// (they also evict what the next step re-reads).

__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(char* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}

struct Tile;
// Descriptor of one operand (rank | slot << 8) on the current tile.
template <class Args>
__device__ __forceinline__ __amdgpu_buffer_rsrc_t operand_rsrc(const Args& a, int32_t w, const Tile& t);

template <int W> struct BufIO;
template <> struct BufIO<16> {
    static __device__ __forceinline__ u32x4 ld(__amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        auto x = __builtin_amdgcn_raw_buffer_load_b128(r, (int)v, (int)s, 0); u32x4 o; __builtin_memcpy(&o, &x, 16); return o; }
    static __device__ __forceinline__ void st(u32x4 d, __amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        decltype(__builtin_amdgcn_raw_buffer_load_b128(r, 0, 0, 0)) x; __builtin_memcpy(&x, &d, 16);
        __builtin_amdgcn_raw_buffer_store_b128(x, r, (int)v, (int)s, 0); }
};
template <> struct BufIO<8> {
    static __device__ __forceinline__ u32x2 ld(__amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        auto x = __builtin_amdgcn_raw_buffer_load_b64(r, (int)v, (int)s, 0); u32x2 o; __builtin_memcpy(&o, &x, 8); return o; }
    static __device__ __forceinline__ void st(u32x2 d, __amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        decltype(__builtin_amdgcn_raw_buffer_load_b64(r, 0, 0, 0)) x; __builtin_memcpy(&x, &d, 8);
        __builtin_amdgcn_raw_buffer_store_b64(x, r, (int)v, (int)s, 0); }
};
template <> struct BufIO<4> {
    static __device__ __forceinline__ uint32_t ld(__amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        return (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(r, (int)v, (int)s, 0); }
    static __device__ __forceinline__ void st(uint32_t d, __amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        __builtin_amdgcn_raw_buffer_store_b32(d, r, (int)v, (int)s, 0); }
};
template <> struct BufIO<2> {
    static __device__ __forceinline__ uint16_t ld(__amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        return (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)v, (int)s, 0); }
    static __device__ __forceinline__ void st(uint16_t d, __amdgpu_buffer_rsrc_t r, uint32_t v, uint32_t s) {
        __builtin_amdgcn_raw_buffer_store_b16(d, r, (int)v, (int)s, 0); }
};

// U vectors per lane, `ustride` bytes apart (one workgroup-wide row each): coalesced rows.
template <int W, int U>
__device__ __forceinline__ void load_rows(typename VecOf<W>::type (&x)[U], __amdgpu_buffer_rsrc_t r,
                                          uint32_t lane_off, uint32_t ustride) {
#pragma unroll
    for (int u = 0; u < U; u++) x[u] = BufIO<W>::ld(r, lane_off, u * ustride);
}
template <int W, int U>
__device__ __forceinline__ void store_rows(const typename VecOf<W>::type (&x)[U], __amdgpu_buffer_rsrc_t r,
                                           uint32_t lane_off, uint32_t ustride) {
#pragma unroll
    for (int u = 0; u < U; u++) BufIO<W>::st(x[u], r, lane_off, u * ustride);
}

// ---- accumulators: how one vector of W bytes is widened, summed and narrowed per dtype
template <int DT, int W> struct Acc;

template <int W> struct Acc<SCCL_I32, W> {           // wrapping sum modulo 2^32
    static constexpr int N = W / 4;
    uint32_t a[N];
    template <typename V> __device__ __forceinline__ void init(V v) { __builtin_memcpy(a, &v, W); }
    template <typename V> __device__ __forceinline__ void add(V v) {
        uint32_t x[N]; __builtin_memcpy(x, &v, W);
#pragma unroll
        for (int i = 0; i < N; i++) a[i] += x[i];
    }
    template <typename V> __device__ __forceinline__ V done() { V v; __builtin_memcpy(&v, a, W); return v; }
};

template <int W> struct Acc<SCCL_F32, W> {           // binary32 add, round to nearest even
    static constexpr int N = W / 4;
    float a[N];
    template <typename V> __device__ __forceinline__ void init(V v) { __builtin_memcpy(a, &v, W); }
    template <typename V> __device__ __forceinline__ void add(V v) {
        float x[N]; __builtin_memcpy(x, &v, W);
#pragma unroll
        for (int i = 0; i < N; i++) a[i] = a[i] + x[i];
    }
    template <typename V> __device__ __forceinline__ V done() { V v; __builtin_memcpy(&v, a, W); return v; }
};

template <int W> struct Acc<SCCL_F16, W> {           // binary16 in memory, binary32 sum, one RNE narrowing
    static constexpr int N = W / 2;
    float a[N];
    template <typename V> __device__ __forceinline__ void init(V v) {
        _Float16 h[N]; __builtin_memcpy(h, &v, W);
#pragma unroll
        for (int i = 0; i < N; i++) a[i] = (float)h[i];
    }
    template <typename V> __device__ __forceinline__ void add(V v) {
        _Float16 h[N]; __builtin_memcpy(h, &v, W);
#pragma unroll
        for (int i = 0; i < N; i++) a[i] = a[i] + (float)h[i];
    }
    template <typename V> __device__ __forceinline__ V done() {
        _Float16 h[N];
#pragma unroll
        for (int i = 0; i < N; i++) h[i] = (_Float16)a[i];     // default rounding mode: nearest even
        V v; __builtin_memcpy(&v, h, W); return v;
    }
};

// What every op of one work item shares.
struct Tile {
    int64_t chunk_bytes;
    int64_t in_chunk;        // byte offset of the tile inside its chunk
    uint32_t bytes;          // bytes of the tile that exist (the last tile of a chunk may be short)
    uint32_t lane_off;       // this lane's byte offset in a row
    uint32_t ustride;        // bytes per row
};

template <class Args>
__device__ __forceinline__ __amdgpu_buffer_rsrc_t operand_rsrc(const Args& a, int32_t w, const Tile& t) {
    char* base = a.bufs[w & OPERAND_RANK_MASK] + (int64_t)(w >> OPERAND_RANK_BITS) * t.chunk_bytes + t.in_chunk;
    return tile_rsrc(base, t.bytes);
}

// NS sources of a reduce group (NS is a compile-time batch size): all scalar work (operand words,
// pointers, descriptors) first, then every load back to back, then the adds in order.  In the
// FIRST batch the accumulators start from the destination's value d0, whose load was issued just
// before this batch's loads, so all of them are in flight together.
template <int DT, int W, int U, int NS, bool FIRST, class Args>
__device__ __forceinline__ void reduce_batch(Acc<DT, W> (&acc)[U], const typename VecOf<W>::type (&d0)[U],
                                             const Args& a, table_ptr srcs, const Tile& t) {
    typedef typename VecOf<W>::type V;
    V x[NS][U];
    __amdgpu_buffer_rsrc_t r[NS];
#pragma unroll
    for (int j = 0; j < NS; j++) r[j] = operand_rsrc(a, srcs[j], t);
#pragma unroll
    for (int j = 0; j < NS; j++) load_rows<W, U>(x[j], r[j], t.lane_off, t.ustride);
    if (FIRST) {
#pragma unroll
        for (int u = 0; u < U; u++) acc[u].init(d0[u]);
    }
#pragma unroll
    for (int j = 0; j < NS; j++)
#pragma unroll
        for (int u = 0; u < U; u++) acc[u].add(x[j][u]);
}

template <int DT, int W, int U, bool FIRST, class Args>
__device__ __forceinline__ void reduce_some(int32_t n, Acc<DT, W> (&acc)[U], const typename VecOf<W>::type (&d0)[U],
                                            const Args& a, table_ptr srcs, const Tile& t) {
    switch (n) {
        case 4:  reduce_batch<DT, W, U, 4, FIRST>(acc, d0, a, srcs, t); break;
        case 3:  reduce_batch<DT, W, U, 3, FIRST>(acc, d0, a, srcs, t); break;
        case 2:  reduce_batch<DT, W, U, 2, FIRST>(acc, d0, a, srcs, t); break;
        default: reduce_batch<DT, W, U, 1, FIRST>(acc, d0, a, srcs, t); break;
    }
}

// One op on one tile: op points at  header | anchor rank | other ranks...  ; returns the word count.
template <int DT, int W, int U, class Args>
__device__ __forceinline__ int32_t do_op(const Args& a, table_ptr op, const Tile& t) {
    typedef typename VecOf<W>::type V;
    const int32_t hdr = op[0];
    const int32_t k = hdr >> 8;
    if ((hdr & OP_KIND_REDUCE) == 0) {
        // copy group: one read, k writes
        const int32_t ws = op[1];
        V x[U];
        load_rows<W, U>(x, operand_rsrc(a, ws, t), t.lane_off, t.ustride);
        for (int32_t d = 0; d < k; d++) {
            const int32_t wd = op[2 + d];
            store_rows<W, U>(x, operand_rsrc(a, wd, t), t.lane_off, t.ustride);
        }
    } else {
        // reduce group: destination first, then the k sources in schedule order
        const int32_t wd = op[1];
        const __amdgpu_buffer_rsrc_t rd = operand_rsrc(a, wd, t);
        Acc<DT, W> acc[U];
        V d0[U];
        load_rows<W, U>(d0, rd, t.lane_off, t.ustride);
        table_ptr srcs = op + 2;
        int32_t left = k;                                  // k >= 1
        int32_t n = left < 4 ? left : 4;
        reduce_some<DT, W, U, true>(n, acc, d0, a, srcs, t);
        srcs += n; left -= n;
        while (left > 0) {                                 // fan-in above 4: further batches, still in order
            n = left < 4 ? left : 4;
            reduce_some<DT, W, U, false>(n, acc, d0, a, srcs, t);
            srcs += n; left -= n;
        }
        V out[U];
#pragma unroll
        for (int u = 0; u < U; u++) out[u] = acc[u].template done<V>();
        store_rows<W, U>(out, rd, t.lane_off, t.ustride);
    }
    return 2 + k;
}

// Persistent kernel: workgroup b takes work items b, b + grid, ... ; a work item is (chunk, tile).
template <int DT, int W, int U>
__global__ void __launch_bounds__(256) sccl_exec_kernel(const ExecArgs a) {
    const uint32_t tile_bytes = blockDim.x * U * W;
    Tile t;
    t.lane_off = threadIdx.x * W;
    t.ustride = blockDim.x * W;
    t.chunk_bytes = a.chunk_bytes;
    table_ptr offs = (table_ptr)a.chunk_off;
    for (int64_t item = blockIdx.x; item < a.num_items; item += gridDim.x) {
        const int32_t c = (int32_t)(item / a.tiles_per_chunk);
        const int32_t tile = (int32_t)(item - (int64_t)c * a.tiles_per_chunk);
        const int64_t in_chunk = (int64_t)tile * tile_bytes;
        const int64_t rest = a.chunk_bytes - in_chunk;
        t.in_chunk = in_chunk;
        t.bytes = rest < (int64_t)tile_bytes ? (uint32_t)rest : tile_bytes;
        table_ptr op = (table_ptr)a.prog + offs[c];
        table_ptr end = (table_ptr)a.prog + offs[c + 1];
        while (op < end) op += do_op<DT, W, U>(a, op, t);
    }
}

// The step-per-launch lowering (paper section 4, "multiple kernels, one per step"): one launch
// executes the groups of ONE step; a work item is (group, tile).  The kernel boundary is the
// global synchronisation between steps.  Kept as a comparator for the fused kernel above.
struct StepArgs {
    const int32_t* step_prog;     // per group: header | anchor | others...
    const int32_t* group_off;     // word offset of every group, in step order
    int64_t chunk_bytes;
    int64_t num_items;            // groups of this step x tiles per chunk
    int32_t first_group;          // index into group_off of this step's first group
    int32_t tiles_per_chunk;
    char* bufs[SCCL_MAX_RANKS];
};

template <int DT, int W, int U>
__global__ void __launch_bounds__(256) sccl_step_kernel(const StepArgs a) {
    const uint32_t tile_bytes = blockDim.x * U * W;
    Tile t;
    t.lane_off = threadIdx.x * W;
    t.ustride = blockDim.x * W;
    t.chunk_bytes = a.chunk_bytes;
    table_ptr goff = (table_ptr)a.group_off;
    for (int64_t item = blockIdx.x; item < a.num_items; item += gridDim.x) {
        const int32_t g = (int32_t)(item / a.tiles_per_chunk);
        const int32_t tile = (int32_t)(item - (int64_t)g * a.tiles_per_chunk);
        table_ptr op = (table_ptr)a.step_prog + goff[a.first_group + g];
        const int64_t in_chunk = (int64_t)tile * tile_bytes;
        const int64_t rest = a.chunk_bytes - in_chunk;
        t.in_chunk = in_chunk;
        t.bytes = rest < (int64_t)tile_bytes ? (uint32_t)rest : tile_bytes;
        do_op<DT, W, U>(a, op, t);
    }
}


// ---- the staged lowering -----------------------------------------------------------------------
// A work item is (chunk, slice): `slice` consecutive vectors of the chunk, in every rank buffer that holds
// it.  The workgroup (1) loads the slice of every cell of the chunk that the schedule reads before writing
// into the local data share, all loads in flight together: one memory round trip; (2) runs the chunk's
// sends there, one dependency level after the other, one lane per (cell write, vector), with a workgroup
// barrier between levels (nothing but program order when the workgroup is a single wavefront); (3) stores
// the slice of every cell the schedule wrote.  Per element the operations and their order are those of the
// schedule, so the bits equal the other lowerings'.  A chunk's chain of sends costs local-memory latency
// per level instead of a cache round trip per group, which is what small buffers are bound by.
// The plan compiler has already propagated copies (a cell that only receives a copy of a value that stays put is
// stored straight from the storage holding that value: plan.cpp), so the levels that arrive here are the reduce
// groups and the few copies that could not be propagated; a non-combining collective arrives with none.
struct StagedArgs {
    const int32_t* table;         // one block per chunk, see plan.hpp
    int64_t chunk_bytes;
    int64_t num_items;            // chunks x slices per chunk
    int64_t vecs_per_chunk;
    int64_t slices_per_chunk;
    int32_t log_slice;            // vectors per slice = 1 << log_slice
    int32_t block_words;          // stride of the chunk blocks, in words (a multiple of 4)
    int32_t cell_words_room;      // words reserved for cell words in every block
    uint32_t identity_off;        // byte offset of the identity storage in a workgroup's cell area
    char* bufs[SCCL_MAX_RANKS];
};

// Base pointer of rank `rank` (any value per lane) out of the wavefront's copy: lane n holds bufs[n].
__device__ __forceinline__ char* rank_base(uint32_t lo, uint32_t hi, int32_t rank) {
    const uint32_t l = (uint32_t)__shfl((int)lo, rank, 64), h = (uint32_t)__shfl((int)hi, rank, 64);
    return (char*)(((uint64_t)h << 32) | l);
}

// Offsets of the parts of one chunk's block inside the local copy, and their sizes.
struct StagedBlock { int32_t n_in, n_out, n_levels, off_out, off_lev, off_task, off_extra; };

// One task record as a lane holds it: destination byte offset | fan-in << 24, overflow index, four source byte offsets.
struct StagedTask { int32_t w0, w1, s[4]; };

// The record of the task lane slot i runs in the level [t_lo, t_hi): task t_lo + (i >> ls), vector i & (slice - 1).
// Slots beyond the level fetch the level's last record instead (valid memory, same code path) and return false.
__device__ __forceinline__ bool fetch_task(StagedTask& t, const int32_t* tab, const StagedBlock& b,
                                           int32_t t_lo, int32_t t_hi, int32_t i, int32_t ls) {
    const int32_t task = t_lo + (i >> ls);
    const int32_t last = t_hi > 0 ? t_hi - 1 : 0;
    const int32_t rd = task < t_hi ? task : last;
    const u32x4* rec = (const u32x4*)(tab + b.off_task + STAGED_TASK_WORDS * rd);     // 16-byte aligned
    const u32x4 lo = rec[0];
    const u32x2 hi = *(const u32x2*)(rec + 1);
    t.w0 = (int32_t)lo.x; t.w1 = (int32_t)lo.y; t.s[0] = (int32_t)lo.z; t.s[1] = (int32_t)lo.w;
    t.s[2] = (int32_t)hi.x; t.s[3] = (int32_t)hi.y;
    return task < t_hi;
}

// What the identity storage holds: adding it changes no bit of any sum (-0.0 for the floating types: x + (-0.0) is x
// for every x, signed zeros and denormals included, in binary32, where binary16 operands are summed too; 0 for int32).
template <int DT, int W>
__device__ __forceinline__ typename VecOf<W>::type identity_vector() {
    typedef typename VecOf<W>::type V;
    uint32_t word = DT == SCCL_F32 ? 0x80000000u : DT == SCCL_F16 ? 0x80008000u : 0u;
    uint32_t w4[4] = {word, word, word, word};
    V v; __builtin_memcpy(&v, w4, W); return v;
}

// One task on one vector, the same instructions whatever the fan-in: the destination's own value first, then four
// sources in schedule order (unused slots name the identity storage), then any further sources; a copy (fan-in 0)
// takes the bits of its source instead of the sum.  `voff` is the byte offset of the lane's vector in a slice.
template <int DT, int W>
__device__ __forceinline__ void run_task(char* cells, const int32_t* tab, const StagedBlock& b,
                                         const StagedTask& t, bool active, uint32_t voff) {
    typedef typename VecOf<W>::type V;
    const int32_t k = t.w0 >> STAGED_TASK_K_SHIFT;
    const uint32_t dst = (uint32_t)(t.w0 & ((1 << STAGED_TASK_K_SHIFT) - 1)) + voff;
    const V d = *(const V*)(cells + dst);
    V x[4];
#pragma unroll
    for (int j = 0; j < 4; j++) x[j] = *(const V*)(cells + (uint32_t)t.s[j] + voff);
    Acc<DT, W> acc;
    acc.init(d);
#pragma unroll
    for (int j = 0; j < 4; j++) acc.add(x[j]);
    for (int32_t j = 4; j < k; j++) acc.add(*(const V*)(cells + (uint32_t)tab[b.off_extra + t.w1 + j - 4] + voff));
    V out = acc.template done<V>();
    if (k == 0) out = x[0];
    if (active) *(V*)(cells + dst) = out;
}

// First task of level l (any l >= 0; beyond the last level: the end) out of the wavefront's copy of the
// level table: lane n holds entries n, n + 64, n + 128, n + 192.  l is the same in every lane.
__device__ __forceinline__ int32_t level_first(const int32_t (&reg)[4], int32_t l, int32_t n_levels) {
    l = l < n_levels ? l : n_levels;
    const int32_t q = l >> 6;
    const int32_t r = q == 0 ? reg[0] : q == 1 ? reg[1] : q == 2 ? reg[2] : reg[3];
    return __builtin_amdgcn_readlane(r, l & 63);
}

// Orders this workgroup's local-memory accesses before and after: a barrier, or for a single wavefront
// (whose local-memory operations execute in program order) only a fence for the compiler.
__device__ __forceinline__ void staged_sync(bool one_wave) {
    if (one_wave) __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    else __syncthreads();
}

template <int DT, int W>
__global__ void __launch_bounds__(1024) sccl_staged_kernel(const StagedArgs a) {
    typedef typename VecOf<W>::type V;
    extern __shared__ __attribute__((aligned(16))) unsigned char staged_lds[];
    const int32_t* tab = (const int32_t*)staged_lds;               // the chunk's block
    V* cells = (V*)(staged_lds + (size_t)a.block_words * 4);
    char* cell_bytes = (char*)cells;
    const int32_t tid = (int32_t)threadIdx.x, BT = (int32_t)blockDim.x;
    const bool one_wave = BT <= 64;
    const int32_t ls = a.log_slice, sv = 1 << ls, vmask = sv - 1;

    // lane n of every wavefront keeps the base pointer of rank n (P <= 64 = lanes of a wavefront)
    const uint64_t mine = (uint64_t)a.bufs[tid & 63];
    const uint32_t base_lo = (uint32_t)mine, base_hi = (uint32_t)(mine >> 32);

    constexpr int UA = 4;                                          // loads a lane keeps in flight in phase 1
    for (int64_t item = blockIdx.x; item < a.num_items; item += gridDim.x) {
        const int32_t c = (int32_t)(item / a.slices_per_chunk);
        const int64_t slice = item - (int64_t)c * a.slices_per_chunk;
        const int64_t v0 = slice << ls;
        const int64_t left = a.vecs_per_chunk - v0;
        const int32_t here = left < sv ? (int32_t)left : sv;       // vectors of this slice that exist
        const int64_t slice_off = v0 * W;
        const bool live = (tid & vmask) < here;                    // this lane's vector exists in this slice

        // Everything this item needs first is fetched in ONE round trip, because where it sits does not depend
        // on the header: the header itself (scalar), the level table into registers, the operand words of the
        // cells to load, and the whole block into the local data share.
        const int32_t* gblock = a.table + (int64_t)c * a.block_words;
        table_ptr h = (table_ptr)gblock;
        const int32_t n_tasks = h[4];
        StagedBlock b;
        b.n_in = h[1]; b.n_out = h[2]; b.n_levels = h[3];
        b.off_lev = STAGED_HEADER_WORDS + a.cell_words_room;
        b.off_out = b.off_lev + b.n_levels + 2;
        b.off_task = (b.off_out + 2 * b.n_out + 3) & ~3;
        b.off_extra = b.off_task + STAGED_TASK_WORDS * n_tasks;
        int32_t levreg[4];                                         // entries past the table are never used
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const int32_t l = STAGED_HEADER_WORDS + a.cell_words_room + (tid & 63) + 64 * q;
            levreg[q] = l < a.block_words ? gblock[l] : 0;
        }
        int32_t w0[UA];                                            // operand words of the first cells this lane loads
#pragma unroll
        for (int u = 0; u < UA; u++) {
            const int32_t i = u * BT + tid;
            w0[u] = (i >> ls) < a.cell_words_room ? gblock[STAGED_HEADER_WORDS + (i >> ls)] : 0;
        }
        {   // the block goes to the local data share, 16 bytes per lane and trip
            const u32x4* src = (const u32x4*)gblock;
            u32x4* dst = (u32x4*)staged_lds;
            for (int32_t i = tid; i < a.block_words / 4; i += BT) dst[i] = src[i];
        }
        if (b.n_levels > 0)                                        // the identity storage, one slice long
            for (int32_t i = tid; i < sv; i += BT) *(V*)(cell_bytes + a.identity_off + (uint32_t)i * W) = identity_vector<DT, W>();

        // ---- (1) load: cell i < n_in is the i-th loaded cell; its operand word comes straight from memory
        const int32_t in_lanes = b.n_in << ls, out_lanes = b.n_out << ls;
        for (int32_t base = 0; base < in_lanes; base += BT * UA) {
            int32_t w[UA]; bool ok[UA]; V x[UA];
#pragma unroll
            for (int u = 0; u < UA; u++) {
                const int32_t i = base + u * BT + tid;
                w[u] = base == 0 ? w0[u] : ((i >> ls) < a.cell_words_room ? gblock[STAGED_HEADER_WORDS + (i >> ls)] : 0);
            }
#pragma unroll
            for (int u = 0; u < UA; u++) {
                const int32_t i = base + u * BT + tid;
                ok[u] = i < in_lanes && (i & vmask) < here;
            }
#pragma unroll
            for (int u = 0; u < UA; u++) {
                const int32_t i = base + u * BT + tid;
                char* p = rank_base(base_lo, base_hi, w[u] & OPERAND_RANK_MASK) +
                          (int64_t)(w[u] >> OPERAND_RANK_BITS) * a.chunk_bytes + slice_off + (int64_t)(i & vmask) * W;
                if (ok[u]) x[u] = *(const V*)p;
            }
#pragma unroll
            for (int u = 0; u < UA; u++) {
                const int32_t i = base + u * BT + tid;
                if (ok[u]) cells[i] = x[u];                        // cell (i >> ls), vector (i & vmask)
            }
        }
        staged_sync(one_wave);

        // ---- (2) the schedule, level by level.  The block is read-only, so a lane fetches its task record of
        // the NEXT level together with the cells of the current one: one local-memory round trip per level.
        // The first cell this lane stores in phase 3, (cell id, operand word), is fetched here too.
        const bool ok0 = tid < out_lanes && live;
        const int32_t out_c0 = ok0 ? tab[b.off_out + 2 * (tid >> ls)] : 0;
        const int32_t out_w0 = ok0 ? tab[b.off_out + 2 * (tid >> ls) + 1] : 0;
        int32_t lo0 = level_first(levreg, 0, b.n_levels), lo1 = level_first(levreg, 1, b.n_levels);
        const uint32_t voff = (uint32_t)(tid & vmask) * W;
        StagedTask cur;
        bool cur_on = false;
        if (b.n_levels > 0) cur_on = fetch_task(cur, tab, b, lo0, lo1, tid, ls);
        for (int32_t lv = 0; lv < b.n_levels; lv++) {
            const int32_t lo2 = level_first(levreg, lv + 2, b.n_levels);
            StagedTask nxt;
            const bool nxt_on = fetch_task(nxt, tab, b, lo1, lo2, tid, ls);
            run_task<DT, W>(cell_bytes, tab, b, cur, cur_on, voff);
            const int32_t lanes = (lo1 - lo0) << ls;
            for (int32_t i = tid + BT; i < lanes; i += BT) {       // levels wider than the workgroup
                StagedTask t;
                const bool on = fetch_task(t, tab, b, lo0, lo1, i, ls);
                run_task<DT, W>(cell_bytes, tab, b, t, on, (uint32_t)(i & vmask) * W);
            }
            cur = nxt; cur_on = nxt_on;
            staged_sync(one_wave);
            lo0 = lo1; lo1 = lo2;
        }

        // ---- (3) store every cell the schedule wrote
        for (int32_t base = 0; base < out_lanes; base += BT) {
            const int32_t i = base + tid;
            const bool ok = i < out_lanes && (i & vmask) < here;
            const int32_t oc = base == 0 ? out_c0 : (ok ? tab[b.off_out + 2 * (i >> ls)] : 0);
            const int32_t ow = base == 0 ? out_w0 : (ok ? tab[b.off_out + 2 * (i >> ls) + 1] : 0);
            char* p = rank_base(base_lo, base_hi, ow & OPERAND_RANK_MASK) +
                      (int64_t)(ow >> OPERAND_RANK_BITS) * a.chunk_bytes + slice_off + (int64_t)(i & vmask) * W;
            if (ok) *(V*)p = *(const V*)(cell_bytes + (uint32_t)oc + (uint32_t)(i & vmask) * W);
        }
        if (item + gridDim.x < a.num_items) staged_sync(one_wave); // the next item overwrites the block and the cells
    }
}

typedef void (*staged_fn)(const StagedArgs);
template <int DT>
staged_fn pick_staged_w(int W) {
    switch (W) {
        case 16: return sccl_staged_kernel<DT, 16>;
        case 8:  return sccl_staged_kernel<DT, 8>;
        default: return sccl_staged_kernel<DT, 4>;
    }
}
staged_fn pick_staged_kernel(sccl_dtype_t dt, int W) {
    switch (dt) {
        case SCCL_I32: return pick_staged_w<SCCL_I32>(W);
        case SCCL_F32: return pick_staged_w<SCCL_F32>(W);
        default:
            if (W == 2) return sccl_staged_kernel<SCCL_F16, 2>;
            return pick_staged_w<SCCL_F16>(W);
    }
}

typedef void (*kernel_fn)(const ExecArgs);
typedef void (*step_kernel_fn)(const StepArgs);

template <int DT, int W>
step_kernel_fn pick_step_u(int U) {
    switch (U) {
        case 1: return sccl_step_kernel<DT, W, 1>;
        case 2: return sccl_step_kernel<DT, W, 2>;
        case 4: return sccl_step_kernel<DT, W, 4>;
        default: return sccl_step_kernel<DT, W, 8>;
    }
}
template <int DT>
step_kernel_fn pick_step_w(int W, int U) {
    switch (W) {
        case 16: return pick_step_u<DT, 16>(U);
        case 8:  return pick_step_u<DT, 8>(U);
        default: return pick_step_u<DT, 4>(U);
    }
}
step_kernel_fn pick_step_kernel(sccl_dtype_t dt, int W, int U) {
    switch (dt) {
        case SCCL_I32: return pick_step_w<SCCL_I32>(W, U);
        case SCCL_F32: return pick_step_w<SCCL_F32>(W, U);
        default:
            if (W == 2) return pick_step_u<SCCL_F16, 2>(U);
            return pick_step_w<SCCL_F16>(W, U);
    }
}

template <int DT, int W>
kernel_fn pick_u(int U) {
    switch (U) {
        case 1: return sccl_exec_kernel<DT, W, 1>;
        case 2: return sccl_exec_kernel<DT, W, 2>;
        case 4: return sccl_exec_kernel<DT, W, 4>;
        default: return sccl_exec_kernel<DT, W, 8>;
    }
}

template <int DT>
kernel_fn pick_w(int W, int U) {
    switch (W) {
        case 16: return pick_u<DT, 16>(U);
        case 8:  return pick_u<DT, 8>(U);
        default: return pick_u<DT, 4>(U);
    }
}

kernel_fn pick_kernel(sccl_dtype_t dt, int W, int U) {
    switch (dt) {
        case SCCL_I32: return pick_w<SCCL_I32>(W, U);
        case SCCL_F32: return pick_w<SCCL_F32>(W, U);
        default:
            if (W == 2) return pick_u<SCCL_F16, 2>(U);
            return pick_w<SCCL_F16>(W, U);
    }
}

}  // namespace

extern "C" {

sccl_status_t sccl_plan_create_ex(const sccl_topology_t* topology, const sccl_collective_t* collective,
                                  const sccl_schedule_t* schedule, const sccl_options_t* options,
                                  sccl_plan_t** out_plan) {
    if (!out_plan) return SCCL_ERR_INVALID_ARG;
    *out_plan = nullptr;
    sccl_plan* plan = new (std::nothrow) sccl_plan();
    if (!plan) return SCCL_ERR_NOMEM;
    const bool host_only = options && (options->flags & SCCL_PLAN_HOST_ONLY);
    int num_cus = 256;
    int dev = -1;
    sccl_status_t st = SCCL_OK;
    try {
        if (!host_only) {
            hipDeviceProp_t prop;
            if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
                delete plan;
                return SCCL_ERR_DEVICE;
            }
            num_cus = prop.multiProcessorCount;
        }
        st = sccl_compile_host(topology, collective, schedule, options, num_cus, plan);
    } catch (const std::bad_alloc&) {
        st = SCCL_ERR_NOMEM;
    }
    if (st != SCCL_OK) { delete plan; return st; }
    static std::atomic<uint64_t> next_plan_id{1};
    plan->id = next_plan_id.fetch_add(1, std::memory_order_relaxed);
    if (!host_only) {
        plan->device = dev;
        plan->num_cus = num_cus;
        const size_t pb = plan->prog.size() * sizeof(int32_t), ob = plan->chunk_off.size() * sizeof(int32_t);
        const size_t sb = plan->step_prog.size() * sizeof(int32_t), gb = plan->group_off.size() * sizeof(int32_t);
        bool good = hipMalloc((void**)&plan->d_step_prog, sb ? sb : 4) == hipSuccess &&
                    hipMalloc((void**)&plan->d_group_off, gb ? gb : 4) == hipSuccess &&
                    (sb == 0 || hipMemcpy(plan->d_step_prog, plan->step_prog.data(), sb, hipMemcpyHostToDevice) == hipSuccess) &&
                    (gb == 0 || hipMemcpy(plan->d_group_off, plan->group_off.data(), gb, hipMemcpyHostToDevice) == hipSuccess) &&
                    hipMalloc((void**)&plan->d_prog, pb ? pb : 4) == hipSuccess &&
                    hipMalloc((void**)&plan->d_chunk_off, ob) == hipSuccess &&
                    (pb == 0 || hipMemcpy(plan->d_prog, plan->prog.data(), pb, hipMemcpyHostToDevice) == hipSuccess) &&
                    hipMemcpy(plan->d_chunk_off, plan->chunk_off.data(), ob, hipMemcpyHostToDevice) == hipSuccess;
        if (!good) { sccl_plan_destroy(plan); return SCCL_ERR_DEVICE; }
        sccl_staged& sg = plan->staged;
        if (sg.available) {
            staged_fn sfn = pick_staged_kernel(plan->dtype, plan->vector_bytes);
            // More than 64 KiB of dynamic local data share has to be asked for, per kernel.  If the runtime
            // refuses, plans that need more cannot be staged: they fall back to the through-memory kernel
            // unless the caller demanded the staged one.
            if (sg.lds_bytes > 64 * 1024 &&
                hipFuncSetAttribute((const void*)sfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)STAGED_LDS_LIMIT) != hipSuccess) {
                (void)hipGetLastError();
                if (plan->opts.lowering == SCCL_LOWER_STAGED) { sccl_plan_destroy(plan); return SCCL_ERR_DEVICE; }
                sg.available = false;
                plan->lowering = SCCL_LOWER_MEMORY;
                plan->stats.lowering = SCCL_LOWER_MEMORY;
                plan->stats.staged_available = 0;
            }
        }
        if (sg.available) {
            const size_t tb = sg.table.size() * sizeof(int32_t);
            const bool staged_ok = hipMalloc((void**)&plan->d_staged, tb) == hipSuccess &&
                                   hipMemcpy(plan->d_staged, sg.table.data(), tb, hipMemcpyHostToDevice) == hipSuccess;
            if (!staged_ok) { sccl_plan_destroy(plan); return SCCL_ERR_DEVICE; }
            // Latency bound: one workgroup per work item while the hardware can queue them (32 per CU), the
            // grid-stride loop only beyond that
            int64_t sgrid = plan->opts.max_workgroups > 0 ? plan->opts.max_workgroups : (int64_t)num_cus * 32;
            if (sgrid > sg.num_slices) sgrid = sg.num_slices;
            sg.grid = (int32_t)sgrid;
        }
        // One persistent workgroup per CU: measured best, because fewer tiles in flight means the
        // values a lane wrote in one step are still in the L2 when it reads them in the next.
        int64_t grid = num_cus;
        if (plan->opts.max_workgroups > 0) grid = plan->opts.max_workgroups;
        if (grid > plan->num_items) grid = plan->num_items;
        plan->grid = (int32_t)grid;
        plan->stats.grid_workgroups = plan->lowering == SCCL_LOWER_STAGED ? sg.grid : plan->grid;
    }
    *out_plan = plan;
    return SCCL_OK;
}

sccl_status_t sccl_plan_create(const sccl_topology_t* topology, const sccl_collective_t* collective,
                               const sccl_schedule_t* schedule, sccl_plan_t** out_plan) {
    return sccl_plan_create_ex(topology, collective, schedule, nullptr, out_plan);
}

// Alignment and pairwise disjointness of the P rank buffers (host arithmetic on the pointer values only).
static sccl_status_t check_pointers(const sccl_plan_t* plan, void* const* rank_buffers) {
    const int32_t P = plan->P;
    const uint64_t bytes = (uint64_t)plan->stats.bytes_per_rank;
    for (int32_t n = 0; n < P; n++) {
        if (!rank_buffers[n]) return SCCL_ERR_INVALID_ARG;
        if ((uintptr_t)rank_buffers[n] & 15u) return SCCL_ERR_ALIGNMENT;
    }
    for (int32_t n = 0; n < P; n++)
        for (int32_t m = n + 1; m < P; m++) {
            const uintptr_t a = (uintptr_t)rank_buffers[n], b = (uintptr_t)rank_buffers[m];
            if (a == b || (a < b ? a + bytes > b : b + bytes > a)) return SCCL_ERR_OVERLAP;
        }
    return SCCL_OK;
}

static sccl_status_t check_buffers(const sccl_plan_t* plan, void* const* rank_buffers) {
    if (!plan || !rank_buffers) return SCCL_ERR_INVALID_ARG;
    if (plan->device < 0) return SCCL_ERR_DEVICE;
    int current = -1;                                    // the step tables live on the device the plan was made on
    if (hipGetDevice(&current) != hipSuccess || current != plan->device) return SCCL_ERR_DEVICE;
    return check_pointers(plan, rank_buffers);
}

sccl_status_t sccl_execute_stepwise(const sccl_plan_t* plan, void* const* rank_buffers, void* stream) {
    const sccl_status_t chk = check_buffers(plan, rank_buffers);
    if (chk != SCCL_OK) return chk;
    if (plan->num_items == 0 || plan->step_prog.empty()) return SCCL_OK;
    StepArgs args;
    std::memset(&args, 0, sizeof(args));
    args.step_prog = plan->d_step_prog;
    args.group_off = plan->d_group_off;
    args.chunk_bytes = plan->stats.chunk_bytes;
    args.tiles_per_chunk = plan->tiles_per_chunk;
    for (int32_t n = 0; n < plan->P; n++) args.bufs[n] = (char*)rank_buffers[n];
    step_kernel_fn fn = pick_step_kernel(plan->dtype, plan->vector_bytes, plan->vectors_per_thread);
    for (int32_t s = 0; s < plan->S; s++) {
        const int32_t first = plan->step_first[(size_t)s], count = plan->step_first[(size_t)s + 1] - first;
        if (count == 0) continue;
        args.first_group = first;
        args.num_items = (int64_t)count * plan->tiles_per_chunk;
        int64_t grid = (int64_t)plan->num_cus * 4;
        if (grid > args.num_items) grid = args.num_items;
        hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3((unsigned)plan->block_threads), 0, (hipStream_t)stream, args);
        if (hipGetLastError() != hipSuccess) return SCCL_ERR_DEVICE;
    }
    return SCCL_OK;
}

sccl_status_t sccl_execute_memcpy(const sccl_plan_t* plan, void* const* rank_buffers, void* stream) {
    const sccl_status_t chk = check_buffers(plan, rank_buffers);
    if (chk != SCCL_OK) return chk;
    if (plan->stats.num_reduce_groups != 0) return SCCL_ERR_INVALID_ARG;     // a copy engine cannot add
    const size_t cs = (size_t)plan->stats.chunk_bytes;
    if (cs == 0) return SCCL_OK;
    for (const auto& t : plan->copy_sends) {
        char* dst = (char*)rank_buffers[t.dst] + (size_t)t.dst_slot * cs;
        const char* src = (const char*)rank_buffers[t.src] + (size_t)t.src_slot * cs;
        if (hipMemcpyAsync(dst, src, cs, hipMemcpyDeviceToDevice, (hipStream_t)stream) != hipSuccess) return SCCL_ERR_DEVICE;
    }
    return SCCL_OK;
}

// The two launches of sccl_execute, with the table and the grid passed in: sccl_execute passes the plan's own
// device copy, sccl_execute_static the library's static array.
static sccl_status_t launch_staged(const sccl_plan_t* plan, const int32_t* table, int32_t grid,
                                   void* const* rank_buffers, void* stream) {
    const sccl_staged& sg = plan->staged;
    StagedArgs args;
    std::memset(&args, 0, sizeof(args));
    args.table = table;
    args.chunk_bytes = plan->stats.chunk_bytes;
    args.num_items = sg.num_slices;
    args.vecs_per_chunk = plan->vecs_per_chunk;
    args.slices_per_chunk = sg.slices_per_chunk;
    args.log_slice = sg.log_slice_vectors;
    args.block_words = sg.max_block_words;
    args.cell_words_room = sg.cell_words_room;
    args.identity_off = (uint32_t)(((int64_t)sg.max_chunk_cells << sg.log_slice_vectors) * plan->vector_bytes);
    for (int32_t n = 0; n < plan->P; n++) args.bufs[n] = (char*)rank_buffers[n];
    staged_fn fn = pick_staged_kernel(plan->dtype, plan->vector_bytes);
    hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3((unsigned)sg.threads), (size_t)sg.lds_bytes, (hipStream_t)stream, args);
    return hipGetLastError() == hipSuccess ? SCCL_OK : SCCL_ERR_DEVICE;
}

static sccl_status_t launch_memory(const sccl_plan_t* plan, const int32_t* prog, const int32_t* chunk_off, int32_t grid,
                                   void* const* rank_buffers, void* stream) {
    ExecArgs args;
    std::memset(&args, 0, sizeof(args));
    args.prog = prog;
    args.chunk_off = chunk_off;
    args.chunk_bytes = plan->stats.chunk_bytes;
    args.num_items = plan->num_items;
    args.tiles_per_chunk = plan->tiles_per_chunk;
    for (int32_t n = 0; n < plan->P; n++) args.bufs[n] = (char*)rank_buffers[n];
    kernel_fn fn = pick_kernel(plan->dtype, plan->vector_bytes, plan->vectors_per_thread);
    hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3((unsigned)plan->block_threads), 0, (hipStream_t)stream, args);
    return hipGetLastError() == hipSuccess ? SCCL_OK : SCCL_ERR_DEVICE;
}

sccl_status_t sccl_execute(const sccl_plan_t* plan, void* const* rank_buffers, void* stream) {
    const sccl_status_t chk = check_buffers(plan, rank_buffers);
    if (chk != SCCL_OK) return chk;
    if (plan->num_items == 0 || plan->prog.empty()) return SCCL_OK;     // nothing to move
    if (plan->lowering == SCCL_LOWER_STAGED) return launch_staged(plan, plan->d_staged, plan->staged.grid, rank_buffers, stream);
    return launch_memory(plan, plan->d_prog, plan->d_chunk_off, plan->grid, rank_buffers, stream);
}

// ---- sccl_execute_static: the step table in a static device array instead of memory the plan allocated.
//
// `scratch` below is part of the code object, so every GPU that loads the library has its own copy at its own
// address, from load time to the end of the process.  In host code the NAME is only a handle for
// hipGetSymbolAddress: the address kernels are given is the one that call returns, looked up once per device
// with that device current, and kept in static_devices[].
constexpr int32_t STATIC_SCRATCH_WORDS = SCCL_STATIC_SCRATCH_BYTES / 4;
static __device__ __align__(256) int32_t scratch[STATIC_SCRATCH_WORDS];

// Table words travel as kernel arguments (by value, read by the kernel from its argument block), so writing
// the table needs no host-to-device copy and is captured by value when the stream is being captured.
constexpr int32_t SCRATCH_WRITE_WORDS = 896;              // 3.5 KiB of a 4 KiB argument block
struct ScratchWriteArgs {
    int32_t* dst;                                         // where in the static array
    int32_t count, pad;
    int32_t words[SCRATCH_WRITE_WORDS];
};

static __global__ void __launch_bounds__(256) sccl_scratch_write_kernel(const ScratchWriteArgs a) {
    for (int32_t i = (int32_t)threadIdx.x; i < a.count; i += 256) a.dst[i] = a.words[i];
}

constexpr int MAX_STATIC_DEVICES = 64;
struct StaticDevice {
    int32_t* ptr = nullptr;                               // device address of `scratch` on this GPU
    int num_cus = 0;
    // Whose table the array holds once everything enqueued so far has run (0: unknown).  Calls are required to be
    // serialised on the GPU, so a call for the same plan need not write the table again.  That bookkeeping is
    // only sound while every write of the array is a call the library sees: a captured call writes it again at
    // every replay of its graph, whenever the caller chooses, so after the first call on a capturing stream
    // (`captured`) nothing is assumed any more and every call writes its table.
    uint64_t resident = 0;
    bool captured = false;
};
static StaticDevice static_devices[MAX_STATIC_DEVICES];
static std::mutex static_mutex;

sccl_status_t sccl_execute_static(const sccl_plan_t* plan, void* const* rank_buffers, void* stream) {
    if (!plan || !rank_buffers) return SCCL_ERR_INVALID_ARG;
    const bool staged = plan->lowering == SCCL_LOWER_STAGED;
    const std::vector<int32_t>& image = staged ? plan->staged.table : plan->static_image;
    if (image.size() > (size_t)STATIC_SCRATCH_WORDS) return SCCL_ERR_SCRATCH;
    const sccl_status_t chk = check_pointers(plan, rank_buffers);
    if (chk != SCCL_OK) return chk;
    if (plan->num_items == 0 || plan->prog.empty()) return SCCL_OK;     // nothing to move
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_STATIC_DEVICES) return SCCL_ERR_DEVICE;

    std::lock_guard<std::mutex> lock(static_mutex);
    StaticDevice& sd = static_devices[dev];
    if (!sd.ptr) {                                        // first call on this GPU
        int32_t* p = nullptr;
        int cus = 0;
        if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
            (void)hipGetLastError();
            return SCCL_ERR_DEVICE;
        }
        sd.num_cus = cus;
        sd.ptr = p;
    }
    if (staged && plan->staged.lds_bytes > 64 * 1024 &&
        hipFuncSetAttribute((const void*)pick_staged_kernel(plan->dtype, plan->vector_bytes),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)STAGED_LDS_LIMIT) != hipSuccess) {
        (void)hipGetLastError();
        return SCCL_ERR_DEVICE;
    }

    // The table first, on the same stream, unless the array is known to hold it already (see StaticDevice).
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing((hipStream_t)stream, &capture) != hipSuccess) {
        (void)hipGetLastError();                          // e.g. the null stream while another stream captures
        capture = hipStreamCaptureStatusActive;           // assume the worst
    }
    if (capture != hipStreamCaptureStatusNone) sd.captured = true;
    if (sd.captured || sd.resident != plan->id) {
        sd.resident = 0;
        ScratchWriteArgs w;
        for (size_t at = 0; at < image.size(); at += SCRATCH_WRITE_WORDS) {
            const size_t n = std::min(image.size() - at, (size_t)SCRATCH_WRITE_WORDS);
            w.dst = sd.ptr + at;
            w.count = (int32_t)n; w.pad = 0;
            std::memcpy(w.words, image.data() + at, n * sizeof(int32_t));
            hipLaunchKernelGGL(sccl_scratch_write_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, w);
            if (hipGetLastError() != hipSuccess) return SCCL_ERR_DEVICE;
        }
        if (!sd.captured) sd.resident = plan->id;
    }
    sccl_status_t st;
    if (staged) {
        int64_t grid = plan->opts.max_workgroups > 0 ? plan->opts.max_workgroups : (int64_t)sd.num_cus * 32;
        grid = std::min(grid, plan->staged.num_slices);
        st = launch_staged(plan, sd.ptr, (int32_t)grid, rank_buffers, stream);
    } else {
        int64_t grid = plan->opts.max_workgroups > 0 ? plan->opts.max_workgroups : (int64_t)sd.num_cus;
        grid = std::min(grid, plan->num_items);
        st = launch_memory(plan, sd.ptr + plan->static_prog_off, sd.ptr, (int32_t)grid, rank_buffers, stream);
    }
    return st;
}

sccl_status_t sccl_plan_stats(const sccl_plan_t* plan, sccl_stats_t* out_stats) {
    if (!plan || !out_stats) return SCCL_ERR_INVALID_ARG;
    *out_stats = plan->stats;
    return SCCL_OK;
}

void sccl_plan_destroy(sccl_plan_t* plan) {
    if (!plan) return;
    if (plan->d_prog) (void)hipFree(plan->d_prog);
    if (plan->d_chunk_off) (void)hipFree(plan->d_chunk_off);
    if (plan->d_step_prog) (void)hipFree(plan->d_step_prog);
    if (plan->d_group_off) (void)hipFree(plan->d_group_off);
    if (plan->d_staged) (void)hipFree(plan->d_staged);
    delete plan;
}

const char* sccl_status_string(sccl_status_t status) {
    switch (status) {
        case SCCL_OK: return "SCCL_OK";
        case SCCL_ERR_INVALID_ARG: return "SCCL_ERR_INVALID_ARG";
        case SCCL_ERR_TOPOLOGY: return "SCCL_ERR_TOPOLOGY";
        case SCCL_ERR_SEND_NO_SOURCE: return "SCCL_ERR_SEND_NO_SOURCE";
        case SCCL_ERR_SEND_NO_LINK: return "SCCL_ERR_SEND_NO_LINK";
        case SCCL_ERR_BANDWIDTH: return "SCCL_ERR_BANDWIDTH";
        case SCCL_ERR_POSTCONDITION: return "SCCL_ERR_POSTCONDITION";
        case SCCL_ERR_HAZARD: return "SCCL_ERR_HAZARD";
        case SCCL_ERR_ALIGNMENT: return "SCCL_ERR_ALIGNMENT";
        case SCCL_ERR_OVERLAP: return "SCCL_ERR_OVERLAP";
        case SCCL_ERR_NOMEM: return "SCCL_ERR_NOMEM";
        case SCCL_ERR_DEVICE: return "SCCL_ERR_DEVICE";
        case SCCL_ERR_SCRATCH: return "SCCL_ERR_SCRATCH";
    }
    return "SCCL_ERR_UNKNOWN";
}

}  // extern "C"
