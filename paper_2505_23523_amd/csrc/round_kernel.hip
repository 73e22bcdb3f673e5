// Fused round kernel for gfx950 and its launcher.
//
// One launch applies ALL ops of one round of a schedule (Sec. 3: a round is a
// set of matchings, each moving one chunk).  The n ranks are n buffers in this
// GPU's HBM, so an op is a streaming pass over one chunk:
//   COPY             dst[c]  = src[c]                       read 1, write 1
//   REDUCE           dst[c]  = rnd(dst[c] + src[c])         read 2, write 1
//   REDUCE_EXCHANGE  t = rnd(src[c] + dst[c]); both = t     read 2, write 2
// The work is purely HBM-bound (at most one add per 12 bytes moved): no LDS, no
// MFMA.  Everything is moved as 16-byte vectors, U of them in flight per
// thread, all loads of a step issued before the first store.
//
// Cache hints.  When the rank buffers together exceed the 256 MiB memory-side
// cache, accesses whose data is dead afterwards, or cannot stay cached until its
// next use anyway, carry the non-temporal hint so that they do not evict chunks
// a later round reads again.  Which accesses those are depends on the schedule
// and on the buffer size (the sar::kHints* sets in launch.hpp); the kernel is
// compiled once per set, because a hint chosen at run time is lost.
//
// Grid: blockIdx.y picks the op, blockIdx.x strides over that op's chunk.  The
// rank pointers and the packed op list travel in the kernel arguments, so a
// launch needs no device-side tables and the library never allocates device
// memory.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

#include "launch.hpp"
#include "plan.hpp"
#include "stream_ops.hpp"

namespace {

using namespace sar::dev;

constexpr int kThreads = 256;
constexpr size_t kMaxBlocksX = (size_t(1) << 24) - 1;   // x kThreads stays below 2^32

// What one launch needs to know about its ops (up to CAP of them; a round with more is split
// into several launches - its ops are independent).  Two layouts behind one interface:
//   resolve(y, ...)  device: op y's chunk start in both rank buffers, its length, its kind
//   set(i, ...)      host:   describe op i
// Up to 32 ranks each op carries its two resolved pointers and its length, so a workgroup is
// ready after one round of scalar loads (measured 2-4 % over looking the ranks up, which takes a
// second, dependent round and some 64-bit arithmetic).  With up to 256 ranks that would not fit
// the 4 KiB of kernel arguments: there the ops are packed words next to one table of rank pointers.
struct OpGeometry {
    size_t elem_bytes, chunk_elems, count;   // of the plan / schedule
    void* const* rank_bufs;
};

template <int CAP>
struct RoundArgs {
    void* bufs[CAP];        // device pointer of each physical rank's buffer
    uint32_t ops[CAP];      // src | dst << 8 | first chunk << 16 | kind << 24
    uint32_t span[CAP / 4]; // consecutive chunks each op covers (ops on adjacent chunks are merged),
                            // one byte per op, four to a word so that the read stays a scalar load
    uint64_t chunk_elems;   // elements per chunk
    uint64_t count;         // elements per rank buffer

    void init(const OpGeometry& g, int n) {
        for (int i = 0; i < CAP; ++i) {
            bufs[i] = i < n ? g.rank_bufs[i] : nullptr;
            ops[i] = 0;
        }
        chunk_elems = g.chunk_elems;
        count = g.count;
    }
    void set(int i, const OpGeometry&, int src, int dst, int first_chunk, int nchunks, int kind) {
        ops[i] = uint32_t(src) | uint32_t(dst) << 8 | uint32_t(first_chunk) << 16 | uint32_t(kind) << 24;
        if (i % 4 == 0) span[i / 4] = 0;
        span[i / 4] |= uint32_t(nchunks) << ((i % 4) * 8);
    }
    __device__ __forceinline__ void resolve(uint32_t y, size_t eb, char*& sbase, char*& dbase, size_t& len,
                                            int& kind) const {
        const uint32_t op = ops[y];
        kind = int(op >> 24);
        const size_t first = size_t((op >> 16) & 0xFFu) * chunk_elems;
        const size_t want = size_t((span[y >> 2] >> ((y & 3u) * 8)) & 0xFFu) * chunk_elems;
        len = count - first;
        if (len > want) len = want;
        sbase = static_cast<char*>(bufs[op & 0xFFu]) + first * eb;
        dbase = static_cast<char*>(bufs[(op >> 8) & 0xFFu]) + first * eb;
    }
};

template <>
struct RoundArgs<32> {
    char* src[32];          // where op i's first chunk starts in the source rank's buffer
    char* dst[32];          // ... and in the destination rank's
    uint64_t len_kind[32];  // elements the op covers | kind << 62

    void init(const OpGeometry&, int) {
        for (int i = 0; i < 32; ++i) {
            src[i] = dst[i] = nullptr;
            len_kind[i] = 0;
        }
    }
    void set(int i, const OpGeometry& g, int src_rank, int dst_rank, int first_chunk, int nchunks, int kind) {
        const size_t first = size_t(first_chunk) * g.chunk_elems;
        size_t len = g.count - first;
        if (len > size_t(nchunks) * g.chunk_elems) len = size_t(nchunks) * g.chunk_elems;
        src[i] = static_cast<char*>(g.rank_bufs[src_rank]) + first * g.elem_bytes;
        dst[i] = static_cast<char*>(g.rank_bufs[dst_rank]) + first * g.elem_bytes;
        len_kind[i] = uint64_t(len) | uint64_t(kind) << 62;
    }
    __device__ __forceinline__ void resolve(uint32_t y, size_t, char*& sbase, char*& dbase, size_t& len,
                                            int& kind) const {
        const uint64_t lk = len_kind[y];
        kind = int(lk >> 62);
        len = size_t(lk & ((uint64_t(1) << 62) - 1));
        sbase = src[y];
        dbase = dst[y];
    }
};

// Streams one chunk for an op of kind KIND.  NT holds that kind's sar::NtBits.
//
// Chunk starts are only 16-byte aligned (a chunk is 1/(n-1) of the buffer), so
// the vector index space is shifted by `lead`, the number of 16-byte vectors
// between the previous 128-byte boundary of dst and the chunk start: slot j
// maps to vector j - lead, slots below `lead` stay empty, and every wavefront's
// 1 KiB access then starts on a 128-byte line in both buffers whenever the rank
// buffers share their alignment (allocator-returned buffers do).
template <int DT, int U, int KIND, uint32_t NT>
__device__ __forceinline__ void stream_chunk(u32x4* __restrict__ s, u32x4* __restrict__ d, size_t nvec) {
    constexpr bool kLs = (NT & sar::NT_LOAD_SRC) != 0, kLd = (NT & sar::NT_LOAD_DST) != 0;
    constexpr bool kSd = (NT & sar::NT_STORE_DST) != 0, kSs = (NT & sar::NT_STORE_SRC) != 0;
    const size_t lead = (reinterpret_cast<uintptr_t>(d) & 127u) / 16;
    const size_t end = lead + nvec;
    const size_t step = size_t(gridDim.x) * (kThreads * U);

    for (size_t j = size_t(blockIdx.x) * (kThreads * U) + threadIdx.x; j < end; j += step) {
        if (j >= lead && j + size_t(U - 1) * kThreads < end) {
            // full step: U vectors per thread, every load issued before the first store
            const size_t i = j - lead;
            u32x4 x[U], y[U];
#pragma unroll
            for (int u = 0; u < U; ++u) x[u] = ld<kLs>(s + i + u * kThreads);
            if (KIND != SAR_COPY) {
#pragma unroll
                for (int u = 0; u < U; ++u) y[u] = ld<kLd>(d + i + u * kThreads);
#pragma unroll
                for (int u = 0; u < U; ++u) x[u] = add_vec<DT>(x[u], y[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) st_stream<kSd>(d + i + u * kThreads, x[u]);
            if (KIND == SAR_REDUCE_EXCHANGE) {
#pragma unroll
                for (int u = 0; u < U; ++u) st_stream<kSs>(s + i + u * kThreads, x[u]);
            }
        } else {
            // first or last step of the chunk: slot by slot
            for (int u = 0; u < U; ++u) {
                const size_t jj = j + size_t(u) * kThreads;
                if (jj < lead || jj >= end) continue;
                const size_t i = jj - lead;
                u32x4 x = ld<kLs>(s + i);
                if (KIND != SAR_COPY) x = add_vec<DT>(x, ld<kLd>(d + i));
                st_stream<kSd>(d + i, x);
                if (KIND == SAR_REDUCE_EXCHANGE) st_stream<kSs>(s + i, x);
            }
        }
    }
}

// NTM: sar::NtBits of the three op kinds, four bits each at bit 4 * kind.
template <int DT, int CAP, int U, uint32_t NTM>
__global__ __launch_bounds__(kThreads) void round_kernel(const RoundArgs<CAP> a) {
    constexpr size_t EB = (DT == SAR_BF16) ? 2 : 4;
    char *sbase, *dbase;
    size_t len;
    int kind;
    a.resolve(blockIdx.y, EB, sbase, dbase, len, kind);
    u32x4* s = reinterpret_cast<u32x4*>(sbase);
    u32x4* d = reinterpret_cast<u32x4*>(dbase);
    const size_t nvec = len * EB / 16;

    if (kind == SAR_COPY)
        stream_chunk<DT, U, SAR_COPY, NTM & 0xFu>(s, d, nvec);
    else if (kind == SAR_REDUCE)
        stream_chunk<DT, U, SAR_REDUCE, (NTM >> 4) & 0xFu>(s, d, nvec);
    else
        stream_chunk<DT, U, SAR_REDUCE_EXCHANGE, (NTM >> 8) & 0xFu>(s, d, nvec);

    // elements past the last whole vector (only the buffer's final chunk can have any)
    if (blockIdx.x == 0) {
        const size_t done = nvec * (16 / EB);
        if (done + threadIdx.x < len) tail_elem<DT>(sbase, dbase, done + threadIdx.x, kind);
    }
}

// ---- rounds whose same-value copies are merged (sar_group_op) ---------------------------------
// A COPY group streams one chunk from one holder to every rank in its destination mask: one load,
// k stores per vector, the value staying in registers (no LDS: each thread stores what it
// loaded).  Reducing ops have one destination and run as in round_kernel.  Up to 32 ranks.
struct GroupArgs {
    char* bufs[32];
    uint32_t op[32];        // kind | src << 8 | first chunk << 16 | chunks covered << 24
    uint32_t dst_mask[32];  // bit r: physical rank r receives (one bit for reducing ops)
    uint64_t chunk_elems, count;
};

template <int DT, int U, uint32_t NT>
__device__ __forceinline__ void multicast_chunk(const GroupArgs& a, const char* sbase, size_t first_byte,
                                                uint32_t mask, size_t len) {
    constexpr size_t EB = (DT == SAR_BF16) ? 2 : 4;
    constexpr bool kLs = (NT & sar::NT_LOAD_SRC) != 0, kSd = (NT & sar::NT_STORE_DST) != 0;
    const u32x4* s = reinterpret_cast<const u32x4*>(sbase);
    const size_t nvec = len * EB / 16;
    const size_t lead = (reinterpret_cast<uintptr_t>(sbase) & 127u) / 16;
    const size_t end = lead + nvec;
    const size_t step = size_t(gridDim.x) * (kThreads * U);
    for (size_t j0 = size_t(blockIdx.x) * (kThreads * U) + threadIdx.x; j0 < end; j0 += step) {
        u32x4 x[U];
        bool live[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t j = j0 + size_t(u) * kThreads;
            live[u] = j >= lead && j < end;
            if (live[u]) x[u] = ld<kLs>(s + (j - lead));
        }
        for (uint32_t m = mask; m != 0; m &= m - 1) {
            u32x4* d = reinterpret_cast<u32x4*>(a.bufs[__builtin_ctz(m)] + first_byte);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (live[u]) st_stream<kSd>(d + (j0 + size_t(u) * kThreads - lead), x[u]);
        }
    }
    // elements past the last whole vector (only the buffer's final chunk can have any)
    const size_t e = nvec * (16 / EB) + threadIdx.x;
    if (blockIdx.x == 0 && e < len) {
        for (uint32_t m = mask; m != 0; m &= m - 1) {
            char* dbase = a.bufs[__builtin_ctz(m)] + first_byte;
            if (DT == SAR_BF16)
                reinterpret_cast<uint16_t*>(dbase)[e] = reinterpret_cast<const uint16_t*>(sbase)[e];
            else
                reinterpret_cast<uint32_t*>(dbase)[e] = reinterpret_cast<const uint32_t*>(sbase)[e];
        }
    }
}

template <int DT, int U, uint32_t NTM>
__global__ __launch_bounds__(kThreads) void group_kernel(const GroupArgs a) {
    constexpr size_t EB = (DT == SAR_BF16) ? 2 : 4;
    const uint32_t op = a.op[blockIdx.y];
    const uint32_t mask = a.dst_mask[blockIdx.y];
    const int kind = int(op & 0xFFu);
    const size_t first = size_t((op >> 16) & 0xFFu) * a.chunk_elems;
    const size_t want = size_t(op >> 24) * a.chunk_elems;
    size_t len = a.count - first;
    if (len > want) len = want;
    char* sbase = a.bufs[(op >> 8) & 0xFFu] + first * EB;
    if (kind == SAR_COPY) {
        multicast_chunk<DT, U, NTM & 0xFu>(a, sbase, first * EB, mask, len);
        return;
    }
    char* dbase = a.bufs[__builtin_ctz(mask)] + first * EB;
    u32x4* s = reinterpret_cast<u32x4*>(sbase);
    u32x4* d = reinterpret_cast<u32x4*>(dbase);
    const size_t nvec = len * EB / 16;
    if (kind == SAR_REDUCE)
        stream_chunk<DT, U, SAR_REDUCE, (NTM >> 4) & 0xFu>(s, d, nvec);
    else
        stream_chunk<DT, U, SAR_REDUCE_EXCHANGE, (NTM >> 8) & 0xFu>(s, d, nvec);
    if (blockIdx.x == 0) {
        const size_t done = nvec * (16 / EB);
        if (done + threadIdx.x < len) tail_elem<DT>(sbase, dbase, done + threadIdx.x, kind);
    }
}

template <int DT, int CAP, int U>
hipError_t launch_nt(uint32_t hints, dim3 grid, hipStream_t stream, const RoundArgs<CAP>& args) {
#define SAR_LAUNCH(M) \
    case M: hipLaunchKernelGGL((round_kernel<DT, CAP, U, M>), grid, dim3(kThreads), 0, stream, args); break;
    switch (hints) {
        SAR_LAUNCH(sar::kHintsNone)
        SAR_LAUNCH(sar::kHintsCompletion)
        SAR_LAUNCH(sar::kHintsCompletionStores)
        SAR_LAUNCH(sar::kHintsCompletionAll)
        SAR_LAUNCH(sar::kHintsPrecondition)
        SAR_LAUNCH(sar::kHintsPreconditionHuge)
        SAR_LAUNCH(sar::kHintsRing)
        SAR_LAUNCH(sar::kHintsRingHuge)
        SAR_LAUNCH(sar::kHintsRingHugest)
        default: return hipErrorInvalidValue;
    }
#undef SAR_LAUNCH
    return hipGetLastError();
}

template <int DT, int U>
hipError_t launch_group_nt(uint32_t hints, dim3 grid, hipStream_t stream, const GroupArgs& args) {
#define SAR_LAUNCH(M) \
    case M: hipLaunchKernelGGL((group_kernel<DT, U, M>), grid, dim3(kThreads), 0, stream, args); break;
    switch (hints) {
        SAR_LAUNCH(sar::kHintsNone)
        SAR_LAUNCH(sar::kHintsCompletion)
        SAR_LAUNCH(sar::kHintsCompletionStores)
        SAR_LAUNCH(sar::kHintsCompletionAll)
        SAR_LAUNCH(sar::kHintsPrecondition)
        SAR_LAUNCH(sar::kHintsPreconditionHuge)
        SAR_LAUNCH(sar::kHintsRing)
        SAR_LAUNCH(sar::kHintsRingHuge)
        SAR_LAUNCH(sar::kHintsRingHugest)
        default: return hipErrorInvalidValue;
    }
#undef SAR_LAUNCH
    return hipGetLastError();
}

template <int DT>
hipError_t launch_group_u(int unroll, uint32_t hints, dim3 grid, hipStream_t stream, const GroupArgs& args) {
    switch (unroll) {
        case 1: return launch_group_nt<DT, 1>(hints, grid, stream, args);
        case 2: return launch_group_nt<DT, 2>(hints, grid, stream, args);
        default: return launch_group_nt<DT, 4>(hints, grid, stream, args);
    }
}

hipError_t launch_group(int dtype, int unroll, uint32_t hints, dim3 grid, hipStream_t stream, const GroupArgs& args) {
    switch (dtype) {
        case SAR_I32: return launch_group_u<SAR_I32>(unroll, hints, grid, stream, args);
        case SAR_F32: return launch_group_u<SAR_F32>(unroll, hints, grid, stream, args);
        default: return launch_group_u<SAR_BF16>(unroll, hints, grid, stream, args);
    }
}

template <int DT, int CAP>
hipError_t launch_u(int unroll, uint32_t hints, dim3 grid, hipStream_t stream, const RoundArgs<CAP>& args) {
    switch (unroll) {
        case 1: return launch_nt<DT, CAP, 1>(hints, grid, stream, args);
        case 2: return launch_nt<DT, CAP, 2>(hints, grid, stream, args);
        default: return launch_nt<DT, CAP, 4>(hints, grid, stream, args);
    }
}

template <int CAP>
hipError_t launch_dt(int dtype, int unroll, uint32_t hints, dim3 grid, hipStream_t stream,
                     const RoundArgs<CAP>& args) {
    switch (dtype) {
        case SAR_I32: return launch_u<SAR_I32, CAP>(unroll, hints, grid, stream, args);
        case SAR_F32: return launch_u<SAR_F32, CAP>(unroll, hints, grid, stream, args);
        default: return launch_u<SAR_BF16, CAP>(unroll, hints, grid, stream, args);
    }
}

// rank_bufs == nullptr: nothing is launched, the launches are only counted.
template <int CAP>
int run_rounds(const sar_plan* plan, const sar_sched& sched, void* const* rank_bufs, hipStream_t stream,
               const sar::LaunchShape& shape, int* launches) {
    const bool dry = rank_bufs == nullptr;
    const OpGeometry geometry{plan->elem_bytes, sched.chunk_elems, plan->count, rank_bufs};
    RoundArgs<CAP> args;
    if (!dry) args.init(geometry, plan->n);
    const size_t vec_per_chunk = sched.chunk_elems * plan->elem_bytes / 16;
    const size_t per_block = size_t(kThreads) * shape.unroll;

    for (const std::vector<sar_op>& ops : sched.rounds) {
        const int total = int(ops.size());
        int k = 0;
        while (k < total) {
            // fill one launch: merge runs of ops that move adjacent chunks between the same two ranks
            int nops = 0;
            int max_span = 1;
            while (k < total && nops < CAP) {
                const sar_op& op = ops[shape.reverse_ops ? total - 1 - k : k];
                int span = 1;
                while (k + span < total && span < 255) {
                    const sar_op& nx = ops[shape.reverse_ops ? total - 1 - (k + span) : k + span];
                    const int want_chunk = shape.reverse_ops ? op.chunk - span : op.chunk + span;
                    if (nx.src != op.src || nx.dst != op.dst || nx.op != op.op || nx.chunk != want_chunk) break;
                    ++span;
                }
                const int first_chunk = shape.reverse_ops ? op.chunk - (span - 1) : op.chunk;
                if (!dry) args.set(nops, geometry, op.src, op.dst, first_chunk, span, op.op);
                if (span > max_span) max_span = span;
                ++nops;
                k += span;
            }
            // slots of the longest op: its vectors plus at most 7 empty leading slots (see stream_chunk)
            const size_t max_bx = (vec_per_chunk * max_span + 7 + per_block - 1) / per_block;
            // one workgroup per tile unless the caller bounds the grid; the kernel strides, so the
            // runtime's limit of 2^32 threads per grid dimension only ever costs extra steps
            size_t bx = shape.total_blocks > 0 ? (size_t(shape.total_blocks) + nops - 1) / nops : max_bx;
            if (bx > max_bx) bx = max_bx;
            if (bx > kMaxBlocksX) bx = kMaxBlocksX;
            if (bx < 1) bx = 1;
            const dim3 grid(static_cast<unsigned>(bx), static_cast<unsigned>(nops));
            ++*launches;
            if (!dry && launch_dt<CAP>(plan->dtype, shape.unroll, shape.hints, grid, stream, args) != hipSuccess)
                return SAR_EDEVICE;
        }
    }
    return SAR_OK;
}

// One launch per round over the round's merged ops (sched.grouped); groups on adjacent chunks with
// the same kind, source and destinations become one streaming op.
int run_groups(const sar_plan* plan, const sar_sched& sched, void* const* rank_bufs, hipStream_t stream,
               const sar::LaunchShape& shape, int* launches) {
    const bool dry = rank_bufs == nullptr;
    GroupArgs args;
    for (int i = 0; i < 32; ++i) {
        args.bufs[i] = !dry && i < plan->n ? static_cast<char*>(rank_bufs[i]) : nullptr;
        args.op[i] = args.dst_mask[i] = 0;
    }
    args.chunk_elems = sched.chunk_elems;
    args.count = plan->count;
    const size_t vec_per_chunk = sched.chunk_elems * plan->elem_bytes / 16;
    const size_t per_block = size_t(kThreads) * shape.unroll;
    for (const std::vector<sar_group_op>& groups : sched.grouped) {
        const int total = int(groups.size());
        int k = 0;
        while (k < total) {
            int nops = 0, max_span = 1;
            while (k < total && nops < 32) {
                const sar_group_op& g = groups[k];
                int span = 1;
                while (k + span < total) {
                    const sar_group_op& nx = groups[k + span];
                    if (nx.kind != g.kind || nx.src != g.src || nx.dst_mask != g.dst_mask || nx.chunk != g.chunk + span) break;
                    ++span;
                }
                args.op[nops] = uint32_t(g.kind) | uint32_t(g.src) << 8 | uint32_t(g.chunk) << 16 | uint32_t(span) << 24;
                args.dst_mask[nops] = g.dst_mask;
                if (span > max_span) max_span = span;
                ++nops;
                k += span;
            }
            const size_t max_bx = (vec_per_chunk * max_span + 7 + per_block - 1) / per_block;
            size_t bx = shape.total_blocks > 0 ? (size_t(shape.total_blocks) + nops - 1) / nops : max_bx;
            if (bx > max_bx) bx = max_bx;
            if (bx > kMaxBlocksX) bx = kMaxBlocksX;
            if (bx < 1) bx = 1;
            const dim3 grid(static_cast<unsigned>(bx), static_cast<unsigned>(nops));
            ++*launches;
            if (!dry && launch_group(plan->dtype, shape.unroll, shape.hints, grid, stream, args) != hipSuccess)
                return SAR_EDEVICE;
        }
    }
    return SAR_OK;
}

}  // namespace

int sar::run_schedule(const sar_plan* plan, int which, void* const* rank_bufs, void* hip_stream,
                      const LaunchShape& shape, int* launches) {
    const sar_sched& sched = plan->sched[which];
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int counted = 0;
    int st;
    if (shape.merge_copies && !sched.grouped.empty())
        st = run_groups(plan, sched, rank_bufs, stream, shape, &counted);
    else if (plan->n <= 32)
        st = run_rounds<32>(plan, sched, rank_bufs, stream, shape, &counted);
    else
        st = run_rounds<SAR_MAX_RANKS>(plan, sched, rank_bufs, stream, shape, &counted);
    if (launches) *launches = counted;
    return st;
}

int sar::device_compute_units(int* out) {
    // cached per device: the attribute query costs a few microseconds per call otherwise
    static std::atomic<int> cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SAR_EDEVICE;
    if (dev >= 0 && dev < 64) {
        const int hit = cache[dev].load(std::memory_order_relaxed);
        if (hit > 0) {
            *out = hit;
            return SAR_OK;
        }
    }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return SAR_EDEVICE;
    if (dev >= 0 && dev < 64) cache[dev].store(cus, std::memory_order_relaxed);
    *out = cus;
    return SAR_OK;
}
