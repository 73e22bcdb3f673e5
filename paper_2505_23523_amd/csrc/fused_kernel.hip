// Single-launch execution of a whole schedule.
//
// Every op of the schedules touches one chunk index only, and an op on chunk c
// depends only on earlier ops on the same elements of chunk c (Alg. 1 moves and
// reduces chunks, never parts of different chunks together).  So a workgroup
// that owns one 4 KiB tile of one chunk index can run ALL rounds' ops on that
// tile by itself, in round order, with no synchronisation between workgroups:
// what it reads in a later round is what it wrote itself in an earlier one.
// Ops are applied in round order.  Two things change against one launch per
// round.  Where an op's source value comes from: when the source cell is one
// this workgroup wrote itself since the value last changed (the planner marks
// such ops), the value is still in registers and the load is skipped.  And
// which stores reach memory: a store that no later op loads and a later op
// overwrites (the planner marks those too) is dropped - the partial sums a ring
// leaves on the ranks it passes through are all of this kind; every cell's final
// content is still written.  For the precondition on its own, whose
// postcondition defines only each on-time rank's own chunk (Sec. 3.1), the other
// chunks of the rank buffers are then left as they were instead of holding
// partial sums.  In the completion every COPY forwards the value produced by the
// chunk's exchange and every store is final, so per chunk index the kernel reads
// 2 cells and writes n.  HBM bytes (s = bytes per rank buffer; in brackets one
// launch per round):
//   completion    per chunk index 2 reads + n writes          (n+2) s    [2n s]
//   precondition  per chunk index n-1 reads + 1 write         n s        [3(n-2) s]
//   ring          per chunk index n reads + n writes          2n s       [5(n-1) s]
// The launches per call drop from one per round to one or two, which is what
// matters for small buffers.
//
// The ops of each chunk index (in round order) travel in the kernel arguments; a
// launch covers as many chunk indices as fit in their 4 KiB.  Two layouts: up to
// 32 ranks (16-bit op words, 1536 of them) and up to 256 ranks (32-bit words, 440
// of them: fewer chunk indices per launch, hence more launches per call).
//
// Besides this general kernel (fused_kernel) the file holds kernels for schedules of a
// particular shape, which need no op lists and compute the same bits:
//   sum_to_all_kernel   every chunk index one exchange whose sum goes to all n ranks (the
//                       completion of Alg. 1), straight-line;
//   exchange_kernel + broadcast_kernel   the same split in two launches per group of chunk
//                       indices: the exchanges, then the sum copied rank by rank, so that
//                       HBM sees few write streams at a time;
//   chain_kernel        every chunk index the same walk around a ring of ranks from its own
//                       start position (the precondition's ReduceScatter, the ring AllReduce).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "launch.hpp"
#include "plan.hpp"
#include "stream_ops.hpp"

namespace {

using namespace sar::dev;

constexpr int kThreads = 256;
constexpr int kMaxChunks = 32;     // chunk indices per launch

// op word: src | dst << B | kind << 2B | forward << (2B + 2) | dead << (2B + 3) | chained << (2B + 4),
// with B = rank index bits.
// Everything a workgroup reads from its arguments is laid out in 32-bit words, so that the op loop
// fetches with scalar loads: a 16-bit array element is fetched with a vector load, whose wait also
// waits for the data stores issued before it and so serialises the whole chain.
template <int CAP>
struct FusedArgs;

template <>
struct FusedArgs<32> {
    static constexpr int kRankBits = 5;
    static constexpr int kMaxOps = 1536;
    void* bufs[32];
    uint32_t ops[kMaxOps / 2 + 2];    // 16-bit op words, two to a word (+ slack: the kernel reads 4 ahead)
    uint32_t first[kMaxChunks + 1];   // ops of chunk chunk0 + y: [first[y], first[y + 1])
    uint32_t chunk0;
    uint64_t chunk_elems;
    uint64_t count;
    __host__ __device__ uint32_t op_at(uint32_t o) const { return (ops[o >> 1] >> ((o & 1u) * 16)) & 0xFFFFu; }
    void set_op(int o, uint32_t w) {
        if (o % 2 == 0) ops[o / 2] = 0;
        ops[o / 2] |= w << ((o % 2) * 16);
    }
};

template <>
struct FusedArgs<256> {
    static constexpr int kRankBits = 8;
    static constexpr int kMaxOps = 440;
    void* bufs[256];
    uint32_t ops[kMaxOps + 4];        // + slack: the kernel reads 4 ahead
    uint32_t first[kMaxChunks + 1];
    uint32_t chunk0;
    uint64_t chunk_elems;
    uint64_t count;
    __host__ __device__ uint32_t op_at(uint32_t o) const { return ops[o]; }
    void set_op(int o, uint32_t w) { ops[o] = w; }
};
static_assert(sizeof(FusedArgs<32>) <= 4096 && sizeof(FusedArgs<256>) <= 4096,
              "kernel arguments are limited to 4 KiB");

template <int DT, int CAP, int U, bool NTL, bool NTS>
__global__ __launch_bounds__(kThreads) void fused_kernel(const FusedArgs<CAP> a) {
    constexpr int B = FusedArgs<CAP>::kRankBits;
    constexpr uint32_t kRankMask = (1u << B) - 1u;
    constexpr size_t EB = (DT == SAR_BF16) ? 2 : 4;
    const uint32_t y = blockIdx.y;
    const size_t first = size_t(a.chunk0 + y) * a.chunk_elems;
    size_t len = a.count - first;
    if (len > a.chunk_elems) len = a.chunk_elems;
    const size_t nvec = len * EB / 16;
    const size_t byte_off = first * EB;

    // slot -> vector shift that puts every wavefront's access on a 128-byte line
    // (rank buffers normally share their alignment; rank 0's is taken)
    const size_t lead = ((reinterpret_cast<uintptr_t>(a.bufs[0]) + byte_off) & 127u) / 16;
    const size_t j0 = size_t(blockIdx.x) * (kThreads * U) + threadIdx.x;
    bool live[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t j = j0 + size_t(u) * kThreads;
        live[u] = j >= lead && j < lead + nvec;
    }
    const size_t i0 = j0 - lead;
    const size_t done = nvec * (16 / EB);
    const size_t te = done + threadIdx.x;      // this thread's element of the ragged tail
    const bool tail = blockIdx.x == 0 && te < len;

    u32x4 x[U];
    uint32_t xt = 0;                           // tail element (low 16 bits for bf16)
#pragma unroll
    for (int u = 0; u < U; ++u) x[u] = u32x4{0, 0, 0, 0};

    const uint32_t end = a.first[y + 1];
    uint32_t o = a.first[y];
    uint32_t op = a.op_at(o);                  // (reading at `end` is safe: the array has slack)
    constexpr int kBatch = 4;
    constexpr uint32_t kChained = 1u << (2 * B + 4);
    while (o < end) {
        // A reduce chain (the hops of a ring): the source is in registers and nothing in between
        // writes the operands, so up to four operand loads go out together; the additions follow
        // in list order.
        if (op & kChained) {
            uint32_t w[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) w[k] = a.op_at(o + k);      // may run past `end`: slack
            int run = 1;
#pragma unroll
            for (int k = 1; k < kBatch; ++k)
                if (run == k && o + k < end && (w[k] & kChained)) run = k + 1;
            char* base[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k)
                base[k] = static_cast<char*>(a.bufs[(w[k] >> B) & kRankMask]) + byte_off;
            u32x4 operand[kBatch][U];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                if (k >= run) continue;
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (live[u]) operand[k][u] = ld<NTL>(reinterpret_cast<u32x4*>(base[k]) + i0 + u * kThreads);
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                if (k >= run) continue;
                const bool keep_k = ((w[k] >> (2 * B + 3)) & 1u) == 0;
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (live[u]) x[u] = add_vec<DT>(x[u], operand[k][u]);
                if (keep_k) {
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        if (live[u]) st<NTS>(reinterpret_cast<u32x4*>(base[k]) + i0 + u * kThreads, x[u]);
                }
                if (tail) {
                    if (DT == SAR_BF16) {
                        uint16_t* dp = reinterpret_cast<uint16_t*>(base[k]) + te;
                        xt = bf16_rne(__uint_as_float(xt << 16) + __uint_as_float(uint32_t(*dp) << 16));
                        if (keep_k) *dp = uint16_t(xt);
                    } else {
                        uint32_t* dp = reinterpret_cast<uint32_t*>(base[k]) + te;
                        xt = add_word<DT>(xt, *dp);
                        if (keep_k) *dp = xt;
                    }
                }
            }
            o += run;
            op = a.op_at(o);
            continue;
        }
        const int kind = int((op >> (2 * B)) & 3u);
        const bool forward = ((op >> (2 * B + 2)) & 1u) != 0;     // source value is already in registers
        const bool keep = ((op >> (2 * B + 3)) & 1u) == 0;        // the store to dst can be observed
        char* sbase = static_cast<char*>(a.bufs[op & kRankMask]) + byte_off;
        char* dbase = static_cast<char*>(a.bufs[(op >> B) & kRankMask]) + byte_off;
        u32x4* s = reinterpret_cast<u32x4*>(sbase) + i0;
        u32x4* d = reinterpret_cast<u32x4*>(dbase) + i0;
        if (!forward) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (live[u]) x[u] = ld<NTL>(s + u * kThreads);
        }
        if (kind != SAR_COPY) {
            u32x4 yv[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (live[u]) yv[u] = ld<NTL>(d + u * kThreads);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (live[u]) x[u] = add_vec<DT>(x[u], yv[u]);
        }
        if (keep) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (live[u]) st<NTS>(d + u * kThreads, x[u]);
        }
        if (kind == SAR_REDUCE_EXCHANGE) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (live[u]) st<NTS>(s + u * kThreads, x[u]);
        }
        if (tail) {
            if (DT == SAR_BF16) {
                uint16_t* sp = reinterpret_cast<uint16_t*>(sbase) + te;
                uint16_t* dp = reinterpret_cast<uint16_t*>(dbase) + te;
                if (!forward) xt = *sp;
                if (kind != SAR_COPY)
                    xt = bf16_rne(__uint_as_float(xt << 16) + __uint_as_float(uint32_t(*dp) << 16));
                if (keep) *dp = uint16_t(xt);
                if (kind == SAR_REDUCE_EXCHANGE) *sp = uint16_t(xt);
            } else {
                uint32_t* sp = reinterpret_cast<uint32_t*>(sbase) + te;
                uint32_t* dp = reinterpret_cast<uint32_t*>(dbase) + te;
                if (!forward) xt = *sp;
                if (kind != SAR_COPY) xt = add_word<DT>(xt, *dp);
                if (keep) *dp = xt;
                if (kind == SAR_REDUCE_EXCHANGE) *sp = xt;
            }
        }

        // The copies that hand this value on (source in registers) are stores only.  They get a
        // loop of their own with no load in it: the hardware counts loads and stores in one
        // counter, and in a loop that may also load the compiler has to wait for that counter to
        // reach zero before every store - which would make each store wait for the one before it.
        // Four at a time, so that the scalar loads of op words and rank pointers overlap.
        constexpr uint32_t kForwardedCopy = 1u << (2 * B + 2);              // kind COPY, forward
        constexpr uint32_t kKindAndForward = (3u << (2 * B)) | kForwardedCopy;
        ++o;
        op = a.op_at(o);
        while (o < end && (op & kKindAndForward) == kForwardedCopy) {
            uint32_t w[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) w[k] = a.op_at(o + k);      // may run past `end`: slack
            int run = 0;                                  // leading forwarded copies of the batch
#pragma unroll
            for (int k = 0; k < kBatch; ++k)
                if (run == k && o + k < end && (w[k] & kKindAndForward) == kForwardedCopy) run = k + 1;
            char* base[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k)
                base[k] = static_cast<char*>(a.bufs[(w[k] >> B) & kRankMask]) + byte_off;
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                if (k >= run || ((w[k] >> (2 * B + 3)) & 1u)) continue;     // past the run, or unobserved
                u32x4* nd = reinterpret_cast<u32x4*>(base[k]) + i0;
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (live[u]) st<NTS>(nd + u * kThreads, x[u]);
                if (tail) {
                    if (DT == SAR_BF16)
                        reinterpret_cast<uint16_t*>(base[k])[te] = uint16_t(xt);
                    else
                        reinterpret_cast<uint32_t*>(base[k])[te] = xt;
                }
            }
            o += run;
            op = a.op_at(o);
        }
    }
}

// `lds` bytes of (unused) dynamic LDS per workgroup cap how many workgroups share a
// compute unit: the kernel is store-dominated, and HBM takes the stores better
// when fewer wavefronts interleave their write streams.
template <int DT, int CAP, int U>
hipError_t launch_nt(bool nt_loads, bool nt_stores, dim3 grid, size_t lds, hipStream_t stream,
                     const FusedArgs<CAP>& args) {
    if (nt_loads && nt_stores)
        hipLaunchKernelGGL((fused_kernel<DT, CAP, U, true, true>), grid, dim3(kThreads), lds, stream, args);
    else if (nt_loads)
        hipLaunchKernelGGL((fused_kernel<DT, CAP, U, true, false>), grid, dim3(kThreads), lds, stream, args);
    else if (nt_stores)
        hipLaunchKernelGGL((fused_kernel<DT, CAP, U, false, true>), grid, dim3(kThreads), lds, stream, args);
    else
        hipLaunchKernelGGL((fused_kernel<DT, CAP, U, false, false>), grid, dim3(kThreads), lds, stream, args);
    return hipGetLastError();
}

template <int DT, int CAP>
hipError_t launch_u(int unroll, bool ntl, bool nts, dim3 grid, size_t lds, hipStream_t stream,
                    const FusedArgs<CAP>& args) {
    switch (unroll) {
        case 1: return launch_nt<DT, CAP, 1>(ntl, nts, grid, lds, stream, args);
        case 2: return launch_nt<DT, CAP, 2>(ntl, nts, grid, lds, stream, args);
        default: return launch_nt<DT, CAP, 4>(ntl, nts, grid, lds, stream, args);
    }
}

template <int CAP>
hipError_t launch(int dtype, int unroll, bool ntl, bool nts, dim3 grid, size_t lds, hipStream_t stream,
                  const FusedArgs<CAP>& args) {
    switch (dtype) {
        case SAR_I32: return launch_u<SAR_I32, CAP>(unroll, ntl, nts, grid, lds, stream, args);
        case SAR_F32: return launch_u<SAR_F32, CAP>(unroll, ntl, nts, grid, lds, stream, args);
        default: return launch_u<SAR_BF16, CAP>(unroll, ntl, nts, grid, lds, stream, args);
    }
}

// Dynamic LDS that lets exactly `wgs` workgroups fit the 160 KiB of a compute unit (0: no cap).
size_t lds_for_workgroups_per_cu(int wgs) {
    switch (wgs) {
        case 2: return 65536;
        case 3: return 53248;
        case 4: return 40960;
        case 5: return 32768;
        case 6: return 26624;
        default: return 0;
    }
}

// ---- the trailing copies of a split schedule (sar_sched::cut) -----------------------------------
// After the producing ops a chunk's value sits in one rank's cell and only has to reach the other
// ranks.  Storing a tile to all of them from one workgroup makes every workgroup write n streams
// at once, which HBM takes 15-25 % worse than sequential writes (the more ranks, the worse).
// Here a workgroup copies ONE tile to ONE rank, and the workgroups are ordered segment by segment
// (a run of `seg` tiles), inside a segment rank by rank, inside a rank tile by tile: at any moment
// only a few destination streams are being written, each in runs of seg x 4 KiB, and a segment's
// source tiles are re-read from L2 - workgroup ids that differ by a multiple of 8 run on the same
// XCD, and seg is a multiple of 8 (except for short chunks, broadcast_segment), so tile t of
// every rank's pass meets the same L2.
struct BroadcastArgs {
    char* bufs[SAR_MAX_RANKS];
    uint32_t route[SAR_MAX_RANKS];   // per chunk index: holder | excluded0 << 8 | excluded1 << 16
    uint32_t dests;                  // ranks written per chunk index
    uint32_t seg;                    // tiles per segment (8, a multiple of the XCD count; fewer for short chunks)
    uint32_t tiles;                  // 4 KiB tiles per chunk (incl. up to 7 empty leading slots)
    uint32_t y0;                     // chunk index of blockIdx.y == 0
    uint64_t chunk_elems, count;
};
static_assert(sizeof(BroadcastArgs) <= 4096, "kernel arguments are limited to 4 KiB");

template <int DT, bool NTS>
__global__ __launch_bounds__(kThreads) void broadcast_kernel(const BroadcastArgs a) {
    constexpr size_t EB = (DT == SAR_BF16) ? 2 : 4;
    const uint32_t y = blockIdx.y + a.y0;
    const uint32_t route = a.route[y];
    const uint32_t per_seg = a.seg * a.dests;
    const uint32_t seg = blockIdx.x / per_seg, rem = blockIdx.x - seg * per_seg;
    const uint32_t ri = rem / a.seg, tile = seg * a.seg + (rem - ri * a.seg);
    if (tile >= a.tiles) return;
    // destination: the ri-th rank outside the excluded set
    const uint32_t e0 = (route >> 8) & 0xFFu, e1 = (route >> 16) & 0xFFu;
    uint32_t r = ri;
    if (r >= e0) ++r;
    if (e1 != e0 && r >= e1) ++r;
    const size_t first = size_t(y) * a.chunk_elems;
    size_t len = a.count - first;
    if (len > a.chunk_elems) len = a.chunk_elems;
    const size_t nvec = len * EB / 16;
    const size_t byte_off = first * EB;
    const char* sbase = a.bufs[route & 0xFFu] + byte_off;
    char* dbase = a.bufs[r] + byte_off;
    const size_t lead = ((reinterpret_cast<uintptr_t>(a.bufs[0]) + byte_off) & 127u) / 16;
    const size_t j = size_t(tile) * kThreads + threadIdx.x;
    if (j >= lead && j < lead + nvec)
        st<NTS>(reinterpret_cast<u32x4*>(dbase) + (j - lead), *(reinterpret_cast<const u32x4*>(sbase) + (j - lead)));
    const size_t te = nvec * (16 / EB) + threadIdx.x;      // the ragged tail, element by element
    if (tile == 0 && te < len) {
        if (DT == SAR_BF16)
            reinterpret_cast<uint16_t*>(dbase)[te] = reinterpret_cast<const uint16_t*>(sbase)[te];
        else
            reinterpret_cast<uint32_t*>(dbase)[te] = reinterpret_cast<const uint32_t*>(sbase)[te];
    }
}

template <int DT>
hipError_t launch_broadcast(bool nts, dim3 grid, hipStream_t stream, const BroadcastArgs& args) {
    if (nts)
        hipLaunchKernelGGL((broadcast_kernel<DT, true>), grid, dim3(kThreads), 0, stream, args);
    else
        hipLaunchKernelGGL((broadcast_kernel<DT, false>), grid, dim3(kThreads), 0, stream, args);
    return hipGetLastError();
}

// ---- the completion's shape in one launch, without an op list -----------------------------------
// Every chunk index is one exchange (two loads, one add) whose sum goes to all n ranks
// (sar_sched::sum_to_all).  Straight-line code instead of the op walk is 3 % faster at 8 ranks;
// each workgroup starts its n stores at a different rank, so that the workgroups running at the
// same time are not all writing the same rank's buffer (another 1 %).  The on-time rank's operand
// is what the precondition stored last and is loaded plainly; the other rank's - the straggler's
// input, untouched since long before - takes its own hint (NTO).
template <int CAP>
struct SumToAllArgsT {
    char* bufs[CAP];
    uint32_t route[CAP];    // per chunk index: the exchange's on-time rank | its other rank << 8
    uint32_t n;
    uint32_t y0;            // chunk index of blockIdx.y == 0
    uint64_t chunk_elems, count;
};
typedef SumToAllArgsT<32> SumToAllArgs;
static_assert(sizeof(SumToAllArgsT<SAR_MAX_RANKS>) <= 4096, "kernel arguments are limited to 4 KiB");

template <int DT, int U, bool NTO, bool NTS>
__global__ __launch_bounds__(kThreads) void sum_to_all_kernel(const SumToAllArgs a) {
    constexpr size_t EB = (DT == SAR_BF16) ? 2 : 4;
    const uint32_t y = blockIdx.y + a.y0;
    const uint32_t route = a.route[y];
    const size_t first = size_t(y) * a.chunk_elems;
    size_t len = a.count - first;
    if (len > a.chunk_elems) len = a.chunk_elems;
    const size_t nvec = len * EB / 16;
    const size_t byte_off = first * EB;
    const size_t lead = ((reinterpret_cast<uintptr_t>(a.bufs[0]) + byte_off) & 127u) / 16;
    const size_t j0 = size_t(blockIdx.x) * (kThreads * U) + threadIdx.x;
    const size_t i0 = j0 - lead;
    const char* sbase = a.bufs[route & 0xFFu] + byte_off;
    const char* dbase = a.bufs[(route >> 8) & 0xFFu] + byte_off;
    const u32x4* s = reinterpret_cast<const u32x4*>(sbase) + i0;
    const u32x4* d = reinterpret_cast<const u32x4*>(dbase) + i0;
    bool live[U];
    u32x4 x[U], yv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t j = j0 + size_t(u) * kThreads;
        live[u] = j >= lead && j < lead + nvec;
        if (live[u]) x[u] = ld<false>(s + u * kThreads);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (live[u]) yv[u] = ld<NTO>(d + u * kThreads);
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (live[u]) x[u] = add_vec<DT>(x[u], yv[u]);
    uint32_t r = (blockIdx.x + y) % a.n;
    for (uint32_t k = 0; k < a.n; ++k) {
        u32x4* o = reinterpret_cast<u32x4*>(a.bufs[r] + byte_off) + i0;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (live[u]) st<NTS>(o + u * kThreads, x[u]);
        if (++r == a.n) r = 0;
    }
    // the ragged tail (fewer than 16 bytes, only the buffer's last chunk has one), element by element
    if (blockIdx.x == 0) {
        const size_t te = nvec * (16 / EB) + threadIdx.x;
        if (te < len) {
            uint32_t xt;
            if (DT == SAR_BF16)
                xt = bf16_rne(__uint_as_float(uint32_t(reinterpret_cast<const uint16_t*>(sbase)[te]) << 16) +
                              __uint_as_float(uint32_t(reinterpret_cast<const uint16_t*>(dbase)[te]) << 16));
            else
                xt = add_word<DT>(reinterpret_cast<const uint32_t*>(sbase)[te], reinterpret_cast<const uint32_t*>(dbase)[te]);
            for (uint32_t k = 0; k < a.n; ++k) {
                if (DT == SAR_BF16)
                    reinterpret_cast<uint16_t*>(a.bufs[k] + byte_off)[te] = uint16_t(xt);
                else
                    reinterpret_cast<uint32_t*>(a.bufs[k] + byte_off)[te] = xt;
            }
        }
    }
}

// The exchanges alone (the producing ops of a split completion): the sum goes back to the two
// ranks it came from.  The exchange's destination (the straggler's cell) is stored plainly - it
// is the cell the broadcast launch reads next (sar_sched::route) and nothing that touches it
// carries a hint (a hinted load of its old content made the broadcast's reads miss: 0.56 vs 0.31
// ms at 32 ranks) - while, with NT, the on-time rank's final copy is stored with the hint.
template <int DT, int U, bool NT, int CAP>
__global__ __launch_bounds__(kThreads) void exchange_kernel(const SumToAllArgsT<CAP> a) {
    constexpr size_t EB = (DT == SAR_BF16) ? 2 : 4;
    const uint32_t y = blockIdx.y + a.y0;
    const uint32_t route = a.route[y];
    const size_t first = size_t(y) * a.chunk_elems;
    size_t len = a.count - first;
    if (len > a.chunk_elems) len = a.chunk_elems;
    const size_t nvec = len * EB / 16;
    const size_t byte_off = first * EB;
    const size_t lead = ((reinterpret_cast<uintptr_t>(a.bufs[0]) + byte_off) & 127u) / 16;
    const size_t j0 = size_t(blockIdx.x) * (kThreads * U) + threadIdx.x;
    const size_t i0 = j0 - lead;
    char* sbase = a.bufs[route & 0xFFu] + byte_off;
    char* dbase = a.bufs[(route >> 8) & 0xFFu] + byte_off;
    u32x4* s = reinterpret_cast<u32x4*>(sbase) + i0;
    u32x4* d = reinterpret_cast<u32x4*>(dbase) + i0;
    bool live[U];
    u32x4 x[U], yv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t j = j0 + size_t(u) * kThreads;
        live[u] = j >= lead && j < lead + nvec;
        if (live[u]) x[u] = ld<false>(s + u * kThreads);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (live[u]) yv[u] = ld<false>(d + u * kThreads);
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (live[u]) x[u] = add_vec<DT>(x[u], yv[u]);
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (live[u]) st<false>(d + u * kThreads, x[u]);
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (live[u]) st<NT>(s + u * kThreads, x[u]);
    if (blockIdx.x == 0) {
        const size_t te = nvec * (16 / EB) + threadIdx.x;
        if (te < len) tail_elem<DT>(sbase, dbase, te, SAR_REDUCE_EXCHANGE);
    }
}

template <int DT, int CAP>
hipError_t launch_exchange(bool nt, dim3 grid, size_t lds, hipStream_t stream, const SumToAllArgsT<CAP>& args) {
    if (nt)
        hipLaunchKernelGGL((exchange_kernel<DT, 2, true, CAP>), grid, dim3(kThreads), lds, stream, args);
    else
        hipLaunchKernelGGL((exchange_kernel<DT, 2, false, CAP>), grid, dim3(kThreads), lds, stream, args);
    return hipGetLastError();
}

template <int DT, int U>
hipError_t launch_sum_to_all_nt(bool nt_other, bool nts, dim3 grid, size_t lds, hipStream_t stream, const SumToAllArgs& args) {
    if (nt_other && nts)
        hipLaunchKernelGGL((sum_to_all_kernel<DT, U, true, true>), grid, dim3(kThreads), lds, stream, args);
    else if (nt_other)
        hipLaunchKernelGGL((sum_to_all_kernel<DT, U, true, false>), grid, dim3(kThreads), lds, stream, args);
    else if (nts)
        hipLaunchKernelGGL((sum_to_all_kernel<DT, U, false, true>), grid, dim3(kThreads), lds, stream, args);
    else
        hipLaunchKernelGGL((sum_to_all_kernel<DT, U, false, false>), grid, dim3(kThreads), lds, stream, args);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_sum_to_all(int unroll, bool nt_other, bool nts, dim3 grid, size_t lds, hipStream_t stream, const SumToAllArgs& args) {
    switch (unroll) {
        case 1: return launch_sum_to_all_nt<DT, 1>(nt_other, nts, grid, lds, stream, args);
        case 2: return launch_sum_to_all_nt<DT, 2>(nt_other, nts, grid, lds, stream, args);
        default: return launch_sum_to_all_nt<DT, 4>(nt_other, nts, grid, lds, stream, args);
    }
}

// 8 tiles = 32 KiB runs per rank.  16 is level up to 40 ranks and behind where chunks are short and
// ranks many - the last segment of a chunk is padded to full length with workgroups that exit at
// once (128 ranks x 16 MiB: 0.50 vs 0.43 ms; 256 ranks x 4 MiB: 0.69 vs 0.37 ms); 32 and more lose.
constexpr uint32_t kSegmentTiles = 8;

// A split run goes through the chunk indices in groups, each group one producing launch and one
// broadcast launch: the broadcast reads what the producing launch stored last, and that has to be
// in the memory-side cache still - with the cells of ALL chunk indices (one rank buffer's worth)
// between the two, the broadcast of 16 ranks x 256 MiB took 1.12 ms instead of 0.63 ms.  Groups of
// at most 100 MiB of such cells, evenly sized: 64 MiB per rank stays one group, 128 MiB becomes
// two (24 ranks: 0.57 ms against 0.62 ms in one), 256 MiB three (group limits of 32 ... 128 MiB
// are within 5 % of each other there).
constexpr size_t kSplitGroupBytes = size_t(100) << 20;

int split_group_chunks(const sar_plan* plan, const sar_sched& sched) {
    const size_t total = sched.chunk_elems * plan->elem_bytes * size_t(sched.parts);
    const size_t groups = (total + kSplitGroupBytes - 1) / kSplitGroupBytes;
    return groups <= 1 ? sched.parts : std::max(1, int((size_t(sched.parts) + groups - 1) / groups));
}

// 4 KiB tiles per chunk (including up to 7 empty leading slots), and tiles per segment.  A chunk's
// last segment is padded to full length with workgroups that exit at once; for short chunks
// (under 64 tiles) that padding costs more than the L2 affinity of 8-tile segments brings, so
// their segments are as many as 8-tile ones would be but of even length (256 ranks x 16 MiB: 17
// tiles per chunk as 3 x 6 instead of 3 x 8, 1.02 -> 0.79 ms; 256 x 1 MiB: 1 tile, 0.36 -> 0.12 ms).
size_t broadcast_tiles(const sar_plan* plan, const sar_sched& sched) {
    return (sched.chunk_elems * plan->elem_bytes / 16 + 7 + kThreads - 1) / kThreads;
}
uint32_t broadcast_segment(size_t tiles) {
    if (tiles >= 64) return kSegmentTiles;
    const size_t segs = (tiles + kSegmentTiles - 1) / kSegmentTiles;
    return uint32_t((tiles + segs - 1) / segs);
}

// Grid of the broadcast launch; x == 0 if it does not fit the grid limits.
dim3 broadcast_grid(const sar_plan* plan, const sar_sched& sched) {
    const size_t tiles = broadcast_tiles(plan, sched);
    const size_t seg = broadcast_segment(tiles);
    const size_t segs = (tiles + seg - 1) / seg;
    const size_t x = segs * seg * size_t(sched.dests);
    if (x >= (size_t(1) << 31) || sched.parts > 65535) return dim3(0, 0);
    return dim3(static_cast<unsigned>(x), static_cast<unsigned>(sched.parts));
}

int run_broadcast(const sar_plan* plan, const sar_sched& sched, void* const* rank_bufs, hipStream_t stream,
                  const sar::LaunchShape& shape, int c0 = 0, int c1 = -1) {
    if (c1 < 0) c1 = sched.parts;
    BroadcastArgs args{};
    for (int i = 0; i < plan->n; ++i) args.bufs[i] = static_cast<char*>(rank_bufs[i]);
    for (int c = 0; c < sched.parts; ++c) args.route[c] = sched.route[c];
    args.dests = uint32_t(sched.dests);
    args.tiles = uint32_t(broadcast_tiles(plan, sched));
    args.seg = broadcast_segment(args.tiles);
    args.chunk_elems = sched.chunk_elems;
    args.count = plan->count;
    dim3 grid = broadcast_grid(plan, sched);
    grid.y = unsigned(c1 - c0);
    args.y0 = uint32_t(c0);
    hipError_t err;
    switch (plan->dtype) {
        case SAR_I32: err = launch_broadcast<SAR_I32>(shape.fused_nt_stores, grid, stream, args); break;
        case SAR_F32: err = launch_broadcast<SAR_F32>(shape.fused_nt_stores, grid, stream, args); break;
        default: err = launch_broadcast<SAR_BF16>(shape.fused_nt_stores, grid, stream, args); break;
    }
    return err == hipSuccess ? SAR_OK : SAR_EDEVICE;
}


// ---- reduce chains of one shape, without an op list --------------------------------------------
// A ring ReduceScatter (the precondition; the first half of the ring AllReduce) is the same walk
// for every chunk index, only started at another rank (sar_sched::chain_ring).  Described by the
// ring and one start position per chunk index it fits one launch's arguments at any rank count,
// where op lists of n to 2n ops per chunk index fill the 4 KiB after a few chunk indices - with
// 64 ranks the precondition is 1 launch instead of 9, with 256 ranks 1 instead of 85.  Operand
// loads go out four at a time, the additions follow in ring order.  ALL: the sum goes to every
// rank of the ring (the ring AllReduce in one launch), each workgroup starting at a different
// one; otherwise to the last rank of the walk only.
struct ChainArgs {
    char* bufs[SAR_MAX_RANKS];
    uint32_t ring[SAR_MAX_RANKS / 4];      // the cyclic rank order, four ranks to a word
    uint32_t start[SAR_MAX_RANKS / 2];     // per chunk index: ring position of its first operand, two to a word
    uint32_t m;                            // ranks in the ring
    uint32_t y0;                           // chunk index of blockIdx.y == 0
    uint64_t chunk_elems, count;
    __device__ uint32_t rank_at(uint32_t pos) const { return (ring[pos >> 2] >> ((pos & 3u) * 8)) & 0xFFu; }
};
static_assert(sizeof(ChainArgs) <= 4096, "kernel arguments are limited to 4 KiB");

template <int DT, int U, bool NTL, bool NTS, bool ALL>
__global__ __launch_bounds__(kThreads) void chain_kernel(const ChainArgs a) {
    constexpr size_t EB = (DT == SAR_BF16) ? 2 : 4;
    constexpr int kBatch = 4;
    const uint32_t y = blockIdx.y + a.y0;
    uint32_t pos = (a.start[y >> 1] >> ((y & 1u) * 16)) & 0xFFFFu;
    const size_t first = size_t(y) * a.chunk_elems;
    size_t len = a.count - first;
    if (len > a.chunk_elems) len = a.chunk_elems;
    const size_t nvec = len * EB / 16;
    const size_t byte_off = first * EB;
    const size_t lead = ((reinterpret_cast<uintptr_t>(a.bufs[0]) + byte_off) & 127u) / 16;
    const size_t j0 = size_t(blockIdx.x) * (kThreads * U) + threadIdx.x;
    const size_t i0 = j0 - lead;
    const size_t te = nvec * (16 / EB) + threadIdx.x;      // this thread's element of the ragged tail
    const bool tail = blockIdx.x == 0 && te < len;
    bool live[U];
    u32x4 x[U];
    uint32_t xt = 0;
    {
        const char* p0 = a.bufs[a.rank_at(pos)] + byte_off;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t j = j0 + size_t(u) * kThreads;
            live[u] = j >= lead && j < lead + nvec;
            if (live[u]) x[u] = ld<NTL>(reinterpret_cast<const u32x4*>(p0) + i0 + u * kThreads);
        }
        if (tail) xt = DT == SAR_BF16 ? uint32_t(reinterpret_cast<const uint16_t*>(p0)[te]) : reinterpret_cast<const uint32_t*>(p0)[te];
    }
    for (uint32_t left = a.m - 1; left > 0;) {
        const int run = left < uint32_t(kBatch) ? int(left) : kBatch;
        const char* base[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) base[k] = a.bufs[a.rank_at((pos + 1 + k) % a.m)] + byte_off;
        u32x4 operand[kBatch][U];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            if (k >= run) continue;
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (live[u]) operand[k][u] = ld<NTL>(reinterpret_cast<const u32x4*>(base[k]) + i0 + u * kThreads);
        }
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            if (k >= run) continue;
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (live[u]) x[u] = add_vec<DT>(x[u], operand[k][u]);
            if (tail) {
                if (DT == SAR_BF16)
                    xt = bf16_rne(__uint_as_float(xt << 16) + __uint_as_float(uint32_t(reinterpret_cast<const uint16_t*>(base[k])[te]) << 16));
                else
                    xt = add_word<DT>(xt, reinterpret_cast<const uint32_t*>(base[k])[te]);
            }
        }
        pos = (pos + run) % a.m;
        left -= run;
    }
    // pos: the last rank of the walk
    if (ALL) pos = (blockIdx.x + y) % a.m;
    for (uint32_t k = 0; k < (ALL ? a.m : 1u); ++k) {
        char* o = a.bufs[a.rank_at(pos)] + byte_off;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (live[u]) st<NTS>(reinterpret_cast<u32x4*>(o) + i0 + u * kThreads, x[u]);
        if (tail) {
            if (DT == SAR_BF16)
                reinterpret_cast<uint16_t*>(o)[te] = uint16_t(xt);
            else
                reinterpret_cast<uint32_t*>(o)[te] = xt;
        }
        if (++pos == a.m) pos = 0;
    }
}

template <int DT, int U, bool ALL>
hipError_t launch_chain_nt(bool ntl, bool nts, dim3 grid, size_t lds, hipStream_t stream, const ChainArgs& args) {
    if (ntl && nts)
        hipLaunchKernelGGL((chain_kernel<DT, U, true, true, ALL>), grid, dim3(kThreads), lds, stream, args);
    else if (ntl)
        hipLaunchKernelGGL((chain_kernel<DT, U, true, false, ALL>), grid, dim3(kThreads), lds, stream, args);
    else if (nts)
        hipLaunchKernelGGL((chain_kernel<DT, U, false, true, ALL>), grid, dim3(kThreads), lds, stream, args);
    else
        hipLaunchKernelGGL((chain_kernel<DT, U, false, false, ALL>), grid, dim3(kThreads), lds, stream, args);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_chain(int unroll, bool all, bool ntl, bool nts, dim3 grid, size_t lds, hipStream_t stream, const ChainArgs& args) {
    if (unroll >= 2)
        return all ? launch_chain_nt<DT, 2, true>(ntl, nts, grid, lds, stream, args) : launch_chain_nt<DT, 2, false>(ntl, nts, grid, lds, stream, args);
    return all ? launch_chain_nt<DT, 1, true>(ntl, nts, grid, lds, stream, args) : launch_chain_nt<DT, 1, false>(ntl, nts, grid, lds, stream, args);
}

// A chain-shaped schedule: in one launch, or - split - in groups of chunk indices, each group a
// chain launch that leaves the sum with the last rank of the walk and a broadcast launch.
int run_chains(const sar_plan* plan, const sar_sched& sched, void* const* rank_bufs, hipStream_t stream,
               const sar::LaunchShape& shape) {
    ChainArgs args{};
    for (int i = 0; i < plan->n; ++i) args.bufs[i] = static_cast<char*>(rank_bufs[i]);
    for (size_t k = 0; k < sched.chain_ring.size(); ++k) args.ring[k >> 2] |= uint32_t(sched.chain_ring[k]) << ((k & 3) * 8);
    for (int c = 0; c < sched.parts; ++c) args.start[c >> 1] |= uint32_t(sched.chain_start[c]) << ((c & 1) * 16);
    args.m = uint32_t(sched.chain_ring.size());
    args.chunk_elems = sched.chunk_elems;
    args.count = plan->count;
    const bool split = shape.fused_split && sched.chain_to_all;
    const int unroll = shape.fused_unroll >= 2 ? 2 : 1;
    const size_t slots = sched.chunk_elems * plan->elem_bytes / 16 + 7;
    const size_t per_block = size_t(kThreads) * unroll;
    const unsigned tiles = static_cast<unsigned>((slots + per_block - 1) / per_block);
    const size_t lds = lds_for_workgroups_per_cu(shape.fused_wgs_per_cu);
    const int group_chunks = split ? split_group_chunks(plan, sched) : sched.parts;
    for (int c0 = 0; c0 < sched.parts; c0 += group_chunks) {
        const int c1 = std::min(sched.parts, c0 + group_chunks);
        args.y0 = uint32_t(c0);
        const dim3 grid(tiles, static_cast<unsigned>(c1 - c0));
        const bool all = sched.chain_to_all && !split;
        // the chain launch of a split stores plainly: the broadcast launch reads that cell next
        const bool nts = shape.fused_nt_stores && !split;
        hipError_t err;
        switch (plan->dtype) {
            case SAR_I32: err = launch_chain<SAR_I32>(unroll, all, shape.fused_nt_loads, nts, grid, lds, stream, args); break;
            case SAR_F32: err = launch_chain<SAR_F32>(unroll, all, shape.fused_nt_loads, nts, grid, lds, stream, args); break;
            default: err = launch_chain<SAR_BF16>(unroll, all, shape.fused_nt_loads, nts, grid, lds, stream, args); break;
        }
        if (err != hipSuccess) return SAR_EDEVICE;
        if (split) {
            const int st = run_broadcast(plan, sched, rank_bufs, stream, shape, c0, c1);
            if (st != SAR_OK) return st;
        }
    }
    return SAR_OK;
}

template <int CAP>
void fill_sum_to_all(const sar_plan* plan, const sar_sched& sched, void* const* rank_bufs, SumToAllArgsT<CAP>& args) {
    for (int i = 0; i < plan->n; ++i) args.bufs[i] = static_cast<char*>(rank_bufs[i]);
    for (int c = 0; c < sched.parts; ++c) {
        const sar_chunk_op& exchange = sched.by_chunk[c][0];
        args.route[c] = uint32_t(exchange.src) | uint32_t(exchange.dst) << 8;
    }
    args.n = uint32_t(plan->n);
    args.chunk_elems = sched.chunk_elems;
    args.count = plan->count;
}

// The split form of a schedule whose chunk indices are each one exchange followed by copies: per
// group of chunk indices the exchange launch, then the broadcast launch.  One exchange launch
// covers all chunk indices of its group at any rank count (op lists would hold 32 per launch).
template <int CAP>
int run_exchange_broadcast(const sar_plan* plan, const sar_sched& sched, void* const* rank_bufs, hipStream_t stream,
                           const sar::LaunchShape& shape) {
    SumToAllArgsT<CAP> args{};
    fill_sum_to_all(plan, sched, rank_bufs, args);
    const size_t slots = sched.chunk_elems * plan->elem_bytes / 16 + 7;
    const size_t per_block = size_t(kThreads) * 2;      // 2 vectors per thread, 4 workgroups per compute unit (measured)
    const size_t lds = lds_for_workgroups_per_cu(4);
    const int per_group = split_group_chunks(plan, sched);
    for (int c0 = 0; c0 < sched.parts; c0 += per_group) {
        const int c1 = std::min(sched.parts, c0 + per_group);
        const dim3 grid(static_cast<unsigned>((slots + per_block - 1) / per_block), static_cast<unsigned>(c1 - c0));
        args.y0 = uint32_t(c0);
        hipError_t err;
        switch (plan->dtype) {
            case SAR_I32: err = launch_exchange<SAR_I32, CAP>(shape.fused_nt_stores, grid, lds, stream, args); break;
            case SAR_F32: err = launch_exchange<SAR_F32, CAP>(shape.fused_nt_stores, grid, lds, stream, args); break;
            default: err = launch_exchange<SAR_BF16, CAP>(shape.fused_nt_stores, grid, lds, stream, args); break;
        }
        if (err != hipSuccess) return SAR_EDEVICE;
        const int st = run_broadcast(plan, sched, rank_bufs, stream, shape, c0, c1);
        if (st != SAR_OK) return st;
    }
    return SAR_OK;
}

// The completion's shape in one launch (up to 32 ranks).
int run_sum_to_all(const sar_plan* plan, const sar_sched& sched, void* const* rank_bufs, hipStream_t stream,
                   const sar::LaunchShape& shape) {
    SumToAllArgs args{};
    fill_sum_to_all(plan, sched, rank_bufs, args);
    const size_t slots = sched.chunk_elems * plan->elem_bytes / 16 + 7;
    const size_t per_block = size_t(kThreads) * shape.fused_unroll;
    const dim3 grid(static_cast<unsigned>((slots + per_block - 1) / per_block), static_cast<unsigned>(sched.parts));
    const size_t lds = lds_for_workgroups_per_cu(shape.fused_wgs_per_cu);
    hipError_t err;
    switch (plan->dtype) {
        case SAR_I32: err = launch_sum_to_all<SAR_I32>(shape.fused_unroll, shape.fused_nt_other_load, shape.fused_nt_stores, grid, lds, stream, args); break;
        case SAR_F32: err = launch_sum_to_all<SAR_F32>(shape.fused_unroll, shape.fused_nt_other_load, shape.fused_nt_stores, grid, lds, stream, args); break;
        default: err = launch_sum_to_all<SAR_BF16>(shape.fused_unroll, shape.fused_nt_other_load, shape.fused_nt_stores, grid, lds, stream, args); break;
    }
    return err == hipSuccess ? SAR_OK : SAR_EDEVICE;
}

// Ops of chunk index c the op-list kernel runs: all of them, or the producing ones of a split.
size_t ops_to_run(const sar_sched& sched, int c, bool split) {
    return split ? size_t(sched.cut[c]) : sched.by_chunk[c].size();
}

template <int CAP>
int run_fused(const sar_plan* plan, const sar_sched& sched, void* const* rank_bufs, hipStream_t stream,
              const sar::LaunchShape& shape) {
    typedef FusedArgs<CAP> Args;
    constexpr int B = Args::kRankBits;
    Args args{};   // zeroed: the kernel reads a few op words past the last one it uses
    for (int i = 0; i < CAP; ++i) args.bufs[i] = i < plan->n ? rank_bufs[i] : nullptr;
    args.chunk_elems = sched.chunk_elems;
    args.count = plan->count;
    // slots per chunk: its vectors plus at most 7 empty leading slots
    const size_t slots = sched.chunk_elems * plan->elem_bytes / 16 + 7;
    const int unroll = shape.fused_unroll;
    const size_t lds = lds_for_workgroups_per_cu(shape.fused_wgs_per_cu);
    const size_t per_block = size_t(kThreads) * unroll;
    const unsigned tiles = static_cast<unsigned>((slots + per_block - 1) / per_block);

    const bool split = shape.fused_split;
    const int group_chunks = split ? split_group_chunks(plan, sched) : sched.parts;
    for (int g0 = 0; g0 < sched.parts; g0 += group_chunks) {
        const int g1 = std::min(sched.parts, g0 + group_chunks);
        int c = g0;
        while (c < g1) {
            int nchunks = 0, nops = 0;
            while (c + nchunks < g1 && nchunks < kMaxChunks &&
                   nops + int(ops_to_run(sched, c + nchunks, split)) <= Args::kMaxOps) {
                args.first[nchunks] = uint32_t(nops);
                const std::vector<sar_chunk_op>& ops = sched.by_chunk[c + nchunks];
                for (size_t k = 0; k < ops_to_run(sched, c + nchunks, split); ++k) {
                    const sar_chunk_op& op = ops[k];
                    args.set_op(nops++, uint32_t(op.src) | uint32_t(op.dst) << B | uint32_t(op.kind) << (2 * B) |
                                            uint32_t(op.forward) << (2 * B + 2) | uint32_t(op.dead) << (2 * B + 3) |
                                            uint32_t(op.chained && shape.fused_batch_chains) << (2 * B + 4));
                }
                ++nchunks;
            }
            if (nchunks == 0) return SAR_EINVAL;   // one chunk index with more ops than a launch carries
            args.first[nchunks] = uint32_t(nops);
            args.chunk0 = uint32_t(c);
            const dim3 grid(tiles, static_cast<unsigned>(nchunks));
            // the producing ops of a split store plainly: the broadcast launch reads that cell next
            if (launch<CAP>(plan->dtype, unroll, shape.fused_nt_loads, shape.fused_nt_stores && !split, grid, lds, stream, args) != hipSuccess)
                return SAR_EDEVICE;
            c += nchunks;
        }
        if (split) {
            const int st = run_broadcast(plan, sched, rank_bufs, stream, shape, g0, g1);
            if (st != SAR_OK) return st;
        }
    }
    return SAR_OK;
}

}  // namespace

bool sar::can_fuse(const sar_plan* plan, int which, bool chain) {
    const sar_sched& sched = plan->sched[which];
    const size_t cap = plan->n <= 32 ? FusedArgs<32>::kMaxOps : FusedArgs<256>::kMaxOps;
    // one workgroup per tile and no striding: the runtime's limit of 2^32 threads per grid
    // dimension bounds the chunk (64 GiB); larger ones take the per-round kernel, which strides
    if ((sched.chunk_elems * plan->elem_bytes / 16 + 7) / kThreads >= (size_t(1) << 24) - 1) return false;
    if (chain && !sched.chain_ring.empty()) return sched.parts <= 65535;     // no op lists involved
    bool any = false;        // a schedule without ops (the precondition of two ranks) has nothing to launch
    for (const std::vector<sar_chunk_op>& ops : sched.by_chunk) {
        if (ops.size() > cap) return false;
        any = any || !ops.empty();
    }
    return any;
}

bool sar::can_split(const sar_plan* plan, int which, bool chain) {
    const sar_sched& sched = plan->sched[which];
    return can_fuse(plan, which, chain) && !sched.cut.empty() && broadcast_grid(plan, sched).x != 0;
}

namespace {
template <int CAP>
int count_launches(const sar_sched& sched, bool split, int group_chunks) {
    int launches = 0;
    for (int g0 = 0; g0 < sched.parts; g0 += group_chunks) {
        const int g1 = std::min(sched.parts, g0 + group_chunks);
        for (int c = g0; c < g1; ++launches) {
            int nchunks = 0, nops = 0;
            while (c + nchunks < g1 && nchunks < kMaxChunks &&
                   nops + int(ops_to_run(sched, c + nchunks, split)) <= FusedArgs<CAP>::kMaxOps) {
                nops += int(ops_to_run(sched, c + nchunks, split));
                ++nchunks;
            }
            if (nchunks == 0) return 0;
            c += nchunks;
        }
        if (split) ++launches;      // the group's broadcast launch
    }
    return launches;
}

// The exchange launch instead of the op-list kernel for the producing ops of a split.
bool exchange_path(const sar_plan*, const sar_sched& sched, bool split) {
    return split && sched.sum_to_all;
}
}  // namespace

int sar::fused_launches(const sar_plan* plan, int which, bool split, bool direct) {
    const sar_sched& sched = plan->sched[which];
    const int group_chunks = split ? split_group_chunks(plan, sched) : sched.parts;
    if (exchange_path(plan, sched, split)) return 2 * ((sched.parts + group_chunks - 1) / group_chunks);
    if (direct && !sched.chain_ring.empty())       // the chain kernel: one launch, or a chain and a broadcast launch per group
        return split && sched.chain_to_all ? 2 * ((sched.parts + group_chunks - 1) / group_chunks) : 1;
    if (direct && !split) return 1;
    return plan->n <= 32 ? count_launches<32>(sched, split, group_chunks) : count_launches<256>(sched, split, group_chunks);
}

int sar::split_groups(const sar_plan* plan, int which) {
    const sar_sched& sched = plan->sched[which];
    const int group_chunks = split_group_chunks(plan, sched);
    return (sched.parts + group_chunks - 1) / group_chunks;
}

int sar::run_schedule_fused(const sar_plan* plan, int which, void* const* rank_bufs, void* hip_stream,
                            const LaunchShape& shape) {
    const sar_sched& sched = plan->sched[which];
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (exchange_path(plan, sched, shape.fused_split))
        return plan->n <= 32 ? run_exchange_broadcast<32>(plan, sched, rank_bufs, stream, shape)
                             : run_exchange_broadcast<SAR_MAX_RANKS>(plan, sched, rank_bufs, stream, shape);
    if (shape.fused_sum_to_all && !shape.fused_split) return run_sum_to_all(plan, sched, rank_bufs, stream, shape);
    if (shape.fused_chain) return run_chains(plan, sched, rank_bufs, stream, shape);
    if (plan->n <= 32) return run_fused<32>(plan, sched, rank_bufs, stream, shape);
    return run_fused<256>(plan, sched, rank_bufs, stream, shape);
}
