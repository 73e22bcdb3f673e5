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
// Grid: blockIdx.y picks the op, blockIdx.x strides over that op's chunk.  The
// rank pointers and the packed op list travel in the kernel arguments, so a
// launch needs no device-side tables and the library never allocates device
// memory.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "plan.hpp"
#include "launch.hpp"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

template <int CAP>
struct RoundArgs {
    void* bufs[CAP];        // device pointer of each physical rank's buffer
    uint32_t ops[CAP];      // src | dst << 8 | chunk << 16 | kind << 24
    uint64_t chunk_elems;   // elements per chunk
    uint64_t count;         // elements per rank buffer
};

// ---- arithmetic on one 16-byte vector --------------------------------------
template <int DT>
__device__ __forceinline__ uint32_t add_word(uint32_t a, uint32_t b);

template <>
__device__ __forceinline__ uint32_t add_word<SAR_I32>(uint32_t a, uint32_t b) {
    return a + b;
}

template <>
__device__ __forceinline__ uint32_t add_word<SAR_F32>(uint32_t a, uint32_t b) {
    return __float_as_uint(__uint_as_float(a) + __uint_as_float(b));
}

// fp32 -> bf16 bits, round to nearest even; NaN stays a quiet NaN
__device__ __forceinline__ uint32_t bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    const uint32_t quiet = (u >> 16) | 0x40u;
    return (u & 0x7FFFFFFFu) > 0x7F800000u ? quiet : rounded;
}

template <>
__device__ __forceinline__ uint32_t add_word<SAR_BF16>(uint32_t a, uint32_t b) {
    const float lo = __uint_as_float(a << 16) + __uint_as_float(b << 16);
    const float hi = __uint_as_float(a & 0xFFFF0000u) + __uint_as_float(b & 0xFFFF0000u);
    return bf16_rne(lo) | (bf16_rne(hi) << 16);
}

template <int DT>
__device__ __forceinline__ u32x4 add_vec(u32x4 a, u32x4 b) {
    u32x4 r;
    r.x = add_word<DT>(a.x, b.x);
    r.y = add_word<DT>(a.y, b.y);
    r.z = add_word<DT>(a.z, b.z);
    r.w = add_word<DT>(a.w, b.w);
    return r;
}

template <int NT>
__device__ __forceinline__ u32x4 ld(const u32x4* p) {
    if (NT >= 2) return __builtin_nontemporal_load(p);
    return *p;
}

template <int NT>
__device__ __forceinline__ void st(u32x4* p, u32x4 v) {
    if (NT >= 1)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// One element of the ragged tail (fewer than 16 bytes), in the element type.
template <int DT>
__device__ __forceinline__ void tail_elem(char* s, char* d, size_t e, int kind) {
    if (DT == SAR_BF16) {
        uint16_t* sp = reinterpret_cast<uint16_t*>(s) + e;
        uint16_t* dp = reinterpret_cast<uint16_t*>(d) + e;
        if (kind == SAR_COPY) {
            *dp = *sp;
        } else {
            const float t = __uint_as_float(uint32_t(*sp) << 16) + __uint_as_float(uint32_t(*dp) << 16);
            const uint16_t v = uint16_t(bf16_rne(t));
            *dp = v;
            if (kind == SAR_REDUCE_EXCHANGE) *sp = v;
        }
    } else {
        uint32_t* sp = reinterpret_cast<uint32_t*>(s) + e;
        uint32_t* dp = reinterpret_cast<uint32_t*>(d) + e;
        if (kind == SAR_COPY) {
            *dp = *sp;
        } else {
            const uint32_t v = add_word<DT>(*sp, *dp);
            *dp = v;
            if (kind == SAR_REDUCE_EXCHANGE) *sp = v;
        }
    }
}

template <int DT, int CAP, int U, int NT>
__global__ __launch_bounds__(kThreads) void round_kernel(const RoundArgs<CAP> a) {
    constexpr size_t EB = (DT == SAR_BF16) ? 2 : 4;
    const uint32_t op = a.ops[blockIdx.y];
    const int kind = int(op >> 24);
    const size_t first = size_t((op >> 16) & 0xFFu) * a.chunk_elems;
    size_t len = a.count - first;
    if (len > a.chunk_elems) len = a.chunk_elems;

    char* sbase = static_cast<char*>(a.bufs[op & 0xFFu]) + first * EB;
    char* dbase = static_cast<char*>(a.bufs[(op >> 8) & 0xFFu]) + first * EB;
    u32x4* __restrict__ s = reinterpret_cast<u32x4*>(sbase);
    u32x4* __restrict__ d = reinterpret_cast<u32x4*>(dbase);

    const size_t nvec = len * EB / 16;
    const size_t step = size_t(gridDim.x) * (kThreads * U);
    size_t i = size_t(blockIdx.x) * (kThreads * U) + threadIdx.x;

    // full steps: U vectors per thread, no bounds checks
    for (; i + size_t(U - 1) * kThreads < nvec; i += step) {
        u32x4 x[U], y[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = ld<NT>(s + i + u * kThreads);
        if (kind != SAR_COPY) {
#pragma unroll
            for (int u = 0; u < U; ++u) y[u] = ld<NT>(d + i + u * kThreads);
#pragma unroll
            for (int u = 0; u < U; ++u) x[u] = add_vec<DT>(x[u], y[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) st<NT>(d + i + u * kThreads, x[u]);
        if (kind == SAR_REDUCE_EXCHANGE) {
#pragma unroll
            for (int u = 0; u < U; ++u) st<NT>(s + i + u * kThreads, x[u]);
        }
    }
    // the last, partial step of this block
    for (; i < nvec; i += kThreads) {
        u32x4 x = ld<NT>(s + i);
        if (kind != SAR_COPY) x = add_vec<DT>(x, ld<NT>(d + i));
        st<NT>(d + i, x);
        if (kind == SAR_REDUCE_EXCHANGE) st<NT>(s + i, x);
    }
    // elements past the last whole vector (only the buffer's final chunk can have any)
    if (blockIdx.x == 0) {
        const size_t done = nvec * (16 / EB);
        if (done + threadIdx.x < len) tail_elem<DT>(sbase, dbase, done + threadIdx.x, kind);
    }
}

template <int DT, int CAP, int U>
hipError_t launch_nt(int nt, dim3 grid, hipStream_t stream, const RoundArgs<CAP>& args) {
    switch (nt) {
        case 0: hipLaunchKernelGGL((round_kernel<DT, CAP, U, 0>), grid, dim3(kThreads), 0, stream, args); break;
        case 1: hipLaunchKernelGGL((round_kernel<DT, CAP, U, 1>), grid, dim3(kThreads), 0, stream, args); break;
        default: hipLaunchKernelGGL((round_kernel<DT, CAP, U, 2>), grid, dim3(kThreads), 0, stream, args); break;
    }
    return hipGetLastError();
}

template <int DT, int CAP>
hipError_t launch_u(int unroll, int nt, dim3 grid, hipStream_t stream, const RoundArgs<CAP>& args) {
    switch (unroll) {
        case 1: return launch_nt<DT, CAP, 1>(nt, grid, stream, args);
        case 2: return launch_nt<DT, CAP, 2>(nt, grid, stream, args);
        case 4: return launch_nt<DT, CAP, 4>(nt, grid, stream, args);
        default: return launch_nt<DT, CAP, 8>(nt, grid, stream, args);
    }
}

template <int CAP>
hipError_t launch_dt(int dtype, int unroll, int nt, dim3 grid, hipStream_t stream, const RoundArgs<CAP>& args) {
    switch (dtype) {
        case SAR_I32: return launch_u<SAR_I32, CAP>(unroll, nt, grid, stream, args);
        case SAR_F32: return launch_u<SAR_F32, CAP>(unroll, nt, grid, stream, args);
        default: return launch_u<SAR_BF16, CAP>(unroll, nt, grid, stream, args);
    }
}

template <int CAP>
int run_rounds(const sar_plan* plan, const sar_sched& sched, void* const* rank_bufs, hipStream_t stream,
               const sar::LaunchShape& shape) {
    RoundArgs<CAP> args;
    for (int i = 0; i < CAP; ++i) {
        args.bufs[i] = i < plan->n ? rank_bufs[i] : nullptr;
        args.ops[i] = 0;
    }
    args.chunk_elems = sched.chunk_elems;
    args.count = plan->count;

    const size_t vec_per_chunk = sched.chunk_elems * plan->elem_bytes / 16;
    const size_t per_block = size_t(kThreads) * shape.unroll;
    const size_t max_bx = (vec_per_chunk + per_block - 1) / per_block;

    for (const std::vector<sar_op>& ops : sched.rounds) {
        const int nops = int(ops.size());
        if (nops == 0) continue;
        for (int k = 0; k < nops; ++k)
            args.ops[k] = uint32_t(ops[k].src) | uint32_t(ops[k].dst) << 8 | uint32_t(ops[k].chunk) << 16 |
                          uint32_t(ops[k].op) << 24;
        size_t bx = (size_t(shape.total_blocks) + nops - 1) / nops;
        if (bx > max_bx) bx = max_bx;
        if (bx < 1) bx = 1;
        const dim3 grid(static_cast<unsigned>(bx), static_cast<unsigned>(nops));
        if (launch_dt<CAP>(plan->dtype, shape.unroll, shape.nontemporal, grid, stream, args) != hipSuccess)
            return SAR_EDEVICE;
    }
    return SAR_OK;
}

}  // namespace

int sar::run_schedule(const sar_plan* plan, int which, void* const* rank_bufs, void* hip_stream,
                      const LaunchShape& shape) {
    const sar_sched& sched = plan->sched[which];
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (plan->n <= 32) return run_rounds<32>(plan, sched, rank_bufs, stream, shape);
    return run_rounds<SAR_MAX_RANKS>(plan, sched, rank_bufs, stream, shape);
}

int sar::device_compute_units(int* out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SAR_EDEVICE;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return SAR_EDEVICE;
    *out = cus;
    return SAR_OK;
}
