// Diagnostic, not part of the library: how does this GPU's HBM take K write streams at once?
//
// The single-launch completion stores every tile of a reduced chunk to all n rank
// buffers (Alg. 1: after its straggler pairing a chunk only has to reach every
// rank).  Done from one workgroup per tile, that is n write streams advancing in
// lockstep.  This probe writes the same total number of bytes (2 GiB by default)
// as K such streams - K separately allocated buffers, each workgroup storing one
// 4 KiB tile to each of them, non-temporal 16-byte stores - for K = 1 ... 32, at
// two occupancies.  K = 1 is plain sequential writing.  The result motivates
// running the completion's copies rank by rank from 16 ranks on.
//
// usage: store_streams_probe [total MiB]        (needs about 2 x total of free HBM)
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                          \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) {                                                           \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);    \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)

struct Streams {
    u32x4* base[32];
    int k;
};

// One workgroup: tile blockIdx.x (256 threads x 16 bytes) of every stream.
__global__ __launch_bounds__(256) void write_streams(const Streams s) {
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    const u32x4 v = u32x4{uint32_t(i), 1u, 2u, 3u};
    for (int k = 0; k < s.k; ++k) __builtin_nontemporal_store(v, s.base[k] + i);
}

int main(int argc, char** argv) {
    const size_t total = (argc > 1 ? strtoull(argv[1], nullptr, 10) : 2048) << 20;
    void* arena[32];
    for (int k = 0; k < 32; ++k) {     // 32 buffers of total / 32 ... and fewer, larger ones reuse them in groups
        CHECK(hipMalloc(&arena[k], total / 32));
        CHECK(hipMemset(arena[k], 0, total / 32));
    }
    void* big = nullptr;               // K = 1 ... 16 need longer streams than total / 32: carve them from one block
    CHECK(hipMalloc(&big, total));
    CHECK(hipMemset(big, 0, total));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    std::printf("write-only, %zu MiB in all, K streams of %zu / K MiB, one 4 KiB tile of every stream per workgroup\n", total >> 20, total >> 20);
    for (int K : {1, 2, 4, 8, 16, 32}) {
        Streams s;
        s.k = K;
        const size_t per_stream = total / K;
        for (int k = 0; k < K; ++k)
            s.base[k] = K == 32 ? static_cast<u32x4*>(arena[k]) : reinterpret_cast<u32x4*>(static_cast<char*>(big) + per_stream * k);
        const unsigned tiles = unsigned(per_stream / 4096);
        for (int wgs : {2, 4, 8}) {    // resident workgroups per compute unit, capped through unused dynamic LDS
            const size_t lds = wgs == 2 ? 65536 : wgs == 4 ? 40960 : 0;
            float best = 1e9f;
            for (int rep = 0; rep < 5; ++rep) {
                CHECK(hipEventRecord(e0, nullptr));
                hipLaunchKernelGGL(write_streams, dim3(tiles), dim3(256), lds, nullptr, s);
                CHECK(hipEventRecord(e1, nullptr));
                CHECK(hipEventSynchronize(e1));
                float ms = 0;
                CHECK(hipEventElapsedTime(&ms, e0, e1));
                best = std::min(best, ms);
            }
            CHECK(hipGetLastError());
            std::printf("K = %2d  %d workgroups per CU : %.4f ms  %5.0f GB/s  (%.3f of 8 TB/s)\n", K, wgs, best, total / best / 1e6, total / best / 1e6 / 8000);
        }
    }
    return 0;
}
