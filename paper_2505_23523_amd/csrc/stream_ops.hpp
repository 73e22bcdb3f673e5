// Device-side building blocks shared by the kernels: 16-byte vector access with
// optional non-temporal hints, and the per-op arithmetic of each dtype.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "stragglar.h"

namespace sar {
namespace dev {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

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

// fp32 -> bf16 bits, round to nearest even, NaN stays a quiet NaN: the conversion the
// language defines for __bf16, which gfx950 has as one instruction for a pair of floats
// (v_cvt_pk_bf16_f32).  Done with integer arithmetic instead it costs four times the
// instructions, and the reducing kernels then stop being purely memory-bound for bf16.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t bf16_rne(float f) {
    return uint32_t(__builtin_bit_cast(uint16_t, static_cast<__bf16>(f)));
}

template <>
__device__ __forceinline__ uint32_t add_word<SAR_BF16>(uint32_t a, uint32_t b) {
    f32x2 sum;
    sum.x = __uint_as_float(a << 16) + __uint_as_float(b << 16);
    sum.y = __uint_as_float(a & 0xFFFF0000u) + __uint_as_float(b & 0xFFFF0000u);
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(sum, bf16x2));
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

// The non-temporal hint must be a compile-time property of the access: a
// run-time "if (nt) hinted else plain" pair is merged by the optimiser into one
// plain access.
template <bool NT>
__device__ __forceinline__ u32x4 ld(const u32x4* p) {
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

template <bool NT>
__device__ __forceinline__ void st(u32x4* p, u32x4 v) {
    if (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
}

// The store of a copy that streams a whole chunk to one other rank buffer (one launch per round):
// the non-temporal hint together with the SC1 scope bit.  A 1 GiB device copy of random data runs
// at 6.47 TB/s with loads and stores hinted `nt` and at 6.69 TB/s with the stores `sc1 nt`; the
// completion's rounds gain 2.5 % at 256 MiB per rank.  The compiler has no builtin for the scope
// bits of a plain vector store, hence the instruction by hand (a vector store; the wait states
// after it cover the rule that a wide store's data registers are not overwritten at once).
// Not for stores that fan one value out to many ranks: those lose up to 30 % with it.
template <bool NT>
__device__ __forceinline__ void st_stream(u32x4* p, u32x4 v) {
    if (NT)
        asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
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

}  // namespace dev
}  // namespace sar
