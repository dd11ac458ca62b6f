// Pieces shared by the product kernels that load straight from global memory into LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "gemm_common.hpp"

namespace nnt {

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* glb_void_ptr;

// s_waitcnt immediate (gfx9 encoding) that constrains only vmcnt
constexpr int wait_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

// A chunk descriptor in scalar registers.  The descriptor tables are constant for the lifetime of
// a launch, but the compiler cannot know that next to the loads that write LDS, so the scalar
// loads are spelled out.
struct ChunkS {
    uint64_t A, B;
    int64_t lda, ldb, strideA, strideB;
    int32_t k, vec_ok;
    int64_t strideA2, strideB2;
};
static_assert(sizeof(ChunkS) == sizeof(GemmChunk) && sizeof(GemmChunk) == 72, "descriptor layout");

__device__ __forceinline__ ChunkS sload_chunk(const GemmChunk* p) {
    typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    u32x8 a;
    u32x4 b, d;
    u32x2 c;
    asm volatile("s_load_dwordx8 %0, %4, 0x0\n\ts_load_dwordx4 %1, %4, 0x20\n\ts_load_dwordx2 %2, %4, 0x30\n\ts_load_dwordx4 %3, %4, 0x38\n\ts_waitcnt lgkmcnt(0)"
                 : "=&s"(a), "=&s"(b), "=&s"(c), "=&s"(d)
                 : "s"(p)
                 : "memory");
    ChunkS r;
    r.A = a[0] | ((uint64_t)a[1] << 32);
    r.B = a[2] | ((uint64_t)a[3] << 32);
    r.lda = (int64_t)(a[4] | ((uint64_t)a[5] << 32));
    r.ldb = (int64_t)(a[6] | ((uint64_t)a[7] << 32));
    r.strideA = (int64_t)(b[0] | ((uint64_t)b[1] << 32));
    r.strideB = (int64_t)(b[2] | ((uint64_t)b[3] << 32));
    r.k = (int32_t)c[0];
    r.vec_ok = (int32_t)c[1];
    r.strideA2 = (int64_t)(d[0] | ((uint64_t)d[1] << 32));
    r.strideB2 = (int64_t)(d[2] | ((uint64_t)d[3] << 32));
    return r;
}

// LDS reads of the pipeline are spelled as inline assembly: the compiler treats every LDS read
// it knows of as possibly touching what the in-flight global->LDS loads write and would wait for
// all of them (vmcnt 0) first, which is exactly what the stages are there to avoid.  The price is
// that the waits for these reads are ours too (wait_frags).
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

}  // namespace nnt
