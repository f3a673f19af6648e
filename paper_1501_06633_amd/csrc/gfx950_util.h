// Small gfx950 device helpers shared by the kernel translation units: vector
// types, a compile-time loop, LDS reads and counter waits issued through inline
// asm, a fence-free workgroup barrier, and division by an invariant.
#ifndef MDNN_GFX950_UTIL_H_
#define MDNN_GFX950_UTIL_H_

#include <hip/hip_runtime.h>

#include <stdint.h>
#include <type_traits>
#include <utility>

namespace mdnn {

typedef float    f32x16 __attribute__((ext_vector_type(16)));
typedef float    f32x4  __attribute__((ext_vector_type(4)));
typedef float    f32x2  __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2  __attribute__((ext_vector_type(2)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

constexpr uint32_t kOutOfRange = 0xFFFFFFFFu;   // beyond any buffer of < 2^32 bytes
constexpr int      kRsrcWord3  = 0x00020000;    // raw 32-bit-data buffer descriptor, gfx9 family

// ---- compile-time loop (asm immediates must be constants)
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// ---- LDS reads the compiler does not see as LDS reads (see header comment)
template <int OFF> __device__ __forceinline__ void lds_read(float& v, uint32_t addr)
{
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
}
template <int OFF> __device__ __forceinline__ void lds_read(f32x2& v, uint32_t addr)
{
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
}
template <int OFF> __device__ __forceinline__ void lds_read(f32x4& v, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
}
template <int OFF> __device__ __forceinline__ void lds_read(u32x2& v, uint32_t addr)
{
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
}
// Wait until at most N LDS operations are outstanding.  The registers that the
// awaited reads fill are threaded through as in/out operands so that nothing
// that consumes them can be scheduled above the wait.
template <int N, class T> __device__ __forceinline__ void lds_wait(T& a)
{
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(N));
}
template <int N, class T, class U> __device__ __forceinline__ void lds_wait(T& a, U& b)
{
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N));
}
template <int N, class T, class U, class V> __device__ __forceinline__ void lds_wait(T& a, U& b, V& c)
{
    asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(a), "+v"(b), "+v"(c) : "n"(N));
}
template <int N, class T, class U, class V, class W>
__device__ __forceinline__ void lds_wait(T& a, U& b, V& c, W& d)
{
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}
template <int N, class T, class U, class V, class W, class X>
__device__ __forceinline__ void lds_wait(T& a, U& b, V& c, W& d, X& e)
{
    asm volatile("s_waitcnt lgkmcnt(%5)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(e) : "n"(N));
}
template <int N> __device__ __forceinline__ void vmem_wait()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// Workgroup barrier without the memory fence __syncthreads() carries: the fence
// would make the compiler drain every outstanding global -> LDS copy here.  The
// waits that matter are placed by hand around it.
__device__ __forceinline__ void bare_barrier()
{
    asm volatile("s_barrier" ::: "memory");
}

// n / d for an invariant d whose (magic, shift) the host prepared; exact for n < 2^32
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t magic, uint32_t shift)
{
    if (magic == 0) return n;                               // d == 1
    const uint32_t t = __umulhi(n, magic);
    return (t + ((n - t) >> 1)) >> shift;
}

}  // namespace mdnn
#endif
