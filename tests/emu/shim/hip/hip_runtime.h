// CPU emulation of the small part of HIP that libvadusa uses: every GPU thread is an OS
// thread, blocks run one after another, wave collectives are rendezvous between lanes.
#pragma once
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <tuple>
#include <utility>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __shared__ static
#define __launch_bounds__(...)
#define __HIP_MEMORY_SCOPE_AGENT 4
#define __HIP_MEMORY_SCOPE_WORKGROUP 2
#define __HIP_MEMORY_SCOPE_SYSTEM 5

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {}
};
struct alignas(8) uint2 { uint32_t x, y; };
struct alignas(16) uint4 { uint32_t x, y, z, w; };
struct alignas(8) float2 { float x, y; };
struct alignas(16) float4 { float x, y, z, w; };
static inline uint2 make_uint2(uint32_t a, uint32_t b) { return uint2{a, b}; }
static inline uint4 make_uint4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) { return uint4{a, b, c, d}; }
static inline float2 make_float2(float a, float b) { return float2{a, b}; }
static inline float4 make_float4(float a, float b, float c, float d) { return float4{a, b, c, d}; }

extern thread_local dim3 threadIdx, blockIdx;
extern dim3 blockDim, gridDim;
extern thread_local const char* emu_where;   // last collective reached (file:line)
extern thread_local int emu_line;
extern char* emu_dyn_lds;

typedef void* hipStream_t;
typedef int hipError_t;
enum { hipSuccess = 0, hipErrorUnknown = 999 };
enum hipMemcpyKind { hipMemcpyHostToDevice, hipMemcpyDeviceToHost, hipMemcpyDeviceToDevice, hipMemcpyDefault };
enum { hipFuncAttributeMaxDynamicSharedMemorySize = 8 };
struct hipDeviceProp_t { int multiProcessorCount; int cooperativeLaunch; };
static inline hipError_t hipMemcpy(void* d, const void* s, size_t n, hipMemcpyKind) { memcpy(d, s, n); return 0; }
static inline hipError_t hipMemcpyAsync(void* d, const void* s, size_t n, hipMemcpyKind, hipStream_t) { memcpy(d, s, n); return 0; }
static inline hipError_t hipMemset(void* d, int v, size_t n) { memset(d, v, n); return 0; }
static inline hipError_t hipMemsetAsync(void* d, int v, size_t n, hipStream_t) { memset(d, v, n); return 0; }
static inline hipError_t hipStreamSynchronize(hipStream_t) { return 0; }
static inline hipError_t hipGetLastError() { return 0; }
static inline const char* hipGetErrorString(hipError_t) { return "emu"; }
static inline hipError_t hipGetDevice(int* d) { *d = 0; return 0; }
#ifndef __align__
#define __align__(n) __attribute__((aligned(n)))
#endif
#define HIP_SYMBOL(x) (&(x))
static inline hipError_t hipGetSymbolAddress(void** p, const void* sym) { *p = (void*)sym; return 0; }
static inline hipError_t hipGetDeviceProperties(hipDeviceProp_t* p, int) {
    const char* e = getenv("EMU_CUS");
    p->multiProcessorCount = e ? atoi(e) : 1;
    p->cooperativeLaunch = 1;
    return 0;
}
enum { hipErrorCooperativeLaunchTooLarge = 720 };
template <class F> static inline hipError_t hipOccupancyMaxActiveBlocksPerMultiprocessor(int* n, F, int, size_t) { *n = 1; return 0; }
static inline hipError_t hipFuncSetAttribute(const void*, int, int) { return 0; }

// ---- launch ----
void emu_launch(const std::function<void()>& body, dim3 grid, dim3 block, size_t shmem, bool coop);
template <class... KA, class... A>
void hipLaunchKernelGGL(void (*k)(KA...), dim3 grid, dim3 block, size_t shmem, hipStream_t, A&&... a) {
    std::tuple<KA...> args(std::forward<A>(a)...);
    emu_launch([=]() { std::apply(k, args); }, grid, block, shmem, false);
}
template <class P>
hipError_t emu_launch_coop(void (*k)(P), dim3 grid, dim3 block, void** args, size_t shmem) {
    P p = *(P*)args[0];
    emu_launch([=]() { k(p); }, grid, block, shmem, true);
    return 0;
}

// ---- block / wave collectives ----
void emu_syncthreads();
uint32_t emu_shfl_xor32(uint32_t v, int mask);
uint32_t emu_shfl_down32(uint32_t v, int delta);
void emu_mfma_16x16x32_bf16(const uint16_t a[8], const uint16_t b[8], float c[4]);
long long emu_clock();
#define EMU_MARK (emu_where = __FILE__, emu_line = __LINE__)
#define __syncthreads() (EMU_MARK, emu_syncthreads())
template <class T> static inline T emu_shfl_xor_t(T v, int m) {
    static_assert(sizeof(T) == 4, "32-bit shuffles only");
    uint32_t u; memcpy(&u, &v, 4); u = emu_shfl_xor32(u, m); memcpy(&v, &u, 4); return v;
}
template <class T> static inline T emu_shfl_down_t(T v, int m) {
    uint32_t u; memcpy(&u, &v, 4); u = emu_shfl_down32(u, m); memcpy(&v, &u, 4); return v;
}
#define __shfl_xor(v, m, w) (EMU_MARK, emu_shfl_xor_t(v, m))
#define __shfl_down(v, m, w) (EMU_MARK, emu_shfl_down_t(v, m))
uint32_t emu_shfl_idx32(uint32_t v, int src);
template <class T> static inline T emu_shfl_idx_t(T v, int src) {
    uint32_t u; memcpy(&u, &v, 4); u = emu_shfl_idx32(u, src); memcpy(&v, &u, 4); return v;
}
int emu_all(int pred);
#define __all(p) (EMU_MARK, emu_all(p))
#define __shfl(v, src, w) (EMU_MARK, emu_shfl_idx_t(v, src))
static inline void __threadfence() { std::atomic_thread_fence(std::memory_order_seq_cst); }
static inline long long wall_clock64() { return emu_clock(); }
#define __builtin_amdgcn_s_sleep(n) emu_yield()
void emu_yield();

typedef __attribute__((ext_vector_type(8))) __bf16 emu_bf16x8;
typedef __attribute__((ext_vector_type(4))) float emu_f32x4;
static inline emu_f32x4 emu_mfma(emu_bf16x8 a, emu_bf16x8 b, emu_f32x4 c) {
    uint16_t ua[8], ub[8]; float fc[4];
    memcpy(ua, &a, 16); memcpy(ub, &b, 16); memcpy(fc, &c, 16);
    emu_mfma_16x16x32_bf16(ua, ub, fc);
    emu_f32x4 r; memcpy(&r, fc, 16); return r;
}
#define __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, x, y, z) (EMU_MARK, emu_mfma(a, b, c))

// ---- atomics ----
template <class T> static inline void emu_atomic_store(T* p, T v) { __atomic_store(p, &v, __ATOMIC_RELAXED); }
template <class T> static inline T emu_atomic_load(const T* p) { T v; __atomic_load(const_cast<T*>(p), &v, __ATOMIC_RELAXED); return v; }
#define __hip_atomic_store(p, v, o, s) emu_atomic_store(p, (__typeof__(*(p)))(v))
#define __hip_atomic_load(p, o, s) emu_atomic_load(p)
#define __hip_atomic_fetch_add(p, v, o, s) __atomic_fetch_add(p, v, __ATOMIC_SEQ_CST)

static inline int atomicAdd(int* p, int v) { return __atomic_fetch_add(p, v, __ATOMIC_SEQ_CST); }

#define __builtin_amdgcn_readfirstlane(x) (x)
// every lane reads lane l of its wave
#define __builtin_amdgcn_readlane(v, l) (EMU_MARK, (int)emu_shfl_idx32((uint32_t)(v), (l)))
// DPP lane permutations used by the kernels (full row and bank masks): quad_perm [1,0,3,2],
// quad_perm [2,3,0,1], row_half_mirror, row_mirror are the pairwise exchanges lane ^ 1, ^ 2, ^ 7, ^ 15
static inline int emu_dpp_mask(int ctrl) {
    switch (ctrl) {
    case 0xB1: return 1;
    case 0x4E: return 2;
    case 0x141: return 7;
    case 0x140: return 15;
    default: __builtin_trap();
    }
}
#define __builtin_amdgcn_update_dpp(old, v, ctrl, rm, bm, bc) \
    (EMU_MARK, (int)emu_shfl_xor32((uint32_t)(v), emu_dpp_mask(ctrl)))

// Row swaps of gfx950 (v_permlane16_swap / v_permlane32_swap): the first operand's odd rows (upper halves) change
// places with the second operand's even rows (lower halves); a row is 16 lanes (a half 32).  First result: the new
// first operand (a lane of an odd row holds the second operand of the lane `bit` below), second result: the new second
// operand (a lane of an even row holds the first operand of the lane `bit` above).
typedef unsigned int emu_u32x2 __attribute__((ext_vector_type(2)));
static inline emu_u32x2 emu_permlane_swap(uint32_t a, uint32_t b, int bit) {
    const int lane = (int)(threadIdx.x & 63);
    const uint32_t b_below = emu_shfl_idx32(b, lane & ~bit), a_above = emu_shfl_idx32(a, lane | bit);
    emu_u32x2 r;
    r.x = (lane & bit) ? b_below : a;
    r.y = (lane & bit) ? b : a_above;
    return r;
}
#define __builtin_amdgcn_permlane16_swap(a, b, fi, bc) (EMU_MARK, emu_permlane_swap((a), (b), 16))
#define __builtin_amdgcn_permlane32_swap(a, b, fi, bc) (EMU_MARK, emu_permlane_swap((a), (b), 32))

// ---- math / bits ----
static inline float __uint_as_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static inline uint32_t __float_as_uint(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static inline float __int_as_float(int u) { float f; memcpy(&f, &u, 4); return f; }
static inline int __float_as_int(float f) { int u; memcpy(&u, &f, 4); return u; }
#define __expf(x) expf(x)
static inline float __frcp_rn(float x) { return 1.0f / x; }
static inline float __builtin_amdgcn_rcpf(float x) { return 1.0f / x; }
static inline float rsqrtf(float x) { return 1.0f / sqrtf(x); }
static inline int min(int a, int b) { return a < b ? a : b; }
static inline int max(int a, int b) { return a > b ? a : b; }
