// CPU stand-in for the parts of the HIP runtime and device language that
// libprep uses.  TEST INFRASTRUCTURE ONLY: it lets the kernels' source be
// compiled by g++ and run on host threads (one OS thread per lane, real
// barriers, 64-lane shuffles), so that host logic and kernel indexing can be
// checked under AddressSanitizer without a GPU.  Nothing in the product
// includes this directory; the shipped library is built by hipcc for gfx950.
#pragma once
#include <algorithm>
#include <atomic>
#include <barrier>
#include <cmath>
#include <condition_variable>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <memory>
#include <mutex>
#include <thread>
#include <vector>

#define __global__
#define __device__
#define __host__
#define __constant__
#define __shared__ static
#define __launch_bounds__(...)
#define __forceinline__ inline

struct dim3 {
    unsigned x, y, z;
    dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
struct uint2 { uint32_t x, y; };
struct uint4 { uint32_t x, y, z, w; };
struct float4 { float x, y, z, w; };
inline uint4 make_uint4(uint32_t x, uint32_t y, uint32_t z, uint32_t w) { return {x, y, z, w}; }
inline float4 make_float4(float x, float y, float z, float w) { return {x, y, z, w}; }

typedef void *hipStream_t;
typedef void *hipEvent_t;
enum hipError_t { hipSuccess = 0, hipErrorUnknown = 1 };
enum hipMemcpyKind { hipMemcpyHostToDevice, hipMemcpyDeviceToHost, hipMemcpyDeviceToDevice };
enum { hipHostMallocDefault = 0, hipEventDisableTiming = 2, hipStreamNonBlocking = 1 };

namespace hip_emul {

struct BlockCtx {
    unsigned nthreads;
    std::barrier<> bar;
    std::vector<std::unique_ptr<std::barrier<>>> wave_bar;
    std::vector<uint64_t> xchg;
    std::atomic<int> orflag[2];
    explicit BlockCtx(unsigned n) : nthreads(n), bar(n), xchg(n)
    {
        orflag[0] = orflag[1] = 0;
        for (unsigned w = 0; w * 64 < n; w++)
            wave_bar.emplace_back(new std::barrier<>(std::min(64u, n - w * 64)));
    }
};

struct ThreadState {
    dim3 tid, bid, bdim, gdim;
    BlockCtx *ctx = nullptr;
    unsigned or_calls = 0;
};
inline thread_local ThreadState tls;

// Run fn once per lane of every workgroup of the grid; workgroups run one after another
// because __shared__ variables are function-level statics here.
void launch(dim3 grid, dim3 block, const std::function<void()> &fn);

template <typename T>
inline uint64_t to_bits(T v) { uint64_t b = 0; memcpy(&b, &v, sizeof(T)); return b; }
template <typename T>
inline T from_bits(uint64_t b) { T v; memcpy(&v, &b, sizeof(T)); return v; }

template <typename T, typename F>
inline T shuffle(T v, F src_of)
{
    ThreadState &t = tls;
    const unsigned tid = t.tid.x, wave = tid >> 6, lane = tid & 63;
    BlockCtx &c = *t.ctx;
    const unsigned wave_n = std::min(64u, c.nthreads - wave * 64);
    c.xchg[tid] = to_bits(v);
    c.wave_bar[wave]->arrive_and_wait();
    const int src = src_of((int)lane);
    T r = (src >= 0 && (unsigned)src < wave_n) ? from_bits<T>(c.xchg[wave * 64 + src]) : v;
    c.wave_bar[wave]->arrive_and_wait();
    return r;
}

}  // namespace hip_emul

#define threadIdx (hip_emul::tls.tid)
#define blockIdx (hip_emul::tls.bid)
#define blockDim (hip_emul::tls.bdim)
#define gridDim (hip_emul::tls.gdim)

inline void __syncthreads() { hip_emul::tls.ctx->bar.arrive_and_wait(); }
inline int __syncthreads_or(int p)
{
    hip_emul::ThreadState &t = hip_emul::tls;
    hip_emul::BlockCtx &c = *t.ctx;
    const int slot = (int)(t.or_calls++ & 1u);
    if (p) c.orflag[slot].store(1);
    c.bar.arrive_and_wait();
    const int r = c.orflag[slot].load();
    c.bar.arrive_and_wait();
    if (t.tid.x == 0) c.orflag[slot].store(0);
    return r;
}
// mask of the lanes of the wave whose predicate is true
inline unsigned long long __ballot(int pred)
{
    hip_emul::ThreadState &t = hip_emul::tls;
    const unsigned tid = t.tid.x, wave = tid >> 6;
    hip_emul::BlockCtx &c = *t.ctx;
    const unsigned wave_n = std::min(64u, c.nthreads - wave * 64);
    c.xchg[tid] = pred ? 1 : 0;
    c.wave_bar[wave]->arrive_and_wait();
    unsigned long long m = 0;
    for (unsigned l = 0; l < wave_n; l++) m |= (unsigned long long)(c.xchg[wave * 64 + l] & 1) << l;
    c.wave_bar[wave]->arrive_and_wait();
    return m;
}
template <typename T>
inline T __shfl(T v, int src, int = 64) { return hip_emul::shuffle(v, [src](int) { return src; }); }
template <typename T>
inline T __shfl_up(T v, unsigned d, int = 64) { return hip_emul::shuffle(v, [d](int l) { return l - (int)d; }); }
template <typename T>
inline T __shfl_down(T v, unsigned d, int = 64) { return hip_emul::shuffle(v, [d](int l) { return l + (int)d; }); }
template <typename T>
inline T __shfl_xor(T v, int d, int = 64) { return hip_emul::shuffle(v, [d](int l) { return l ^ d; }); }

inline uint32_t atomicOr(uint32_t *p, uint32_t v) { return __atomic_fetch_or(p, v, __ATOMIC_SEQ_CST); }
inline uint32_t atomicAdd(uint32_t *p, uint32_t v) { return __atomic_fetch_add(p, v, __ATOMIC_SEQ_CST); }
inline int32_t atomicMin(int32_t *p, int32_t v)
{
    int32_t old = __atomic_load_n(p, __ATOMIC_SEQ_CST);
    while (old > v && !__atomic_compare_exchange_n(p, &old, v, false, __ATOMIC_SEQ_CST, __ATOMIC_SEQ_CST)) {}
    return old;
}
inline uint32_t atomicMin(uint32_t *p, uint32_t v)
{
    uint32_t old = __atomic_load_n(p, __ATOMIC_SEQ_CST);
    while (old > v && !__atomic_compare_exchange_n(p, &old, v, false, __ATOMIC_SEQ_CST, __ATOMIC_SEQ_CST)) {}
    return old;
}
// ({hi,lo} >> (shift & 31)) truncated to 32 bits, as V_ALIGNBIT_B32 computes it
inline uint32_t __builtin_amdgcn_alignbit(uint32_t hi, uint32_t lo, uint32_t shift)
{
    return (uint32_t)(((((uint64_t)hi) << 32) | lo) >> (shift & 31u));
}
// V_CVT_PK_U8_F32: v rounded to the nearest integer (half-way to even), clamped to 0..255,
// into byte `lane` of `word`
inline uint32_t __builtin_amdgcn_cvt_pk_u8_f32(float v, uint32_t lane, uint32_t word)
{
    const float r = __builtin_nearbyintf(v);
    const uint32_t b = !(r > 0.0f) ? 0u : r >= 255.0f ? 255u : (uint32_t)r;
    const uint32_t sh = 8u * (lane & 3u);
    return (word & ~(255u << sh)) | (b << sh);
}
// V_BFE_U32: `width` bits of v from bit `offset` up; 0 for width 0
inline uint32_t __builtin_amdgcn_ubfe(uint32_t v, uint32_t offset, uint32_t width)
{
    offset &= 31u;
    width &= 31u;
    return width == 0 ? 0u : (v >> offset) & ((1u << width) - 1u);
}
inline int32_t __builtin_amdgcn_sbfe(int32_t v, uint32_t offset, uint32_t width)
{
    offset &= 31u;
    width &= 31u;
    if (width == 0) return 0;
    const uint32_t field = ((uint32_t)v >> offset) & ((1u << width) - 1u);
    return (field >> (width - 1)) ? (int32_t)(field | ~((1u << width) - 1u)) : (int32_t)field;
}
// the value of the wave's first active lane; used only where all lanes hold the same value
inline int __builtin_amdgcn_readfirstlane(int v) { return v; }
inline int __mul24(int a, int b) { return a * b; }
inline int __popcll(unsigned long long v) { return __builtin_popcountll(v); }

template <typename T> inline T min(T a, T b) { return b < a ? b : a; }
template <typename T> inline T max(T a, T b) { return a < b ? b : a; }

#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...) \
    hip_emul::launch((grid), (block), [&]() { kernel(__VA_ARGS__); })

// ---- runtime API: the "device" is the host heap --------------------------------------
inline hipError_t hipGetDeviceCount(int *n) { *n = 1; return hipSuccess; }
inline hipError_t hipSetDevice(int) { return hipSuccess; }
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipDeviceSynchronize() { return hipSuccess; }
inline hipError_t hipMalloc(void **p, size_t n) { *p = malloc(n ? n : 1); return *p ? hipSuccess : hipErrorUnknown; }
inline hipError_t hipFree(void *p) { free(p); return hipSuccess; }
inline hipError_t hipHostMalloc(void **p, size_t n, unsigned) { return hipMalloc(p, n); }
inline hipError_t hipHostFree(void *p) { free(p); return hipSuccess; }
inline hipError_t hipMemcpy(void *d, const void *s, size_t n, hipMemcpyKind) { memcpy(d, s, n); return hipSuccess; }
inline hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, hipMemcpyKind, hipStream_t) { memcpy(d, s, n); return hipSuccess; }
inline hipError_t hipMemset(void *d, int v, size_t n) { memset(d, v, n); return hipSuccess; }
inline hipError_t hipMemsetAsync(void *d, int v, size_t n, hipStream_t) { memset(d, v, n); return hipSuccess; }
inline hipError_t hipMemcpy2D(void *d, size_t dp, const void *s, size_t sp, size_t w, size_t h, hipMemcpyKind)
{
    for (size_t r = 0; r < h; r++) memcpy((char *)d + r * dp, (const char *)s + r * sp, w);
    return hipSuccess;
}
inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
inline hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned) { *s = malloc(1); return hipSuccess; }
inline hipError_t hipStreamDestroy(hipStream_t s) { free(s); return hipSuccess; }
inline hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
inline hipError_t hipEventCreate(hipEvent_t *e) { *e = malloc(1); return hipSuccess; }
inline hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { *e = malloc(1); return hipSuccess; }
inline hipError_t hipEventDestroy(hipEvent_t e) { free(e); return hipSuccess; }
inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
inline hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
inline hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.0f; return hipSuccess; }
