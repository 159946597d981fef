// gs_mixprobe.hip -- measurement aid, not part of the product path: kernels with the memory traffic
// of the fused step (k bf16 gradient streams and three fp32 state streams in; three fp32 streams
// and one bf16 stream out, 2k+26 bytes per element) and no arithmetic beyond what keeps the
// compiler from dropping the accesses.  bench.py times them next to gs_accum_adamw so that the
// step's bandwidth can be held against what the same device gives the same mix of streams:
//   mode 0  the step kernel's own shape without its arithmetic: one tile per workgroup, the
//           three state loads first, gradient loads one at a time, the four stores one by one;
//   mode 1  the same tile with every load in flight at once and the stores back to back;
//   mode 2  the read half only (the 2k+12 bytes in), loads one at a time;
//   mode 3  the write half only (the 14 bytes out), stores one by one.
// Modes 2 and 3 launched together on two streams put the same bytes on the memory system from
// separate workgroups: if that pair is no faster than mode 0, the mix itself -- not the way one
// kernel interleaves its loads and stores -- sets the rate.
//
// Outputs are written out of place (po/mo/vo/w), so the caller's states survive; with mask = 0 the
// values written are the values read.  Built into its own shared library; libgs.so does not
// contain or call any of this.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxK = 32;

struct MixArgs {
    const uint32_t *p, *m, *v;   // fp32 streams read as raw words
    uint32_t *po, *mo, *vo;
    uint16_t *w;
    const uint16_t *g[kMaxK];
    int k;
    int64_t n;                   // elements; a multiple of 4
    uint32_t mask;               // 0 at run time; unknown to the compiler
    uint32_t *sink;
};

template <typename T> __device__ __forceinline__ T ld_stream(const T *p) { return __builtin_nontemporal_load(p); }
template <typename T> __device__ __forceinline__ void st_stream(T *p, T v) { __builtin_nontemporal_store(v, p); }

__device__ __forceinline__ void wait_vm_idle()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
}

template <int BLOCK, int MODE>
__global__ __launch_bounds__(BLOCK) void k_mix(MixArgs A)
{
    const int64_t lo = ((int64_t)blockIdx.x * BLOCK + threadIdx.x) * 4;
    if (lo >= A.n) return;
    if constexpr (MODE == 3) {
        const uint32_t x = A.mask | threadIdx.x;
        st_stream(reinterpret_cast<u32x4 *>(A.po + lo), u32x4{x, x, x, x});
        wait_vm_idle();
        st_stream(reinterpret_cast<u32x4 *>(A.mo + lo), u32x4{x, x, x, x});
        wait_vm_idle();
        st_stream(reinterpret_cast<u32x4 *>(A.vo + lo), u32x4{x, x, x, x});
        wait_vm_idle();
        st_stream(reinterpret_cast<u32x2 *>(A.w + lo), u32x2{x, x});
        return;
    }
    u32x4 p = ld_stream(reinterpret_cast<const u32x4 *>(A.p + lo));
    u32x4 m = ld_stream(reinterpret_cast<const u32x4 *>(A.m + lo));
    u32x4 v = ld_stream(reinterpret_cast<const u32x4 *>(A.v + lo));
    u32x2 acc = u32x2{0u, 0u};
    if constexpr (MODE == 1) {
        u32x2 gv[kMaxK];
#pragma unroll
        for (int j = 0; j < kMaxK; ++j)
            if (j < A.k) gv[j] = ld_stream(reinterpret_cast<const u32x2 *>(A.g[j] + lo));
#pragma unroll
        for (int j = 0; j < kMaxK; ++j)
            if (j < A.k) acc ^= gv[j];
    } else {
#pragma unroll 1
        for (int j = 0; j < A.k; ++j) acc ^= ld_stream(reinterpret_cast<const u32x2 *>(A.g[j] + lo));
    }
    const uint32_t t = (acc.x ^ acc.y) & A.mask;      // 0 at run time
    if constexpr (MODE == 2) {
        const uint32_t s = (p.x ^ p.y ^ p.z ^ p.w ^ m.x ^ m.y ^ m.z ^ m.w ^ v.x ^ v.y ^ v.z ^ v.w) & A.mask;
        if ((s | t) != 0u) A.sink[0] = s | t;         // never taken
        return;
    }
    p.x ^= t; m.y ^= t; v.z ^= t;
    u32x2 wv;
    wv.x = (p.x >> 16) | (p.y & 0xffff0000u);
    wv.y = (p.z >> 16) | (p.w & 0xffff0000u);
    __builtin_amdgcn_sched_barrier(0);
    st_stream(reinterpret_cast<u32x4 *>(A.po + lo), p);
    if constexpr (MODE == 0) wait_vm_idle();
    st_stream(reinterpret_cast<u32x4 *>(A.mo + lo), m);
    if constexpr (MODE == 0) wait_vm_idle();
    st_stream(reinterpret_cast<u32x4 *>(A.vo + lo), v);
    if constexpr (MODE == 0) wait_vm_idle();
    st_stream(reinterpret_cast<u32x2 *>(A.w + lo), wv);
}

template <int MODE>
hipError_t launch(const MixArgs &A, int block, hipStream_t s)
{
    const int64_t tiles = (A.n / 4 + block - 1) / block;
    if (tiles < 1 || tiles > 0x7fffffff) return hipErrorInvalidValue;
    if (block == 64) k_mix<64, MODE><<<(int)tiles, 64, 0, s>>>(A);
    else if (block == 128) k_mix<128, MODE><<<(int)tiles, 128, 0, s>>>(A);
    else if (block == 256) k_mix<256, MODE><<<(int)tiles, 256, 0, s>>>(A);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace

// Returns 0, -1 for a rejected argument, or the hipError_t of a failed launch.  All tensor pointers
// are device addresses, 16-byte aligned; n is a multiple of 4; grads is a host table of k device
// pointers; block is 64, 128 or 256 lanes per workgroup; sink is a device word (mode 2).
extern "C" int gs_mixprobe_launch(int mode, int block, const float *p, const float *m, const float *v,
                                  float *po, float *mo, float *vo, uint16_t *w,
                                  const uint16_t *const *grads, int k, int64_t n,
                                  uint32_t mask, uint32_t *sink, void *stream)
{
    if (mode < 0 || mode > 3 || k < 1 || k > kMaxK || n < 4 || (n & 3)) return -1;
    if (!grads || !sink) return -1;
    if (mode != 3 && (!p || !m || !v)) return -1;
    if (mode != 2 && (!po || !mo || !vo || !w)) return -1;
    const void *ptrs[] = {p, m, v, po, mo, vo, w};
    for (const void *q : ptrs)
        if (reinterpret_cast<uintptr_t>(q) & 15u) return -1;
    MixArgs A = {};
    A.p = reinterpret_cast<const uint32_t *>(p);
    A.m = reinterpret_cast<const uint32_t *>(m);
    A.v = reinterpret_cast<const uint32_t *>(v);
    A.po = reinterpret_cast<uint32_t *>(po);
    A.mo = reinterpret_cast<uint32_t *>(mo);
    A.vo = reinterpret_cast<uint32_t *>(vo);
    A.w = w;
    for (int j = 0; j < k; ++j) {
        if (!grads[j] || (reinterpret_cast<uintptr_t>(grads[j]) & 15u)) return -1;
        A.g[j] = grads[j];
    }
    A.k = k;
    A.n = n;
    A.mask = mask;
    A.sink = sink;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    switch (mode) {
    case 0: e = launch<0>(A, block, s); break;
    case 1: e = launch<1>(A, block, s); break;
    case 2: e = launch<2>(A, block, s); break;
    default: e = launch<3>(A, block, s); break;
    }
    return (int)e;
}
