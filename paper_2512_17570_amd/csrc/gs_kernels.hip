// gs_kernels.hip -- gfx950 kernels of the per-layer optimizer step and their launchers.
//
// The work is one streaming pass over 2k+26 bytes per parameter (k bf16 gradient streams and
// the fp32 p/m/v streams in, p/m/v and the bf16 weight out) with ~100 VALU lane-ops per
// element: HBM-bound, so there is no MFMA here.  Measured on MI355X, what decides the achieved
// bandwidth of such a many-stream read+write pass is the shape of the memory traffic:
//   * every wave-level memory instruction covers whole, contiguous 128-byte lines -- a lane owns
//     4 consecutive elements, i.e. one 8-byte load per bf16 stream (512 B per wave) and one
//     16-byte load/store per fp32 stream (1 KB per wave); lanes that own 8 elements would split
//     each fp32 line across two instructions and fetch it twice;
//   * workgroups are NOT persistent: one 512-element tile per 128-lane workgroup, dispatched in
//     order, keeps the set of addresses in flight compact, which HBM rewards (a grid-stride loop
//     costs 30-40 % on stores on this part);
//   * a wave keeps its memory queues shallow in the step kernels: the three state loads up
//     front, then one gradient load in flight at a time, then the four stores one by one;
//   * every stream is touched once, so loads and stores carry the non-temporal hint.
// The norm pass is read-only and does best with short contiguous spans of tiles per workgroup.
//
// Partition independence (Sec. 6.5 of the paper: results must not depend on the partition
// ratio): every element goes through the same update function `adamw_element`, compiled with
// floating-point contraction off, whether it is reached through the 4-wide body or through
// the per-element path used for ragged range ends.  Grouping is by ABSOLUTE element index
// (groups of 4 starting at multiples of 4), so a range split at any point is processed with
// bit-identical arithmetic.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gs_internal.h"

#pragma clang fp contract(off)

namespace gs {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---- memory access helpers: streams are touched exactly once => non-temporal ------------
template <typename T>
__device__ __forceinline__ T ld_stream(const T *p)
{
    return __builtin_nontemporal_load(p);
}
template <typename T>
__device__ __forceinline__ void st_stream(T *p, T v)
{
    __builtin_nontemporal_store(v, p);
}

// s_waitcnt vmcnt(0) (expcnt and lgkmcnt left at their maxima), pinned in place
__device__ __forceinline__ void wait_vm_idle()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_sched_barrier(0);
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// fp32 -> bf16, round to nearest even; NaN stays NaN (quiet bit forced).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    uint32_t r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    uint32_t nan = (u >> 16) | 0x0040u;
    return ((u & 0x7fffffffu) > 0x7f800000u) ? nan : r;
}

// Clip coefficient from the total squared norm (Sec. 2.1: global L2 norm for clipping).
__device__ __forceinline__ float clip_coefficient(const double *d_sqnorm, float max_norm)
{
    if (d_sqnorm == nullptr || !(max_norm > 0.0f)) return 1.0f;
    float norm = (float)sqrt(*d_sqnorm);
    float c = max_norm / (norm + 1e-6f);
    return c < 1.0f ? c : 1.0f;
}

// The element update: clip, moments, master weight (Sec. 2.2: three fp32 states per weight,
// updated element-wise).  One rounding per operation, no fused multiply-add.
__device__ __forceinline__ void adamw_element(float a, float c, const StepConsts &s, float &p, float &m, float &v)
{
    float g = c * a;
    float t1 = s.beta1 * m;
    float t2 = s.omb1 * g;
    float mn = t1 + t2;
    float gg = g * g;
    float t3 = s.beta2 * v;
    float t4 = s.omb2 * gg;
    float vn = t3 + t4;
    float d = __builtin_sqrtf(vn) / s.rsbc2;
    d = d + s.eps;
    float u = mn / d;
    float t5 = p * s.decay;
    float t6 = s.step_size * u;
    p = t5 - t6;
    m = mn;
    v = vn;
}

// k-way accumulation of one 4-element group, j ascending from +0 (Sec. 2.1: micro-batch
// gradients are accumulated in full precision).  K > 0: compile-time count; K == 0: runtime.
// DEPTH is how many gradient loads a wave keeps in flight:
//   0  all of them (compile-time K) or four and two at a time (runtime k) -- what the read-only
//      norm kernel wants;
//   1  one: each load is consumed before the next is issued -- the kernels that mix many read
//      streams with the four write streams of a step do best with shallow memory queues;
//   2  two at a time -- the optimum measured for the staged norm kernel (k reads + one write).
__device__ __forceinline__ void add_pair(float (&a)[4], u32x2 g)
{
    a[0] += bf16_lo(g.x); a[1] += bf16_hi(g.x);
    a[2] += bf16_lo(g.y); a[3] += bf16_hi(g.y);
}

template <int K, int DEPTH>
__device__ __forceinline__ void accumulate_group(const GradTable &gt, int k, int64_t lo, float (&a)[4])
{
#pragma unroll
    for (int e = 0; e < 4; ++e) a[e] = 0.0f;
    if constexpr (K > 0 && DEPTH == 0) {
        u32x2 gv[K];
#pragma unroll
        for (int j = 0; j < K; ++j) gv[j] = ld_stream(reinterpret_cast<const u32x2 *>(gt.g[j] + lo));
#pragma unroll
        for (int j = 0; j < K; ++j) add_pair(a, gv[j]);
    } else if constexpr (K > 0) {
#pragma unroll
        for (int j = 0; j < K; j += DEPTH) {
            u32x2 gv[DEPTH];
#pragma unroll
            for (int q = 0; q < DEPTH; ++q)
                if (j + q < K) gv[q] = ld_stream(reinterpret_cast<const u32x2 *>(gt.g[j + q] + lo));
#pragma unroll
            for (int q = 0; q < DEPTH; ++q)
                if (j + q < K) add_pair(a, gv[q]);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        // runtime k; the adds stay in ascending order of j
        int j = 0;
        if constexpr (DEPTH == 0) {
            for (; j + 4 <= k; j += 4) {
                u32x2 gv[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) gv[q] = ld_stream(reinterpret_cast<const u32x2 *>(gt.g[j + q] + lo));
#pragma unroll
                for (int q = 0; q < 4; ++q) add_pair(a, gv[q]);
            }
        }
        if constexpr (DEPTH == 0 || DEPTH == 2) {
#pragma unroll 1
            for (; j + 2 <= k; j += 2) {
                u32x2 g0 = ld_stream(reinterpret_cast<const u32x2 *>(gt.g[j] + lo));
                u32x2 g1 = ld_stream(reinterpret_cast<const u32x2 *>(gt.g[j + 1] + lo));
                add_pair(a, g0);
                add_pair(a, g1);
            }
        }
#pragma unroll 1
        for (; j < k; ++j) add_pair(a, ld_stream(reinterpret_cast<const u32x2 *>(gt.g[j] + lo)));
    }
}

__device__ __forceinline__ float accumulate_one(const GradTable &gt, int k, int64_t i)
{
    float a = 0.0f;
    for (int j = 0; j < k; ++j) a += __uint_as_float((uint32_t)gt.g[j][i] << 16);
    return a;
}

// ---- block reduction used by the norm kernels ----------------------------------------------
// Per-lane fp64 partial (each square is exact in fp64) -> wave64 butterfly -> LDS across the
// block's waves -> one partial per block; a second tiny kernel folds the block partials in a
// fixed order, so the result is deterministic.
__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

template <int BLOCK>
__device__ __forceinline__ double block_sum(double x, double *lds)
{
    constexpr int NW = BLOCK / 64;
    x = wave_sum(x);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) lds[wave] = x;
    __syncthreads();
    double t = 0.0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 0; w < NW; ++w) t += lds[w];
    }
    return t;   // valid in thread 0
}

// ---- fused accumulate + clip + AdamW + bf16 emit -----------------------------------------
// The group of 4 elements starting at `lo` (a multiple of 4): whole-group vector path when the
// group lies inside [begin,end), per-element path for ragged range ends -- same arithmetic.
// States are read from A.p/m/v and written to A.po/mo/vo (the same arrays for the in-place
// entry points).  NORM: also add the squares of the accumulated gradients to acc0/acc1.
template <int K, bool NORM, int DEPTH = 1>
__device__ __forceinline__ void step_group(const StepArgs &A, int k, int64_t lo, float c, const StepConsts &s,
                                           double &acc0, double &acc1)
{
    if (lo >= A.begin && lo + 4 <= A.end) {
        f32x4 p, m, v;
        float a[4];
        if constexpr (K < 0) {
            // four fp32 read streams against four write streams (a 1:1 mix): here even the loads
            // do best one at a time -- 3.75 ms against 4.05 ms with the four in flight together
            // (805 M elements)
            p = ld_stream(reinterpret_cast<const f32x4 *>(A.p + lo));
            wait_vm_idle();
            m = ld_stream(reinterpret_cast<const f32x4 *>(A.m + lo));
            wait_vm_idle();
            v = ld_stream(reinterpret_cast<const f32x4 *>(A.v + lo));
            wait_vm_idle();
            f32x4 av = ld_stream(reinterpret_cast<const f32x4 *>(A.acc + lo));
            a[0] = av.x; a[1] = av.y; a[2] = av.z; a[3] = av.w;
        } else {
            // State loads go first.  With many gradient streams they stay in flight while the
            // gradient loads are walked one by one (k = 16: 7.46 ms against 7.83 ms when each state
            // load is waited for); with few (where reads and writes are nearly balanced) waiting
            // for each wins by 2-4 %, as in the staged case above.
            p = ld_stream(reinterpret_cast<const f32x4 *>(A.p + lo));
            if (DEPTH != 0 && k <= GS_STATE_WAIT_MAX_K) wait_vm_idle();
            m = ld_stream(reinterpret_cast<const f32x4 *>(A.m + lo));
            if (DEPTH != 0 && k <= GS_STATE_WAIT_MAX_K) wait_vm_idle();
            v = ld_stream(reinterpret_cast<const f32x4 *>(A.v + lo));
            if (DEPTH != 0 && k <= GS_STATE_WAIT_MAX_K) wait_vm_idle();
            accumulate_group<K, DEPTH>(A.gt, k, lo, a);
        }
        float P[4] = {p.x, p.y, p.z, p.w};
        float M[4] = {m.x, m.y, m.z, m.w};
        float V[4] = {v.x, v.y, v.z, v.w};
        if constexpr (NORM) {
            acc0 = fma((double)a[0], (double)a[0], acc0);
            acc1 = fma((double)a[1], (double)a[1], acc1);
            acc0 = fma((double)a[2], (double)a[2], acc0);
            acc1 = fma((double)a[3], (double)a[3], acc1);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) adamw_element(a[e], c, s, P[e], M[e], V[e]);
        u32x2 wv;
        wv.x = f32_to_bf16_bits(P[0]) | (f32_to_bf16_bits(P[1]) << 16);
        wv.y = f32_to_bf16_bits(P[2]) | (f32_to_bf16_bits(P[3]) << 16);
        if constexpr (DEPTH == 0) {
            st_stream(reinterpret_cast<f32x4 *>(A.po + lo), f32x4{P[0], P[1], P[2], P[3]});
            st_stream(reinterpret_cast<f32x4 *>(A.mo + lo), f32x4{M[0], M[1], M[2], M[3]});
            st_stream(reinterpret_cast<f32x4 *>(A.vo + lo), f32x4{V[0], V[1], V[2], V[3]});
            st_stream(reinterpret_cast<u32x2 *>(A.w + lo), wv);
        } else {
            // like the gradient loads, the four stores of a wave go out one at a time (each waits
            // for the previous one): another ~3 % on MI355X from keeping the queues shallow
            __builtin_amdgcn_sched_barrier(0);
            st_stream(reinterpret_cast<f32x4 *>(A.po + lo), f32x4{P[0], P[1], P[2], P[3]});
            wait_vm_idle();
            st_stream(reinterpret_cast<f32x4 *>(A.mo + lo), f32x4{M[0], M[1], M[2], M[3]});
            wait_vm_idle();
            st_stream(reinterpret_cast<f32x4 *>(A.vo + lo), f32x4{V[0], V[1], V[2], V[3]});
            wait_vm_idle();
            st_stream(reinterpret_cast<u32x2 *>(A.w + lo), wv);
        }
    } else {
        const int64_t i0 = lo > A.begin ? lo : A.begin;
        const int64_t i1 = lo + 4 < A.end ? lo + 4 : A.end;
        for (int64_t i = i0; i < i1; ++i) {
            float a;
            if constexpr (K < 0) a = A.acc[i]; else a = accumulate_one(A.gt, k, i);
            if constexpr (NORM) acc0 = fma((double)a, (double)a, acc0);
            float pi = A.p[i], mi = A.m[i], vi = A.v[i];
            adamw_element(a, c, s, pi, mi, vi);
            A.po[i] = pi;
            A.mo[i] = mi;
            A.vo[i] = vi;
            A.w[i] = (uint16_t)f32_to_bf16_bits(pi);
        }
    }
}

// One workgroup = one tile of BLOCK*4 consecutive elements, one group of 4 per lane.  BLOCK is 64
// (one wave) up to 14 gradient streams and for the staged step, 128 from 15 on: measured on
// 805 M elements, single-wave workgroups are 1-3.5 % faster for k = 1..14 (k = 8: 5.50 ms against
// 5.70 ms) and level or 1 % slower at k = 16; 256 lanes lose 4-6 % everywhere.  Tiles start at multiples of the tile size counted from element 0 of the arrays, not from
// `begin`: the grouping does not move with the range (partition independence), and a wave's
// 1 KB accesses stay line-aligned for any `begin` (a split point in the middle of a layer would
// otherwise make every wave straddle two extra lines).
template <int K, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_accum_adamw(StepArgs A)
{
    constexpr int TILE = BLOCK * 4;
    const int k = (K > 0) ? K : A.k;     // K < 0: gradients come as one staged fp32 sum (A.acc)
    const int64_t lo = (A.begin / TILE + (int64_t)blockIdx.x) * TILE + (int64_t)threadIdx.x * 4;
    if (lo >= A.end || lo + 4 <= A.begin) return;
    const float c = clip_coefficient(A.d_sqnorm, A.max_norm);
    double unused0 = 0.0, unused1 = 0.0;
    step_group<K, false>(A, k, lo, c, A.c, unused0, unused1);
}

// Speculative single pass (Sec. 2.1 of the paper: prior work steps before the global norm is
// known because clipping rarely changes the gradients): the step is applied with c = 1 and the
// squared norm of the same accumulated gradients is reduced on the way, so the gradients are
// read once.  Every workgroup leaves a partial.  Fast shape: the step kernel's own 512-element
// tiles, one per workgroup, shallow queues (needs a workspace of one double per tile);
// fallback for the fixed-size workspace: 4096-element tiles, all loads in flight, `span` tiles
// per workgroup.
template <int K, int BLOCK, int DEPTH>
__global__ __launch_bounds__(BLOCK) void k_accum_adamw_spec(StepArgs A, double *partials, int span)
{
    constexpr int TILE = BLOCK * 4;
    __shared__ double lds[BLOCK / 64];
    const int k = (K > 0) ? K : A.k;
    const int64_t first = (A.begin / TILE + (int64_t)blockIdx.x * span) * TILE + (int64_t)threadIdx.x * 4;
    double acc0 = 0.0, acc1 = 0.0;
    for (int it = 0; it < span; ++it) {
        const int64_t lo = first + (int64_t)it * TILE;
        if (lo >= A.end) break;
        if (lo + 4 <= A.begin) continue;
        step_group<K, true, DEPTH>(A, k, lo, 1.0f, A.c, acc0, acc1);
    }
    double t = block_sum<BLOCK>(acc0 + acc1, lds);
    if (threadIdx.x == 0) partials[blockIdx.x] = t;
}

// ---- squared norm of the accumulated gradient --------------------------------------------
// Workgroup b reads `span` consecutive tiles starting at tile b*span (tiles counted from the
// GS_TILE-aligned start of the range): a short contiguous run per workgroup is what the read
// path likes best.
// STAGE: also write the fp32 sum a_i to A.acc (the staged two-pass variant: the step then reads
// one fp32 stream instead of re-reading k bf16 streams).  Once a store stream is involved, runs
// of tiles per workgroup cost bandwidth again (stores want in-order, one-tile workgroups), so
// the staged kernel uses 1024-lane workgroups (4096-element tiles) and a span of 1 wherever the
// partials still fit the workspace.
template <int K, bool STAGE, int BLOCK, int DEPTH>
__global__ __launch_bounds__(BLOCK) void k_grad_sqnorm(SqnormArgs A, int span)
{
    constexpr int TILE = BLOCK * 4;
    __shared__ double lds[BLOCK / 64];
    const int k = (K > 0) ? K : A.k;
    const int64_t first = (A.begin / TILE + (int64_t)blockIdx.x * span) * TILE + (int64_t)threadIdx.x * 4;
    double acc0 = 0.0, acc1 = 0.0;
    for (int it = 0; it < span; ++it) {
        const int64_t lo = first + (int64_t)it * TILE;
        if (lo >= A.end) break;
        if (lo + 4 <= A.begin) continue;
        if (lo >= A.begin && lo + 4 <= A.end) {
            float a[4];
            accumulate_group<K, DEPTH>(A.gt, k, lo, a);
            if constexpr (STAGE) st_stream(reinterpret_cast<f32x4 *>(A.acc + lo), f32x4{a[0], a[1], a[2], a[3]});
            acc0 = fma((double)a[0], (double)a[0], acc0);
            acc1 = fma((double)a[1], (double)a[1], acc1);
            acc0 = fma((double)a[2], (double)a[2], acc0);
            acc1 = fma((double)a[3], (double)a[3], acc1);
        } else {
            const int64_t i0 = lo > A.begin ? lo : A.begin;
            const int64_t i1 = lo + 4 < A.end ? lo + 4 : A.end;
            for (int64_t i = i0; i < i1; ++i) {
                float a = accumulate_one(A.gt, k, i);
                if constexpr (STAGE) A.acc[i] = a;
                acc0 = fma((double)a, (double)a, acc0);
            }
        }
    }
    double t = block_sum<BLOCK>(acc0 + acc1, lds);
    if (threadIdx.x == 0) A.partials[blockIdx.x] = t;
}

// ---- accumulate as you go ------------------------------------------------------------------
// The paper's GPU keeps one full-precision accumulation buffer per layer and each micro-batch's
// backward adds its gradient into it (Sec. 3.4, Sec. 4.3).  acc = (FIRST ? +0 : acc) + widen(g):
// 2 + 4 bytes read and 4 written per element (2 + 4 for the first micro-batch).  NORM: the call
// that adds the last micro-batch also reduces the squared norm of the finished sum.
template <bool FIRST, bool NORM, int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_accum_add(AccumAddArgs A, int span)
{
    constexpr int TILE = BLOCK * 4;
    __shared__ double lds[BLOCK / 64];
    const int64_t first = (A.begin / TILE + (int64_t)blockIdx.x * span) * TILE + (int64_t)threadIdx.x * 4;
    double acc0 = 0.0, acc1 = 0.0;
    for (int it = 0; it < span; ++it) {
        const int64_t lo = first + (int64_t)it * TILE;
        if (lo >= A.end) break;
        if (lo + 4 <= A.begin) continue;
        if (lo >= A.begin && lo + 4 <= A.end) {
            const u32x2 g = ld_stream(reinterpret_cast<const u32x2 *>(A.g + lo));
            f32x4 a = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            if constexpr (!FIRST) {
                wait_vm_idle();          // one load at a time per wave: +1-2 % on this 2:1 read/write mix
                a = ld_stream(reinterpret_cast<const f32x4 *>(A.acc + lo));
            }
            a.x += bf16_lo(g.x); a.y += bf16_hi(g.x);
            a.z += bf16_lo(g.y); a.w += bf16_hi(g.y);
            st_stream(reinterpret_cast<f32x4 *>(A.acc + lo), a);
            if constexpr (NORM) {
                acc0 = fma((double)a.x, (double)a.x, acc0);
                acc1 = fma((double)a.y, (double)a.y, acc1);
                acc0 = fma((double)a.z, (double)a.z, acc0);
                acc1 = fma((double)a.w, (double)a.w, acc1);
            }
        } else {
            const int64_t i0 = lo > A.begin ? lo : A.begin;
            const int64_t i1 = lo + 4 < A.end ? lo + 4 : A.end;
            for (int64_t i = i0; i < i1; ++i) {
                float a = FIRST ? 0.0f : A.acc[i];
                a += __uint_as_float((uint32_t)A.g[i] << 16);
                A.acc[i] = a;
                if constexpr (NORM) acc0 = fma((double)a, (double)a, acc0);
            }
        }
    }
    if constexpr (NORM) {
        double t = block_sum<BLOCK>(acc0 + acc1, lds);
        if (threadIdx.x == 0) A.partials[blockIdx.x] = t;
    }
}

// Norm of a finished fp32 accumulation buffer (the buffer gs_accum_add builds, or one that came
// back from a reduction across devices): 4 bytes read per element, the read-only shape of the
// gradient norm -- a short contiguous run of tiles per workgroup.
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_acc_sqnorm(const float *acc, int64_t begin, int64_t end, double *partials, int span)
{
    constexpr int TILE = BLOCK * 4;
    __shared__ double lds[BLOCK / 64];
    const int64_t first = (begin / TILE + (int64_t)blockIdx.x * span) * TILE + (int64_t)threadIdx.x * 4;
    double acc0 = 0.0, acc1 = 0.0;
    for (int it = 0; it < span; ++it) {
        const int64_t lo = first + (int64_t)it * TILE;
        if (lo >= end) break;
        if (lo + 4 <= begin) continue;
        if (lo >= begin && lo + 4 <= end) {
            const f32x4 a = ld_stream(reinterpret_cast<const f32x4 *>(acc + lo));
            acc0 = fma((double)a.x, (double)a.x, acc0);
            acc1 = fma((double)a.y, (double)a.y, acc1);
            acc0 = fma((double)a.z, (double)a.z, acc0);
            acc1 = fma((double)a.w, (double)a.w, acc1);
        } else {
            const int64_t i0 = lo > begin ? lo : begin;
            const int64_t i1 = lo + 4 < end ? lo + 4 : end;
            for (int64_t i = i0; i < i1; ++i) acc0 = fma((double)acc[i], (double)acc[i], acc0);
        }
    }
    double t = block_sum<BLOCK>(acc0 + acc1, lds);
    if (threadIdx.x == 0) partials[blockIdx.x] = t;
}

// Folding the workgroup partials, in a fixed order (deterministic).  Up to 262144 partials are too
// many for one workgroup to read quickly, so large counts go through GS_FINAL_SLICES workgroups
// that each fold a contiguous slice into the tail of the workspace, then one workgroup folds those.
__global__ __launch_bounds__(GS_FINAL_BLOCK) void k_sqnorm_fold_slices(const double *partials, int nparts, double *slices)
{
    __shared__ double lds[GS_FINAL_BLOCK / 64];
    const int per = (nparts + GS_FINAL_SLICES - 1) / GS_FINAL_SLICES;
    const int lo = blockIdx.x * per;
    const int hi = lo + per < nparts ? lo + per : nparts;
    double x = 0.0;
    for (int i = lo + threadIdx.x; i < hi; i += GS_FINAL_BLOCK) x += partials[i];
    double t = block_sum<GS_FINAL_BLOCK>(x, lds);
    if (threadIdx.x == 0) slices[blockIdx.x] = t;
}

__global__ __launch_bounds__(GS_FINAL_BLOCK) void k_sqnorm_finalize(const double *partials, int nparts, double *out, int accumulate)
{
    __shared__ double lds[GS_FINAL_BLOCK / 64];
    double x = 0.0;
    for (int i = threadIdx.x; i < nparts; i += GS_FINAL_BLOCK) x += partials[i];
    double t = block_sum<GS_FINAL_BLOCK>(x, lds);
    if (threadIdx.x == 0) *out = accumulate ? (*out + t) : t;
}

static hipError_t launch_fold(double *partials, int64_t cap, int nparts, double *d_out, int accumulate, hipStream_t stream)
{
    if (nparts > GS_FINAL_DIRECT_MAX) {
        double *slices = partials + cap;          // the last GS_FINAL_SLICES doubles of the workspace
        k_sqnorm_fold_slices<<<GS_FINAL_SLICES, GS_FINAL_BLOCK, 0, stream>>>(partials, nparts, slices);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        k_sqnorm_finalize<<<1, GS_FINAL_BLOCK, 0, stream>>>(slices, GS_FINAL_SLICES, d_out, accumulate);
    } else {
        k_sqnorm_finalize<<<1, GS_FINAL_BLOCK, 0, stream>>>(partials, nparts, d_out, accumulate);
    }
    return hipGetLastError();
}

// ---- launchers -----------------------------------------------------------------------------
static int64_t tiles_of(int64_t begin, int64_t end, int64_t tile = GS_TILE)
{
    if (end <= begin) return 0;
    return (end - 1) / tile - begin / tile + 1;
}

hipError_t launch_accum_adamw(const StepArgs &A, hipStream_t stream)
{
    const bool wide = !A.acc && A.k >= GS_STEP_WIDE_MIN_K;
    const int64_t tiles = tiles_of(A.begin, A.end, (int64_t)(wide ? GS_STEP_BLOCK : GS_WAVE_BLOCK) * 4);
    if (tiles < 1 || tiles > 0x7fffffff) return hipErrorInvalidValue;
    const int grid = (int)tiles;
    if (A.acc) {
        k_accum_adamw<-1, GS_WAVE_BLOCK><<<grid, GS_WAVE_BLOCK, 0, stream>>>(A);
        return hipGetLastError();
    }
    // k = 1, 2 unrolled; every other k takes the runtime loop, which keeps one gradient load in
    // flight per wave with the fewest registers (27 VGPRs: full occupancy) and measured as fast
    // as or faster than unrolled bodies for k = 4, 8, 16
    if (wide) {
        k_accum_adamw<0, GS_STEP_BLOCK><<<grid, GS_STEP_BLOCK, 0, stream>>>(A);
        return hipGetLastError();
    }
    switch (A.k) {
    case 1: k_accum_adamw<1, GS_WAVE_BLOCK><<<grid, GS_WAVE_BLOCK, 0, stream>>>(A); break;
    case 2: k_accum_adamw<2, GS_WAVE_BLOCK><<<grid, GS_WAVE_BLOCK, 0, stream>>>(A); break;
    default: k_accum_adamw<0, GS_WAVE_BLOCK><<<grid, GS_WAVE_BLOCK, 0, stream>>>(A); break;
    }
    return hipGetLastError();
}

// Partials the workspace can hold (its last GS_FINAL_SLICES doubles serve the folding stage).
static int64_t partial_capacity(size_t workspace_bytes)
{
    return (int64_t)(workspace_bytes / sizeof(double)) - GS_FINAL_SLICES;
}

hipError_t launch_accum_adamw_spec(const StepArgs &A, double *partials, size_t workspace_bytes, double *d_out,
                                   int accumulate, hipStream_t stream)
{
    const int64_t cap = partial_capacity(workspace_bytes);
    // fastest shape the workspace has room for: one tile per workgroup, runtime gradient loop,
    // shallow queues -- single-wave workgroups (k = 16: 7.42 ms, k = 8: 5.28 ms on 805 M elements),
    // else two waves (7.58 / 5.54 ms)
    int64_t tiles = tiles_of(A.begin, A.end, (int64_t)GS_WAVE_BLOCK * 4);
    if (tiles < 1) tiles = 1;
    if (tiles <= cap && tiles <= 0x7fffffff) {
        const int grid = (int)tiles;
        k_accum_adamw_spec<0, GS_WAVE_BLOCK, 1><<<grid, GS_WAVE_BLOCK, 0, stream>>>(A, partials, 1);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        return launch_fold(partials, cap, grid, d_out, accumulate, stream);
    }
    tiles = tiles_of(A.begin, A.end, (int64_t)GS_STEP_BLOCK * 4);
    if (tiles < 1) tiles = 1;
    if (tiles <= cap && tiles <= 0x7fffffff) {
        const int grid = (int)tiles;
        k_accum_adamw_spec<0, GS_STEP_BLOCK, 1><<<grid, GS_STEP_BLOCK, 0, stream>>>(A, partials, 1);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        return launch_fold(partials, cap, grid, d_out, accumulate, stream);
    }
    tiles = tiles_of(A.begin, A.end, (int64_t)GS_STAGE_BLOCK * 4);
    if (tiles < 1) tiles = 1;
    int64_t span = 1;
    if (tiles > cap) span = (tiles + cap - 1) / cap;
    if (span > 0x7fffffff) return hipErrorInvalidValue;
    const int grid = (int)((tiles + span - 1) / span);
    const int sp = (int)span;
    switch (A.k) {
    case 1: k_accum_adamw_spec<1, GS_STAGE_BLOCK, 0><<<grid, GS_STAGE_BLOCK, 0, stream>>>(A, partials, sp); break;
    case 2: k_accum_adamw_spec<2, GS_STAGE_BLOCK, 0><<<grid, GS_STAGE_BLOCK, 0, stream>>>(A, partials, sp); break;
    case 4: k_accum_adamw_spec<4, GS_STAGE_BLOCK, 0><<<grid, GS_STAGE_BLOCK, 0, stream>>>(A, partials, sp); break;
    case 8: k_accum_adamw_spec<8, GS_STAGE_BLOCK, 0><<<grid, GS_STAGE_BLOCK, 0, stream>>>(A, partials, sp); break;
    case 16: k_accum_adamw_spec<16, GS_STAGE_BLOCK, 0><<<grid, GS_STAGE_BLOCK, 0, stream>>>(A, partials, sp); break;
    default: k_accum_adamw_spec<0, GS_STAGE_BLOCK, 0><<<grid, GS_STAGE_BLOCK, 0, stream>>>(A, partials, sp); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_fold(partials, cap, grid, d_out, accumulate, stream);
}

hipError_t launch_grad_sqnorm(const SqnormArgs &A, size_t workspace_bytes, double *d_out, int accumulate,
                              hipStream_t stream)
{
    const int64_t cap = partial_capacity(workspace_bytes);
    const bool stage = A.acc != nullptr;
    if (stage) {
        // staged norm, fast shapes: one tile per workgroup, two gradient loads in flight -- single-wave
        // workgroups up to 8 streams (k = 4: 1.44 ms against 1.47 ms on 805 M elements; level at k = 8),
        // two waves beyond (k = 16: 4.65 ms against 4.72 ms)
        const int64_t t64 = tiles_of(A.begin, A.end, (int64_t)GS_WAVE_BLOCK * 4);
        if (A.k <= 8 && t64 >= 1 && t64 <= cap && t64 <= 0x7fffffff) {
            const int grid = (int)t64;
            k_grad_sqnorm<0, true, GS_WAVE_BLOCK, 2><<<grid, GS_WAVE_BLOCK, 0, stream>>>(A, 1);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            return launch_fold(A.partials, cap, grid, d_out, accumulate, stream);
        }
        int64_t t128 = tiles_of(A.begin, A.end, (int64_t)GS_STEP_BLOCK * 4);
        if (t128 < 1) t128 = 1;
        if (t128 <= cap && t128 <= 0x7fffffff) {
            const int grid = (int)t128;
            k_grad_sqnorm<0, true, GS_STEP_BLOCK, 2><<<grid, GS_STEP_BLOCK, 0, stream>>>(A, 1);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            return launch_fold(A.partials, cap, grid, d_out, accumulate, stream);
        }
    }
    const int block = stage ? GS_STAGE_BLOCK : GS_BLOCK;
    int64_t tiles = tiles_of(A.begin, A.end, (int64_t)block * 4);
    if (tiles < 1) tiles = 1;
    int64_t span = stage ? 1 : GS_NORM_SPAN;
    if ((tiles + span - 1) / span > cap) span = (tiles + cap - 1) / cap;
    if (span > 0x7fffffff) return hipErrorInvalidValue;
    const int grid = (int)((tiles + span - 1) / span);
    const int sp = (int)span;
#define GS_NORM_CASE(KK)                                                                                 \
    if (stage) k_grad_sqnorm<KK, true, GS_STAGE_BLOCK, 0><<<grid, GS_STAGE_BLOCK, 0, stream>>>(A, sp);   \
    else k_grad_sqnorm<KK, false, GS_BLOCK, 0><<<grid, GS_BLOCK, 0, stream>>>(A, sp);                    \
    break
    switch (A.k) {
    case 1: GS_NORM_CASE(1);
    case 2: GS_NORM_CASE(2);
    case 4: GS_NORM_CASE(4);
    case 8: GS_NORM_CASE(8);
    case 16: GS_NORM_CASE(16);
    default: GS_NORM_CASE(0);
    }
#undef GS_NORM_CASE
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_fold(A.partials, cap, grid, d_out, accumulate, stream);
}

hipError_t launch_acc_sqnorm(const float *acc, int64_t begin, int64_t end, double *partials, size_t workspace_bytes,
                             double *d_out, int accumulate, hipStream_t stream)
{
    const int64_t cap = partial_capacity(workspace_bytes);
    int64_t tiles = tiles_of(begin, end, GS_TILE);
    if (tiles < 1) tiles = 1;
    int64_t span = GS_NORM_SPAN;
    if ((tiles + span - 1) / span > cap) span = (tiles + cap - 1) / cap;
    if (span > 0x7fffffff) return hipErrorInvalidValue;
    const int grid = (int)((tiles + span - 1) / span);
    k_acc_sqnorm<GS_BLOCK><<<grid, GS_BLOCK, 0, stream>>>(acc, begin, end, partials, (int)span);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_fold(partials, cap, grid, d_out, accumulate, stream);
}

hipError_t launch_accum_add(const AccumAddArgs &A, int first, size_t workspace_bytes, double *d_out, int accumulate,
                            hipStream_t stream)
{
    if (!d_out) {
        // no partials to leave behind: single-wave workgroups over 256-element tiles measured best
        // (1.17 ms against 1.23 ms with two waves per workgroup, 805 M elements)
        const int64_t t64 = tiles_of(A.begin, A.end, 64 * 4);
        if (t64 > 0x7fffffff) return hipErrorInvalidValue;
        const int grid = (int)(t64 < 1 ? 1 : t64);
        if (first) k_accum_add<true, false, 64><<<grid, 64, 0, stream>>>(A, 1);
        else k_accum_add<false, false, 64><<<grid, 64, 0, stream>>>(A, 1);
        return hipGetLastError();
    }
    const int64_t cap = partial_capacity(workspace_bytes);
    int grid;
    const int64_t tiles64 = tiles_of(A.begin, A.end, (int64_t)GS_WAVE_BLOCK * 4);
    int64_t tiles = tiles_of(A.begin, A.end, (int64_t)GS_STEP_BLOCK * 4);
    if (tiles64 >= 1 && tiles64 <= cap && tiles64 <= 0x7fffffff) {
        // single-wave workgroups here too: 1.24 ms against 1.29 ms with two waves (805 M elements)
        grid = (int)tiles64;
        if (first) k_accum_add<true, true, GS_WAVE_BLOCK><<<grid, GS_WAVE_BLOCK, 0, stream>>>(A, 1);
        else k_accum_add<false, true, GS_WAVE_BLOCK><<<grid, GS_WAVE_BLOCK, 0, stream>>>(A, 1);
    } else if (tiles >= 1 && tiles <= cap && tiles <= 0x7fffffff) {
        grid = (int)tiles;
        if (first) k_accum_add<true, true, GS_STEP_BLOCK><<<grid, GS_STEP_BLOCK, 0, stream>>>(A, 1);
        else k_accum_add<false, true, GS_STEP_BLOCK><<<grid, GS_STEP_BLOCK, 0, stream>>>(A, 1);
    } else {
        tiles = tiles_of(A.begin, A.end, (int64_t)GS_STAGE_BLOCK * 4);
        if (tiles < 1) tiles = 1;
        int64_t span = 1;
        if (tiles > cap) span = (tiles + cap - 1) / cap;
        if (span > 0x7fffffff) return hipErrorInvalidValue;
        grid = (int)((tiles + span - 1) / span);
        const int sp = (int)span;
        if (first) k_accum_add<true, true, GS_STAGE_BLOCK><<<grid, GS_STAGE_BLOCK, 0, stream>>>(A, sp);
        else k_accum_add<false, true, GS_STAGE_BLOCK><<<grid, GS_STAGE_BLOCK, 0, stream>>>(A, sp);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_fold(A.partials, cap, grid, d_out, accumulate, stream);
}

}  // namespace gs
