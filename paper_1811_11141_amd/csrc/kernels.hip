// gfx950 kernels of the merged-gradient data path.
//
//   k_fused   pack + N-way reduce + unpack (+ update) in one pass: element i of layer l is
//             read from the N workers' tensors, summed in worker order, scaled by 1/N (Eq. 2)
//             and written to the per-layer output; the merged buffer of Algorithm 2 never
//             touches memory.
//   k_pack    Algorithm 2's layer buffer: each worker's layers of a group laid end to end.
//   k_reduce  Eq. 2 over N contiguous merged buffers.
//   k_unpack  merged buffer back to per-layer tensors (+ update of Eq. 1-2 with momentum).
//   k_fused_gated  k_fused over the whole plan as one launch whose workgroups wait, tile by tile,
//             for the arrival counter of the tile's group (Algorithm 2's communication thread
//             on the device); k_signal and k_await are its helpers.
//
// The path is bound by HBM bandwidth (0.2-0.3 flop per byte); there is nothing for the matrix
// cores to do.  In the reductions (k_fused, k_reduce) one workgroup of 128 lanes (2 wave64) owns
// one tile.  Full aligned tiles, the bulk of the bytes, run fast_tile(): 128-bit streaming loads
// and stores written out as instructions, one load in flight per wave at full occupancy,
// stores after all loads.  The rest (ragged tails, misaligned tensors, gather tiles of many
// tiny layers) runs compiler-scheduled loops that issue the N loads of an element before the
// first add.  The copy-like steps (k_pack, k_unpack) want the opposite shape: one workgroup per
// 512-element piece of a tile, one 16-byte access per lane (see "Copy-like steps").
// Arithmetic order is fixed (worker 0 first, one rounding per operation; the file is compiled
// with -ffp-contract=off) so results are reproducible bit for bit.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <utility>

#include "../../include/mgwfbp.h"
#include "plan.hpp"

namespace mgwfbp {

namespace {

constexpr int kBlock = 128;  // 2 wave64 per workgroup

typedef float v4f __attribute__((ext_vector_type(4)));

// Every tensor, table and workspace pointer handed to the kernels is device global memory.
// Saying so lets the compiler emit global_load/global_store (scalar base + lane offset) in
// place of flat accesses, which would also have to test for the LDS and scratch apertures.
#define MGWFBP_GLOBAL __attribute__((address_space(1)))

template <bool NT, class T>
__device__ __forceinline__ T ld(const T *p)
{
    const MGWFBP_GLOBAL T *gp = (const MGWFBP_GLOBAL T *)p;
    if constexpr (NT) return __builtin_nontemporal_load(gp);
    else return *gp;
}

template <bool NT, class T>
__device__ __forceinline__ void st(T *p, T x)
{
    MGWFBP_GLOBAL T *gp = (MGWFBP_GLOBAL T *)p;
    if constexpr (NT) __builtin_nontemporal_store(x, gp);
    else *gp = x;
}

// The plan tables (tiles, segments, pointer arrays) are written once by the host and never by
// a kernel.  Reading them through the constant address space tells the compiler so, and a
// load whose address is uniform over the wave then becomes a scalar load into SGPRs.
#define MGWFBP_CONST __attribute__((address_space(4)))

template <class T>
__device__ __forceinline__ T table_load(const T *p)
{
    return *(const MGWFBP_CONST T *)p;
}

// A tile descriptor is three 64-bit words: start | seg, nseg | n, pad (pad = elements of
// padding that follow the tile in the merged order; only with the padded layout).
__device__ __forceinline__ TileDev load_tile(const TileDev *p)
{
    const uint64_t *q = reinterpret_cast<const uint64_t *>(p);
    const uint64_t w1 = table_load(q + 1), w2 = table_load(q + 2);
    TileDev t;
    t.start = table_load(q);
    t.seg = static_cast<uint32_t>(w1);
    t.nseg = static_cast<uint32_t>(w1 >> 32);
    t.n = static_cast<uint32_t>(w2);
    t.pad = static_cast<uint32_t>(w2 >> 32);
    return t;
}

// The fields of a segment descriptor the kernels need (plan offset and flags).
__device__ __forceinline__ SegDev load_seg(const SegDev *p)
{
    SegDev sg{};
    sg.plan_off = table_load(&p->plan_off);
    sg.flags = table_load(&p->flags);
    return sg;
}

// v = mu*v + g ; w = w - lr*v with one rounding per operation.
template <class T>
__device__ __forceinline__ void sgd_momentum(T g, T &w, T &v, float lr, float mu)
{
    const T mv = v * mu;
    const T vn = mv + g;
    const T step = vn * lr;
    v = vn;
    w = w - step;
}

// Sum of the N workers' values at index i (in units of T), worker 0 first, times 1/N.
// Fixed N: every load is issued before the first add so that N 128-bit requests per lane are
// in flight at once.
template <int NW, bool NT, class T>
__device__ __forceinline__ T nway_mean_fixed(const float *const (&sp)[NW], uint32_t i, float inv_n)
{
    T x[NW];
#pragma unroll
    for (int g = 0; g < NW; ++g) x[g] = ld<NT>(reinterpret_cast<const T *>(sp[g]) + i);
    T acc = x[0];
#pragma unroll
    for (int g = 1; g < NW; ++g) acc = acc + x[g];
    return acc * inv_n;
}

// Loads with the device-scope bit: served from where every compute die's writes are visible
// instead of this die's L2, for data that a kernel running at the same time produced.  There is
// no 128-bit atomic load to ask the compiler for, so the 128-bit form is written as instructions;
// the compiler's wait-count bookkeeping does not see them, so each statement ends with its own
// wait and the values are complete when it returns.
__device__ __forceinline__ void ld_device(const float *p, float &a)
{
    a = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ld_device(const v4f *p, v4f &a)
{
    asm volatile("global_load_dwordx4 %0, %1, off sc1 nt\n\ts_waitcnt vmcnt(0)" : "=&v"(a) : "v"(p));
}
__device__ __forceinline__ void ld_device4(const float *pa, const float *pb, const float *pc, const float *pd,
                                           float &a, float &b, float &c, float &d)
{
    a = __hip_atomic_load(pa, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    b = __hip_atomic_load(pb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    c = __hip_atomic_load(pc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    d = __hip_atomic_load(pd, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ld_device4(const v4f *pa, const v4f *pb, const v4f *pc, const v4f *pd,
                                           v4f &a, v4f &b, v4f &c, v4f &d)
{
    asm volatile("global_load_dwordx4 %0, %4, off sc1 nt\n\t"
                 "global_load_dwordx4 %1, %5, off sc1 nt\n\t"
                 "global_load_dwordx4 %2, %6, off sc1 nt\n\t"
                 "global_load_dwordx4 %3, %7, off sc1 nt\n\t"
                 "s_waitcnt vmcnt(0)"
                 : "=&v"(a), "=&v"(b), "=&v"(c), "=&v"(d)
                 : "v"(pa), "v"(pb), "v"(pc), "v"(pd));
}

// Run-time N: `ptr(g)` yields worker g's base pointer; loads go out four at a time.
// COH: with device-scope loads.
template <bool NT, class T, bool COH = false, class PtrFn>
__device__ __forceinline__ T nway_mean_dyn(PtrFn ptr, int nw, uint32_t i, float inv_n)
{
    if constexpr (COH) {
        // workers 0..3 together, then 4..7, ...: N = 8 is two round trips
        T acc;
        int g = 0;
        if (nw >= 4) {
            T b, c, d;
            ld_device4(reinterpret_cast<const T *>(ptr(0)) + i, reinterpret_cast<const T *>(ptr(1)) + i,
                       reinterpret_cast<const T *>(ptr(2)) + i, reinterpret_cast<const T *>(ptr(3)) + i,
                       acc, b, c, d);
            acc = acc + b;
            acc = acc + c;
            acc = acc + d;
            g = 4;
        } else {
            ld_device(reinterpret_cast<const T *>(ptr(0)) + i, acc);
            g = 1;
        }
        for (; g + 4 <= nw; g += 4) {
            T a, b, c, d;
            ld_device4(reinterpret_cast<const T *>(ptr(g)) + i, reinterpret_cast<const T *>(ptr(g + 1)) + i,
                       reinterpret_cast<const T *>(ptr(g + 2)) + i, reinterpret_cast<const T *>(ptr(g + 3)) + i,
                       a, b, c, d);
            acc = acc + a;
            acc = acc + b;
            acc = acc + c;
            acc = acc + d;
        }
        for (; g < nw; ++g) {
            T a;
            ld_device(reinterpret_cast<const T *>(ptr(g)) + i, a);
            acc = acc + a;
        }
        return acc * inv_n;
    } else {
        T acc = ld<NT>(reinterpret_cast<const T *>(ptr(0)) + i);
        int g = 1;
        for (; g + 4 <= nw; g += 4) {
            const T a = ld<NT>(reinterpret_cast<const T *>(ptr(g)) + i);
            const T b = ld<NT>(reinterpret_cast<const T *>(ptr(g + 1)) + i);
            const T c = ld<NT>(reinterpret_cast<const T *>(ptr(g + 2)) + i);
            const T d = ld<NT>(reinterpret_cast<const T *>(ptr(g + 3)) + i);
            acc = acc + a;
            acc = acc + b;
            acc = acc + c;
            acc = acc + d;
        }
        for (; g < nw; ++g) acc = acc + ld<NT>(reinterpret_cast<const T *>(ptr(g)) + i);
        return acc * inv_n;
    }
}

// Write the averaged value and, when STEP, apply the update.  Pointers are in units of float.
template <bool STEP, bool NT, class T>
__device__ __forceinline__ void finish(T avg, float *outp, float *wp, float *vp, uint32_t i,
                                       float lr, float mu)
{
    if constexpr (STEP) {
        T w = ld<NT>(reinterpret_cast<const T *>(wp) + i);
        T v = ld<NT>(reinterpret_cast<const T *>(vp) + i);
        sgd_momentum(avg, w, v, lr, mu);
        st<NT>(reinterpret_cast<T *>(vp) + i, v);
        st<NT>(reinterpret_cast<T *>(wp) + i, w);
    }
    if (outp) st<NT>(reinterpret_cast<T *>(outp) + i, avg);
}

// Offsets (relative to the tile start) and lengths of the segments a gather tile spans go to
// LDS; each lane then finds the segment holding its element by binary search.  With the padded
// layout the run has holes between the layers: position k lies in a hole when it is past the
// end of the segment that starts at or before it.
__device__ __forceinline__ void stage_gather_offsets(const DeviceTables &dt, const TileDev &tl,
                                                     uint32_t *s_rel, uint32_t *s_len)
{
    for (uint32_t k = threadIdx.x; k < tl.nseg; k += kBlock) {
        s_rel[k] = static_cast<uint32_t>(dt.segs[tl.seg + k].plan_off - tl.start);
        s_len[k] = static_cast<uint32_t>(dt.segs[tl.seg + k].n);
    }
    __syncthreads();
}

__device__ __forceinline__ uint32_t find_segment(const uint32_t *s_rel, uint32_t nseg, uint32_t k)
{
    uint32_t lo = 0, hi = nseg - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (s_rel[mid] <= k) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

// Global -> LDS and LDS -> global copies of n floats whose global side has arbitrary 4-byte
// alignment: a scalar head up to the next 16-byte boundary, a 128-bit body, a scalar tail.
template <bool NT>
__device__ __forceinline__ void global_to_lds(const float *src, float *lds, uint32_t n)
{
    uint32_t head = static_cast<uint32_t>((16u - (reinterpret_cast<uintptr_t>(src) & 15u)) & 15u) >> 2;
    head = head < n ? head : n;
    if (threadIdx.x < head) lds[threadIdx.x] = ld<NT>(src + threadIdx.x);
    const uint32_t nb = (n - head) >> 2;
    const v4f *s4 = reinterpret_cast<const v4f *>(src + head);
    for (uint32_t i = threadIdx.x; i < nb; i += kBlock) {
        const v4f x = ld<NT>(s4 + i);
        float *d = lds + head + 4 * i;
        d[0] = x.x;
        d[1] = x.y;
        d[2] = x.z;
        d[3] = x.w;
    }
    for (uint32_t i = head + 4 * nb + threadIdx.x; i < n; i += kBlock) lds[i] = ld<NT>(src + i);
}

template <bool NT>
__device__ __forceinline__ void lds_to_global(const float *lds, float *dst, uint32_t n)
{
    uint32_t head = static_cast<uint32_t>((16u - (reinterpret_cast<uintptr_t>(dst) & 15u)) & 15u) >> 2;
    head = head < n ? head : n;
    if (threadIdx.x < head) st<NT>(dst + threadIdx.x, lds[threadIdx.x]);
    const uint32_t nb = (n - head) >> 2;
    v4f *d4 = reinterpret_cast<v4f *>(dst + head);
    for (uint32_t i = threadIdx.x; i < nb; i += kBlock) {
        const float *s = lds + head + 4 * i;
        v4f x;
        x.x = s[0];
        x.y = s[1];
        x.z = s[2];
        x.w = s[3];
        st<NT>(d4 + i, x);
    }
    for (uint32_t i = head + 4 * nb + threadIdx.x; i < n; i += kBlock) st<NT>(dst + i, lds[i]);
}

// ------------------------------------------------------------------------------------------
// Fused single pass
// ------------------------------------------------------------------------------------------

// 128-bit streaming (non-temporal) load at (uniform base pointer) + (32-bit lane byte offset):
// the form the hardware addresses with a scalar register pair plus one vector register.  The
// loads of the fast path are written as instructions so that their order and the number in
// flight are exactly what the code says (left to itself the compiler hoists all N*U loads of
// a tile to the top, ~270 registers, one wave per SIMD).  Such a load is invisible to the
// compiler's own wait-count bookkeeping, so its result is passed through wait_all_loads()
// before the first use.
// COH: the load also carries the device-scope bit, so it is served from where every compute
// die's writes are visible instead of this die's L2 (for data another running kernel produced).
template <int OFF, bool COH = false>
__device__ __forceinline__ v4f ld_stream(const char *base, uint32_t voff)
{
    v4f r;
    if constexpr (COH)
        asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3 sc1 nt" : "=v"(r) : "v"(voff), "s"(base), "n"(OFF));
    else
        asm volatile("global_load_dwordx4 %0, %1, %2 offset:%3 nt" : "=v"(r) : "v"(voff), "s"(base), "n"(OFF));
    return r;
}

// Same load, ordered after the computation of `dep` (an in/out operand that is not touched).
template <int OFF, bool COH = false>
__device__ __forceinline__ v4f ld_stream_after(const char *base, uint32_t voff, v4f &dep)
{
    v4f r;
    if constexpr (COH)
        asm volatile("global_load_dwordx4 %0, %2, %3 offset:%4 sc1 nt"
                     : "=v"(r), "+v"(dep)
                     : "v"(voff), "s"(base), "n"(OFF));
    else
        asm volatile("global_load_dwordx4 %0, %2, %3 offset:%4 nt"
                     : "=v"(r), "+v"(dep)
                     : "v"(voff), "s"(base), "n"(OFF));
    return r;
}

// 128-bit streaming store in the same addressing form (the compiler, left to choose, builds a
// 64-bit address per lane and per piece: two registers and two additions each).
template <int OFF>
__device__ __forceinline__ void st_stream(char *base, uint32_t voff, const v4f &x)
{
    asm volatile("global_store_dwordx4 %0, %1, %2 offset:%3 nt"
                 :
                 : "v"(voff), "v"(x), "s"(base), "n"(OFF)
                 : "memory");
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a
// compile-time constant in every iteration.
template <int... J, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, J...>, F f)
{
    (f(std::integral_constant<int, J>{}), ...);
}

template <int N, class F>
__device__ __forceinline__ void static_for(F f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// Block until at most K of this wave's vector-memory loads are outstanding.  Loads return in
// issue order, so this covers x when K loads were issued after it.  x is an in/out operand only
// to pin the wait between the load and its first use.
template <int K>
__device__ __forceinline__ void wait_loads(v4f &x)
{
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(x) : "n"(K));
}

__device__ __forceinline__ void wait_all_loads(v4f &x) { wait_loads<0>(x); }

// A uniform pointer moved into scalar registers whatever the compiler thought of it.
// An SGPR written by a vector instruction (v_readfirstlane) must not be read by a vector
// memory instruction for 5 wait states.  The compiler pads its own memory instructions, but it
// does not look inside the hand-written loads, so the padding is done here: the s_nop takes
// both halves as operands, which places it after the readfirstlanes and before any use.
__device__ __forceinline__ const char *scalar_ptr(const void *p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
    uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
    asm volatile("s_nop 4" : "+s"(lo), "+s"(hi));
    return reinterpret_cast<const char *>((static_cast<uint64_t>(hi) << 32) | lo);
}

// Short pause between two loads of a wave (units of ~64 clocks).
__device__ __forceinline__ void pace_wave(int pace)
{
    for (int k = 0; k < pace; ++k) __builtin_amdgcn_s_sleep(1);
}

// A full tile of U*kBlock float4 per worker, every pointer 16-byte aligned.  Each lane owns U
// float4 (lane-interleaved, so every wave access is one contiguous KiB).  What measurement on
// MI355X says about streaming N buffers into one:
//   * one load in flight per wave, at full occupancy (8 waves per SIMD), beats any deeper
//     pipelining: a second outstanding load of the same wave costs 5-10 % of the bandwidth,
//     more when it goes to another worker's buffer (loads of a wave must return in order);
//   * visit one worker's buffer for all U pieces before moving to the next worker;
//   * read the whole tile before writing anything: stores mixed into the load stream cost
//     another 10-15 %;
//   * a pause of ~64 clocks between loads gains a further 1-2 %.
// So: U accumulators in registers, worker-major loop (which is also the fixed summation
// order: worker g is added after worker g-1), every load waited for before the next is
// issued, all stores at the end.
//
// src(g) yields worker g's tile base pointer (uniform over the workgroup).  SCALE = false
// skips the multiplication by 1/N: with NW = 1 the tile is then moved bit for bit, which is
// what pack and unpack need.
#ifndef MGWFBP_STEP_BATCH
#define MGWFBP_STEP_BATCH 4
#endif

//
// NW = 0: the number of workers `nw` is only known at run time.  The walk is the same with a
// loop over the workers that is not unrolled (worker 0 is peeled off: it initialises the
// accumulators); short launches keep the U pieces of one worker in flight instead of a ring
// across workers.
template <int NW, int U, bool STEP, int D, bool SCALE, bool COH = false, class SrcFn>
__device__ __forceinline__ void fast_tile(SrcFn src, float *outp, float *wp, float *vp,
                                          float inv_n, float lr, float mu, int pace, int nw = NW)
{
    // Lane offset of piece 0 (+BIAS); piece u sits u KiB further on, which the load and store
    // instructions add as their immediate offset (13 bits, signed: -4096 .. 4095), so one
    // register addresses the whole tile.  Each wave walks its own contiguous U KiB.
    // Pieces 8 and up (U = 16) sit 8 KiB further on: the scalar base is moved instead.
    constexpr int BIAS = U * 1024 > 4096 ? 4096 : 0;
    static_assert(U >= 1 && U <= 16, "piece offsets must fit the immediate plus one base step");
    const uint32_t vo = (threadIdx.x >> 6) * (U * 1024u) + (threadIdx.x & 63u) * 16u + BIAS;
#define MGWFBP_OFF(u) (((u) % 8) * 1024 - BIAS)
#define MGWFBP_HI(u) (((u) / 8) * 8192)
    v4f res[U];
    if constexpr (NW == 0 && D == 1) {
        {
            const char *sb = scalar_ptr(src(0));
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                v4f x;
                if constexpr (u == 0) x = ld_stream<MGWFBP_OFF(u), COH>(sb, vo);
                else x = ld_stream_after<MGWFBP_OFF(u), COH>(sb + MGWFBP_HI(u), vo, res[u - 1]);
                wait_all_loads(x);
                res[u] = x;
                pace_wave(pace);
            });
        }
#pragma unroll 1
        for (int g = 1; g < nw; ++g) {
            const char *sb = scalar_ptr(src(g));
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                v4f x = ld_stream_after<MGWFBP_OFF(u), COH>(sb + MGWFBP_HI(u), vo, res[u == 0 ? U - 1 : u - 1]);
                wait_all_loads(x);
                res[u] = res[u] + x;
                pace_wave(pace);
            });
        }
    } else if constexpr (NW == 0) {
        // latency-bound launches: the U pieces of a worker go out together
        {
            const char *sb = scalar_ptr(src(0));
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                res[u] = ld_stream<MGWFBP_OFF(u), COH>(sb + MGWFBP_HI(u), vo);
            });
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                wait_loads<U - 1 - u>(res[u]);
            });
        }
#pragma unroll 1
        for (int g = 1; g < nw; ++g) {
            const char *sb = scalar_ptr(src(g));
            v4f x[U];
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                // ordered after the previous worker's last add, so that no more than U loaded
                // values are live
                x[u] = ld_stream_after<MGWFBP_OFF(u), COH>(sb + MGWFBP_HI(u), vo, res[U - 1]);
            });
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                wait_loads<U - 1 - u>(x[u]);
                res[u] = res[u] + x[u];
            });
        }
    } else if constexpr (D == 1) {
        static_for<NW>([&](auto gc) {
            constexpr int g = decltype(gc)::value;
            const char *sb = scalar_ptr(src(g));
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                // the load is ordered after the previous add through its operand res[..]
                v4f x;
                if constexpr (g == 0 && u == 0) x = ld_stream<MGWFBP_OFF(u), COH>(sb, vo);
                else x = ld_stream_after<MGWFBP_OFF(u), COH>(sb + MGWFBP_HI(u), vo, res[u == 0 ? U - 1 : u - 1]);
                wait_all_loads(x);
                if constexpr (g == 0) res[u] = x;
                else res[u] = res[u] + x;
                pace_wave(pace);
            });
        });
    } else {
        // Launches too small to fill the chip are bound by latency, not bandwidth: keep D
        // loads in flight through a register ring (same visiting and summation order).
        constexpr int T = NW * U;
        constexpr int DD = D < T ? D : T;
        const char *sb[NW];
#pragma unroll
        for (int g = 0; g < NW; ++g) sb[g] = scalar_ptr(src(g));
        v4f x[DD];
        static_for<DD>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            x[j] = ld_stream<MGWFBP_OFF(j % U), COH>(sb[j / U] + MGWFBP_HI(j % U), vo);
        });
        static_for<T>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            constexpr int g = j / U, u = j % U;
            constexpr int newer = T - 1 - j < DD - 1 ? T - 1 - j : DD - 1;  // loads issued after load j
            wait_loads<newer>(x[j % DD]);
            if constexpr (g == 0) res[u] = x[j % DD];
            else res[u] = res[u] + x[j % DD];
            // the next load re-uses the slot just consumed; naming res[u] as an operand keeps
            // the add above ahead of it, so no more than DD loaded values are ever live
            if constexpr (j + DD < T)
                x[j % DD] = ld_stream_after<MGWFBP_OFF((j + DD) % U), COH>(sb[(j + DD) / U] + MGWFBP_HI((j + DD) % U), vo, res[u]);
        });
    }
    if constexpr (SCALE) {
#pragma unroll
        for (int u = 0; u < U; ++u) res[u] = res[u] * inv_n;
    }
    if constexpr (STEP) {
        // weights and momentum: read a batch, update, write the batch
        const char *wb = scalar_ptr(wp);
        const char *vb = scalar_ptr(vp);
        constexpr int UB = U < MGWFBP_STEP_BATCH ? U : MGWFBP_STEP_BATCH;  // float4 of w and of v held at once
        static_for<U / UB>([&](auto bc) {
            constexpr int u0 = decltype(bc)::value * UB;
            v4f w[UB], v[UB];
            static_for<UB>([&](auto kc) {
                constexpr int k = decltype(kc)::value;
                w[k] = ld_stream_after<MGWFBP_OFF(u0 + k), COH>(wb + MGWFBP_HI(u0 + k), vo, res[u0 + k]);
                wait_all_loads(w[k]);
                v[k] = ld_stream_after<MGWFBP_OFF(u0 + k), COH>(vb + MGWFBP_HI(u0 + k), vo, w[k]);
                wait_all_loads(v[k]);
            });
#pragma unroll
            for (int k = 0; k < UB; ++k) sgd_momentum(res[u0 + k], w[k], v[k], lr, mu);
            static_for<UB>([&](auto kc) {
                constexpr int k = decltype(kc)::value;
                st_stream<MGWFBP_OFF(u0 + k)>(const_cast<char *>(vb) + MGWFBP_HI(u0 + k), vo, v[k]);
                st_stream<MGWFBP_OFF(u0 + k)>(const_cast<char *>(wb) + MGWFBP_HI(u0 + k), vo, w[k]);
            });
        });
    }
    // without the update the averaged gradient is the only output, so out[] is always bound
    if (!STEP || outp) {
        char *ob = const_cast<char *>(scalar_ptr(outp));
        static_for<U>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            st_stream<MGWFBP_OFF(u)>(ob + MGWFBP_HI(u), vo, res[u]);
        });
    }
#undef MGWFBP_OFF
#undef MGWFBP_HI
}

// U > 0: full aligned tiles of U*kBlock float4 take fast_tile; everything else (ragged tails,
// misaligned tensors, gather tiles) takes the general path below.
// COH: the gradients were written by a kernel that ran while this one was already running (the
// gated launch): every load of a gradient carries the device-scope bit (the run-time-N code only).
template <int NW, int U, bool STEP, bool NT, int D, bool COH = false>
__device__ __forceinline__ void fused_tile(const DeviceTables &dt, uint32_t tile_index, int nw, float inv_n,
                                           float lr, float mu, int pace, float *merged_out, uint64_t base_off,
                                           uint32_t *s_rel, uint32_t *s_len)
{
    // merged_out != nullptr: the averaged values go to a merged buffer (the layer buffer of
    // Algorithm 2, already reduced) at their packed position instead of the per-layer out[].
    const TileDev tl = load_tile(dt.tiles + tile_index);

    if (tl.nseg == 1) {
        const uint32_t flags = table_load(&dt.segs[tl.seg].flags);
        const float *const *sp_tbl = dt.src + static_cast<size_t>(tl.seg) * nw;
        float *outp;
        uint32_t need = SEG_SRC_ALIGNED | SEG_WV_ALIGNED;
        bool merged_al = true;
        if (!STEP && merged_out) {  // the update never targets a merged buffer
            const uint64_t moff = table_load(&dt.segs[tl.seg].plan_off) - base_off + tl.start;
            outp = merged_out + moff;
            merged_al = !(moff & 3);
        } else {
            outp = dt.out ? table_load(dt.out + tl.seg) + tl.start : nullptr;
            need |= SEG_OUT_ALIGNED;
        }
        float *wp = STEP ? table_load(dt.w + tl.seg) + tl.start : nullptr;
        float *vp = STEP ? table_load(dt.v + tl.seg) + tl.start : nullptr;
        const uint32_t n = tl.n;
        const bool vec = (flags & need) == need && merged_al;
        if constexpr (U > 0) {
            if (vec && n == U * kBlock * 4) {
                const uint64_t start = tl.start;
                fast_tile<NW, U, STEP, D, true, COH>(
                    [sp_tbl, start](int g) { return table_load(sp_tbl + g) + start; }, outp, wp, vp,
                    inv_n, lr, mu, pace, nw);
                return;
            }
        }
        if (!STEP && merged_out && threadIdx.x < tl.pad) st<NT>(outp + n + threadIdx.x, 0.0f);
        const uint32_t n4 = vec ? (n >> 2) : 0;
        if constexpr (NW > 0) {
            // per-worker base pointers of this tile (uniform over the workgroup)
            const float *sp[NW];
#pragma unroll
            for (int g = 0; g < NW; ++g) sp[g] = table_load(sp_tbl + g) + tl.start;
#pragma unroll 1
            for (uint32_t i = threadIdx.x; i < n4; i += kBlock) {
                const v4f avg = nway_mean_fixed<NW, NT, v4f>(sp, i, inv_n);
                finish<STEP, NT, v4f>(avg, outp, wp, vp, i, lr, mu);
            }
#pragma unroll 1
            for (uint32_t i = (n4 << 2) + threadIdx.x; i < n; i += kBlock) {
                const float avg = nway_mean_fixed<NW, NT, float>(sp, i, inv_n);
                finish<STEP, NT, float>(avg, outp, wp, vp, i, lr, mu);
            }
        } else {
            const uint64_t start = tl.start;
            auto ptr = [sp_tbl, start](int g) { return sp_tbl[g] + start; };
#pragma unroll 1
            for (uint32_t i = threadIdx.x; i < n4; i += kBlock) {
                const v4f avg = nway_mean_dyn<NT, v4f, COH>(ptr, nw, i, inv_n);
                finish<STEP, NT, v4f>(avg, outp, wp, vp, i, lr, mu);
            }
#pragma unroll 1
            for (uint32_t i = (n4 << 2) + threadIdx.x; i < n; i += kBlock) {
                const float avg = nway_mean_dyn<NT, float, COH>(ptr, nw, i, inv_n);
                finish<STEP, NT, float>(avg, outp, wp, vp, i, lr, mu);
            }
        }
    } else {
        stage_gather_offsets(dt, tl, s_rel, s_len);
#pragma unroll 1
        for (uint32_t k = threadIdx.x; k < tl.n; k += kBlock) {
            const uint32_t s = find_segment(s_rel, tl.nseg, k);
            const uint32_t si = tl.seg + s;
            const uint32_t i = k - s_rel[s];
            if (i >= s_len[s]) {  // padding between two layers: zero in a merged buffer, else nothing
                if (!STEP && merged_out) st<NT>(merged_out + (tl.start - base_off) + k, 0.0f);
                continue;
            }
            const float *const *sp_tbl = dt.src + static_cast<size_t>(si) * nw;
            const float avg = nway_mean_dyn<NT, float, COH>([sp_tbl](int g) { return sp_tbl[g]; }, nw, i, inv_n);
            if (!STEP && merged_out)  // a gather tile is one contiguous run of the merged buffer
                st<NT>(merged_out + (tl.start - base_off) + k, avg);
            else
                finish<STEP, NT, float>(avg, dt.out ? dt.out[si] : nullptr, STEP ? dt.w[si] : nullptr,
                                        STEP ? dt.v[si] : nullptr, i, lr, mu);
        }
    }
}

template <int NW, int U, bool STEP, bool NT, int D>
__global__ void __launch_bounds__(kBlock)
k_fused(DeviceTables dt, uint32_t tile_begin, int nw, float inv_n, float lr, float mu, int pace,
        float *merged_out, uint64_t base_off)
{
    __shared__ uint32_t s_rel[kMaxGatherSegs], s_len[kMaxGatherSegs];
    fused_tile<NW, U, STEP, NT, D>(dt, tile_begin + blockIdx.x, nw, inv_n, lr, mu, pace, merged_out, base_off,
                                   s_rel, s_len);
}

// ------------------------------------------------------------------------------------------
// Algorithm 2's communication thread as one launch
// ------------------------------------------------------------------------------------------
// Algorithm 2 sends a group when its lowest layer arrives from the backward pass.  Launching a
// kernel per group costs 3.5 us each for groups that hold a few kilobytes (a dependent launch
// cannot be shorter on this part), 90 of the 232 us of ResNet-50's 33 launches.  Here the whole
// plan is ONE launch over a list of the tiles in arrival order.  Its workgroups stay: workgroup b
// takes tiles b, b + gridDim.x, ... of the list and, before each, waits until the tile's group
// has arrived, which is when the group's counter in device memory has reached this iteration's
// number.  Whoever produces the gradients (here: the stand-ins of the backward pass) bumps the
// group's counter with a release store behind its work.
//   * Every wait is bounded: after max_polls polls of about a microsecond the workgroup sets
//     the give-up word and ends, and every other workgroup ends at its next look at that word,
//     so the launch always drains; the host then reports the failure.
//   * The caller launches fewer workgroups than the chip holds at once, so the kernels that
//     bump the counters find free slots (kernels that need whole SIMDs do not: every compute
//     unit has some of this launch's workgroups).
//   * The gradients were written while this kernel was already running, by a kernel that may
//     have run on another compute die, and each die has its own L2.  The polls read the counter
//     with device-scope loads that order nothing (an acquiring load drops the die's cached
//     lines each time: 30 us more per ResNet-50 pass when every tile did it).  The gradients
//     are then read with device-scope loads as well, which costs nothing measurable, and the
//     tables stay in the die's L2.
//   * The worker loop is the run-time one (any N), one load in flight per wave.
__device__ __forceinline__ uint32_t load_agent(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t peek_agent(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kGatedReserve = 2;         // workgroup slots per compute unit the gated launch leaves free at least
constexpr int kGatedDefaultReserve = 4;  // and by default

// *ctl: the give-up word, zero when the launch starts
template <int U, bool STEP>
__global__ void __launch_bounds__(kBlock)
k_fused_gated(DeviceTables dt, uint32_t tile_begin, uint32_t n_tiles, int nw, float inv_n, float lr, float mu,
              int pace, const uint32_t *ready, uint32_t epoch, uint32_t *ctl, uint64_t max_polls)
{
    __shared__ uint32_t s_rel[kMaxGatherSegs], s_len[kMaxGatherSegs];
    __shared__ uint32_t s_go;
#pragma unroll 1
    for (uint32_t i = blockIdx.x; i < n_tiles; i += gridDim.x) {
        // the tables are the host's and never change: the tile's descriptor is read before the wait
        // (its second word holds the first segment, whose group is the tile's)
        const uint32_t seg = static_cast<uint32_t>(
            table_load(reinterpret_cast<const uint64_t *>(dt.tiles + tile_begin + i) + 1));
        const uint32_t grp = table_load(&dt.segs[seg].group);
        if (threadIdx.x == 0) {
            uint32_t go = 0;
            for (uint64_t k = 0; k < max_polls; ++k) {
                const uint32_t stop = peek_agent(ctl), seen = peek_agent(ready + grp);  // both in flight
                if (stop != 0) break;
                // counters only grow; the difference is taken modulo 2^32
                if (static_cast<int32_t>(seen - epoch) >= 0) {
                    go = 1;
                    break;
                }
                __builtin_amdgcn_s_sleep(16);
            }
            if (!go) __hip_atomic_store(ctl, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_go = go;
        }
        __syncthreads();
        const uint32_t go = s_go;
        __syncthreads();  // s_go and the gather tables are rewritten in the next pass
        if (!go) return;  // the same for every lane of the workgroup
        fused_tile<0, U, STEP, true, 1, true>(dt, tile_begin + i, nw, inv_n, lr, mu, pace, nullptr, 0, s_rel, s_len);
    }
}

// The kernels in front of this one in its stream have ended, which made what they wrote visible
// to the whole device; the store itself needs to order nothing more.
__global__ void __launch_bounds__(64) k_signal(uint32_t *counter, uint32_t epoch)
{
    if (threadIdx.x == 0) __hip_atomic_store(counter, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void __launch_bounds__(64)
k_await(const uint32_t *word, uint32_t value, uint32_t *result, uint64_t max_polls)
{
    if (threadIdx.x != 0) return;
    uint32_t seen = 2u;
    for (uint64_t i = 0; i < max_polls; ++i) {
        if (load_agent(word) == value) {
            seen = 1u;
            break;
        }
        __builtin_amdgcn_s_sleep(32);
    }
    __hip_atomic_store(result, seen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ------------------------------------------------------------------------------------------
// Materialised path
// ------------------------------------------------------------------------------------------
// Workspace: N packed replica buffers of `epad` floats each, then the reduced buffer.
// `base_off` is the plan offset of the scope's first element (0 for the whole plan).

template <int NW, bool NT, int U, int D>
__global__ void __launch_bounds__(kBlock)
k_reduce(float *ws, uint64_t epad, uint64_t elems, uint32_t tile, int nw, float inv_n, int pace)
{
    const uint64_t t0 = static_cast<uint64_t>(blockIdx.x) * tile;
    const uint32_t n = static_cast<uint32_t>(elems - t0 < tile ? elems - t0 : tile);
    float *outp = ws + static_cast<uint64_t>(nw) * epad + t0;
    if constexpr (U > 0) {
        if (n == U * kBlock * 4) {
            fast_tile<NW, U, false, D, true>(
                [ws, epad, t0](int g) { return ws + static_cast<uint64_t>(g) * epad + t0; }, outp,
                nullptr, nullptr, inv_n, 0.0f, 0.0f, pace, nw);
            return;
        }
    }
    const uint32_t n4 = n >> 2;  // workspace and epad keep every buffer 16-byte aligned
    if constexpr (NW > 0) {
        const float *sp[NW];
#pragma unroll
        for (int g = 0; g < NW; ++g) sp[g] = ws + static_cast<uint64_t>(g) * epad + t0;
#pragma unroll 1
        for (uint32_t i = threadIdx.x; i < n4; i += kBlock)
            st<NT>(reinterpret_cast<v4f *>(outp) + i, nway_mean_fixed<NW, NT, v4f>(sp, i, inv_n));
        for (uint32_t i = (n4 << 2) + threadIdx.x; i < n; i += kBlock)
            st<NT>(outp + i, nway_mean_fixed<NW, NT, float>(sp, i, inv_n));
    } else {
        auto ptr = [ws, epad, t0](int g) { return ws + static_cast<uint64_t>(g) * epad + t0; };
#pragma unroll 1
        for (uint32_t i = threadIdx.x; i < n4; i += kBlock)
            st<NT>(reinterpret_cast<v4f *>(outp) + i, nway_mean_dyn<NT, v4f>(ptr, nw, i, inv_n));
        for (uint32_t i = (n4 << 2) + threadIdx.x; i < n; i += kBlock)
            st<NT>(outp + i, nway_mean_dyn<NT, float>(ptr, nw, i, inv_n));
    }
}

// ------------------------------------------------------------------------------------------
// Copy-like steps in small pieces
// ------------------------------------------------------------------------------------------
// Streams that are half writes want the opposite of the N-way reduction.  Measured on MI355X
// with plain copy kernels over 512 MiB buffers: one 16-byte access per lane and workgroup
// (2 KiB per workgroup, 262 144 workgroups) copies at 84 % of the HBM peak, two per lane at
// 80 %, four or eight at 74 % -- the vendor's own device-to-device copy reaches 66 %.  Short
// workgroups keep everything the chip has in flight inside a window of a few MiB that sweeps
// through the buffers in address order; long ones spread it over tens of MiB.
//
// So pack and unpack do not run one workgroup per tile: a tile of the plan's list is cut into
// pieces of SV * kBlock float4 (512 elements for SV = 1), one workgroup each, `subs` pieces per
// tile, consecutive workgroups taking consecutive pieces.  A piece that lies beyond the end of
// a ragged tile exits at once.  Pieces of a tile whose two sides disagree on 16-byte alignment
// are realigned through a piece-sized LDS buffer; a gather tile (many tiny layers) is handled
// whole by its first piece with 32-bit accesses.
//
// Where a piece starts matters on the side that is written: a wave's 1 KiB store that begins
// 16 or 32 bytes past a 64-byte boundary leaves a partly written 64-byte sector at both ends,
// and the same copy kernel drops from 84 % to 76 % of peak (a pure fill from 75 % to 52 %);
// misaligned reads cost 3 points.  The merged offset of a layer is whatever the layers before
// it add up to, so the pieces of a tile are laid out from the first 128-byte boundary of the
// written side: the tile's first `head` elements (under 32) ride with piece 0, and piece k
// covers [head + k * kElems, head + (k + 1) * kElems).
template <int SV>
struct Piece {
    static constexpr uint32_t kElems = SV * kBlock * 4;
};

// x / d for a workgroup-uniform x with the host's m = floor(2^32 / d) (2^32 - 1 for d = 1):
// the estimate mulhi(x, m) is the quotient or one less, so one correction makes it exact for
// every 32-bit x.  Multiply-high, multiply, compare: all on the scalar unit (a plain `/` goes
// through the vector unit's reciprocal and back).
struct Divisor {
    uint32_t d, m;
};
__device__ __forceinline__ uint32_t div_uniform(uint32_t x, Divisor dv)
{
    uint32_t q = __umulhi(x, dv.m);
    if (x - q * dv.d >= dv.d) ++q;
    return q;
}

// Elements from the start of a tile to the first 128-byte boundary of `written` (a 16-byte
// aligned address): 0, 4, .. 28.
__device__ __forceinline__ uint32_t head_elems(const float *written)
{
    return (32u - (static_cast<uint32_t>(reinterpret_cast<uintptr_t>(written) >> 2) & 31u)) & 31u;
}

// Range [lo, hi) of piece `sub` in a tile of n elements whose pieces start `head` elements in.
template <int SV>
__device__ __forceinline__ bool piece_range(uint32_t sub, uint32_t head, uint32_t n, uint32_t &lo, uint32_t &hi)
{
    const uint32_t base = head + sub * Piece<SV>::kElems;
    lo = sub == 0 ? 0 : base;
    hi = base + Piece<SV>::kElems < n ? base + Piece<SV>::kElems : n;
    return lo < n;
}

// Copy elements [lo, hi) of a tile whose two sides are 16-byte aligned at element 0 (lo, head
// multiples of four).  Every lane moves up to SV float4 of the piece proper, loads first; the
// first lanes of piece 0 also move the head, the last piece the 1-3 trailing elements.
template <bool NT, int SV>
__device__ __forceinline__ void copy_piece_aligned(const float *src, float *dst, uint32_t lo, uint32_t hi,
                                                   uint32_t head)
{
    const uint32_t body = lo == 0 ? head : lo;  // where the 128-byte aligned part of the piece starts
    const uint32_t i0 = (body >> 2) + threadIdx.x, n4 = hi >> 2;
    v4f x[SV], h;
    const bool has_head = lo == 0 && threadIdx.x < (head >> 2) && threadIdx.x < n4;
    if (has_head) h = ld<NT>(reinterpret_cast<const v4f *>(src) + threadIdx.x);
#pragma unroll
    for (int k = 0; k < SV; ++k)
        if (i0 + k * kBlock < n4) x[k] = ld<NT>(reinterpret_cast<const v4f *>(src) + i0 + k * kBlock);
    if (has_head) st<NT>(reinterpret_cast<v4f *>(dst) + threadIdx.x, h);
#pragma unroll
    for (int k = 0; k < SV; ++k)
        if (i0 + k * kBlock < n4) st<NT>(reinterpret_cast<v4f *>(dst) + i0 + k * kBlock, x[k]);
    const uint32_t t = (n4 << 2) + threadIdx.x;
    if (t >= lo && t < hi) st<NT>(dst + t, ld<NT>(src + t));
}

template <bool NT, int SV>
__global__ void __launch_bounds__(kBlock)
k_pack(DeviceTables dt, uint32_t tile_begin, Divisor subs, Divisor workers, float *ws, uint64_t epad,
       uint64_t base_off, bool worker_fastest)
{
    __shared__ float s_buf[Piece<SV>::kElems];
    __shared__ uint32_t s_rel[kMaxGatherSegs], s_len[kMaxGatherSegs];
    // consecutive workgroups take the same piece of consecutive workers (measured against one
    // worker's whole buffer after the other: 261 against 270-290 us on ResNet-50 sizes, 2890
    // against 2900-3080 us on VGG-16 sizes); a grid too long for one dimension puts the worker
    // into the second one
    const int nw = static_cast<int>(workers.d);
    uint32_t lin = blockIdx.x, g = blockIdx.y;
    if (worker_fastest) {
        lin = div_uniform(blockIdx.x, workers);
        g = blockIdx.x - lin * workers.d;
    }
    const uint32_t t = div_uniform(lin, subs), sub = lin - t * subs.d;
    const TileDev tl = load_tile(dt.tiles + tile_begin + t);
    float *merged = ws + static_cast<uint64_t>(g) * epad;
    if (tl.nseg == 1) {
        const SegDev sg = load_seg(dt.segs + tl.seg);
        const float *src = table_load(dt.src + static_cast<size_t>(tl.seg) * nw + g) + tl.start;
        const uint64_t moff = sg.plan_off - base_off + tl.start;
        float *dst = merged + moff;
        const bool aligned = (sg.flags & SEG_SRC_ALIGNED) && !(moff & 3);
        const uint32_t head = aligned ? head_elems(dst) : 0;
        uint32_t lo, hi;
        if (!piece_range<SV>(sub, head, tl.n, lo, hi)) return;
        if (hi == tl.n && threadIdx.x < tl.pad) st<NT>(dst + tl.n + threadIdx.x, 0.0f);  // padding after the layer
        if (aligned) {
            copy_piece_aligned<NT, SV>(src, dst, lo, hi, head);
        } else {
            global_to_lds<NT>(src + lo, s_buf, hi - lo);
            __syncthreads();
            lds_to_global<NT>(s_buf, dst + lo, hi - lo);
        }
    } else {
        if (sub != 0) return;
        stage_gather_offsets(dt, tl, s_rel, s_len);
        float *run = merged + (tl.start - base_off);
        for (uint32_t k = threadIdx.x; k < tl.n; k += kBlock) {
            const uint32_t s = find_segment(s_rel, tl.nseg, k);
            const uint32_t i = k - s_rel[s];
            const float *src = dt.src[static_cast<size_t>(tl.seg + s) * nw + g];
            st<NT>(run + k, i < s_len[s] ? ld<NT>(src + i) : 0.0f);  // zero in the padding between layers
        }
    }
}

template <bool STEP, bool NT, int SV>
__global__ void __launch_bounds__(kBlock)
k_unpack(DeviceTables dt, uint32_t tile_begin, Divisor subs, const float *reduced,
         uint64_t base_off, float lr, float mu)
{
    __shared__ float s_buf[Piece<SV>::kElems];
    __shared__ uint32_t s_rel[kMaxGatherSegs], s_len[kMaxGatherSegs];
    const uint32_t t = div_uniform(blockIdx.x, subs), sub = blockIdx.x - t * subs.d;
    const TileDev tl = load_tile(dt.tiles + tile_begin + t);
    if (tl.nseg == 1) {
        const SegDev sg = load_seg(dt.segs + tl.seg);
        const uint64_t moff = sg.plan_off - base_off + tl.start;
        const float *src = reduced + moff;
        float *outp = dt.out ? table_load(dt.out + tl.seg) + tl.start : nullptr;
        float *wp = STEP ? table_load(dt.w + tl.seg) + tl.start : nullptr;
        float *vp = STEP ? table_load(dt.v + tl.seg) + tl.start : nullptr;
        const bool tensors_al = (sg.flags & (SEG_OUT_ALIGNED | SEG_WV_ALIGNED)) ==
                                (SEG_OUT_ALIGNED | SEG_WV_ALIGNED);
        const bool aligned = tensors_al && !(moff & 3);
        // the pieces follow the 128-byte boundaries of the tensor that is written (the weights
        // when there is an update; momentum and out[] usually share their alignment)
        const uint32_t head = aligned ? head_elems(STEP ? wp : outp) : 0;
        uint32_t lo, hi;
        if (!piece_range<SV>(sub, head, tl.n, lo, hi)) return;
        if (aligned) {
            if constexpr (!STEP) {
                copy_piece_aligned<NT, SV>(src, outp, lo, hi, head);
            } else {
                const uint32_t body = lo == 0 ? head : lo;
                const uint32_t i0 = (body >> 2) + threadIdx.x, n4 = hi >> 2;
                if (lo == 0 && threadIdx.x < (head >> 2) && threadIdx.x < n4)
                    finish<STEP, NT, v4f>(ld<NT>(reinterpret_cast<const v4f *>(src) + threadIdx.x), outp, wp, vp,
                                          threadIdx.x, lr, mu);
                v4f g[SV], w[SV], v[SV];
#pragma unroll
                for (int k = 0; k < SV; ++k) {
                    const uint32_t i = i0 + k * kBlock;
                    if (i < n4) {
                        g[k] = ld<NT>(reinterpret_cast<const v4f *>(src) + i);
                        w[k] = ld<NT>(reinterpret_cast<const v4f *>(wp) + i);
                        v[k] = ld<NT>(reinterpret_cast<const v4f *>(vp) + i);
                    }
                }
#pragma unroll
                for (int k = 0; k < SV; ++k) {
                    const uint32_t i = i0 + k * kBlock;
                    if (i < n4) {
                        sgd_momentum(g[k], w[k], v[k], lr, mu);
                        st<NT>(reinterpret_cast<v4f *>(vp) + i, v[k]);
                        st<NT>(reinterpret_cast<v4f *>(wp) + i, w[k]);
                        if (outp) st<NT>(reinterpret_cast<v4f *>(outp) + i, g[k]);
                    }
                }
                const uint32_t tt = (n4 << 2) + threadIdx.x;
                if (tt >= lo && tt < hi) finish<STEP, NT, float>(ld<NT>(src + tt), outp, wp, vp, tt, lr, mu);
            }
        } else {
            const uint32_t cnt = hi - lo;
            global_to_lds<NT>(src + lo, s_buf, cnt);
            __syncthreads();
            uint32_t done = 0;
            if (tensors_al) {  // head = 0 here, so lo is a multiple of four: the tensor side is aligned
                const uint32_t n4 = cnt >> 2;
                for (uint32_t i = threadIdx.x; i < n4; i += kBlock) {
                    const v4f avg = *reinterpret_cast<const v4f *>(s_buf + 4 * i);
                    finish<STEP, NT, v4f>(avg, outp ? outp + lo : nullptr, STEP ? wp + lo : nullptr,
                                          STEP ? vp + lo : nullptr, i, lr, mu);
                }
                done = n4 << 2;
            }
            for (uint32_t i = done + threadIdx.x; i < cnt; i += kBlock)
                finish<STEP, NT, float>(s_buf[i], outp, wp, vp, lo + i, lr, mu);
        }
    } else {
        if (sub != 0) return;
        stage_gather_offsets(dt, tl, s_rel, s_len);
        const float *run = reduced + (tl.start - base_off);
        for (uint32_t k = threadIdx.x; k < tl.n; k += kBlock) {
            const uint32_t s = find_segment(s_rel, tl.nseg, k);
            const uint32_t si = tl.seg + s;
            const uint32_t i = k - s_rel[s];
            if (i >= s_len[s]) continue;  // padding between two layers
            finish<STEP, NT, float>(ld<NT>(run + k), dt.out ? dt.out[si] : nullptr, STEP ? dt.w[si] : nullptr,
                                    STEP ? dt.v[si] : nullptr, i, lr, mu);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Stand-in for one layer's backward computation: one wave that waits until `ticks` of the
// constant-rate real-time counter have passed.  It touches no memory.  The loop ends when the
// counter has advanced far enough; the iteration cap is a second, independent exit.
// ------------------------------------------------------------------------------------------
// mode 0: wait `ticks` from now; then, if `clock` is given, publish the counter's value there.
// mode 1: wait until `ticks` after the value published in `clock` (an absolute deadline, so the
//         gaps between consecutive stand-ins do not add up).
// arrive != nullptr: at its end the stand-in also bumps a group's arrival counter for the gated
// launch, as the kernel that produces the group's last gradients would (a release store: what
// the kernel wrote is visible to the device before the counter is).
__global__ void __launch_bounds__(64)
k_spin(uint64_t ticks, uint64_t max_polls, uint64_t *clock, int mode, uint32_t *arrive, uint32_t epoch)
{
    const uint64_t t0 = mode == 1 ? __builtin_nontemporal_load(clock) : __builtin_amdgcn_s_memrealtime();
    for (uint64_t i = 0; i < max_polls; ++i) {
        if (__builtin_amdgcn_s_memrealtime() - t0 >= ticks) break;
        __builtin_amdgcn_s_sleep(32);
    }
    if (mode == 0 && clock != nullptr && threadIdx.x == 0)
        __builtin_nontemporal_store(static_cast<uint64_t>(__builtin_amdgcn_s_memrealtime()), clock);
    if (arrive != nullptr && threadIdx.x == 0)
        __hip_atomic_store(arrive, epoch, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

int check_launch(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error(std::string(what) + ": " + hipGetErrorString(e));
        return MGWFBP_EHIP;
    }
    return MGWFBP_OK;
}

// The fast path exists for tiles of U*kBlock float4, U = 2, 4 or 8 (1024, 2048, 4096 elements),
// for the worker counts 1, 2, 4, 8, 16 with the worker loop unrolled and for any other count with
// a run-time loop (NW = 0).
// deep = launch too small to fill the chip (latency-bound): 8 loads in flight per wave.
template <int NW, bool STEP, bool NT>
void fused_launch_u(int u, bool deep, dim3 grid, size_t cap_lds, hipStream_t s, const DeviceTables &dt,
                    uint32_t tb, int nw, float inv_n, float lr, float mu, int pace, float *merged_out,
                    uint64_t base_off)
{
    // grid.x == 0 asks for the kernel to be looked up in the runtime, not launched
#define MGWFBP_LAUNCH(UU, DD)                                                                  \
    do {                                                                                       \
        if (grid.x == 0) {                                                                     \
            hipFuncAttributes fa;                                                              \
            (void)hipFuncGetAttributes(&fa, reinterpret_cast<const void *>(&k_fused<NW, UU, STEP, NT, DD>)); \
        } else {                                                                               \
            k_fused<NW, UU, STEP, NT, DD><<<grid, kBlock, cap_lds, s>>>(dt, tb, nw, inv_n, lr, mu, pace, merged_out, base_off); \
        }                                                                                      \
    } while (0)
    if constexpr (NT) {
        if (u == 2) { if (deep) MGWFBP_LAUNCH(2, 8); else MGWFBP_LAUNCH(2, 1); return; }
        if (u == 4) { if (deep) MGWFBP_LAUNCH(4, 8); else MGWFBP_LAUNCH(4, 1); return; }
        if (u == 8) { if (deep) MGWFBP_LAUNCH(8, 8); else MGWFBP_LAUNCH(8, 1); return; }
        if constexpr (!STEP) {
            // the longer tiles of the alternative whole-plan list (reduce pass only)
            if (u == 16) { if (deep) MGWFBP_LAUNCH(16, 8); else MGWFBP_LAUNCH(16, 1); return; }
            if (u == 10) { MGWFBP_LAUNCH(10, 1); return; }
            if (u == 12) { MGWFBP_LAUNCH(12, 1); return; }
            if (u == 14) { MGWFBP_LAUNCH(14, 1); return; }
        }
    }
    MGWFBP_LAUNCH(0, 1);
#undef MGWFBP_LAUNCH
}

template <bool STEP, bool NT>
void fused_dispatch(int nw, int u, bool deep, dim3 grid, size_t cap_lds, hipStream_t s,
                    const DeviceTables &dt, uint32_t tb, float inv_n, float lr, float mu, int pace,
                    float *merged_out, uint64_t base_off)
{
    switch (nw) {
    case 1: fused_launch_u<1, STEP, NT>(u, deep, grid, cap_lds, s, dt, tb, nw, inv_n, lr, mu, pace, merged_out, base_off); break;
    case 2: fused_launch_u<2, STEP, NT>(u, deep, grid, cap_lds, s, dt, tb, nw, inv_n, lr, mu, pace, merged_out, base_off); break;
    case 4: fused_launch_u<4, STEP, NT>(u, deep, grid, cap_lds, s, dt, tb, nw, inv_n, lr, mu, pace, merged_out, base_off); break;
    case 8: fused_launch_u<8, STEP, NT>(u, deep, grid, cap_lds, s, dt, tb, nw, inv_n, lr, mu, pace, merged_out, base_off); break;
    case 16: fused_launch_u<16, STEP, NT>(u, deep, grid, cap_lds, s, dt, tb, nw, inv_n, lr, mu, pace, merged_out, base_off); break;
    default: fused_launch_u<0, STEP, NT>(u, deep, grid, cap_lds, s, dt, tb, nw, inv_n, lr, mu, pace, merged_out, base_off); break;
    }
}

// Run fn(U_const, D_const) for the (U, deep) pair chosen at run time; U = 0 selects the general
// code only.
template <class Fn>
void with_shape(bool fast, int u, bool deep, Fn fn)
{
    using std::integral_constant;
    if (fast && u == 2) { if (deep) fn(integral_constant<int, 2>{}, integral_constant<int, 8>{}); else fn(integral_constant<int, 2>{}, integral_constant<int, 1>{}); return; }
    if (fast && u == 4) { if (deep) fn(integral_constant<int, 4>{}, integral_constant<int, 8>{}); else fn(integral_constant<int, 4>{}, integral_constant<int, 1>{}); return; }
    if (fast && u == 8) { if (deep) fn(integral_constant<int, 8>{}, integral_constant<int, 8>{}); else fn(integral_constant<int, 8>{}, integral_constant<int, 1>{}); return; }
    fn(integral_constant<int, 0>{}, integral_constant<int, 1>{});
}

template <int NW>
void reduce_launch(bool nt, int u, bool deep, dim3 grid, hipStream_t s, float *ws, uint64_t epad,
                   uint64_t elems, uint32_t tile, int nw, float inv_n, int pace)
{
    if (!nt) {
        k_reduce<NW, false, 0, 1><<<grid, kBlock, 0, s>>>(ws, epad, elems, tile, nw, inv_n, pace);
        return;
    }
    {
        // longer tiles, chosen by launch_reduce
#define MGWFBP_REDUCE_LONG(UU)                                                                  \
    if (u == UU && !deep) {                                                                      \
        k_reduce<NW, true, UU, 1><<<grid, kBlock, 0, s>>>(ws, epad, elems, tile, nw, inv_n, pace); \
        return;                                                                                  \
    }
        MGWFBP_REDUCE_LONG(10)
        MGWFBP_REDUCE_LONG(12)
        MGWFBP_REDUCE_LONG(14)
        MGWFBP_REDUCE_LONG(16)
#undef MGWFBP_REDUCE_LONG
    }
    with_shape(true, u, deep, [&](auto uc, auto dc) {
        k_reduce<NW, true, decltype(uc)::value, decltype(dc)::value>
            <<<grid, kBlock, 0, s>>>(ws, epad, elems, tile, nw, inv_n, pace);
    });
}

}  // namespace

namespace {
// Pause between two loads of a wave (MGWFBP_OPT_PACE; -1 = chosen here).  Measured on MI355X over
// launches of 3 k to 40 k workgroups: a launch that fits the chip in about one and a half batches
// of resident workgroups (ResNet-50, GoogLeNet sized) is fastest with almost no pause, because a
// slower workgroup lengthens the partly filled last batch; from about 1.6 batches on, thinning the
// request stream gains (N = 8: +3 to +5 % at 12 near 8 k workgroups, +2.5 % AlexNet sized;
// N = 16: +1.5 % at 8 near 7 k, +4 % VGG-16 sized; more than that loses again).  The update
// kernel pauses only in its gradient phase: N = 8 gains 1-2 % at 8 on long launches, N = 16
// peaks at 4.
enum class Stream { reduce, update };
int pace_for(const mgwfbp_plan_t &pl, Stream kind, uint64_t workgroups)
{
    if (pl.opt.pace >= 0) return pl.opt.pace;
    // the steps were found on 256 compute units at 6656, 7680 and 8192 workgroups: 26, 30 and 32 per unit
    const uint64_t cus = static_cast<uint64_t>(pl.n_cus > 0 ? pl.n_cus : 256);
    switch (kind) {
    case Stream::reduce:
        if (workgroups < 26 * cus) return 2;
        if (pl.N >= 16) return 8;
        return workgroups < 30 * cus ? 8 : 12;
    default: return workgroups < 32 * cus ? 2 : pl.N >= 16 ? 4 : 8;
    }
}
}  // namespace

namespace {
constexpr int kCopyFloat4 = 1;  // float4 per lane and workgroup in pack / unpack (512-element pieces)

// Pieces that cover the longest direct tile of the scope's list.  Full tiles have tile_elems
// elements; a lone layer just under the gather threshold is a direct tile of its own and can be
// longer than the shortened tiles of a group's list.
uint32_t pieces_per_tile(const mgwfbp_plan_t &pl, const LaunchScope &sc, uint32_t piece_elems)
{
    const uint32_t longest = std::max(sc.tile_elems, std::min(pl.opt.small_elems, pl.opt.tile_elems));
    return (longest + piece_elems - 1) / piece_elems;
}

Divisor divisor(uint32_t d)
{
    return Divisor{d, d <= 1 ? 0xffffffffu : static_cast<uint32_t>((uint64_t(1) << 32) / d)};
}
}  // namespace

int launch_fused(const mgwfbp_plan_t &pl, const LaunchScope &sc, bool step, float lr, float mu,
                 void *stream, float *merged_out)
{
    const uint64_t base_off = sc.base_off;
    if (sc.n_tiles == 0) return MGWFBP_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid(sc.resolve_only ? 0u : sc.n_tiles);
    const float inv_n = 1.0f / static_cast<float>(pl.N);
    const bool nt = pl.opt.nontemporal != 0;
    const int u = static_cast<int>(sc.tile_elems / (kBlock * 4));  // float4 per lane per worker
    // a compute unit has 4 SIMDs x 8 waves = 32 wave slots = 16 workgroups; below about half of
    // that over the whole chip the launch cannot saturate HBM with one load per wave and is bound
    // by latency instead
    const bool deep = sc.n_tiles < 8u * static_cast<uint32_t>(pl.n_cus > 0 ? pl.n_cus : 256);
    // the update runs on one tile length; what it can choose per launch is the workgroups per CU
    const uint32_t occupancy_lds = step && !sc.occupancy_lds && nt && u == 8
        ? update_occupancy_lds(pl.N, pl.n_cus, pl.lds_per_cu, sc.n_tiles, pl.opt.update_wgs_per_cu)
        : sc.occupancy_lds;
    // fewer workgroups per CU already thin the request stream: a capped update launch keeps the
    // short pause whatever its length (measured: the long-launch pause on top costs 3-5 %)
    const int pace = sc.pace >= 0 ? sc.pace
                     : step && occupancy_lds && pl.opt.pace < 0 ? 2
                     : pace_for(pl, step ? Stream::update : Stream::reduce, sc.n_tiles);
    if (step) {
        if (nt) fused_dispatch<true, true>(pl.N, u, deep, grid, occupancy_lds, s, pl.dt, sc.tile_begin, inv_n, lr, mu, pace, merged_out, base_off);
        else fused_dispatch<true, false>(pl.N, u, deep, grid, occupancy_lds, s, pl.dt, sc.tile_begin, inv_n, lr, mu, pace, merged_out, base_off);
    } else {
        if (nt) fused_dispatch<false, true>(pl.N, u, deep, grid, occupancy_lds, s, pl.dt, sc.tile_begin, inv_n, lr, mu, pace, merged_out, base_off);
        else fused_dispatch<false, false>(pl.N, u, deep, grid, occupancy_lds, s, pl.dt, sc.tile_begin, inv_n, lr, mu, pace, merged_out, base_off);
    }
    return check_launch("fused kernel launch");
}

// Workgroups of the gated launch: at most the chosen number per compute unit, and every workgroup
// the same number of tiles (the last pass aside).  0 if the device holds too few.
uint32_t gated_grid(const mgwfbp_plan_t &pl, bool step)
{
    const int holds = pl.gated_resident_per_cu[step ? 1 : 0][pl.gated_tile_elems == 4096 ? 1 : 0];
    if (holds <= kGatedReserve || pl.ordered_tile_count == 0) return 0;
    // by default four workgroup slots (eight waves, two per SIMD) of every compute unit stay free,
    // which is what a producer with 256-lane workgroups needs to be placed at all; the option may
    // go up to two free slots, enough for one-wave kernels like the stand-ins only
    const int want = pl.opt.gated_wgs_per_cu > 0 ? pl.opt.gated_wgs_per_cu : std::max(1, holds - kGatedDefaultReserve);
    int cus = pl.n_cus > 0 ? pl.n_cus : 256;
    if (pl.opt.gated_cus > 0) cus = std::min(cus, pl.opt.gated_cus);  // the caller's stream is confined to these
    const uint32_t cap = static_cast<uint32_t>(std::min(want, holds - kGatedReserve)) * static_cast<uint32_t>(cus);
    const uint32_t nt = pl.ordered_tile_count, passes = (nt + cap - 1) / cap;
    return (nt + passes - 1) / passes;
}

int launch_fused_gated(const mgwfbp_plan_t &pl, bool step, float lr, float mu, const uint32_t *ready,
                       uint32_t epoch, uint32_t *ctl, uint64_t max_polls, void *stream)
{
    const bool lng = pl.gated_tile_elems == 4096;  // else 1024
    hipStream_t s = static_cast<hipStream_t>(stream);
    // cleared by a kernel, not a memset: the caller may be capturing a graph
    k_signal<<<1, 64, 0, s>>>(ctl, 0u);
    if (int rc = check_launch("launch that clears the give-up word")) return rc;
    if (pl.ordered_tile_count == 0) return MGWFBP_OK;
    // the launch takes fewer workgroups per compute unit than the unit can hold of this kernel
    // (16 by wave slots; the update form's registers allow 14) and so leaves room for the kernels
    // that bump the counters: a chip filled with waiting workgroups would never see a counter move
    const int holds = pl.gated_resident_per_cu[step ? 1 : 0][lng ? 1 : 0];
    if (holds <= kGatedReserve) {
        set_error("the gated launch needs a device that holds more than " + std::to_string(kGatedReserve) +
                  " of its workgroups per compute unit");
        return MGWFBP_ESTATE;
    }
    const dim3 grid(gated_grid(pl, step));
    const float inv_n = 1.0f / static_cast<float>(pl.N);
    const int pace = pl.opt.pace >= 0 ? pl.opt.pace : 2;
    const uint32_t tb = pl.ordered_tile_begin, nt = pl.ordered_tile_count;
    if (lng) {
        if (step) k_fused_gated<8, true><<<grid, kBlock, 0, s>>>(pl.dt, tb, nt, pl.N, inv_n, lr, mu, pace, ready, epoch, ctl, max_polls);
        else k_fused_gated<8, false><<<grid, kBlock, 0, s>>>(pl.dt, tb, nt, pl.N, inv_n, lr, mu, pace, ready, epoch, ctl, max_polls);
    } else {
        if (step) k_fused_gated<2, true><<<grid, kBlock, 0, s>>>(pl.dt, tb, nt, pl.N, inv_n, lr, mu, pace, ready, epoch, ctl, max_polls);
        else k_fused_gated<2, false><<<grid, kBlock, 0, s>>>(pl.dt, tb, nt, pl.N, inv_n, lr, mu, pace, ready, epoch, ctl, max_polls);
    }
    return check_launch("gated launch");
}

int gated_resident_per_cu(bool step, bool long_tiles, int *per_cu)
{
    int n = 0;
    hipError_t e;
    if (long_tiles)
        e = step ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_fused_gated<8, true>, kBlock, 0)
                 : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_fused_gated<8, false>, kBlock, 0);
    else
        e = step ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_fused_gated<2, true>, kBlock, 0)
                 : hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k_fused_gated<2, false>, kBlock, 0);
    if (e != hipSuccess) {
        set_error(std::string("hipOccupancyMaxActiveBlocksPerMultiprocessor: ") + hipGetErrorString(e));
        return MGWFBP_EHIP;
    }
    *per_cu = n;
    return MGWFBP_OK;
}

int launch_signal(uint32_t *counter, uint32_t epoch, void *stream)
{
    k_signal<<<1, 64, 0, static_cast<hipStream_t>(stream)>>>(counter, epoch);
    return check_launch("signal launch");
}

int launch_await(const uint32_t *word, uint32_t value, uint32_t *result, uint64_t max_polls, void *stream)
{
    k_await<<<1, 64, 0, static_cast<hipStream_t>(stream)>>>(word, value, result, max_polls);
    return check_launch("handshake launch");
}

int launch_pack(const mgwfbp_plan_t &pl, const LaunchScope &sc, float *ws, uint64_t epad,
                void *stream)
{
    if (sc.n_tiles == 0) return MGWFBP_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t subs = pieces_per_tile(pl, sc, Piece<kCopyFloat4>::kElems);
    const uint64_t per_worker = static_cast<uint64_t>(sc.n_tiles) * subs;
    const uint64_t all = per_worker * static_cast<uint64_t>(pl.N);
    if (per_worker > 0x7fffffffull) {
        set_error("pack: too many pieces for one launch");
        return MGWFBP_EINVAL;
    }
    const bool flat = all <= 0x7fffffffull;
    const dim3 grid = flat ? dim3(static_cast<uint32_t>(all))
                           : dim3(static_cast<uint32_t>(per_worker), static_cast<uint32_t>(pl.N));
    if (pl.opt.nontemporal)
        k_pack<true, kCopyFloat4><<<grid, kBlock, 0, s>>>(pl.dt, sc.tile_begin, divisor(subs), divisor(pl.N), ws, epad, sc.base_off, flat);
    else
        k_pack<false, kCopyFloat4><<<grid, kBlock, 0, s>>>(pl.dt, sc.tile_begin, divisor(subs), divisor(pl.N), ws, epad, sc.base_off, flat);
    return check_launch("pack kernel launch");
}

int launch_reduce(const mgwfbp_plan_t &pl, const LaunchScope &sc, float *ws, uint64_t epad,
                  void *stream)
{
    if (sc.elems == 0) return MGWFBP_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // contiguous buffers need no tile table; the same rule as for the fused pass picks the tile
    // length that fills the chip's batches of workgroups best
    uint32_t tile = sc.tile_elems;
    if (tile == 4096 && pl.opt.long_tiles == -1 && pl.opt.nontemporal) {
        uint64_t counts[kTileChoices];
        for (int c = 0; c < kTileChoices; ++c) counts[c] = (sc.elems + kTileChoice[c] - 1) / kTileChoice[c];
        tile = kTileChoice[best_tile_choice(pl.N, pl.n_cus, counts)];
    }
    const dim3 grid(static_cast<uint32_t>((sc.elems + tile - 1) / tile));
    const float inv_n = 1.0f / static_cast<float>(pl.N);
    const int u = static_cast<int>(tile / (kBlock * 4));
    const bool deep = grid.x < 8u * static_cast<uint32_t>(pl.n_cus > 0 ? pl.n_cus : 256);
    const int pace = pace_for(pl, Stream::reduce, grid.x);
    const bool nt = pl.opt.nontemporal != 0;
    switch (pl.N) {
    case 1: reduce_launch<1>(nt, u, deep, grid, s, ws, epad, sc.elems, tile, pl.N, inv_n, pace); break;
    case 2: reduce_launch<2>(nt, u, deep, grid, s, ws, epad, sc.elems, tile, pl.N, inv_n, pace); break;
    case 4: reduce_launch<4>(nt, u, deep, grid, s, ws, epad, sc.elems, tile, pl.N, inv_n, pace); break;
    case 8: reduce_launch<8>(nt, u, deep, grid, s, ws, epad, sc.elems, tile, pl.N, inv_n, pace); break;
    case 16: reduce_launch<16>(nt, u, deep, grid, s, ws, epad, sc.elems, tile, pl.N, inv_n, pace); break;
    default: reduce_launch<0>(nt, u, deep, grid, s, ws, epad, sc.elems, tile, pl.N, inv_n, pace); break;
    }
    return check_launch("reduce kernel launch");
}

int launch_unpack(const mgwfbp_plan_t &pl, const LaunchScope &sc, const float *reduced, bool step,
                  float lr, float mu, void *stream)
{
    if (sc.n_tiles == 0) return MGWFBP_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t subs = pieces_per_tile(pl, sc, Piece<kCopyFloat4>::kElems);
    const uint64_t all = static_cast<uint64_t>(sc.n_tiles) * subs;
    if (all > 0x7fffffffull) {
        set_error("unpack: too many pieces for one launch");
        return MGWFBP_EINVAL;
    }
    const dim3 grid(static_cast<uint32_t>(all));
    const bool nt = pl.opt.nontemporal != 0;
#define MGWFBP_UNPACK(STEP, NT) \
    k_unpack<STEP, NT, kCopyFloat4><<<grid, kBlock, 0, s>>>(pl.dt, sc.tile_begin, divisor(subs), reduced, sc.base_off, lr, mu)
    if (step) {
        if (nt) MGWFBP_UNPACK(true, true); else MGWFBP_UNPACK(true, false);
    } else {
        if (nt) MGWFBP_UNPACK(false, true); else MGWFBP_UNPACK(false, false);
    }
#undef MGWFBP_UNPACK
    return check_launch("unpack kernel launch");
}

// s_memrealtime counts at a constant 100 MHz on this family; ask the runtime to be sure
int wall_clock_khz()
{
    static int khz = 0;
    if (khz == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeWallClockRate, dev) == hipSuccess && v > 0)
            khz = v;
        else
            khz = 100000;
    }
    return khz;
}

namespace {
int spin(double ms, uint64_t *clock, int mode, void *stream, uint32_t *arrive = nullptr, uint32_t epoch = 0)
{
    if (!(ms > 0.0)) ms = 0.0;
    const uint64_t ticks = static_cast<uint64_t>(ms * wall_clock_khz());
    // one poll takes at least ~2048 clocks of sleep (~1 us); cap generously at 50x the target
    const uint64_t max_polls = 1000 + static_cast<uint64_t>(ms * 1000.0 * 50.0);
    k_spin<<<1, 64, 0, static_cast<hipStream_t>(stream)>>>(ticks, max_polls, clock, mode, arrive, epoch);
    return check_launch("backward stand-in launch");
}
}  // namespace

int launch_spin(double ms, void *stream, uint64_t *publish_clock) { return spin(ms, publish_clock, 0, stream); }

int launch_spin_until(double deadline_ms, uint64_t *clock, void *stream, uint32_t *arrive, uint32_t epoch)
{
    return spin(deadline_ms, clock, 1, stream, arrive, epoch);
}

}  // namespace mgwfbp
