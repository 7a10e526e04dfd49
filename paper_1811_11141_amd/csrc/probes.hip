// Bandwidth probes (include/mgwfbp_probe.h): plain streaming kernels the benchmark times next to
// the data path and uses to calibrate the hardware counters.  Nothing here belongs to the method.
#include <hip/hip_runtime.h>

#include <string>

#include "../../include/mgwfbp.h"
#include "../../include/mgwfbp_probe.h"
#include "plan.hpp"

namespace {

constexpr int kBlock = 128;
typedef float v4f __attribute__((ext_vector_type(4)));
#define PROBE_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ v4f ld_nt(const v4f *p) { return __builtin_nontemporal_load((const PROBE_GLOBAL v4f *)p); }
__device__ __forceinline__ void st_nt(v4f *p, v4f x) { __builtin_nontemporal_store(x, (PROBE_GLOBAL v4f *)p); }

// one float4 per lane and workgroup: n4 float4 in all
__global__ void __launch_bounds__(kBlock) k_probe_copy(const v4f *src, v4f *dst, uint64_t n4)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i < n4) st_nt(dst + i, ld_nt(src + i));
}

__global__ void __launch_bounds__(kBlock) k_probe_fill(v4f *dst, float value, uint64_t n4)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i < n4) st_nt(dst + i, v4f{value, value, value, value});
}

// four float4 per lane, all in flight; the sum only keeps the loads alive
constexpr int kReadPieces = 4;
__global__ void __launch_bounds__(kBlock) k_probe_read(const v4f *src, uint64_t n4, v4f *sink)
{
    const uint64_t base = static_cast<uint64_t>(blockIdx.x) * (kBlock * kReadPieces) + threadIdx.x;
    v4f x[kReadPieces];
#pragma unroll
    for (int k = 0; k < kReadPieces; ++k) {
        const uint64_t i = base + static_cast<uint64_t>(k) * kBlock;
        x[k] = i < n4 ? ld_nt(src + i) : v4f{0, 0, 0, 0};
    }
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < kReadPieces; ++k) s += x[k].x + x[k].y + x[k].z + x[k].w;
    if (s == 1.2345e38f) *sink = x[0];
}

constexpr uint32_t kStreamsTile = 8192;
template <int NW>
__global__ void __launch_bounds__(kBlock)
k_probe_streams(const float *src, uint64_t stride, uint64_t n, float *dst, float inv_n)
{
    const uint64_t t0 = static_cast<uint64_t>(blockIdx.x) * kStreamsTile;
    const uint32_t cnt = static_cast<uint32_t>(n - t0 < kStreamsTile ? n - t0 : kStreamsTile) >> 2;
    for (uint32_t i = threadIdx.x; i < cnt; i += kBlock) {
        v4f x[NW];
#pragma unroll
        for (int g = 0; g < NW; ++g) x[g] = ld_nt(reinterpret_cast<const v4f *>(src + static_cast<uint64_t>(g) * stride + t0) + i);
        v4f acc = x[0];
#pragma unroll
        for (int g = 1; g < NW; ++g) acc = acc + x[g];
        st_nt(reinterpret_cast<v4f *>(dst + t0) + i, acc * inv_n);
    }
}

int bad(const char *msg)
{
    mgwfbp::set_error(msg);
    return MGWFBP_EINVAL;
}

int launched(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return MGWFBP_OK;
    mgwfbp::set_error(std::string(what) + ": " + hipGetErrorString(e));
    return MGWFBP_EHIP;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// workgroups for n4 float4 at `per` float4 each; 0 if that does not fit one grid dimension
uint32_t grid_for(uint64_t n4, uint64_t per)
{
    const uint64_t g = (n4 + per - 1) / per;
    return g <= 0x7fffffffull ? static_cast<uint32_t>(g) : 0u;
}

}  // namespace

extern "C" {

int mgwfbp_probe_copy(const float *src, float *dst, uint64_t n_elems, void *hip_stream)
{
    return mgwfbp::guarded([&]() -> int {
        if (!src || !dst) return bad("src or dst is NULL");
        if (misaligned(src) || misaligned(dst) || (n_elems & 3u))
            return bad("probe buffers must be 16-byte aligned and n_elems a multiple of 4");
        if (n_elems == 0) return MGWFBP_OK;
        const uint32_t grid = grid_for(n_elems / 4, kBlock);
        if (!grid) return bad("probe: too many elements for one launch");
        k_probe_copy<<<grid, kBlock, 0, static_cast<hipStream_t>(hip_stream)>>>(
            reinterpret_cast<const v4f *>(src), reinterpret_cast<v4f *>(dst), n_elems / 4);
        return launched("probe copy launch");
    });
}

int mgwfbp_probe_read(const float *src, uint64_t n_elems, float *sink, void *hip_stream)
{
    return mgwfbp::guarded([&]() -> int {
        if (!src || !sink) return bad("src or sink is NULL");
        if (misaligned(src) || misaligned(sink) || (n_elems & 3u))
            return bad("probe buffers must be 16-byte aligned and n_elems a multiple of 4");
        if (n_elems == 0) return MGWFBP_OK;
        const uint32_t grid = grid_for(n_elems / 4, kBlock * kReadPieces);
        if (!grid) return bad("probe: too many elements for one launch");
        k_probe_read<<<grid, kBlock, 0, static_cast<hipStream_t>(hip_stream)>>>(
            reinterpret_cast<const v4f *>(src), n_elems / 4, reinterpret_cast<v4f *>(sink));
        return launched("probe read launch");
    });
}

int mgwfbp_probe_fill(float *dst, float value, uint64_t n_elems, void *hip_stream)
{
    return mgwfbp::guarded([&]() -> int {
        if (!dst) return bad("dst is NULL");
        if (misaligned(dst) || (n_elems & 3u))
            return bad("probe buffers must be 16-byte aligned and n_elems a multiple of 4");
        if (n_elems == 0) return MGWFBP_OK;
        const uint32_t grid = grid_for(n_elems / 4, kBlock);
        if (!grid) return bad("probe: too many elements for one launch");
        k_probe_fill<<<grid, kBlock, 0, static_cast<hipStream_t>(hip_stream)>>>(reinterpret_cast<v4f *>(dst), value,
                                                                               n_elems / 4);
        return launched("probe fill launch");
    });
}

int mgwfbp_probe_streams(const float *src, int32_t n_streams, uint64_t stride_elems,
                         uint64_t n_elems, float *dst, void *hip_stream)
{
    return mgwfbp::guarded([&]() -> int {
        if (!src || !dst) return bad("src or dst is NULL");
        if (misaligned(src) || misaligned(dst) || (n_elems & 3u) || (stride_elems & 3u) || stride_elems < n_elems)
            return bad("probe buffers must be 16-byte aligned, n_elems and stride multiples of 4, stride >= n_elems");
        if (n_elems == 0) return MGWFBP_OK;
        const uint32_t grid = grid_for(n_elems, kStreamsTile);
        if (!grid) return bad("probe: too many elements for one launch");
        hipStream_t s = static_cast<hipStream_t>(hip_stream);
        const float inv_n = 1.0f / static_cast<float>(n_streams);
        switch (n_streams) {
        case 1: k_probe_streams<1><<<grid, kBlock, 0, s>>>(src, stride_elems, n_elems, dst, inv_n); break;
        case 2: k_probe_streams<2><<<grid, kBlock, 0, s>>>(src, stride_elems, n_elems, dst, inv_n); break;
        case 4: k_probe_streams<4><<<grid, kBlock, 0, s>>>(src, stride_elems, n_elems, dst, inv_n); break;
        case 8: k_probe_streams<8><<<grid, kBlock, 0, s>>>(src, stride_elems, n_elems, dst, inv_n); break;
        case 16: k_probe_streams<16><<<grid, kBlock, 0, s>>>(src, stride_elems, n_elems, dst, inv_n); break;
        default: return bad("probe_streams: n_streams must be 1, 2, 4, 8 or 16");
        }
        return launched("probe streams launch");
    });
}

}  // extern "C"
