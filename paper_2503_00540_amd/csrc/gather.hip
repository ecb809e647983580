// Reload of the retrieved KV: a block copy of whole frames, selected by a device index
// list, from the K and V arenas into one dense buffer per question.  Pure data movement:
// every thread moves 16 bytes per access, a workgroup moves one 16 KB slice of one frame of
// K or of V, so the grid has many more workgroups than the chip has compute units.
#include "common.h"

namespace rekv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int GATHER_THREADS = 256;
constexpr int UNROLL = 4;
constexpr size_t SLICE = (size_t)GATHER_THREADS * 16 * UNROLL;   // bytes per workgroup

__global__ __launch_bounds__(GATHER_THREADS) void gather_kernel(
    const char* __restrict__ src_k, const char* __restrict__ src_v, int n_src_frames,
    const int32_t* __restrict__ idx, size_t frame_bytes, char* __restrict__ dst_k,
    char* __restrict__ dst_v) {
    const int64_t blk = blockIdx.x;              // over (question, selected slot)
    const int f = idx[blk];
    const char* src = (blockIdx.z ? src_v : src_k) + (size_t)(f < 0 ? 0 : f) * frame_bytes;
    char* dst = (blockIdx.z ? dst_v : dst_k) + (size_t)blk * frame_bytes;
    const bool have = f >= 0 && f < n_src_frames;
    const size_t off0 = (size_t)blockIdx.y * SLICE + (size_t)threadIdx.x * 16;
    u32x4 v[UNROLL];
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) {
        const size_t off = off0 + (size_t)i * GATHER_THREADS * 16;
        v[i] = u32x4{0u, 0u, 0u, 0u};
        if (have && off < frame_bytes) v[i] = *reinterpret_cast<const u32x4*>(src + off);
    }
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) {
        const size_t off = off0 + (size_t)i * GATHER_THREADS * 16;
        if (off < frame_bytes) *reinterpret_cast<u32x4*>(dst + off) = v[i];
    }
}

}  // namespace

hipError_t gather_launch(const void* src_k, const void* src_v, int n_src_frames, const int32_t* idx,
                         int n_blocks, size_t frame_bytes, void* dst_k, void* dst_v,
                         hipStream_t stream) {
    dim3 grid((unsigned)n_blocks, (unsigned)((frame_bytes + SLICE - 1) / SLICE), 2);
    hipLaunchKernelGGL(gather_kernel, grid, dim3(GATHER_THREADS), 0, stream,
                       static_cast<const char*>(src_k), static_cast<const char*>(src_v), n_src_frames,
                       idx, frame_bytes, static_cast<char*>(dst_k), static_cast<char*>(dst_v));
    return hipGetLastError();
}

}  // namespace rekv
