// Reload of the retrieved KV: a block copy of whole frames, selected by a device index
// list, from the K and V arenas into one dense buffer per question.  Pure data movement:
// every thread moves 16 bytes per access, a workgroup moves one 16 KB slice of one frame of
// K or of V, so the grid has many more workgroups than the chip has compute units.
#include "common.h"

namespace rekv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
constexpr int GATHER_THREADS = 256;
constexpr int UNROLL = 4;
constexpr size_t SLICE = (size_t)GATHER_THREADS * 16 * UNROLL;   // bytes per workgroup

__global__ __launch_bounds__(GATHER_THREADS) void gather_kernel(
    const char* __restrict__ src_k, const char* __restrict__ src_v, int n_src_frames,
    const int32_t* __restrict__ idx, size_t frame_bytes, char* __restrict__ dst_k,
    char* __restrict__ dst_v, int z_first) {
    const int64_t blk = blockIdx.x;              // over (question, selected slot)
    const int f = idx[blk];
    const int z = blockIdx.z + z_first;          // 0: keys, 1: values
    const char* src = (z ? src_v : src_k) + (size_t)(f < 0 ? 0 : f) * frame_bytes;
    char* dst = (z ? dst_v : dst_k) + (size_t)blk * frame_bytes;
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
        if (off < frame_bytes) __builtin_nontemporal_store(v[i], reinterpret_cast<u32x4*>(dst + off));
    }
}

// The same block copy for several layers in one launch (every layer retrieves its own frames from
// its own arenas): the arenas' base pointers travel in the kernel arguments.
struct LayerArenas {
    const char* k[MAX_GATHER_LAYERS];
    const char* v[MAX_GATHER_LAYERS];
};

__global__ __launch_bounds__(GATHER_THREADS) void gather_layers_kernel(
    LayerArenas arenas, int blocks_per_layer, int n_src_frames, const int32_t* __restrict__ idx,
    size_t frame_bytes, char* __restrict__ dst_k, char* __restrict__ dst_v) {
    const int64_t blk = blockIdx.x;              // over (layer, question, selected slot)
    const int layer = (int)(blk / blocks_per_layer);
    const int f = idx[blk];
    const int z = blockIdx.z;                    // 0: keys, 1: values
    const char* src = (z ? arenas.v[layer] : arenas.k[layer]) + (size_t)(f < 0 ? 0 : f) * frame_bytes;
    char* dst = (z ? dst_v : dst_k) + (size_t)blk * frame_bytes;
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
        if (off < frame_bytes) __builtin_nontemporal_store(v[i], reinterpret_cast<u32x4*>(dst + off));
    }
}

// Keys of the selected frames, turned to their positions in the question-answering context.
// A unit of work is one (token, KV head, column chunk c): the 16-byte chunk at dims
// [c*EPC, (c+1)*EPC) and its partner at + D/2, which hold both members of EPC rotary pairs
// ("half" layout: element e of the first chunk pairs with element e of the second) or EPC/2
// whole pairs each ("interleaved": neighbours pair up).  The pair frequencies theta_i =
// base^(-2i/D) are set up once per workgroup in double precision; the angle position * theta_i
// is formed and reduced to a fraction of a turn in double precision too, so positions in the
// hundreds of thousands lose nothing, and the hardware sine and cosine take it from there.
template <bool BF16>
__global__ __launch_bounds__(GATHER_THREADS) void gather_rope_kernel(
    const char* __restrict__ src_k, int n_src_frames, const int32_t* __restrict__ idx, int k_slots,
    int n_f, int n_kv_heads, int d, char* __restrict__ dst_k, RopeArgs ra) {
    constexpr int EPC = BF16 ? 8 : 4;            // elements per 16-byte chunk
    __shared__ double theta[128];                // D / 2 <= 128 pair frequencies
    const int half = d / 2;
    for (int i = threadIdx.x; i < half; i += GATHER_THREADS)
        theta[i] = exp2(-(2.0 * i / d) * ra.log2_base);
    __syncthreads();
    const int64_t blk = blockIdx.x;              // over (question, selected slot)
    const int f = idx[blk];
    const bool have = f >= 0 && f < n_src_frames;
    const int slot = (int)(blk % k_slots);
    const int cpr = half / EPC;                  // chunk pairs per head row
    const int units = n_f * n_kv_heads * cpr;
    const size_t row_bytes = (size_t)n_kv_heads * d * (BF16 ? 2 : 4);
    const char* src = src_k + (size_t)(have ? f : 0) * n_f * row_bytes;
    char* dst = dst_k + (size_t)blk * n_f * row_bytes;
    for (int u = blockIdx.y * GATHER_THREADS + threadIdx.x; u < units; u += gridDim.y * GATHER_THREADS) {
        const int c = u % cpr, th = u / cpr;     // th = token * Hkv + head
        const int tok = th / n_kv_heads;
        const size_t off = ((size_t)th * d + (size_t)c * EPC) * (BF16 ? 2 : 4);
        u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};
        if (have) {
            lo = *reinterpret_cast<const u32x4*>(src + off);
            hi = *reinterpret_cast<const u32x4*>(src + off + (size_t)half * (BF16 ? 2 : 4));
            const int64_t new_pos = ra.pos_offset + (ra.is_static ? 0 : (int64_t)slot * n_f + tok);
            const int64_t old_pos = ra.src_rotated ? ra.src_pos_offset + (int64_t)f * n_f + tok : 0;
            const double delta = (double)(new_pos - old_pos);
            float x[2 * EPC];                    // first chunk, then its partner
            if (BF16) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    x[2 * i] = __uint_as_float(lo[i] << 16);
                    x[2 * i + 1] = __uint_as_float(lo[i] & 0xffff0000u);
                    x[EPC + 2 * i] = __uint_as_float(hi[i] << 16);
                    x[EPC + 2 * i + 1] = __uint_as_float(hi[i] & 0xffff0000u);
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    x[i] = __uint_as_float(lo[i]);
                    x[EPC + i] = __uint_as_float(hi[i]);
                }
            }
#pragma unroll
            for (int e = 0; e < EPC; ++e) {
                // pair e of this unit: its frequency index and its two members in x[]
                int ti, ia, ib;
                if (ra.interleaved) {
                    const int in_hi = e >= EPC / 2, m = e - in_hi * (EPC / 2);
                    ti = (in_hi ? half / 2 : 0) + c * (EPC / 2) + m;
                    ia = in_hi * EPC + 2 * m;
                    ib = ia + 1;
                } else {
                    ti = c * EPC + e;
                    ia = e;
                    ib = EPC + e;
                }
                const double turns = delta * theta[ti] * 0.15915494309189535;   // 1 / (2 pi)
                const float fr = (float)(turns - rint(turns));                    // in [-0.5, 0.5]
                const float cs = __builtin_amdgcn_cosf(fr), sn = __builtin_amdgcn_sinf(fr);
                const float a_ = x[ia], b_ = x[ib];
                x[ia] = a_ * cs - b_ * sn;
                x[ib] = a_ * sn + b_ * cs;
            }
            if (BF16) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    f32x2 pl = {x[2 * i], x[2 * i + 1]}, ph = {x[EPC + 2 * i], x[EPC + 2 * i + 1]};
                    lo[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pl, bf16x2));
                    hi[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(ph, bf16x2));
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    lo[i] = __float_as_uint(x[i]);
                    hi[i] = __float_as_uint(x[EPC + i]);
                }
            }
        }
        __builtin_nontemporal_store(lo, reinterpret_cast<u32x4*>(dst + off));
        __builtin_nontemporal_store(hi, reinterpret_cast<u32x4*>(dst + off + (size_t)half * (BF16 ? 2 : 4)));
    }
}

}  // namespace

hipError_t gather_rope_launch(const void* src_k, const void* src_v, int n_src_frames, const int32_t* idx,
                              int n_questions, int k_slots, int n_f, int n_kv_heads, int d, int dtype,
                              void* dst_k, void* dst_v, const RopeArgs& ra, hipStream_t stream) {
    const int n_blocks = n_questions * k_slots;
    const size_t es = dtype == REKV_BF16 ? 2 : 4;
    const size_t frame_bytes = (size_t)n_f * n_kv_heads * d * es;
    hipError_t e = hipSuccess;
    if (dst_v) {                       // values: the plain block copy (skipped when only keys are wanted)
        dim3 vgrid((unsigned)n_blocks, (unsigned)((frame_bytes + SLICE - 1) / SLICE), 1);
        hipLaunchKernelGGL(gather_kernel, vgrid, dim3(GATHER_THREADS), 0, stream, static_cast<const char*>(src_k),
                           static_cast<const char*>(src_v), n_src_frames, idx, frame_bytes,
                           static_cast<char*>(dst_k), static_cast<char*>(dst_v), 1);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const int units = n_f * n_kv_heads * (d / 2) / (dtype == REKV_BF16 ? 8 : 4);
    int gy = (units + GATHER_THREADS * 4 - 1) / (GATHER_THREADS * 4);      // about 4 units per thread
    if (gy < 1) gy = 1;
    dim3 kgrid((unsigned)n_blocks, (unsigned)gy, 1);
    if (dtype == REKV_BF16)
        hipLaunchKernelGGL(gather_rope_kernel<true>, kgrid, dim3(GATHER_THREADS), 0, stream,
                           static_cast<const char*>(src_k), n_src_frames, idx, k_slots, n_f, n_kv_heads, d,
                           static_cast<char*>(dst_k), ra);
    else
        hipLaunchKernelGGL(gather_rope_kernel<false>, kgrid, dim3(GATHER_THREADS), 0, stream,
                           static_cast<const char*>(src_k), n_src_frames, idx, k_slots, n_f, n_kv_heads, d,
                           static_cast<char*>(dst_k), ra);
    return hipGetLastError();
}

hipError_t gather_layers_launch(const void* const* src_k, const void* const* src_v, int n_layers, int n_src_frames,
                                const int32_t* idx, int blocks_per_layer, size_t frame_bytes, void* dst_k, void* dst_v,
                                hipStream_t stream) {
    LayerArenas arenas;
    for (int i = 0; i < MAX_GATHER_LAYERS; ++i) {
        arenas.k[i] = static_cast<const char*>(src_k[i < n_layers ? i : 0]);
        arenas.v[i] = static_cast<const char*>(src_v[i < n_layers ? i : 0]);
    }
    dim3 grid((unsigned)(n_layers * blocks_per_layer), (unsigned)((frame_bytes + SLICE - 1) / SLICE), 2);
    hipLaunchKernelGGL(gather_layers_kernel, grid, dim3(GATHER_THREADS), 0, stream, arenas, blocks_per_layer,
                       n_src_frames, idx, frame_bytes, static_cast<char*>(dst_k), static_cast<char*>(dst_v));
    return hipGetLastError();
}

hipError_t gather_launch(const void* src_k, const void* src_v, int n_src_frames, const int32_t* idx,
                         int n_blocks, size_t frame_bytes, void* dst_k, void* dst_v,
                         hipStream_t stream) {
    dim3 grid((unsigned)n_blocks, (unsigned)((frame_bytes + SLICE - 1) / SLICE), 2);
    hipLaunchKernelGGL(gather_kernel, grid, dim3(GATHER_THREADS), 0, stream,
                       static_cast<const char*>(src_k), static_cast<const char*>(src_v), n_src_frames,
                       idx, frame_bytes, static_cast<char*>(dst_k), static_cast<char*>(dst_v), 0);
    return hipGetLastError();
}

}  // namespace rekv
