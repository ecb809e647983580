// Measurement probes: what this GPU sustains on the two resources the hot path is priced
// against.  Neither is an operation of the method.
//   probe_copy_kernel  plain streaming copy (HBM read + write), also the known-size kernel the
//                      HBM byte counters are calibrated on
//   probe_mfma_kernel  register-resident loop of independent bf16 32x32x16 MFMAs
#include "common.h"

namespace rekv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int COPY_THREADS = 256;
constexpr int COPY_UNROLL = 4;   // 16-byte loads in flight per lane

__global__ __launch_bounds__(COPY_THREADS) void probe_copy_kernel(const u32x4* __restrict__ src,
                                                                   u32x4* __restrict__ dst, int64_t n16) {
    const int64_t per_block = (int64_t)COPY_THREADS * COPY_UNROLL;
    for (int64_t base = (int64_t)blockIdx.x * per_block; base < n16; base += (int64_t)gridDim.x * per_block) {
        u32x4 v[COPY_UNROLL];
#pragma unroll
        for (int u = 0; u < COPY_UNROLL; ++u) {
            const int64_t i = base + (int64_t)u * COPY_THREADS + threadIdx.x;
            if (i < n16) v[u] = __builtin_nontemporal_load(src + i);
        }
#pragma unroll
        for (int u = 0; u < COPY_UNROLL; ++u) {
            const int64_t i = base + (int64_t)u * COPY_THREADS + threadIdx.x;
            if (i < n16) __builtin_nontemporal_store(v[u], dst + i);
        }
    }
}

constexpr int MFMA_THREADS = 256;
constexpr int MFMA_CHAINS = 4;   // independent accumulators per wavefront

constexpr int MFMA_FRAGS = 8;    // distinct A and B operand fragments cycled through

__global__ __launch_bounds__(MFMA_THREADS) void probe_mfma_kernel(float* __restrict__ sink, int n_iters) {
    // Operands: approximately N(0, 1) values (sum of four hashed bytes, centred and scaled), a
    // different fragment pair for every MFMA of an unrolled group, so that signs, exponents and
    // mantissas at the multiplier inputs toggle the way activations make them toggle.  The sustained
    // clock, and with it the rate, depends on that: constant or small-integer operands run far
    // faster than any real kernel can.  The sums are random walks and stay finite.
    bf16x8 a[MFMA_FRAGS], b[MFMA_FRAGS];
    auto normal_like = [](uint32_t h) {
        const int sum = (int)(h & 255u) + (int)((h >> 8) & 255u) + (int)((h >> 16) & 255u) + (int)(h >> 24);
        return (__bf16)((float)(sum - 510) * (1.f / 147.8f));
    };
#pragma unroll
    for (int f = 0; f < MFMA_FRAGS; ++f)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t idx = (threadIdx.x * MFMA_FRAGS + f) * 8u + i + 1u;
            a[f][i] = normal_like(idx * 2654435761u);
            b[f][i] = normal_like((idx ^ 0x5bd1e995u) * 2246822519u);
        }
    f32x16 acc[MFMA_CHAINS];
#pragma unroll
    for (int c = 0; c < MFMA_CHAINS; ++c)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[c][j] = 0.f;
    for (int it = 0; it < n_iters; it += MFMA_FRAGS) {
#pragma unroll
        for (int u = 0; u < MFMA_FRAGS; ++u)
#pragma unroll
            for (int c = 0; c < MFMA_CHAINS; ++c)
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + c) % MFMA_FRAGS], b[(u * 3 + c) % MFMA_FRAGS],
                                                                 acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < MFMA_CHAINS; ++c)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[c][j];
    sink[(int64_t)blockIdx.x * MFMA_THREADS + threadIdx.x] = s;
}

}  // namespace

hipError_t launch_probe_copy(void* dst, const void* src, int64_t n_bytes, hipStream_t stream) {
    const int64_t n16 = n_bytes / 16;
    const int64_t per_block = (int64_t)COPY_THREADS * COPY_UNROLL;
    int64_t blocks = (n16 + per_block - 1) / per_block;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)blocks), dim3(COPY_THREADS), 0, stream,
                       static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), n16);
    return hipGetLastError();
}

hipError_t launch_probe_mfma(float* sink, int32_t n_workgroups, int32_t n_iters, hipStream_t stream) {
    hipLaunchKernelGGL(probe_mfma_kernel, dim3((unsigned)n_workgroups), dim3(MFMA_THREADS), 0, stream, sink, n_iters);
    return hipGetLastError();
}

double probe_mfma_flop(int32_t n_workgroups, int32_t n_iters) {
    n_iters = (n_iters + MFMA_FRAGS - 1) / MFMA_FRAGS * MFMA_FRAGS;   // the loop runs whole groups
    return 2.0 * 32 * 32 * 16 * MFMA_CHAINS * (MFMA_THREADS / 64) * (double)n_workgroups * (double)n_iters;
}

}  // namespace rekv
