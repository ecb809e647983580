// fp32 attention for Eq. 1 / Eq. 3 when Q/K/V are stored in fp32.  All arithmetic is fp32
// on the vector ALU (no matrix cores: the fp32 path exists for accuracy, for the small
// configuration whose tolerance is 1e-4).  One wavefront per query row (token, head):
// for 64 keys at a time each lane scores one key, the wavefront takes the running maximum
// and sum, and the lanes then own the output dimensions for the P.V accumulation.
#include "common.h"

namespace rekv {
namespace {

constexpr int ROWS_PER_BLOCK = 4;   // one wavefront each
constexpr int MAX_D = 256;

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__global__ __launch_bounds__(ROWS_PER_BLOCK * 64) void attn_f32_kernel(AttnProblem p) {
    __shared__ float q_lds[ROWS_PER_BLOCK][MAX_D];
    __shared__ float p_lds[ROWS_PER_BLOCK][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int D = p.head_dim;
    const int G = p.n_q_heads / p.n_kv_heads;
    const int item = blockIdx.y;
    const int64_t r = (int64_t)blockIdx.x * ROWS_PER_BLOCK + wave;   // over (token, head)
    if (r >= (int64_t)p.len_q * p.n_q_heads) return;                 // whole wavefront leaves
    const int tok = (int)(r / p.n_q_heads), h = (int)(r % p.n_q_heads), kvh = h / G;
    const ItemSegs seg = item_segments(p, item);
    const int64_t row_stride = (int64_t)p.n_kv_heads * D;
    const bool k_dense = p.a_index && p.a_k_dense;      // re-positioned keys in a dense per-item buffer
    const float* ka = static_cast<const float*>(p.k_a) + (k_dense ? (int64_t)item * p.len_a : seg.a_off) * row_stride + kvh * D;
    const float* va = static_cast<const float*>(p.v_a) + seg.a_off * row_stride + kvh * D;
    const float* kb = static_cast<const float*>(p.k_b) + seg.b_off * row_stride + kvh * D;
    const float* vb = static_cast<const float*>(p.v_b) + seg.b_off * row_stride + kvh * D;
    const int64_t qo = (((int64_t)item * p.len_q + tok) * p.n_q_heads + h) * D;
    const float* q = static_cast<const float*>(p.q) + qo;
    for (int d = lane; d < D; d += 64) q_lds[wave][d] = q[d];
    // q_lds[wave] and p_lds[wave] are private to this wavefront: wave-level ordering suffices
    __builtin_amdgcn_wave_barrier();

    float o[MAX_D / 64] = {0.f, 0.f, 0.f, 0.f};
    // row of segment A's token j in k_a / v_a: j itself, or through the frame index list
    auto a_row = [&](int j) -> int64_t {
        if (!p.a_index) return j;
        const int slot = j / p.n_f;
        int f = p.a_index[(int64_t)item * p.a_index_stride + slot];
        f = f < 0 ? 0 : (f < p.n_src_frames ? f : p.n_src_frames - 1);
        return (int64_t)f * p.n_f + (j - slot * p.n_f);
    };
    float m = -INFINITY, l = 0.f;
    const int n_vis_b = tok + (p.len_b - p.len_q) + 1;   // causal part: text tokens up to itself
    const int n_keys = seg.len_a + n_vis_b;
    for (int j0 = 0; j0 < n_keys; j0 += 64) {
        const int j = j0 + lane;
        float s = -INFINITY;
        const float* vrow = nullptr;
        if (j < n_keys) {
            const float* krow = j < seg.len_a ? ka + (k_dense ? (int64_t)j : a_row(j)) * row_stride
                                              : kb + (int64_t)(j - seg.len_a) * row_stride;
            float acc = 0.f;
            for (int d = 0; d < D; d += 4) {
                const float4 kv = *reinterpret_cast<const float4*>(krow + d);
                acc = fmaf(kv.x, q_lds[wave][d], acc);
                acc = fmaf(kv.y, q_lds[wave][d + 1], acc);
                acc = fmaf(kv.z, q_lds[wave][d + 2], acc);
                acc = fmaf(kv.w, q_lds[wave][d + 3], acc);
            }
            s = acc * p.scale;
        }
        const float m_new = fmaxf(m, wave_max(s));      // finite: key j0 is visible
        const float alpha = expf(m - m_new);            // 0 on the first pass (m = -inf)
        const float pj = (j < n_keys) ? expf(s - m_new) : 0.f;
        l = l * alpha + wave_sum(pj);
        m = m_new;
        p_lds[wave][lane] = pj;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < MAX_D / 64; ++i) o[i] *= alpha;
        const int cnt = n_keys - j0 < 64 ? n_keys - j0 : 64;
        for (int jj = 0; jj < cnt; ++jj) {
            const int jk = j0 + jj;
            vrow = jk < seg.len_a ? va + a_row(jk) * row_stride
                                  : vb + (int64_t)(jk - seg.len_a) * row_stride;
            const float pv = p_lds[wave][jj];
#pragma unroll
            for (int i = 0; i < MAX_D / 64; ++i) {
                const int d = lane + 64 * i;
                if (d < D) o[i] = fmaf(pv, vrow[d], o[i]);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    float* out = static_cast<float*>(p.out) + qo;
    const float inv = 1.f / l;
#pragma unroll
    for (int i = 0; i < MAX_D / 64; ++i) {
        const int d = lane + 64 * i;
        if (d < D) out[d] = o[i] * inv;
    }
}

}  // namespace

hipError_t attn_f32_launch(const AttnProblem& p, hipStream_t stream) {
    const int64_t rows = (int64_t)p.len_q * p.n_q_heads;
    dim3 grid((unsigned)((rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK), (unsigned)p.n_items);
    hipLaunchKernelGGL(attn_f32_kernel, grid, dim3(ROWS_PER_BLOCK * 64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace rekv
