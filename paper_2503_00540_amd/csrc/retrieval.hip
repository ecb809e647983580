// Internal retrieval: frame vectors (mean key per frame), pooled question vector, Eq. 2
// cosine scores with tau = 1, and exact top-k selection.  All of it is memory-bound: the
// kernels read each input once with 16-byte coalesced accesses and keep reductions in
// registers / wavefront shuffles.
#include "common.h"

namespace rekv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// ---------------------------------------------------------------------------------------
// Frame vectors: v_f = (1/N_f) sum_j k_{f,j}, heads concatenated.
// Block = 16 row groups x 16 column lanes; a column lane owns 16 bytes of the key row
// (8 bf16 or 4 fp32).  grid = (frames, column blocks).
// ---------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void frame_keys_kernel(const void* __restrict__ k, int n_f,
                                                         int d_prime, float* __restrict__ out) {
    constexpr int VEC = BF16 ? 8 : 4;
    __shared__ float red[16][16 * VEC + 1];
    const int cl = threadIdx.x & 15, rg = threadIdx.x >> 4;
    const int col = (blockIdx.y * 16 + cl) * VEC;
    const int64_t frame = blockIdx.x;
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    if (col < d_prime) {
        const char* base = static_cast<const char*>(k) +
            ((frame * n_f) * (int64_t)d_prime + col) * (BF16 ? 2 : 4);
        const int64_t pitch = (int64_t)d_prime * (BF16 ? 2 : 4);
#pragma unroll 4
        for (int j = rg; j < n_f; j += 16) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(base + j * pitch);
            if (BF16) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[2 * i] += bf16_lo(w[i]);
                    acc[2 * i + 1] += bf16_hi(w[i]);
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i] += __uint_as_float(w[i]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) red[rg][cl * VEC + i] = acc[i];
    __syncthreads();
    // 16*VEC columns, summed over the 16 row groups by the first 16*VEC threads
    if (threadIdx.x < 16 * VEC) {
        float s = 0.f;
#pragma unroll
        for (int g = 0; g < 16; ++g) s += red[g][threadIdx.x];
        const int c = blockIdx.y * 16 * VEC + threadIdx.x;
        if (c < d_prime) out[frame * d_prime + c] = s / (float)n_f;
    }
}

// ---------------------------------------------------------------------------------------
// Question vector and Eq. 2.  The token mean of a question's queries, per query head, comes
// from the same column-mean kernel as the frame vectors (the question is a "frame" of N_q
// rows of Hq*D columns).  The score kernel finishes the pooling - the mean over the G query
// heads of each KV group - while it stages the question vectors in LDS, then one wavefront
// per frame computes <v,q> and |v|^2 for up to QB questions at a time.
// grid = (frame blocks, question blocks); wavefronts stride over the frames.
// ---------------------------------------------------------------------------------------
constexpr int QB = 8;            // questions sharing one pass over a frame-key table
constexpr int SCORE_WAVES = 4;

__global__ __launch_bounds__(SCORE_WAVES * 64) void score_kernel(
    const float* __restrict__ frame_keys, int64_t fk_stride, int n_frames, int hq, int hkv, int d,
    const float* __restrict__ q_heads, int n_questions, int qb, float* __restrict__ scores) {
    extern __shared__ float qs[];            // [qb][d_prime] then [qb] squared norms
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int d_prime = hkv * d, g_sz = hq / hkv;
    // qb questions share one pass over the table (1 when every question has its own table)
    const int q0 = blockIdx.y * qb;
    const int nq_here = n_questions - q0 < qb ? n_questions - q0 : qb;
    float* qn = qs + qb * d_prime;
    const float inv_g = 1.f / (float)g_sz;
    for (int i = threadIdx.x; i < nq_here * d_prime; i += blockDim.x) {
        const int w = i / d_prime, c = i - w * d_prime;
        const int g = c / d, dd = c - g * d;
        const float* src = q_heads + ((int64_t)(q0 + w) * hq + g * g_sz) * d + dd;
        float acc = 0.f;
        for (int j = 0; j < g_sz; ++j) acc += src[j * d];
        qs[i] = acc * inv_g;
    }
    __syncthreads();
    for (int w = wave; w < nq_here; w += SCORE_WAVES) {
        float s = 0.f;
        for (int i = lane; i < d_prime; i += 64) s += qs[w * d_prime + i] * qs[w * d_prime + i];
        s = wave_sum(s);
        if (lane == 0) qn[w] = s;
    }
    __syncthreads();
    const float* table = frame_keys + (int64_t)q0 * fk_stride;
    for (int f = blockIdx.x * SCORE_WAVES + wave; f < n_frames; f += gridDim.x * SCORE_WAVES) {
        const float* v = table + (int64_t)f * d_prime;
        float dot[QB], vv = 0.f;
#pragma unroll
        for (int w = 0; w < QB; ++w) dot[w] = 0.f;
        for (int i = lane * 4; i < d_prime; i += 256) {
            const float4 x = *reinterpret_cast<const float4*>(v + i);
            vv += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
#pragma unroll
            for (int w = 0; w < QB; ++w)
                if (w < nq_here) {
                    const float4 y = *reinterpret_cast<const float4*>(qs + w * d_prime + i);
                    dot[w] += x.x * y.x + x.y * y.y + x.z * y.z + x.w * y.w;
                }
        }
        vv = wave_sum(vv);
#pragma unroll
        for (int w = 0; w < QB; ++w)
            if (w < nq_here) {
                const float dsum = wave_sum(dot[w]);
                if (lane == 0) {
                    const float den = sqrtf(vv) * sqrtf(qn[w]);
                    scores[(int64_t)(q0 + w) * n_frames + f] = den > 0.f ? dsum / den : 0.f;
                }
            }
    }
}

// ---------------------------------------------------------------------------------------
// Exact top-k of one question's scores.  Scores become order-preserving 32-bit keys; a
// 4-pass radix select (8 bits per pass, histogram in LDS) finds the k-th largest key T;
// then one ordered pass over the frames writes, in ascending frame index, every frame with
// key > T and the first (k - count) frames with key == T - the lower index wins ties.
// One block per question.
// ---------------------------------------------------------------------------------------
constexpr int TOPK_THREADS = 256;

__device__ inline uint32_t order_key(float s) {
    uint32_t u = __float_as_uint(s);
    if (u == 0x80000000u) u = 0u;          // -0 and +0 are the same score
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exclusive scan of one int per thread over the block; returns this thread's prefix and
// the block total through `total`
__device__ inline int block_excl_scan(int v, int* wave_tot, int& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int n = __shfl_up(inc, o);
        if (lane >= o) inc += n;
    }
    __syncthreads();                       // wave_tot may still be read from the last call
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    int before = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < TOPK_THREADS / 64; ++w) {
        const int t = wave_tot[w];
        if (w < wave) before += t;
        total += t;
    }
    return before + inc - v;
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_kernel(const float* __restrict__ scores,
                                                            int n_frames, int k,
                                                            int32_t* __restrict__ idx,
                                                            int32_t* __restrict__ n_sel) {
    __shared__ int hist[256];
    __shared__ int wave_tot[TOPK_THREADS / 64];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_need;
    const int64_t qi = blockIdx.x;
    const float* s = scores + qi * n_frames;
    int32_t* out = idx + qi * k;
    const int tid = threadIdx.x;

    if (k >= n_frames) {                   // everything is selected
        for (int f = tid; f < k; f += TOPK_THREADS) out[f] = f < n_frames ? f : -1;
        if (tid == 0 && n_sel) n_sel[qi] = n_frames;
        return;
    }

    uint32_t prefix = 0;                   // high bits of T found so far
    int need = k;                          // rank of T among keys matching the prefix
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        hist[tid] = 0;                     // TOPK_THREADS == 256 bins
        __syncthreads();
        const uint32_t hi_mask = pass ? (0xFFFFFFFFu << (shift + 8)) : 0u;
        for (int f = tid; f < n_frames; f += TOPK_THREADS) {
            const uint32_t key = order_key(s[f]);
            if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255], 1);
        }
        __syncthreads();
        // bin b is chosen iff (#keys in bins above b) < need <= (#keys in bins >= b)
        const int mine = hist[tid];
        int total;
        const int below = block_excl_scan(mine, wave_tot, total);   // keys in bins < tid
        const int above = total - below - mine;
        if (above < need && need <= above + mine) {
            sh_prefix = prefix | ((uint32_t)tid << shift);
            sh_need = need - above;
        }
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
        __syncthreads();
    }
    const uint32_t T = prefix;             // the k-th largest key; `need` of its copies are taken

    int base_gt = 0, base_eq = 0;          // selected / equal frames before this sweep
    for (int f0 = 0; f0 < n_frames; f0 += TOPK_THREADS) {
        const int f = f0 + tid;
        const uint32_t key = f < n_frames ? order_key(s[f]) : 0u;
        const int gt = (f < n_frames && key > T) ? 1 : 0;
        const int eq = (f < n_frames && key == T) ? 1 : 0;
        int tot_gt, tot_eq;
        const int pre_gt = block_excl_scan(gt, wave_tot, tot_gt);
        const int pre_eq = block_excl_scan(eq, wave_tot, tot_eq);
        const int eq_before = base_eq + pre_eq;
        if (gt || (eq && eq_before < need)) {
            const int eq_sel_before = eq_before < need ? eq_before : need;
            out[base_gt + pre_gt + eq_sel_before] = f;
        }
        base_gt += tot_gt;
        base_eq += tot_eq;
    }
    if (tid == 0 && n_sel) n_sel[qi] = k;
}

}  // namespace

hipError_t frame_keys_launch(const void* k, int n_frames, int tokens_per_frame, int d_prime,
                             int dtype, float* frame_keys, hipStream_t stream) {
    const int vec = dtype == REKV_BF16 ? 8 : 4;
    dim3 grid((unsigned)n_frames, (unsigned)((d_prime + 16 * vec - 1) / (16 * vec)));
    if (dtype == REKV_BF16)
        hipLaunchKernelGGL(frame_keys_kernel<true>, grid, dim3(256), 0, stream, k, tokens_per_frame,
                           d_prime, frame_keys);
    else
        hipLaunchKernelGGL(frame_keys_kernel<false>, grid, dim3(256), 0, stream, k, tokens_per_frame,
                           d_prime, frame_keys);
    return hipGetLastError();
}

hipError_t retrieve_launch(const RetrieveArgs& a, hipStream_t stream) {
    const int d_prime = a.n_kv_heads * a.head_dim;
    // token mean per query head: [n_questions, Hq * D] fp32 in a.q_vec
    hipError_t e = frame_keys_launch(a.q_question, a.n_questions, a.n_q_tokens, a.n_q_heads * a.head_dim,
                                     a.dtype, a.q_vec, stream);
    if (e != hipSuccess) return e;

    // questions per block: up to QB on a shared table, as many as fit 48 KB of LDS
    int qb = a.frame_keys_stride ? 1 : QB;
    while (qb > 1 && (size_t)qb * (d_prime + 1) * sizeof(float) > 48 * 1024) qb >>= 1;
    int fblocks = (a.n_frames + SCORE_WAVES - 1) / SCORE_WAVES;
    if (fblocks > 4096) fblocks = 4096;
    dim3 sg((unsigned)fblocks, (unsigned)((a.n_questions + qb - 1) / qb));
    const size_t lds = (size_t)qb * (d_prime + 1) * sizeof(float);
    hipLaunchKernelGGL(score_kernel, sg, dim3(SCORE_WAVES * 64), lds, stream, a.frame_keys,
                       a.frame_keys_stride, a.n_frames, a.n_q_heads, a.n_kv_heads, a.head_dim, a.q_vec,
                       a.n_questions, qb, a.scores);
    e = hipGetLastError();
    if (e != hipSuccess) return e;

    hipLaunchKernelGGL(topk_kernel, dim3((unsigned)a.n_questions), dim3(TOPK_THREADS), 0, stream,
                       a.scores, a.n_frames, a.k, a.idx, a.n_sel);
    return hipGetLastError();
}

}  // namespace rekv
