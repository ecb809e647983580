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
// One workgroup streams one frame (a contiguous N_f x D' block) front to back: LPR lanes
// cover a key row with 16-byte loads (8 bf16 or 4 fp32 each), the 256 / LPR row groups take
// alternate rows, eight loads are in flight per thread, and the row groups' partial sums
// meet in LDS.  Rows wider than 256 lanes are split over blockIdx.y.
// ---------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void frame_keys_kernel(const void* __restrict__ k, int n_f,
                                                         int d_prime, int lpr_log2,
                                                         float* __restrict__ out) {
    constexpr int VEC = BF16 ? 8 : 4;
    constexpr int ES = BF16 ? 2 : 4;
    __shared__ float red[256 * VEC];
    const int lpr = 1 << lpr_log2, n_rg = 256 >> lpr_log2;
    const int cl = threadIdx.x & (lpr - 1), rg = threadIdx.x >> lpr_log2;
    const int col = (blockIdx.y * lpr + cl) * VEC;
    const int64_t frame = blockIdx.x;
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    if (col < d_prime) {
        const char* base = static_cast<const char*>(k) + ((frame * n_f) * (int64_t)d_prime + col) * ES;
        const int64_t pitch = (int64_t)d_prime * ES;
        auto add = [&](const u32x4& w) {
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
        };
        constexpr int U = 8;
        int j = rg;
        for (; j + n_rg * (U - 1) < n_f; j += n_rg * U) {
            u32x4 w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (j + n_rg * u) * pitch));
#pragma unroll
            for (int u = 0; u < U; ++u) add(w[u]);
        }
        for (; j < n_f; j += n_rg) add(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + j * pitch)));
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) red[(rg * lpr + cl) * VEC + i] = acc[i];
    __syncthreads();
    // lpr * VEC columns, summed over the row groups
    for (int c = threadIdx.x; c < lpr * VEC; c += 256) {
        float sum = 0.f;
        for (int g = 0; g < n_rg; ++g) sum += red[g * lpr * VEC + c];
        const int oc = blockIdx.y * lpr * VEC + c;
        if (oc < d_prime) out[frame * d_prime + oc] = sum / (float)n_f;
    }
}

// ---------------------------------------------------------------------------------------
// Question vector and Eq. 2.  The token mean of a question's queries, per query head, comes
// from the same column-mean kernel as the frame vectors (the question is a "frame" of N_q
// rows of Hq*D columns); a small kernel then averages the G query heads of each KV group.
// The score kernel stages the question vectors in LDS.  A wavefront then takes FR frames x
// QBT questions at a time: every lane accumulates the FR*QBT partial dot
// products (and the FR partial |v|^2) over its slice of the D' columns, and a transposing
// butterfly leaves each total in one lane with one shuffle per total instead of six.
// grid = (frame-group blocks, question blocks); wavefronts stride over the frame groups.
// ---------------------------------------------------------------------------------------
constexpr int SCORE_WAVES = 4;

// q_vec[q][g*D + dd] = mean over the G heads of group g of q_heads[q][(g*G + i)*D + dd]
__global__ __launch_bounds__(256) void group_mean_kernel(const float* __restrict__ q_heads, int hq, int hkv,
                                                         int d, float* __restrict__ q_vec) {
    const int d_prime = hkv * d, g_sz = hq / hkv;
    const int c = blockIdx.y * 256 + threadIdx.x;
    if (c >= d_prime) return;
    const int g = c / d, dd = c - g * d;
    const float* src = q_heads + ((int64_t)blockIdx.x * hq + g * g_sz) * d + dd;
    float acc = 0.f;
    for (int j = 0; j < g_sz; ++j) acc += src[j * d];
    q_vec[(int64_t)blockIdx.x * d_prime + c] = acc / (float)g_sz;
}

// Sums v[i] over the 64 lanes for all i at once.  Returns, in every lane, the total of the
// value whose index is the lane's top log2(N) bits (lane >> (6 - log2 N)).
template <int N>
__device__ inline float transpose_reduce(float (&v)[N], int lane) {
    int n = N;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        if (n > 1) {
            const int half = n / 2;
            const bool up = (lane & off) != 0;
#pragma unroll
            for (int i = 0; i < half; ++i) {
                const float keep = up ? v[i + half] : v[i];
                const float send = up ? v[i] : v[i + half];
                v[i] = keep + __shfl_xor(send, off);
            }
            n = half;
        } else {
            v[0] += __shfl_xor(v[0], off);
        }
    }
    return v[0];
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

// exclusive scan over the block of two counts per thread, packed into one 64-bit value
// (high word, low word); returns this thread's prefix and the block total through `total`
__device__ inline uint64_t block_excl_scan(uint64_t v, uint64_t* wave_tot, uint64_t& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint64_t n = __shfl_up(inc, o);
        if (lane >= o) inc += n;
    }
    __syncthreads();                       // wave_tot may still be read from the last call
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    uint64_t before = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < TOPK_THREADS / 64; ++w) {
        const uint64_t t = wave_tot[w];
        if (w < wave) before += t;
        total += t;
    }
    return before + inc - v;
}

// The whole block works on one question: s its n_frames scores, out its k index slots, n_sel_q
// its count (may be NULL).
__device__ inline void topk_block(const float* s, int n_frames, int k, int32_t* out, int32_t* n_sel_q) {
    // Scores of one question cluster in a few exponent bins, so a single histogram would serialise
    // its LDS atomics on one address: threads spread over NSUB copies, and each thread first adds
    // up runs of equal bins among its own keys.
    // The kernel runs once per question on cold instruction caches, so its loops stay rolled: the
    // code is a few hundred instructions, not thousands.
    constexpr int NSUB = 8;
    constexpr int SPAN = 16;               // consecutive frames a thread owns in the ordered sweep
    __shared__ int hist[NSUB][256];
    __shared__ __attribute__((aligned(16))) uint32_t keys[SPAN * TOPK_THREADS];
    __shared__ uint64_t wave_tot[TOPK_THREADS / 64];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_need;
    const int tid = threadIdx.x;

    if (k >= n_frames) {                   // everything is selected
        for (int f = tid; f < k; f += TOPK_THREADS) out[f] = f < n_frames ? f : -1;
        if (tid == 0 && n_sel_q) *n_sel_q = n_frames;
        return;
    }

    // Up to 256 frames (one per thread): count, for every frame, the frames with a higher key - all
    // keys in LDS, read as broadcasts - and take those with fewer than k above them.  That is the
    // answer unless equal keys straddle the cut, which shows as more than k taken; then (rarely)
    // the radix select below decides.
    if (n_frames <= TOPK_THREADS) {
        const int n4 = (n_frames + 3) >> 2;        // keys are read four at a time; key 0 pads the tail
        for (int f = tid; f < n4 * 4; f += TOPK_THREADS) keys[f] = f < n_frames ? order_key(s[f]) : 0u;
        __syncthreads();
        const uint4* keys4 = reinterpret_cast<const uint4*>(keys);
        const uint32_t mine = tid < n_frames ? keys[tid] : 0xFFFFFFFFu;
        int above = 0;                             // padding keys (0) are above nothing
#pragma unroll 8
        for (int j4 = 0; j4 < n4; ++j4) {
            const uint4 o = keys4[j4];
            above += o.x > mine;
            above += o.y > mine;
            above += o.z > mine;
            above += o.w > mine;
        }
        const bool take = tid < n_frames && above < k;
        uint64_t tot;
        const uint64_t pre = block_excl_scan((uint64_t)take, wave_tot, tot);
        if ((int)tot == k) {                       // uniform over the block
            if (take) out[(int)pre] = tid;
            if (tid == 0 && n_sel_q) *n_sel_q = k;
            return;
        }
        __syncthreads();                           // keys[] is laid out anew below
    }

    // Up to 4096 frames the keys live in LDS (frame f at [f % SPAN][f / SPAN], which both the
    // strided and the owner-contiguous access below reach without bank conflicts), so the scores
    // cross the memory system once instead of once per pass.
    const bool resident = n_frames <= TOPK_THREADS * SPAN;
    if (resident) {
#pragma unroll 1
        for (int f = tid; f < n_frames; f += TOPK_THREADS)
            keys[(f % SPAN) * TOPK_THREADS + f / SPAN] = order_key(s[f]);
        __syncthreads();
    }
    auto key_at = [&](int f) -> uint32_t {
        return resident ? keys[(f % SPAN) * TOPK_THREADS + f / SPAN] : order_key(s[f]);
    };

    uint32_t prefix = 0;                   // high bits of T found so far
    int need = k;                          // rank of T among keys matching the prefix
#pragma unroll 1
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
#pragma unroll 1
        for (int sub = 0; sub < NSUB; ++sub) hist[sub][tid] = 0;    // TOPK_THREADS == 256 bins
        __syncthreads();
        const uint32_t hi_mask = pass ? (0xFFFFFFFFu << (shift + 8)) : 0u;
        int* my_hist = hist[tid % NSUB];
        int run_bin = -1, run_len = 0;
#pragma unroll 1
        for (int f = tid; f < n_frames; f += TOPK_THREADS) {
            const uint32_t key = key_at(f);
            if ((key & hi_mask) != prefix) continue;
            const int bin = (int)((key >> shift) & 255u);
            if (bin == run_bin) {
                ++run_len;
            } else {
                if (run_len) atomicAdd(&my_hist[run_bin], run_len);
                run_bin = bin;
                run_len = 1;
            }
        }
        if (run_len) atomicAdd(&my_hist[run_bin], run_len);
        __syncthreads();
        // bin b is chosen iff (#keys in bins above b) < need <= (#keys in bins >= b)
        int mine = 0;
#pragma unroll 1
        for (int sub = 0; sub < NSUB; ++sub) mine += hist[sub][tid];
        uint64_t total;
        const int below = (int)block_excl_scan((uint64_t)mine, wave_tot, total);   // keys in bins < tid
        const int above = (int)total - below - mine;
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

    // ordered sweep: a thread owns SPAN consecutive frames, so one block scan orders 4096 frames
    int base_gt = 0, base_eq = 0;          // frames above T / equal to T before this sweep
#pragma unroll 1
    for (int f0 = 0; f0 < n_frames; f0 += TOPK_THREADS * SPAN) {
        const int fa = f0 + tid * SPAN;
        uint32_t gt_mask = 0, eq_mask = 0;
#pragma unroll 1
        for (int i = 0; i < SPAN; ++i)
            if (fa + i < n_frames) {
                const uint32_t key = key_at(fa + i);
                gt_mask |= (uint32_t)(key > T) << i;
                eq_mask |= (uint32_t)(key == T) << i;
            }
        uint64_t tot;
        const uint64_t pre = block_excl_scan(((uint64_t)__popc(gt_mask) << 32) | (uint64_t)__popc(eq_mask),
                                             wave_tot, tot);
        int n_gt = base_gt + (int)(pre >> 32), n_eq = base_eq + (int)(pre & 0xFFFFFFFFu);
#pragma unroll 1
        for (int i = 0; i < SPAN; ++i) {
            const bool gt = (gt_mask >> i) & 1, eq = (eq_mask >> i) & 1;
            if (gt || (eq && n_eq < need)) out[n_gt + (n_eq < need ? n_eq : need)] = fa + i;
            n_gt += gt;
            n_eq += eq;
        }
        base_gt += (int)(tot >> 32);
        base_eq += (int)(tot & 0xFFFFFFFFu);
    }
    if (tid == 0 && n_sel_q) *n_sel_q = k;
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_kernel(const float* __restrict__ scores,
                                                            int n_frames, int k,
                                                            int32_t* __restrict__ idx,
                                                            int32_t* __restrict__ n_sel) {
    const int64_t qi = blockIdx.x;
    topk_block(scores + qi * n_frames, n_frames, k, idx + qi * k, n_sel ? n_sel + qi : nullptr);
}


// For the single-question score kernel: the per-head token means it averages into the question
// vector itself (NULL: q_vec is given), which saves the group-mean launch.
struct QuestionHeads {
    const float* q_heads;   // [n_questions, Hq * D] or NULL
    int hq, hkv, d;
};

template <int FR, int QBT, bool POOL>
__global__ __launch_bounds__(SCORE_WAVES * 64) void score_kernel(
    const float* __restrict__ frame_keys, int64_t fk_stride, int n_frames, int d_prime,
    const float* __restrict__ q_vec, int n_questions, float inv_tau, float* __restrict__ scores, QuestionHeads ft) {
    static_assert(!POOL || QBT == 1, "in-kernel group mean serves one question per block");
    static_assert(FR * QBT <= 64 && (FR & (FR - 1)) == 0 && (QBT & (QBT - 1)) == 0, "butterfly sizes");
    extern __shared__ float qs[];            // [QBT][d_prime] then [QBT] squared norms
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q0 = blockIdx.y * QBT;
    const int nq_here = n_questions - q0 < QBT ? n_questions - q0 : QBT;
    float* qn = qs + QBT * d_prime;
    if (POOL && ft.q_heads) {
        // the question vector: mean of the G query heads of each KV group (same order of sums as
        // group_mean_kernel)
        const int g_sz = ft.hq / ft.hkv;
        for (int i = threadIdx.x; i < d_prime; i += blockDim.x) {
            const int g = i / ft.d, dd = i - g * ft.d;
            const float* src = ft.q_heads + ((int64_t)q0 * ft.hq + g * g_sz) * ft.d + dd;
            float acc = 0.f;
            for (int j = 0; j < g_sz; ++j) acc += src[j * ft.d];
            qs[i] = acc / (float)g_sz;
        }
    } else {
        for (int i = threadIdx.x; i < QBT * d_prime; i += blockDim.x)     // absent questions stay zero
            qs[i] = i < nq_here * d_prime ? q_vec[(int64_t)q0 * d_prime + i] : 0.f;
    }
    __syncthreads();
    for (int w = wave; w < QBT; w += SCORE_WAVES) {
        float s = 0.f;
        for (int i = lane; i < d_prime; i += 64) s += qs[w * d_prime + i] * qs[w * d_prime + i];
        s = wave_sum(s);
        if (lane == 0) qn[w] = s;
    }
    __syncthreads();
    const float* table = frame_keys + (int64_t)q0 * fk_stride;
    constexpr int LOG_N = __builtin_ctz(FR * QBT), LOG_FR = __builtin_ctz(FR);
    for (int f0 = (blockIdx.x * SCORE_WAVES + wave) * FR; f0 < n_frames; f0 += gridDim.x * SCORE_WAVES * FR) {
        float acc[FR * QBT], vv[FR];
#pragma unroll
        for (int i = 0; i < FR * QBT; ++i) acc[i] = 0.f;
#pragma unroll
        for (int i = 0; i < FR; ++i) vv[i] = 0.f;
        const float* vrow[FR];
#pragma unroll
        for (int fr = 0; fr < FR; ++fr) {
            const int f = f0 + fr < n_frames ? f0 + fr : n_frames - 1;   // tail: re-read the last frame
            vrow[fr] = table + (int64_t)f * d_prime;
        }
        for (int i = lane * 4; i < d_prime; i += 256) {
            float4 x[FR];
#pragma unroll
            for (int fr = 0; fr < FR; ++fr) {
                x[fr] = *reinterpret_cast<const float4*>(vrow[fr] + i);
                vv[fr] += x[fr].x * x[fr].x + x[fr].y * x[fr].y + x[fr].z * x[fr].z + x[fr].w * x[fr].w;
            }
#pragma unroll
            for (int w = 0; w < QBT; ++w) {
                const float4 y = *reinterpret_cast<const float4*>(qs + w * d_prime + i);
#pragma unroll
                for (int fr = 0; fr < FR; ++fr)
                    acc[fr * QBT + w] += x[fr].x * y.x + x[fr].y * y.y + x[fr].z * y.z + x[fr].w * y.w;
            }
        }
        const float dsum = transpose_reduce<FR * QBT>(acc, lane);
        const float vsum = transpose_reduce<FR>(vv, lane);
        const int idx = lane >> (6 - LOG_N);                 // = fr * QBT + w
        const int fr = lane >> (6 - LOG_FR), w = idx & (QBT - 1);
        const bool writer = (lane & ((1 << (6 - LOG_N)) - 1)) == 0;
        if (writer && f0 + fr < n_frames && w < nq_here) {
            const float den = sqrtf(vsum) * sqrtf(qn[w]);
            scores[(int64_t)(q0 + w) * n_frames + f0 + fr] = den > 0.f ? dsum / den * inv_tau : 0.f;
        }
    }
}

}  // namespace

hipError_t frame_keys_launch(const void* k, int n_frames, int tokens_per_frame, int d_prime,
                             int dtype, float* frame_keys, hipStream_t stream) {
    const int vec = dtype == REKV_BF16 ? 8 : 4;
    const int lanes = (d_prime + vec - 1) / vec;          // 16-byte lanes per key row
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < lanes && lpr_log2 < 8) ++lpr_log2;
    dim3 grid((unsigned)n_frames, (unsigned)((lanes + (1 << lpr_log2) - 1) >> lpr_log2));
    if (dtype == REKV_BF16)
        hipLaunchKernelGGL(frame_keys_kernel<true>, grid, dim3(256), 0, stream, k, tokens_per_frame,
                           d_prime, lpr_log2, frame_keys);
    else
        hipLaunchKernelGGL(frame_keys_kernel<false>, grid, dim3(256), 0, stream, k, tokens_per_frame,
                           d_prime, lpr_log2, frame_keys);
    return hipGetLastError();
}

namespace {

// Frames of the selected blocks, in block order.  One workgroup per question; slot j*b + t of
// the output is frame block[j]*b + t, or -1 past the end of the stream or of the selection.
// Because blocks come in ascending order, only the last selected block can be the stream's
// short one, so the -1 slots are always at the tail.
__global__ __launch_bounds__(256) void expand_blocks_kernel(const int32_t* __restrict__ block_idx,
                                                            int k_blocks, int b, int n_frames,
                                                            int32_t* __restrict__ frame_idx,
                                                            int32_t* __restrict__ n_sel) {
    __shared__ int count;
    const int q = blockIdx.x;
    if (threadIdx.x == 0) count = 0;
    __syncthreads();
    const int n_slots = k_blocks * b;
    int mine = 0;
    for (int s = threadIdx.x; s < n_slots; s += 256) {
        const int blk = block_idx[(int64_t)q * k_blocks + s / b];
        const int64_t f = (int64_t)blk * b + s % b;
        const bool ok = blk >= 0 && f < n_frames;
        frame_idx[(int64_t)q * n_slots + s] = ok ? (int32_t)f : -1;
        mine += ok;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off);
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(&count, mine);
    __syncthreads();
    if (threadIdx.x == 0 && n_sel) n_sel[q] = count;
}

}  // namespace

hipError_t block_keys_launch(const float* frame_keys, int n_frames, int b, int d_prime, float* block_keys,
                             hipStream_t stream) {
    // a block vector is the mean of b rows of the fp32 frame table: the frame-vector kernel
    // with b "tokens" per "frame"; the stream's short last block gets a launch of its own
    const int n_full = n_frames / b, rest = n_frames % b;
    hipError_t e = hipSuccess;
    if (n_full > 0) e = frame_keys_launch(frame_keys, n_full, b, d_prime, REKV_F32, block_keys, stream);
    if (e == hipSuccess && rest > 0)
        e = frame_keys_launch(frame_keys + (int64_t)n_full * b * d_prime, 1, rest, d_prime, REKV_F32,
                              block_keys + (int64_t)n_full * d_prime, stream);
    return e;
}

hipError_t expand_blocks_launch(const int32_t* block_idx, int n_questions, int k_blocks, int b, int n_frames,
                                int32_t* frame_idx, int32_t* n_sel, hipStream_t stream) {
    hipLaunchKernelGGL(expand_blocks_kernel, dim3((unsigned)n_questions), dim3(256), 0, stream, block_idx,
                       k_blocks, b, n_frames, frame_idx, n_sel);
    return hipGetLastError();
}

hipError_t retrieve_launch(const RetrieveArgs& a, hipStream_t stream) {
    const int d_prime = a.dim > 0 ? a.dim : a.n_kv_heads * a.head_dim;
    // Many questions on one table: 8 frames x 8 questions per wavefront (if 8 question vectors
    // fit 48 KB of LDS), after a group-mean launch.  Otherwise one question per block row, 4 frames
    // per wavefront, and the kernel averages the query heads itself.
    const bool batched = a.frame_keys_stride == 0 && a.n_questions > 1 &&
                         (size_t)8 * (d_prime + 1) * sizeof(float) <= 48 * 1024;
    const float* q_vec = a.q_vec_given;
    hipError_t e = hipSuccess;
    if (!q_vec) {
        // token mean per query head: [n_questions, Hq * D] fp32
        e = frame_keys_launch(a.q_question, a.n_questions, a.n_q_tokens, a.n_q_heads * a.head_dim,
                              a.dtype, a.q_heads, stream);
        if (e != hipSuccess) return e;
        if (batched) {                 // then the group mean: [n_questions, D']
            hipLaunchKernelGGL(group_mean_kernel, dim3((unsigned)a.n_questions, (unsigned)((d_prime + 255) / 256)),
                               dim3(256), 0, stream, a.q_heads, a.n_q_heads, a.n_kv_heads, a.head_dim, a.q_vec);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            q_vec = a.q_vec;
        }
    }
    const int fr = batched ? 8 : 4, qbt = batched ? 8 : 1;
    int fblocks = (a.n_frames + SCORE_WAVES * fr - 1) / (SCORE_WAVES * fr);
    if (fblocks > 4096) fblocks = 4096;
    dim3 sg((unsigned)fblocks, (unsigned)((a.n_questions + qbt - 1) / qbt));
    const size_t lds = (size_t)qbt * (d_prime + 1) * sizeof(float);
    QuestionHeads ft;
    ft.q_heads = q_vec ? nullptr : a.q_heads;
    ft.hq = a.n_q_heads; ft.hkv = a.n_kv_heads; ft.d = a.head_dim;
    if (batched)
        hipLaunchKernelGGL((score_kernel<8, 8, false>), sg, dim3(SCORE_WAVES * 64), lds, stream, a.frame_keys,
                           a.frame_keys_stride, a.n_frames, d_prime, q_vec, a.n_questions, a.inv_tau, a.scores, ft);
    else
        hipLaunchKernelGGL((score_kernel<4, 1, true>), sg, dim3(SCORE_WAVES * 64), lds, stream, a.frame_keys,
                           a.frame_keys_stride, a.n_frames, d_prime, q_vec, a.n_questions, a.inv_tau, a.scores, ft);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(topk_kernel, dim3((unsigned)a.n_questions), dim3(TOPK_THREADS), 0, stream,
                       a.scores, a.n_frames, a.k, a.idx, a.n_sel);
    return hipGetLastError();
}

}  // namespace rekv
