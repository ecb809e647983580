// Internal retrieval: frame vectors (mean key per frame), pooled question vector, Eq. 2
// cosine scores with tau = 1, and exact top-k selection.  All of it is memory-bound: the
// kernels read each input once with 16-byte coalesced accesses and keep reductions in
// registers / wavefront shuffles.
#include "common.h"

namespace rekv {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// 16-byte load that is not kept in the caches (a table row is read once per pass)
__device__ inline float4 load_stream(const float* p) {
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

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
// Question vector (the mean of the question's N_q query vectors; the G query heads of a KV
// group averaged so that the vector has D' = Hkv * D entries, like a frame vector).
// One workgroup per (question, KV group): its columns are the G * D contiguous elements of
// that group in every token row.  16-byte loads, fp32 sums, the row groups' partial sums and
// then the G heads meet in LDS.
// ---------------------------------------------------------------------------------------
constexpr int POOL_MAX_COLS = 4096;            // G * D per KV group that fits the LDS buffer

template <bool BF16>
__global__ __launch_bounds__(256) void pool_question_kernel(const void* __restrict__ q, int n_q_tokens, int hq,
                                                            int hkv, int d, float* __restrict__ q_vec) {
    constexpr int VEC = BF16 ? 8 : 4;
    constexpr int ES = BF16 ? 2 : 4;
    __shared__ float red[256 * VEC];
    __shared__ float colsum[POOL_MAX_COLS];
    const int g_sz = hq / hkv, cols = g_sz * d;
    const int lpr = cols / VEC;                      // 16-byte lanes per row of this group's columns
    const int lw = lpr < 256 ? lpr : 256;            // lanes working on a row at a time
    const int n_rg = 256 / lw;                       // row groups
    const int cl = threadIdx.x % lw, rg = threadIdx.x / lw;
    const int64_t pitch = (int64_t)hq * d * ES;
    const char* base = static_cast<const char*>(q) + (int64_t)blockIdx.x * n_q_tokens * pitch +
                       (int64_t)blockIdx.y * cols * ES;
    for (int c0 = 0; c0 < lpr; c0 += lw) {
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
        const bool on = rg < n_rg && c0 + cl < lpr;
        if (on) {
            const char* col = base + (int64_t)(c0 + cl) * 16;
            constexpr int U = 16;
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
            int j = rg;
            for (; j + n_rg * (U - 1) < n_q_tokens; j += n_rg * U) {
                u32x4 w[U];
#pragma unroll
                for (int u = 0; u < U; ++u) w[u] = *reinterpret_cast<const u32x4*>(col + (j + n_rg * u) * pitch);
#pragma unroll
                for (int u = 0; u < U; ++u) add(w[u]);
            }
            for (; j < n_q_tokens; j += n_rg) add(*reinterpret_cast<const u32x4*>(col + j * pitch));
        }
#pragma unroll
        for (int i = 0; i < VEC; ++i) red[threadIdx.x * VEC + i] = acc[i];
        __syncthreads();
        for (int c = threadIdx.x; c < lw * VEC; c += 256) {
            float sum = 0.f;
            for (int g = 0; g < n_rg; ++g) sum += red[(g * lw) * VEC + c];
            if (c0 * VEC + c < cols) colsum[c0 * VEC + c] = sum;
        }
        __syncthreads();
    }
    const float inv = 1.f / ((float)g_sz * (float)n_q_tokens);
    for (int dd = threadIdx.x; dd < d; dd += 256) {
        float sum = 0.f;
        for (int g = 0; g < g_sz; ++g) sum += colsum[g * d + dd];
        q_vec[(int64_t)blockIdx.x * hkv * d + (int64_t)blockIdx.y * d + dd] = sum * inv;
    }
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

// ---------------------------------------------------------------------------------------
// Top-k for the common sizes (257..4096 frames, k <= 64) without a radix select: few phases,
// each one pass over registers or a short LDS list.
//   1. 1024 threads hold up to 4 keys each; frame f belongs to group f mod 128, so all of a
//      thread's keys are in group (thread mod 128) and every group is non-empty.
//   2. The 128 group maxima are 128 different frames, so the k-th largest of them, T0, is a lower
//      bound of the k-th largest key overall: every frame of the answer has key >= T0.
//      Typically fewer than 2k frames pass that test.
//   3. The survivors are ranked among themselves by (key descending, frame ascending) - all
//      pairs, spread over the 1024 threads - and those of rank < k are the answer, exactly,
//      ties going to the lower frame.  One wavefront puts them in ascending frame order.
// Many equal keys at the cut only make the survivor list longer (all-pairs work grows with
// its square), never wrong.  One workgroup per question.
// ---------------------------------------------------------------------------------------
constexpr int SEL_GROUPS = 128;
constexpr int SEL_MAX_FRAMES = 4096;
constexpr int SEL_MAX_K = 64;
constexpr int SEL_MIN_FRAMES = 257;

template <int SEL_THREADS>      // a multiple of 128 that divides 4096
__global__ __launch_bounds__(SEL_THREADS) void topk_groupmax_kernel(const float* __restrict__ scores,
                                                                   int n_frames, int k,
                                                                   int32_t* __restrict__ idx,
                                                                   int32_t* __restrict__ n_sel) {
    // a candidate is one 64-bit word: key in the high half, ~frame in the low half, so that a
    // larger word means "ranks before" (higher key, or equal key and lower frame)
    __shared__ uint32_t gmax[SEL_GROUPS];
    __shared__ __attribute__((aligned(16))) uint64_t cand[SEL_MAX_FRAMES];
    __shared__ int32_t rank_of[SEL_MAX_FRAMES];
    __shared__ int32_t sel[SEL_MAX_K];
    __shared__ uint32_t sh_t0;
    __shared__ int32_t n_cand, n_taken;
    const int tid = threadIdx.x, lane = tid & 63;
    const int64_t qi = blockIdx.x;
    const float* s = scores + qi * n_frames;
    int32_t* out = idx + qi * k;

    constexpr int KPT = SEL_MAX_FRAMES / SEL_THREADS;      // keys per thread
    uint32_t key[KPT];
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const int f = tid + j * SEL_THREADS;
        key[j] = f < n_frames ? order_key(s[f]) : 0u;        // 0 lies below the key of every number
    }
#pragma unroll
    for (int j = 0; j < KPT; ++j) rank_of[tid + j * SEL_THREADS] = 0;
    if (tid < SEL_GROUPS) gmax[tid] = 0u;
    if (tid == 0) { n_cand = 0; n_taken = 0; }
    __syncthreads();
    uint32_t mine = key[0];
#pragma unroll
    for (int j = 1; j < KPT; ++j) mine = max(mine, key[j]);
    atomicMax(&gmax[tid & (SEL_GROUPS - 1)], mine);          // tid mod 128 == the group of all its keys
    __syncthreads();
    if (tid < SEL_GROUPS) {
        const uint32_t v = gmax[tid];
        int above = 0;
#pragma unroll 16
        for (int j = 0; j < SEL_GROUPS; ++j) {
            const uint32_t o = gmax[j];                      // same address in every lane: a broadcast
            above += (o > v) || (o == v && j < tid);
        }
        if (above == k - 1) sh_t0 = v;
    }
    __syncthreads();
    const uint32_t t0 = sh_t0;
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const int f = tid + j * SEL_THREADS;
        const bool pass = f < n_frames && key[j] >= t0;
        const uint64_t mask = __builtin_amdgcn_ballot_w64(pass);
        if (mask != 0) {                                     // wave-uniform
            int base = 0;
            if (lane == 0) base = atomicAdd(&n_cand, __popcll(mask));
            base = __builtin_amdgcn_readfirstlane(base);
            if (pass) {
                const int slot = base + __popcll(mask & ((1ull << lane) - 1ull));
                cand[slot] = ((uint64_t)key[j] << 32) | (uint32_t)~f;
            }
        }
    }
    __syncthreads();
    const int n = n_cand;                                    // k <= n <= n_frames
    // all pairs: candidate i against the candidates of slice sl; a wavefront's lanes share the slice
    const int n_up = (n + 63) & ~63;
    const int n_slices = n_up < SEL_THREADS ? SEL_THREADS / n_up : 1;
    const int sl = __builtin_amdgcn_readfirstlane(tid / n_up);
    if (sl < n_slices) {
        const int j0 = (int)((int64_t)n * sl / n_slices), j1 = (int)((int64_t)n * (sl + 1) / n_slices);
        for (int i = tid - sl * n_up; i < n; i += SEL_THREADS) {
            const uint64_t ci = cand[i];
            int above = 0;
            int j = j0;
            for (; j + 8 <= j1; j += 8) {
                uint64_t c[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) c[u] = cand[j + u];
#pragma unroll
                for (int u = 0; u < 8; ++u) above += c[u] > ci;
            }
            for (; j < j1; ++j) above += cand[j] > ci;
            if (n_slices > 1) atomicAdd(&rank_of[i], above);
            else rank_of[i] = above;
        }
    }
    __syncthreads();
    for (int i = tid; i < n; i += SEL_THREADS)
        if (rank_of[i] < k) sel[atomicAdd(&n_taken, 1)] = (int32_t)~(uint32_t)cand[i];    // exactly k of them
    __syncthreads();
    if (tid < k) {
        const int32_t f = sel[tid];
        int before = 0;
        for (int j = 0; j < k; ++j) before += sel[j] < f;
        out[before] = f;
    }
    if (tid == 0 && n_sel) n_sel[qi] = k;
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_kernel(const float* __restrict__ scores,
                                                            int n_frames, int k,
                                                            int32_t* __restrict__ idx,
                                                            int32_t* __restrict__ n_sel) {
    const int64_t qi = blockIdx.x;
    topk_block(scores + qi * n_frames, n_frames, k, idx + qi * k, n_sel ? n_sel + qi : nullptr);
}


// ---------------------------------------------------------------------------------------
// Eq. 2, one question per pass over a table (a question with its own table, or few questions
// on a shared one): a wavefront takes FR frame rows at a time, the lanes split the D' columns,
// 16-byte loads of the rows and of the question vector are all issued before the first use,
// and a transposing butterfly leaves each row's dot product and squared norm in one lane.
// grid = (frame groups, questions).
// ---------------------------------------------------------------------------------------
constexpr int SCORE_WAVES = 4;
constexpr int SCORE_FR = 8;

// NI > 0: D' <= NI * 256 and the column loop is unrolled NI times, so that all of a row group's
// loads are in flight at once; NI = 0: any D'.
template <int NI>
__global__ __launch_bounds__(SCORE_WAVES * 64) void score_rows_kernel(
    const float* __restrict__ frame_keys, int64_t fk_stride, int n_frames, int d_prime,
    const float* __restrict__ q_vec, float inv_tau, float* __restrict__ scores) {
    constexpr int FR = SCORE_FR;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int qi = blockIdx.y;
    const float* table = frame_keys + (int64_t)qi * fk_stride;
    const float* qv = q_vec + (int64_t)qi * d_prime;
    for (int f0 = (blockIdx.x * SCORE_WAVES + wave) * FR; f0 < n_frames; f0 += gridDim.x * SCORE_WAVES * FR) {
        float acc[FR], vv[FR], qq = 0.f;
#pragma unroll
        for (int i = 0; i < FR; ++i) acc[i] = vv[i] = 0.f;
        const float* vrow[FR];
#pragma unroll
        for (int fr = 0; fr < FR; ++fr) {
            const int f = f0 + fr < n_frames ? f0 + fr : n_frames - 1;   // tail: re-read the last frame
            vrow[fr] = table + (int64_t)f * d_prime;
        }
        auto fold = [&](const float4 (&x)[FR], const float4& y) {
            qq += y.x * y.x + y.y * y.y + y.z * y.z + y.w * y.w;
#pragma unroll
            for (int fr = 0; fr < FR; ++fr) {
                vv[fr] += x[fr].x * x[fr].x + x[fr].y * x[fr].y + x[fr].z * x[fr].z + x[fr].w * x[fr].w;
                acc[fr] += x[fr].x * y.x + x[fr].y * y.y + x[fr].z * y.z + x[fr].w * y.w;
            }
        };
        if (NI > 0) {
            float4 x[NI > 0 ? NI : 1][FR], y[NI > 0 ? NI : 1];
#pragma unroll
            for (int it = 0; it < NI; ++it) {
                const int i = lane * 4 + it * 256;
                const bool on = i < d_prime;
                y[it] = on ? *reinterpret_cast<const float4*>(qv + i) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int fr = 0; fr < FR; ++fr) x[it][fr] = on ? load_stream(vrow[fr] + i) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int it = 0; it < NI; ++it) fold(x[it], y[it]);
        } else {
            for (int i = lane * 4; i < d_prime; i += 256) {
                float4 x[FR];
#pragma unroll
                for (int fr = 0; fr < FR; ++fr) x[fr] = load_stream(vrow[fr] + i);
                fold(x, *reinterpret_cast<const float4*>(qv + i));
            }
        }
        const float dsum = transpose_reduce<FR>(acc, lane);
        const float vsum = transpose_reduce<FR>(vv, lane);
        qq = wave_sum(qq);
        const int fr = lane >> 3;
        if ((lane & 7) == 0 && f0 + fr < n_frames) {
            const float den = sqrtf(vsum) * sqrtf(qq);
            scores[(int64_t)qi * n_frames + f0 + fr] = den > 0.f ? dsum / den * inv_tau : 0.f;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Eq. 2, many questions on one table: a skinny fp32 matrix product, still bound by the table's
// bytes.  A workgroup owns a tile of 32 frames x 32 questions.  Slabs of 128 columns of the
// table rows and of the question vectors are staged in LDS with row-contiguous loads (the next
// slab travels into registers while the current one is used); its 8 wavefronts each take 16
// of the slab's columns and run fp32 MFMAs (v_mfma_f32_32x32x2_f32: full fp32 products, fp32
// sums) on operands read with one 16-byte LDS read per four MFMAs: lane (r, h) holds 4
// consecutive columns of frame r (and of question r), h choosing which 4 of a group of 8.
// Rows are padded by 4 floats, so the 16 lanes of a quarter-wave read 16 different bank
// groups.  The squared norms come from the same registers; the eight partial tiles meet in
// LDS.  The table is read once per 32 questions.  grid = (frame tiles, question tiles).
// ---------------------------------------------------------------------------------------
constexpr int SM_WAVES = 8, SM_TILE = 32, SM_COLS = 128, SM_PITCH = SM_COLS + 4;

typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(SM_WAVES * 64) void score_shared_mfma_kernel(
    const float* __restrict__ table, int n_frames, int d_prime, const float* __restrict__ q_vec,
    int n_questions, float inv_tau, float* __restrict__ scores) {
    // the staging tiles and the partial results share storage: the partials are written after the last slab
    constexpr int STAGE_FLOATS = 2 * SM_TILE * SM_PITCH, PART_FLOATS = SM_WAVES * 16 * 64;
    __shared__ __attribute__((aligned(16))) float lds[STAGE_FLOATS > PART_FLOATS ? STAGE_FLOATS : PART_FLOATS];
    __shared__ float vpart[SM_WAVES][64], qpart[SM_WAVES][64];
    float* tile_a = lds;
    float* tile_b = lds + SM_TILE * SM_PITCH;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, h = lane >> 5;
    const int f0 = blockIdx.x * SM_TILE, q0 = blockIdx.y * SM_TILE;
    // staging: thread t moves float4 number t and t + 512 of each 32 x 32-float4 slab; DEPTH slabs are
    // in flight from memory to registers, because one slab's MFMAs are far shorter than a memory round trip
    constexpr int PER = SM_TILE * (SM_COLS / 4) / (SM_WAVES * 64);       // 2
    constexpr int DEPTH = 4;
    f32x4 xa[DEPTH][PER], xb[DEPTH][PER];
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    // Loads are unconditional (rows and columns past the end are clamped to valid ones, their
    // values replaced by zero or never stored): straight-line code, so the waits for a slab's
    // loads leave the later slabs' loads in flight.
    auto fetch = [&](f32x4 (&ra)[PER], f32x4 (&rb)[PER], int c0) {
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int i = threadIdx.x + u * SM_WAVES * 64;
            const int row = i / (SM_COLS / 4);
            int col = c0 + (i % (SM_COLS / 4)) * 4;
            col = col < d_prime ? col : 0;                                  // D' is a multiple of 4
            const int fr = f0 + row < n_frames ? f0 + row : n_frames - 1;
            const int qr = q0 + row < n_questions ? q0 + row : n_questions - 1;
            ra[u] = *reinterpret_cast<const f32x4*>(table + (int64_t)fr * d_prime + col);
            rb[u] = *reinterpret_cast<const f32x4*>(q_vec + (int64_t)qr * d_prime + col);
        }
    };
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    float vv = 0.f, qq = 0.f;
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) fetch(xa[d], xb[d], d * SM_COLS);
    // Whole rounds of DEPTH slabs, no branch inside a round: slabs past D' are fetched from
    // clamped columns and enter the tiles as zeros.
    const int n_rounds = (d_prime + DEPTH * SM_COLS - 1) / (DEPTH * SM_COLS);
    for (int round = 0; round < n_rounds; ++round) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int cc = (round * DEPTH + d) * SM_COLS;
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int i = threadIdx.x + u * SM_WAVES * 64;
                const int off = (i / (SM_COLS / 4)) * SM_PITCH + (i % (SM_COLS / 4)) * 4;
                const bool on = cc + (i % (SM_COLS / 4)) * 4 < d_prime;   // columns past D' count as zero
                *reinterpret_cast<f32x4*>(tile_a + off) = on ? xa[d][u] : zero;
                *reinterpret_cast<f32x4*>(tile_b + off) = on ? xb[d][u] : zero;
            }
            __syncthreads();
            fetch(xa[d], xb[d], cc + DEPTH * SM_COLS);
#pragma unroll
            for (int g = 0; g < SM_COLS / 8 / SM_WAVES; ++g) {           // this wave's groups of 8 columns
                const int off = r * SM_PITCH + (wave * (SM_COLS / 8 / SM_WAVES) + g) * 8 + 4 * h;
                const f32x4 a = *reinterpret_cast<const f32x4*>(tile_a + off);
                const f32x4 b = *reinterpret_cast<const f32x4*>(tile_b + off);
                vv += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
                qq += b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b[j], acc[j], 0, 0, 0);
            }
            __syncthreads();
        }
    }
    float* part = lds;                               // [wave][16][64]
#pragma unroll
    for (int j = 0; j < 16; ++j) part[(wave * 16 + j) * 64 + lane] = (acc[0][j] + acc[1][j]) + (acc[2][j] + acc[3][j]);
    vpart[wave][lane] = vv;
    qpart[wave][lane] = qq;
    __syncthreads();
    // element (frame fl, question ql) of the tile sits in lane ql + 32 * ((fl / 4) % 2), register
    // (fl / 8) * 4 + fl % 4 of every wave's accumulator
    for (int e = threadIdx.x; e < SM_TILE * SM_TILE; e += SM_WAVES * 64) {
        const int fl = e & 31, ql = e >> 5;
        if (f0 + fl >= n_frames || q0 + ql >= n_questions) continue;
        const int l = ql + 32 * ((fl >> 2) & 1), j = (fl >> 3) * 4 + (fl & 3);
        float dot = 0.f, v2 = 0.f, q2 = 0.f;
#pragma unroll
        for (int w = 0; w < SM_WAVES; ++w) {
            dot += part[(w * 16 + j) * 64 + l];
            v2 += vpart[w][fl] + vpart[w][fl + 32];
            q2 += qpart[w][ql] + qpart[w][ql + 32];
        }
        const float den = sqrtf(v2) * sqrtf(q2);
        scores[(int64_t)(q0 + ql) * n_frames + f0 + fl] = den > 0.f ? dot / den * inv_tau : 0.f;
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
    const float* q_vec = a.q_vec_given;
    hipError_t e = hipSuccess;
    if (!q_vec) {                      // pooled question vectors: [n_questions, D']
        dim3 grid((unsigned)a.n_questions, (unsigned)a.n_kv_heads);
        if (a.dtype == REKV_BF16)
            hipLaunchKernelGGL(pool_question_kernel<true>, grid, dim3(256), 0, stream, a.q_question, a.n_q_tokens,
                               a.n_q_heads, a.n_kv_heads, a.head_dim, a.q_vec);
        else
            hipLaunchKernelGGL(pool_question_kernel<false>, grid, dim3(256), 0, stream, a.q_question, a.n_q_tokens,
                               a.n_q_heads, a.n_kv_heads, a.head_dim, a.q_vec);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        q_vec = a.q_vec;
    }
    // Four or more questions on one table: the matrix-core kernel reads the table once per 32 questions.
    // Otherwise one pass over the (question's own) table per question.
    if (a.frame_keys_stride == 0 && a.n_questions >= 4) {
        dim3 grid((unsigned)((a.n_frames + SM_TILE - 1) / SM_TILE), (unsigned)((a.n_questions + SM_TILE - 1) / SM_TILE));
        hipLaunchKernelGGL(score_shared_mfma_kernel, grid, dim3(SM_WAVES * 64), 0, stream, a.frame_keys, a.n_frames,
                           d_prime, q_vec, a.n_questions, a.inv_tau, a.scores);
    } else {
        int fblocks = (a.n_frames + SCORE_WAVES * SCORE_FR - 1) / (SCORE_WAVES * SCORE_FR);
        if (fblocks > 4096) fblocks = 4096;
        dim3 grid((unsigned)fblocks, (unsigned)a.n_questions);
        const int ni = d_prime <= 1024 ? (d_prime + 255) / 256 : 0;
        auto kern = ni == 1 ? score_rows_kernel<1> : ni == 2 ? score_rows_kernel<2> : ni == 3 ? score_rows_kernel<3>
                  : ni == 4 ? score_rows_kernel<4> : score_rows_kernel<0>;
        hipLaunchKernelGGL(kern, grid, dim3(SCORE_WAVES * 64), 0, stream, a.frame_keys,
                           a.frame_keys_stride, a.n_frames, d_prime, q_vec, a.inv_tau, a.scores);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.n_frames >= SEL_MIN_FRAMES && a.n_frames <= SEL_MAX_FRAMES && a.k <= SEL_MAX_K && a.k < a.n_frames)
        hipLaunchKernelGGL(topk_groupmax_kernel<1024>, dim3((unsigned)a.n_questions), dim3(1024), 0, stream,
                           a.scores, a.n_frames, a.k, a.idx, a.n_sel);
    else
        hipLaunchKernelGGL(topk_kernel, dim3((unsigned)a.n_questions), dim3(TOPK_THREADS), 0, stream,
                           a.scores, a.n_frames, a.k, a.idx, a.n_sel);
    return hipGetLastError();
}

}  // namespace rekv
