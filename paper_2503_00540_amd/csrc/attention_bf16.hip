// bf16 MFMA attention for gfx950: the contraction of Eq. 1 (sliding-window chunk encode)
// and Eq. 3 (question answering over retrieved KV), fp32 accumulation and softmax.
//
// Work split.  A workgroup of 4 wavefronts owns BM = 128 query rows of one (item, KV head):
// the G = Hq / Hkv query heads that share the KV head are stacked into the row dimension
// (row = token * G + head-in-group), so one K/V tile staged in LDS serves all of them.
// The key range (segment A unmasked, then segment B causal) is walked in tiles of 64 keys;
// optionally several workgroups split the tile list (split-KV) and a merge kernel combines
// their (max, sum, unnormalised O) partial results.
//
// Each wavefront computes S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16, so
// that a query is an MFMA column: it lives in one lane (and its partner lane + 32), softmax
// statistics need no cross-lane traffic beyond one exchange with that partner, and the
// S^T accumulator registers are, after packing to bf16, exactly the B operand of the PV
// product.  V is transposed on its way into LDS so that its A operand is one 16-byte read.
#include "common.h"

namespace rekv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BN = 64;        // keys per tile
constexpr int WAVES = 4;
constexpr int WM = 32;        // query rows per wavefront (one MFMA column block)
constexpr int BM = WAVES * WM;
constexpr int THREADS = WAVES * 64;
constexpr float RESCALE_GAP = 8.0f;  // log2 units the running max may lag before O is rescaled

template <int D>
struct Tile {
    static constexpr int KP = D + 8;    // K tile row pitch in elements: 16 B of padding
    static constexpr int VP = BN + 8;   // V^T tile row pitch
    static constexpr int K_ELEMS = BN * KP;
    static constexpr int V_ELEMS = D * VP;
    static constexpr int STAGE = K_ELEMS + V_ELEMS;
    static constexpr int K_LOADS = BN * (D / 8) / THREADS;  // 16-byte loads per thread
    static constexpr size_t LDS_BYTES = 2 * STAGE * sizeof(bf16_t);
};

struct KernelArgs {
    AttnProblem p;
    int32_t n_splits, m_tiles;
    float* part_o;    // [item*Hkv + kvh][split][m_tiles*BM][D]
    float* part_ml;   // [item*Hkv + kvh][split][m_tiles*BM][2]
};

// Blocks are dealt to the 8 XCDs round-robin by hardware; give each XCD one contiguous
// range of logical blocks so that blocks sharing K/V tiles share an L2.
__device__ inline int xcd_remap(int bid, int nb) {
    const int x = bid & 7, per = nb >> 3, rem = nb & 7;
    return x * per + (x < rem ? x : rem) + (bid >> 3);
}

template <int D>
struct Staged {
    u32x4 k[Tile<D>::K_LOADS];
    u32x4 v[4];
};

template <int D>
__device__ inline void load_tile(Staged<D>& st, const bf16_t* kseg, const bf16_t* vseg,
                                 int key0, int seg_len, int64_t row_stride, int tid) {
    constexpr int CH = D / 8;
#pragma unroll
    for (int i = 0; i < Tile<D>::K_LOADS; ++i) {
        const int id = tid + THREADS * i;
        const int key = id / CH, c = id % CH;
        u32x4 val = {0u, 0u, 0u, 0u};
        if (key0 + key < seg_len)
            val = *reinterpret_cast<const u32x4*>(kseg + (int64_t)(key0 + key) * row_stride + c * 8);
        st.k[i] = val;
    }
    const int r = tid & 15, c = tid >> 4;
    if (c < CH) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int key = key0 + 4 * r + i;
            u32x4 val = {0u, 0u, 0u, 0u};
            if (key < seg_len)
                val = *reinterpret_cast<const u32x4*>(vseg + (int64_t)key * row_stride + c * 8);
            st.v[i] = val;
        }
    }
}

template <int D>
__device__ inline void store_tile(const Staged<D>& st, bf16_t* kl, bf16_t* vl, int tid) {
    constexpr int CH = D / 8;
#pragma unroll
    for (int i = 0; i < Tile<D>::K_LOADS; ++i) {
        const int id = tid + THREADS * i;
        const int key = id / CH, c = id % CH;
        *reinterpret_cast<u32x4*>(kl + key * Tile<D>::KP + c * 8) = st.k[i];
    }
    // V^T: thread (r, c) holds keys 4r..4r+3 x dims 8c..8c+7.  Inside each group of 16 keys the
    // quads are stored in the order 0,2,1,3, which is the order the PV product's k-slots take
    // them from the S^T accumulator registers.
    const int r = tid & 15, c = tid >> 4;
    if (c < CH) {
        const int q = r & 3;
        const int pos = (r >> 2) * 16 + (((q & 1) << 1) | (q >> 1)) * 4;
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const uint32_t a = st.v[0][e2], b = st.v[1][e2], c2 = st.v[2][e2], d2 = st.v[3][e2];
            u32x2 lo, hi;
            lo.x = __builtin_amdgcn_perm(b, a, 0x05040100u);   // (a.lo, b.lo)
            lo.y = __builtin_amdgcn_perm(d2, c2, 0x05040100u);
            hi.x = __builtin_amdgcn_perm(b, a, 0x07060302u);   // (a.hi, b.hi)
            hi.y = __builtin_amdgcn_perm(d2, c2, 0x07060302u);
            *reinterpret_cast<u32x2*>(vl + (c * 8 + 2 * e2) * Tile<D>::VP + pos) = lo;
            *reinterpret_cast<u32x2*>(vl + (c * 8 + 2 * e2 + 1) * Tile<D>::VP + pos) = hi;
        }
    }
}

template <int D>
__global__ __launch_bounds__(THREADS) void attn_bf16_kernel(KernelArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    bf16_t* lds = reinterpret_cast<bf16_t*>(lds_raw);
    const AttnProblem& p = a.p;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, hh = lane >> 5;
    const int G = p.n_q_heads / p.n_kv_heads;

    const int nb = gridDim.x;
    int L = xcd_remap(blockIdx.x, nb);
    const int mt = L % a.m_tiles; L /= a.m_tiles;
    const int split = L % a.n_splits; L /= a.n_splits;
    const int kvh = L % p.n_kv_heads;
    const int item = L / p.n_kv_heads;

    const ItemSegs seg = item_segments(p, item);
    const int64_t row_stride = (int64_t)p.n_kv_heads * D;
    const bf16_t* ka = static_cast<const bf16_t*>(p.k_a) + seg.a_off * row_stride + kvh * D;
    const bf16_t* va = static_cast<const bf16_t*>(p.v_a) + seg.a_off * row_stride + kvh * D;
    const bf16_t* kb = static_cast<const bf16_t*>(p.k_b) + seg.b_off * row_stride + kvh * D;
    const bf16_t* vb = static_cast<const bf16_t*>(p.v_b) + seg.b_off * row_stride + kvh * D;

    const int m_rows = p.len_b * G;
    const int m0 = mt * BM;
    const int row = m0 + wave * WM + col;        // this lane's query row
    const int tok = row / G;                      // its token inside the item
    const bool row_ok = row < m_rows;

    // tile list: tiles_a unmasked tiles, then the causal tiles this row block can see
    const int tiles_a = (seg.len_a + BN - 1) / BN;
    const int tiles_b_all = (p.len_b + BN - 1) / BN;
    int last_tok = (m0 + BM - 1) / G;
    if (last_tok > p.len_b - 1) last_tok = p.len_b - 1;
    const int n_tiles = tiles_a + last_tok / BN + 1;
    const int per_split = (tiles_a + tiles_b_all + a.n_splits - 1) / a.n_splits;
    const int t_begin = split * per_split;
    int t_end = t_begin + per_split;
    if (t_end > n_tiles) t_end = n_tiles;

    // Q fragments (B operand of S^T = K Q^T): lane holds row `row`, dims ks*16 + hh*8 .. +8
    bf16x8 qf[D / 16];
    {
        const bf16_t* qrow = static_cast<const bf16_t*>(p.q) +
            (((int64_t)item * p.len_b + tok) * p.n_q_heads + kvh * G + (row - tok * G)) * D;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (row_ok) v = *reinterpret_cast<const u32x4*>(qrow + ks * 16 + hh * 8);
            qf[ks] = __builtin_bit_cast(bf16x8, v);
        }
    }

    f32x16 o[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[i][j] = 0.f;
    float m_ref = -INFINITY, l_part = 0.f;
    const float sc = p.scale * 1.4426950408889634f;

    Staged<D> st;
    auto fetch = [&](int t) {
        if (t < tiles_a) load_tile<D>(st, ka, va, t * BN, seg.len_a, row_stride, tid);
        else load_tile<D>(st, kb, vb, (t - tiles_a) * BN, p.len_b, row_stride, tid);
    };
    if (t_begin < t_end) fetch(t_begin);
    int buf = 0;
    for (int t = t_begin; t < t_end; ++t) {
        bf16_t* kl = lds + buf * Tile<D>::STAGE;
        bf16_t* vl = kl + Tile<D>::K_ELEMS;
        store_tile<D>(st, kl, vl, tid);
        __syncthreads();
        if (t + 1 < t_end) fetch(t + 1);

        // ---- S^T = K Q^T: two 32-key blocks x 32 queries
        f32x16 s[2];
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk) {
#pragma unroll
            for (int j = 0; j < 16; ++j) s[kbk][j] = 0.f;
            const bf16_t* kr = kl + (kbk * 32 + col) * Tile<D>::KP + hh * 8;
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                const bf16x8 af = *reinterpret_cast<const bf16x8*>(kr + ks * 16);
                s[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, qf[ks], s[kbk], 0, 0, 0);
            }
        }

        // ---- visibility: keys [0, lim) of this tile are visible to this lane's row
        const bool in_b = t >= tiles_a;
        const int key0 = (in_b ? t - tiles_a : t) * BN;
        int lim = (in_b ? (tok + 1 < p.len_b ? tok + 1 : p.len_b) : seg.len_a) - key0;
        const bool need_mask = in_b || key0 + BN > seg.len_a;
        if (need_mask) {
#pragma unroll
            for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int key = kbk * 32 + (j >> 2) * 8 + hh * 4 + (j & 3);
                    s[kbk][j] = key < lim ? s[kbk][j] : -INFINITY;
                }
        }

        // ---- online softmax, one query per lane pair (lane, lane ^ 32)
        float mx = s[0][0];
#pragma unroll
        for (int j = 1; j < 16; ++j) mx = fmaxf(mx, s[0][j]);
#pragma unroll
        for (int j = 0; j < 16; ++j) mx = fmaxf(mx, s[1][j]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float mt2 = mx * sc;
        if (__builtin_amdgcn_ballot_w64(mt2 > m_ref + RESCALE_GAP) != 0) {
            const float m_new = fmaxf(m_ref, mt2);
            const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_ref - m_new);
            l_part *= alpha;
#pragma unroll
            for (int i = 0; i < D / 32; ++i)
#pragma unroll
                for (int j = 0; j < 16; ++j) o[i][j] *= alpha;
            m_ref = m_new;
        }
        const float mr = (m_ref == -INFINITY) ? 0.f : m_ref;
        bf16x8 pf[4];
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                float e[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    e[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kbk][h2 * 8 + j], sc, -mr));
                    l_part += e[j];
                }
                bf16x8 pk;
#pragma unroll
                for (int j = 0; j < 8; j += 2) {
                    f32x2 two = {e[j], e[j + 1]};
                    bf16x2 b2 = __builtin_convertvector(two, bf16x2);
                    pk[j] = b2[0];
                    pk[j + 1] = b2[1];
                }
                pf[kbk * 2 + h2] = pk;
            }

        // ---- O^T += V^T P^T
#pragma unroll
        for (int g16 = 0; g16 < 4; ++g16) {
            const bf16_t* vr = vl + col * Tile<D>::VP + g16 * 16 + hh * 8;
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const bf16x8 af = *reinterpret_cast<const bf16x8*>(vr + db * 32 * Tile<D>::VP);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, pf[g16], o[db], 0, 0, 0);
            }
        }
        buf ^= 1;
    }

    const float l_tot = l_part + __shfl_xor(l_part, 32);
    if (a.n_splits == 1) {
        if (row_ok) {
            const float inv = 1.f / l_tot;
            bf16_t* orow = static_cast<bf16_t*>(p.out) +
                (((int64_t)item * p.len_b + tok) * p.n_q_heads + kvh * G + (row - tok * G)) * D;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int j4 = 0; j4 < 4; ++j4) {
                    f32x2 lo = {o[db][j4 * 4] * inv, o[db][j4 * 4 + 1] * inv};
                    f32x2 hi = {o[db][j4 * 4 + 2] * inv, o[db][j4 * 4 + 3] * inv};
                    bf16x2 blo = __builtin_convertvector(lo, bf16x2);
                    bf16x2 bhi = __builtin_convertvector(hi, bf16x2);
                    u32x2 w;
                    w.x = __builtin_bit_cast(uint32_t, blo);
                    w.y = __builtin_bit_cast(uint32_t, bhi);
                    *reinterpret_cast<u32x2*>(orow + db * 32 + j4 * 8 + hh * 4) = w;
                }
        }
    } else {
        const int64_t rows_pad = (int64_t)a.m_tiles * BM;
        const int64_t base = (((int64_t)item * p.n_kv_heads + kvh) * a.n_splits + split) * rows_pad + row;
        float* po = a.part_o + base * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) {
                f32x4 w = {o[db][j4 * 4], o[db][j4 * 4 + 1], o[db][j4 * 4 + 2], o[db][j4 * 4 + 3]};
                *reinterpret_cast<f32x4*>(po + db * 32 + j4 * 8 + hh * 4) = w;
            }
        if (hh == 0) {
            f32x2 ml = {m_ref, l_tot};
            *reinterpret_cast<f32x2*>(a.part_ml + base * 2) = ml;
        }
    }
}

// Combines the split-KV partial results of one query row: the usual log-sum-exp merge.
template <int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(KernelArgs a) {
    const AttnProblem& p = a.p;
    constexpr int TPR = D / 4;                 // threads per row
    const int G = p.n_q_heads / p.n_kv_heads;
    const int m_rows = p.len_b * G;
    const int64_t rows_pad = (int64_t)a.m_tiles * BM;
    const int r_in_block = threadIdx.x / TPR, dq = threadIdx.x % TPR;
    const int64_t gr = (int64_t)blockIdx.x * (256 / TPR) + r_in_block;   // over (item, kvh, row)
    const int64_t ik = gr / m_rows;
    const int row = (int)(gr % m_rows);
    if (ik >= (int64_t)p.n_items * p.n_kv_heads) return;
    const int item = (int)(ik / p.n_kv_heads), kvh = (int)(ik % p.n_kv_heads);
    float m_all = -INFINITY;
    for (int s = 0; s < a.n_splits; ++s)
        m_all = fmaxf(m_all, a.part_ml[((ik * a.n_splits + s) * rows_pad + row) * 2]);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float l_all = 0.f;
    for (int s = 0; s < a.n_splits; ++s) {
        const int64_t base = (ik * a.n_splits + s) * rows_pad + row;
        const float ms = a.part_ml[base * 2], ls = a.part_ml[base * 2 + 1];
        const float w = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - m_all);
        l_all += w * ls;
        const f32x4 v = *reinterpret_cast<const f32x4*>(a.part_o + base * D + dq * 4);
        acc += v * w;
    }
    const float inv = 1.f / l_all;
    const int tok = row / G;
    bf16_t* orow = static_cast<bf16_t*>(p.out) +
        (((int64_t)item * p.len_b + tok) * p.n_q_heads + kvh * G + (row - tok * G)) * D + dq * 4;
    f32x2 lo = {acc[0] * inv, acc[1] * inv}, hi = {acc[2] * inv, acc[3] * inv};
    u32x2 w;
    w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
    w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
    *reinterpret_cast<u32x2*>(orow) = w;
}

template <int D>
hipError_t launch(const AttnProblem& p, const AttnPlan& plan, void* workspace, hipStream_t stream) {
    KernelArgs a;
    a.p = p;
    a.n_splits = plan.n_splits;
    a.m_tiles = plan.m_tiles;
    a.part_o = nullptr;
    a.part_ml = nullptr;
    const int64_t ik = (int64_t)p.n_items * p.n_kv_heads;
    if (plan.n_splits > 1) {
        a.part_o = static_cast<float*>(workspace);
        a.part_ml = a.part_o + ik * plan.n_splits * plan.m_tiles * BM * (int64_t)D;
    }
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_kernel<D>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)Tile<D>::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t nb = ik * plan.n_splits * plan.m_tiles;
    hipLaunchKernelGGL(attn_bf16_kernel<D>, dim3((unsigned)nb), dim3(THREADS), Tile<D>::LDS_BYTES,
                       stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (plan.n_splits > 1) {
        const int64_t rows = ik * p.len_b * (p.n_q_heads / p.n_kv_heads);
        const int rpb = 256 / (D / 4);
        hipLaunchKernelGGL(attn_merge_kernel<D>, dim3((unsigned)((rows + rpb - 1) / rpb)), dim3(256),
                           0, stream, a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace

AttnPlan attn_bf16_plan(const AttnProblem& p) {
    AttnPlan plan;
    const int G = p.n_q_heads / p.n_kv_heads;
    plan.m_tiles = (p.len_b * G + BM - 1) / BM;
    const int64_t base = (int64_t)p.n_items * p.n_kv_heads * plan.m_tiles;
    // longest tile list of any item (encode: a full window; QA: all retrieved tokens)
    const int len_a_max = p.is_encode ? p.l_l : p.len_a;
    const int n_tiles = (len_a_max + BN - 1) / BN + (p.len_b + BN - 1) / BN;
    int splits = 1;
    const int64_t target = 512;              // about two workgroups per CU
    if (base < target) {
        splits = (int)((target + base - 1) / base);
        const int cap = n_tiles / 4 > 1 ? n_tiles / 4 : 1;   // at least 4 tiles per split
        if (splits > cap) splits = cap;
    }
    plan.n_splits = splits;
    plan.workspace_bytes = 0;
    if (splits > 1)
        plan.workspace_bytes = (size_t)p.n_items * p.n_kv_heads * splits * plan.m_tiles * BM *
                               (size_t)(p.head_dim + 2) * sizeof(float);
    return plan;
}

hipError_t attn_bf16_launch(const AttnProblem& p, const AttnPlan& plan, void* workspace,
                            hipStream_t stream) {
    if (p.head_dim == 128) return launch<128>(p, plan, workspace, stream);
    if (p.head_dim == 64) return launch<64>(p, plan, workspace, stream);
    return hipErrorInvalidValue;
}

}  // namespace rekv
