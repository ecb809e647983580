// bf16 MFMA attention for gfx950: the contraction of Eq. 1 (sliding-window chunk encode)
// and Eq. 3 (question answering over retrieved KV), fp32 accumulation and softmax.
//
// Work split.  A workgroup of 4 wavefronts owns BM = 128 query rows of one (item, KV head):
// the G = Hq / Hkv query heads that share the KV head are stacked into the row dimension
// (row = token * G + head-in-group), so one K/V tile staged in LDS serves all of them.
// The key range (segment A unmasked, then segment B causal) is walked in tiles of 32 keys;
// optionally several workgroups split the tile list (split-KV) and a merge kernel combines
// their (max, sum, unnormalised O) partial results.
//
// Each wavefront computes S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16, so
// that a query is an MFMA column: it lives in one lane (and its partner lane + 32), softmax
// statistics need no cross-lane traffic beyond one exchange with that partner, and the
// S^T accumulator registers are, after packing to bf16, exactly the B operand of the PV
// product.
//
// Data movement.  K and V tiles go from global memory straight into LDS (global_load_lds,
// 16 bytes per lane, no staging registers), row-major [key][D] with the 16-byte chunks of a
// row XOR-swizzled by the key index so that neither the K operand reads (ds_read_b128, 16
// consecutive keys per quarter-wave) nor the V operand reads hit a bank twice.  The V^T
// operand is read with ds_read_b64_tr_b16, which transposes 4 keys x 16 dims among 16 lanes.
//
// Pipeline.  Tiles are 32 keys; per tile t one barrier.  While the softmax of tile t runs on
// the vector ALU, the matrix cores compute S^T of tile t+1 and the PV product of tile t;
// K(t+4) and V(t+3) are being fetched, so a load has three steps to land.  The four K and
// four V stages sit in one LDS array and the loop is unrolled by four, so every stage is an
// immediate offset of its ds_read.  Steps whose tiles are whole tiles of segment A run a
// variant without masking and with constant load offsets.  Every step issues the same number
// of loads per wave (past the end of the tile list the last tile is fetched again into a stage
// nobody reads), so "all but the newest N loads have landed" is one s_waitcnt vmcnt(N).
//
// Variants (template parameters): ENCODE - Eq. 1's window + chunk inside one cache, otherwise
// Eq. 3's retrieved KV + text KV (question prefill and decode steps); INDEXED - segment A read
// from the KV arena through a frame index list; STREAM - non-temporal tile loads when no
// other workgroup reads the same keys.
#include <type_traits>

#include "common.h"

namespace rekv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define LDS_AS __attribute__((address_space(3)))
#define GLOBAL_AS __attribute__((address_space(1)))

constexpr int BN = 32;        // keys per tile (one MFMA row block of S^T)
constexpr int STAGES = 4;     // LDS stages per tensor
constexpr int WAVES = 4;
constexpr int WM = 32;        // query rows per wavefront (one MFMA column block)
constexpr int BM = WAVES * WM;
constexpr int THREADS = WAVES * 64;
constexpr float RESCALE_GAP = 8.0f;  // log2 units the running max may lag before O is rescaled

template <int D>
struct Cfg {
    static constexpr int CH = D / 8;                 // 16-byte chunks per key row
    static constexpr int RPI = 64 / CH;              // key rows one 1 KB wave-wide load covers
    static constexpr int N_DMA = BN / RPI;           // such loads per tile and tensor
    static constexpr int DMA_PER_WAVE = N_DMA / WAVES;
    static constexpr int TILE_ELEMS = BN * D;
};

// Swizzle of the chunk index inside a key row: the two 2-bit fields of (key mod 16) swapped.
// 16 consecutive keys get 16 different values; 4 consecutive keys differ in the upper field.
template <int D>
__device__ inline int swz(int key) {
    return (((key & 3) << 2) | ((key >> 2) & 3)) & (Cfg<D>::CH - 1);
}

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

__device__ inline void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

// One 16-byte-per-lane load from global memory straight into LDS: lane i's 16 bytes land at
// lds_addr + 16 * i.  Written as asm so that the loads stay invisible to the compiler's
// wait-count bookkeeping: with more than a handful of such loads in a loop it would drain
// all of them before any LDS read.  Ordering is explicit instead (step_barrier).
// The source address is a wave-uniform base plus a 32-bit per-lane byte offset.
// NT marks the load non-temporal: for keys and values that no other workgroup will read again
// (a decode step), so they stream past the caches instead of displacing what is reused.
template <bool NT>
__device__ inline void dma16(const void* base, uint32_t lane_off, uint32_t lds_addr) {
    if (NT)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                     ::"v"(lane_off), "s"(base), "s"(__builtin_amdgcn_readfirstlane(lds_addr)) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     ::"v"(lane_off), "s"(base), "s"(__builtin_amdgcn_readfirstlane(lds_addr)) : "memory", "m0");
}
__device__ inline uint32_t lds_addr_of(const void* p) {
    return (uint32_t)(uintptr_t)(LDS_AS const void*)p;
}

// A query's two lanes (lane, lane ^ 32) combine a value without touching LDS:
// v_permlane32_swap hands every lane both halves' values.
__device__ inline float pair_max(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float pair_sum(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// End of a pipeline step: this wave's loads except the newest N have landed, its LDS reads
// have returned, then the workgroup barrier.  No fence: a fence would drain the newest loads.
template <int N>
__device__ inline void step_barrier() {
    static_assert(N >= 0 && N < 64, "vmcnt immediate");
    __builtin_amdgcn_sched_barrier(0);     // nothing of this step sinks below its barrier
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
    __builtin_amdgcn_sched_barrier(0);
}

template <int I>
using IC = std::integral_constant<int, I>;

// ENCODE selects the segment layout (Eq. 1 window + chunk in one cache, or Eq. 3 retrieved KV +
// question) at compile time; the two instantiations also show up under separate names in a trace.
// INDEXED: segment A is read from the KV arena through a frame index list (no gathered copy).
constexpr int MAX_INDEXED_FRAMES = 1024;   // index entries staged in LDS per workgroup

// STREAM: every K/V tile is read by this workgroup only (one row block per item), see dma16.
template <int D, bool ENCODE, bool INDEXED, bool STREAM>
__global__ __launch_bounds__(THREADS, 2) void attn_bf16_kernel(KernelArgs a) {
    static_assert(!(ENCODE && INDEXED), "the encode window is contiguous");
    static_assert(!(STREAM && (ENCODE || INDEXED)), "streaming loads serve the plain QA / decode layout");
    typedef Cfg<D> C;
    __shared__ int32_t frame_of_slot[INDEXED ? MAX_INDEXED_FRAMES : 1];
    // K stages 0..3, then V stages 0..3; one array so that every stage is a constant offset
    __shared__ __attribute__((aligned(1024))) bf16_t lds[2 * STAGES * C::TILE_ELEMS];
    constexpr uint32_t TILE_B = C::TILE_ELEMS * 2;           // bytes per stage

    AttnProblem p = a.p;
    p.is_encode = ENCODE;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, hh = lane >> 5;
    const int G = p.n_q_heads / p.n_kv_heads;

    const int nb = gridDim.x;
    int L = xcd_remap(blockIdx.x, nb);
    const int mt = L % a.m_tiles; L /= a.m_tiles;
    const int split = L % a.n_splits; L /= a.n_splits;
    // KV head slowest: an XCD then works through consecutive chunks of one KV head, whose
    // windows overlap, so its L2 keeps serving the same K/V rows
    const int item = L % p.n_items;
    const int kvh = L / p.n_items;

    const ItemSegs seg = item_segments(p, item);
    const int64_t row_stride = (int64_t)p.n_kv_heads * D;
    const uint32_t row_stride_b = (uint32_t)row_stride * 2u;
    // keys of an indexed segment A may sit in a dense per-item buffer (re-positioned copies)
    const bool k_dense = INDEXED && p.a_k_dense;
    const int64_t ka_off = k_dense ? (int64_t)item * p.len_a : seg.a_off;
    const char* ka = reinterpret_cast<const char*>(static_cast<const bf16_t*>(p.k_a) + ka_off * row_stride + kvh * D);
    const char* va = reinterpret_cast<const char*>(static_cast<const bf16_t*>(p.v_a) + seg.a_off * row_stride + kvh * D);
    const char* kb = reinterpret_cast<const char*>(static_cast<const bf16_t*>(p.k_b) + seg.b_off * row_stride + kvh * D);
    const char* vb = reinterpret_cast<const char*>(static_cast<const bf16_t*>(p.v_b) + seg.b_off * row_stride + kvh * D);

    const int m_rows = p.len_q * G;
    const int m0 = mt * BM;
    const int row = m0 + wave * WM + col;        // this lane's query row
    const int tok = row / G;                      // its token inside the item
    const bool row_ok = row < m_rows;
    // A wavefront whose 32 rows all lie past the last query row (the tail of the last row block;
    // three of four in a decode step, which has only G rows) keeps fetching its share of the
    // tiles and joining the barriers in a loop of its own, and computes nothing.
    const bool wave_active = m0 + wave * WM < m_rows;

    // tile list: tiles_a tiles of segment A (the first a_full of them whole and unmasked), then
    // the causal tiles of segment B this row block can see
    const int tiles_a = (seg.len_a + BN - 1) / BN;
    const int a_full = seg.len_a / BN;
    const int tiles_b_all = (p.len_b + BN - 1) / BN;
    const int q_pos0 = p.len_b - p.len_q;         // position of query token 0 inside segment B
    int last_tok = (m0 + BM - 1) / G;
    if (last_tok > p.len_q - 1) last_tok = p.len_q - 1;
    const int n_tiles = tiles_a + (last_tok + q_pos0) / BN + 1;
    const int per_split = (tiles_a + tiles_b_all + a.n_splits - 1) / a.n_splits;
    const int t_begin = split * per_split;
    int t_end = t_begin + per_split;
    if (t_end > n_tiles) t_end = n_tiles;

    // ---- lane-constant addressing -----------------------------------------------------
    const uint32_t lds0 = lds_addr_of(lds);
    // global -> LDS: load j of this wave fills LDS rows dma_row + j*RPI, chunk slot dma_p
    const int dma_row = wave * C::DMA_PER_WAVE * C::RPI + lane / C::CH;
    const int dma_p = lane % C::CH;
    uint32_t dma_coff[C::DMA_PER_WAVE];          // byte offset of the chunk to fetch inside its row
    uint32_t dma_off[C::DMA_PER_WAVE];           // byte offset of that chunk inside a whole tile
#pragma unroll
    for (int j = 0; j < C::DMA_PER_WAVE; ++j) {
        dma_coff[j] = (uint32_t)(dma_p ^ swz<D>(dma_row + j * C::RPI)) * 16u;
        dma_off[j] = (uint32_t)(dma_row + j * C::RPI) * row_stride_b + dma_coff[j];
    }
    const uint32_t dma_lds = lds0 + (uint32_t)(wave * C::DMA_PER_WAVE) * 1024u;   // + stage, + j KB
    // K operand (A of S^T = K Q^T): key row col, dims ks*16 + hh*8 .. +8; LDS byte addresses
    uint32_t k_addr[D / 16];
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks)
        k_addr[ks] = lds0 + (uint32_t)(col * D + (((ks * 2 + hh) ^ swz<D>(col)) * 8)) * 2u;
    // V^T operand (A of O^T = V^T P^T) through the transposing read: this lane supplies the
    // address of 4 dims of one key; which key and dims follows from the lane's place in its
    // group of 16.  r picks the first or second set of 4 k-slots of the MFMA.
    uint32_t v_addr[2][D / 32];
    {
        const int gq = lane >> 4, i16 = lane & 15, qd = i16 & 3, jk = i16 >> 2;
        const int cl = (gq & 1) * 2 + (qd >> 1), half = qd & 1;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int keyl = r * 8 + hh * 4 + jk;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
                v_addr[r][db] = lds0 + STAGES * TILE_B +
                    (uint32_t)(keyl * D + (((db * 4 + cl) ^ swz<D>(keyl)) * 8) + half * 4) * 2u;
        }
    }

    // Indexed segment A: the index row of this item, clamped into the arena, staged in LDS.
    const float inv_n_f = INDEXED ? 1.f / (float)p.n_f : 0.f;
    if (INDEXED) {
        const int n_slots = (seg.len_a + p.n_f - 1) / p.n_f;
        for (int i = tid; i < n_slots; i += THREADS) {
            int f = p.a_index[(int64_t)item * p.a_index_stride + i];
            f = f < 0 ? 0 : (f < p.n_src_frames ? f : p.n_src_frames - 1);
            frame_of_slot[i] = f;
        }
        __syncthreads();
    }
    // A tile of the indexed segment A (t < tiles_a): every lane looks up the frame of its row.
    // Rows are below 2^23, so the float quotient is off by at most one and is corrected exactly.
    auto dma_indexed = [&](const char* arena, int t, uint32_t stage_b) {
        const int key0 = t * BN;
        const int n_valid = seg.len_a - key0;
#pragma unroll
        for (int j = 0; j < C::DMA_PER_WAVE; ++j) {
            int r = dma_row + j * C::RPI;
            r = (r < n_valid - 1 ? r : n_valid - 1) + key0;
            int slot = (int)((float)r * inv_n_f);
            int within = r - slot * p.n_f;
            if (within < 0) { --slot; within += p.n_f; }
            if (within >= p.n_f) { ++slot; within -= p.n_f; }
            const uint32_t src_row = (uint32_t)(frame_of_slot[slot] * p.n_f + within);
            dma16<STREAM>(arena, src_row * row_stride_b + dma_coff[j], dma_lds + stage_b + j * 1024u);
        }
    };
    // A whole tile inside segment A: constant per-lane offsets, only the base moves.
    auto dma_fast = [&](const char* base, uint32_t stage_b) {
#pragma unroll
        for (int j = 0; j < C::DMA_PER_WAVE; ++j) dma16<STREAM>(base, dma_off[j], dma_lds + stage_b + j * 1024u);
    };
    const int64_t tile_stride_b = BN * (int64_t)row_stride_b;
    const char* k_run = nullptr;                 // next K / V tile of the plain steps
    const char* v_run = nullptr;
    // Any tile (clamped to the last tile of this workgroup's list); a segment's ragged last
    // tile re-reads the segment's last key for the rows past its end.
    auto dma_any = [&](const char* seg_a, const char* seg_b, int t, uint32_t stage_b, bool through_index = true) {
        t = t < t_end - 1 ? t : t_end - 1;
        const bool in_b = t >= tiles_a;
        if (INDEXED && !in_b && through_index) {
            dma_indexed(seg_a, t, stage_b);
            return;
        }
        const int key0 = (in_b ? t - tiles_a : t) * BN;
        const int n_valid = (in_b ? p.len_b : seg.len_a) - key0;
        const char* base = (in_b ? seg_b : seg_a) + (int64_t)key0 * row_stride_b;
#pragma unroll
        for (int j = 0; j < C::DMA_PER_WAVE; ++j) {
            int r = dma_row + j * C::RPI;
            r = r < n_valid - 1 ? r : n_valid - 1;
            dma16<STREAM>(base, (uint32_t)r * row_stride_b + dma_coff[j], dma_lds + stage_b + j * 1024u);
        }
    };
    constexpr int DMA_PER_STEP = 2 * C::DMA_PER_WAVE;

    // Q fragments (B operand of S^T = K Q^T): lane holds row `row`, dims ks*16 + hh*8 .. +8
    bf16x8 qf[D / 16];
    {
        const bf16_t* qrow = static_cast<const bf16_t*>(p.q) +
            (((int64_t)item * p.len_q + tok) * p.n_q_heads + kvh * G + (row - tok * G)) * D;
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

    typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 tr4_t;

    // S^T of one tile (32 keys x 32 queries) from K fragments already in registers
    auto qk = [&](const bf16x8 (&kf)[D / 16], f32x16& s) {
#pragma unroll
        for (int j = 0; j < 16; ++j) s[j] = 0.f;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], s, 0, 0, 0);
    };
    auto load_k = [&](uint32_t stage_b, bf16x8 (&kf)[D / 16]) {
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
            kf[ks] = *reinterpret_cast<LDS_AS const bf16x8*>(k_addr[ks] + stage_b);
    };

    // One pipeline step for tile t.  s_cur holds S^T(t); S^T(t+1) goes to s_next.  Stage KN
    // holds K(t+1), stage VC holds V(t); K(t+4) and V(t+3) are fetched into stages KL / VL,
    // whose tiles (K(t), V(t-1)) were consumed in the step before.  PLAIN steps are those
    // whose tile and whose fetched tiles are whole tiles of segment A: no mask, no clamping.
    auto step = [&](int t, f32x16& s_cur, f32x16& s_next, auto kn, auto kl, auto vc, auto vl, auto plain) {
        constexpr uint32_t KN = decltype(kn)::value * TILE_B, KL = decltype(kl)::value * TILE_B;
        constexpr uint32_t VC = decltype(vc)::value * TILE_B, VL = decltype(vl)::value * TILE_B;
        constexpr bool PLAIN = decltype(plain)::value;
        if (PLAIN && INDEXED) {
            if (k_dense) {
                dma_fast(k_run, KL);
                k_run += tile_stride_b;
            } else {
                dma_indexed(ka, t + 4, KL);
            }
            dma_indexed(va, t + 3, STAGES * TILE_B + VL);
        } else if (PLAIN) {
            dma_fast(k_run, KL);
            dma_fast(v_run, STAGES * TILE_B + VL);
            k_run += tile_stride_b;
            v_run += tile_stride_b;
        } else {
            dma_any(ka, kb, t + 4, KL, !k_dense);
            dma_any(va, vb, t + 3, STAGES * TILE_B + VL);
        }
        // All LDS operand reads of this step are issued first; the running-maximum work below
        // covers their latency, and the MFMAs then issue back to back.
        bf16x8 kf[D / 16];
        load_k(KN, kf);
        bf16x8 vf[2][D / 32];
        auto load_v = [&](int g16) {
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const tr4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    reinterpret_cast<LDS_AS tr4_t*>(v_addr[0][db] + VC + g16 * 16 * D * 2));
                const tr4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                    reinterpret_cast<LDS_AS tr4_t*>(v_addr[1][db] + VC + g16 * 16 * D * 2));
                vf[g16][db] = __builtin_shufflevector(__builtin_bit_cast(bf16x4, lo),
                                                      __builtin_bit_cast(bf16x4, hi), 0, 1, 2, 3, 4, 5, 6, 7);
            }
        };
        load_v(0);
        __builtin_amdgcn_sched_barrier(0);
        if (!PLAIN) {
            // ---- visibility: keys [0, lim) of this tile are visible to this lane's row
            const bool in_b = t >= tiles_a;
            const int key0 = (in_b ? t - tiles_a : t) * BN;
            if (in_b || key0 + BN > seg.len_a) {
                const int lim = (in_b ? (tok + q_pos0 + 1 < p.len_b ? tok + q_pos0 + 1 : p.len_b) : seg.len_a) - key0;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int key = (j >> 2) * 8 + hh * 4 + (j & 3);
                    s_cur[j] = key < lim ? s_cur[j] : -INFINITY;
                }
            }
        }
        // ---- running maximum, one query per lane pair (lane, lane ^ 32)
        float mx = s_cur[0];
#pragma unroll
        for (int j = 1; j < 16; ++j) mx = fmaxf(mx, s_cur[j]);
        mx = pair_max(mx);
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

        // ---- matrix cores: S^T(t+1); vector ALU: exp of tile t; then O^T += V^T P^T
        __builtin_amdgcn_s_setprio(3);     // the MFMA-carrying part of the step goes first on this SIMD
        qk(kf, s_next);            // past the last tile this works on a stale stage and is unused
        load_v(1);
#pragma unroll
        for (int g16 = 0; g16 < 2; ++g16) {
            float e[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                e[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[g16 * 8 + j], sc, -mr));
                l_part += e[j];
            }
            bf16x8 pf;
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
                f32x2 two = {e[j], e[j + 1]};
                bf16x2 b2 = __builtin_convertvector(two, bf16x2);
                pf[j] = b2[0];
                pf[j + 1] = b2[1];
            }
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[g16][db], pf, o[db], 0, 0, 0);
        }
        // Order asked of the scheduler for the part above: one MFMA, then its share of the vector
        // work (and, in the first half, one of the second V group's LDS reads).
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < 8) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        }
        __builtin_amdgcn_s_setprio(0);
        step_barrier<2 * DMA_PER_STEP>();   // the loads of this step and the one before may be in flight
    };

    if (t_begin < t_end) {
        f32x16 s_a, s_b;
        constexpr uint32_t VB = STAGES * TILE_B;
        dma_any(ka, kb, t_begin, 0, !k_dense);
        dma_any(ka, kb, t_begin + 1, TILE_B, !k_dense);
        dma_any(ka, kb, t_begin + 2, 2 * TILE_B, !k_dense);
        dma_any(ka, kb, t_begin + 3, 3 * TILE_B, !k_dense);
        dma_any(va, vb, t_begin, VB);
        dma_any(va, vb, t_begin + 1, VB + TILE_B);
        dma_any(va, vb, t_begin + 2, VB + 2 * TILE_B);
        step_barrier<0>();
        if (wave_active) {
            bf16x8 kf0[D / 16];
            load_k(0, kf0);
            qk(kf0, s_a);
        }
        step_barrier<0>();         // K(t_begin) is consumed: its stage is refilled in the first step
        // Everything this wave has loaded so far (the Q fragments among it) has landed.  Saying so in
        // a form the compiler's wait-count bookkeeping sees keeps it from putting a vmcnt(0) in front
        // of the loop's first MFMA, where it would also wait for the tile loads the loop has just
        // issued (those are asm and invisible to it).
        wait_vmem();
        // Step i (mod 4) of this workgroup: S(t) in s_a / s_b alternately, K(t+1) in stage i+1,
        // V(t) in stage i; K(t+4) goes to stage i, V(t+3) to stage i+3.  Groups of four steps
        // run the plain variant while all their tiles, and the tiles they fetch, are whole
        // unmasked tiles of segment A; the rest runs the general variant.
        int t = t_begin;
        if (!wave_active) {
            for (; t < t_end; ++t) {           // same loads into the same stages as the steps below
                const uint32_t i4 = (uint32_t)(t - t_begin) & 3u;
                dma_any(ka, kb, t + 4, i4 * TILE_B, !k_dense);
                dma_any(va, vb, t + 3, VB + ((i4 + 3u) & 3u) * TILE_B);
                step_barrier<2 * DMA_PER_STEP>();
            }
        }
        const int t_plain = (a_full < t_end ? a_full : t_end) - 8;   // t + 3 + 4 < a_full for the group
        const std::false_type general;
        const std::true_type plain;
        k_run = ka + (t + 4) * tile_stride_b;
        v_run = va + (t + 3) * tile_stride_b;
        for (; t <= t_plain; t += 4) {
            step(t, s_a, s_b, IC<1>{}, IC<0>{}, IC<0>{}, IC<3>{}, plain);
            step(t + 1, s_b, s_a, IC<2>{}, IC<1>{}, IC<1>{}, IC<0>{}, plain);
            step(t + 2, s_a, s_b, IC<3>{}, IC<2>{}, IC<2>{}, IC<1>{}, plain);
            step(t + 3, s_b, s_a, IC<0>{}, IC<3>{}, IC<3>{}, IC<2>{}, plain);
        }
        while (t < t_end) {
            step(t, s_a, s_b, IC<1>{}, IC<0>{}, IC<0>{}, IC<3>{}, general);
            if (++t == t_end) break;
            step(t, s_b, s_a, IC<2>{}, IC<1>{}, IC<1>{}, IC<0>{}, general);
            if (++t == t_end) break;
            step(t, s_a, s_b, IC<3>{}, IC<2>{}, IC<2>{}, IC<1>{}, general);
            if (++t == t_end) break;
            step(t, s_b, s_a, IC<0>{}, IC<3>{}, IC<3>{}, IC<2>{}, general);
            ++t;
        }
        wait_vmem();               // no load may still be writing LDS when the workgroup retires
    }

    const float l_tot = pair_sum(l_part);
    if (a.n_splits == 1) {
        if (row_ok) {
            const float inv = 1.f / l_tot;
            bf16_t* orow = static_cast<bf16_t*>(p.out) +
                (((int64_t)item * p.len_q + tok) * p.n_q_heads + kvh * G + (row - tok * G)) * D;
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
        if (row_ok) {                  // the merge reads only real rows
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int j4 = 0; j4 < 4; ++j4) {
                    f32x4 w = {o[db][j4 * 4], o[db][j4 * 4 + 1], o[db][j4 * 4 + 2], o[db][j4 * 4 + 3]};
                    *reinterpret_cast<f32x4*>(po + db * 32 + j4 * 8 + hh * 4) = w;
                }
        }
        if (hh == 0 && row_ok) {
            f32x2 ml = {m_ref, l_tot};
            *reinterpret_cast<f32x2*>(a.part_ml + base * 2) = ml;
        }
    }
}

// Combines the split-KV partial results of one query row (the usual log-sum-exp merge).  One
// workgroup per row: the splits are spread over 256 / (D/4) thread groups, each thread owning
// four output dimensions, and the groups' sums meet in LDS.
template <int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(KernelArgs a) {
    const AttnProblem& p = a.p;
    constexpr int TPR = D / 4;                 // threads per row
    constexpr int NG = 256 / TPR;              // split groups
    __shared__ float red_m[NG];
    __shared__ float red_l[NG];
    __shared__ f32x4 red_o[NG][TPR];
    const int G = p.n_q_heads / p.n_kv_heads;
    const int m_rows = p.len_q * G;
    const int64_t rows_pad = (int64_t)a.m_tiles * BM;
    const int64_t ik = blockIdx.x / m_rows;    // (item, KV head)
    const int row = (int)(blockIdx.x % m_rows);
    const int item = (int)(ik / p.n_kv_heads), kvh = (int)(ik % p.n_kv_heads);
    const int64_t base0 = ik * a.n_splits * rows_pad + row;
    const int tid = threadIdx.x;

    // each group folds its splits into one (m, l, O) triple; all loads of a group are
    // independent, so the kernel pays one memory round trip when n_splits <= NG
    const int g = tid / TPR, dq = tid % TPR;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;
    for (int s = g; s < a.n_splits; s += NG) {
        const int64_t base = base0 + s * rows_pad;
        const f32x2 ml = *reinterpret_cast<const f32x2*>(a.part_ml + base * 2);
        const f32x4 v = *reinterpret_cast<const f32x4*>(a.part_o + base * D + dq * 4);
        const float m_new = fmaxf(m, ml[0]);
        const float w_old = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - m_new);
        const float w_new = (ml[0] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ml[0] - m_new);
        l = l * w_old + ml[1] * w_new;
        acc = acc * w_old + v * w_new;
        m = m_new;
    }
    red_o[g][dq] = acc;
    if (dq == 0) {
        red_m[g] = m;
        red_l[g] = l;
    }
    __syncthreads();
    if (tid < TPR) {
        float m_all = red_m[0];
#pragma unroll
        for (int i = 1; i < NG; ++i) m_all = fmaxf(m_all, red_m[i]);
        f32x4 sum = {0.f, 0.f, 0.f, 0.f};
        float l_all = 0.f;
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const float w = (red_m[i] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(red_m[i] - m_all);
            sum += red_o[i][tid] * w;
            l_all += red_l[i] * w;
        }
        const float inv = 1.f / l_all;
        const int tok = row / G;
        bf16_t* orow = static_cast<bf16_t*>(p.out) +
            (((int64_t)item * p.len_q + tok) * p.n_q_heads + kvh * G + (row - tok * G)) * D + tid * 4;
        f32x2 lo = {sum[0] * inv, sum[1] * inv}, hi = {sum[2] * inv, sum[3] * inv};
        u32x2 w;
        w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
        w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
        *reinterpret_cast<u32x2*>(orow) = w;
    }
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
    const int64_t nb = ik * plan.n_splits * plan.m_tiles;
    if (p.is_encode)
        hipLaunchKernelGGL((attn_bf16_kernel<D, true, false, false>), dim3((unsigned)nb), dim3(THREADS), 0, stream, a);
    else if (p.a_index)
        hipLaunchKernelGGL((attn_bf16_kernel<D, false, true, false>), dim3((unsigned)nb), dim3(THREADS), 0, stream, a);
    else if (plan.m_tiles == 1)
        hipLaunchKernelGGL((attn_bf16_kernel<D, false, false, true>), dim3((unsigned)nb), dim3(THREADS), 0, stream, a);
    else
        hipLaunchKernelGGL((attn_bf16_kernel<D, false, false, false>), dim3((unsigned)nb), dim3(THREADS), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (plan.n_splits > 1) {
        const int64_t rows = ik * p.len_q * (p.n_q_heads / p.n_kv_heads);
        hipLaunchKernelGGL(attn_merge_kernel<D>, dim3((unsigned)rows), dim3(256), 0, stream, a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace

AttnPlan attn_bf16_plan(const AttnProblem& p) {
    AttnPlan plan;
    const int G = p.n_q_heads / p.n_kv_heads;
    plan.m_tiles = (p.len_q * G + BM - 1) / BM;
    const int64_t base = (int64_t)p.n_items * p.n_kv_heads * plan.m_tiles;
    // longest tile list of any item (encode: a full window; QA: all retrieved tokens)
    const int len_a_max = p.is_encode ? p.l_l : p.len_a;
    const int n_tiles = (len_a_max + BN - 1) / BN + (p.len_b + BN - 1) / BN;
    int splits = 1;
    const int64_t target = 512;              // about two workgroups per CU
    if (base < target) {
        // the largest split count that still fits one round of resident workgroups: one more
        // workgroup than that costs a whole second round
        splits = (int)(target / base);
        if (splits < 1) splits = 1;
        // at least 8 tiles (256 keys) per split; 2 when only one wavefront per workgroup has rows
        // (a decode step), where latency rather than the pipeline's fill cost decides
        const int min_tiles = p.len_q * G <= WM ? 2 : 8;
        const int cap = n_tiles / min_tiles > 1 ? n_tiles / min_tiles : 1;
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
