// Internal declarations shared by the HIP sources of librekv (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rekv.h"

namespace rekv {

typedef __bf16 bf16_t;

// One attention problem family: every batch item (a chunk of the stream, or a question)
// attends to two key segments.  Segment A is visible to every query row; segment B is the
// item's text tokens, visible causally: the len_q query tokens are the last len_q tokens of
// B, so query token i sees B-token j iff j <= i + (len_b - len_q).
//   encode (Eq. 1): A = local window in the cache, B = the chunk's own K/V in the cache
//   QA     (Eq. 3): A = retrieved KV of the question, B = the question's own K/V
//   decode (Eq. 3): A = retrieved KV, B = question + generated tokens, queries = the new ones
struct AttnProblem {
    const void* q;      // [n_items * len_q, Hq, D]
    void* out;          // same shape
    const void* k_a;    // encode: k_cache; QA: k_ret
    const void* v_a;
    const void* k_b;    // encode: k_cache; QA: k_self
    const void* v_b;
    int64_t first_token;  // encode only
    int32_t l_l;          // encode only: window length in tokens
    int32_t len_a;        // QA only: retrieved tokens per question
    int32_t len_b;        // l_x, N_q, or the text tokens so far
    int32_t len_q;        // query tokens per item: len_b, or the new tokens of a decode step
    int64_t b_stride;     // QA / decode: tokens between consecutive items' B segments
    int32_t n_items;      // chunks or questions
    int32_t is_encode;
    int32_t n_q_heads, n_kv_heads, head_dim;
    float scale;
    // Indexed segment A (QA / decode straight from the KV arena, no gathered copy): A-token j of
    // item i is token a_index[i * a_index_stride + j / n_f] * n_f + j % n_f of k_a / v_a.
    const int32_t* a_index;   // NULL: segment A is contiguous
    int64_t a_index_stride;
    int32_t n_f;              // tokens per frame
    int32_t n_src_frames;     // frames in the arena; index entries are clamped into [0, n_src_frames)
    // QA / decode: frames actually retrieved per item (device int32 [n_items], NULL = all): item i
    // attends to the first min(a_valid_frames[i] * n_f, len_a) tokens of its segment A only.
    const int32_t* a_valid_frames;
    // With a_index: the KEYS of segment A come from a dense per-item buffer [n_items, len_a, Hkv, D]
    // at k_a (keys re-positioned by a pre-pass over the index list) while the values are still
    // read in place through the index list.
    int32_t a_k_dense;
};

// Resolves one item's segment bases (in elements) and lengths.  Device only: it reads the
// per-item count of retrieved frames.
struct ItemSegs {
    int64_t a_off, b_off;  // token offsets into k_a/v_a and k_b/v_b
    int32_t len_a;
};
__device__ inline ItemSegs item_segments(const AttnProblem& p, int item) {
    ItemSegs s;
    if (p.is_encode) {
        const int64_t t0 = p.first_token + (int64_t)item * p.len_b;
        const int64_t w0 = t0 > p.l_l ? t0 - p.l_l : 0;
        s.a_off = w0;
        s.b_off = t0;
        s.len_a = (int32_t)(t0 - w0);
    } else {
        s.a_off = p.a_index ? 0 : (int64_t)item * p.len_a;
        s.b_off = (int64_t)item * p.b_stride;
        s.len_a = p.len_a;
        if (p.a_valid_frames) {
            const int32_t nv = p.a_valid_frames[item];
            const int64_t lim = (int64_t)(nv > 0 ? nv : 0) * p.n_f;
            if (lim < s.len_a) s.len_a = (int32_t)lim;
        }
    }
    return s;
}

// Split-KV workspace need of the bf16 kernel, in bytes (0 when one split suffices).
struct AttnPlan {
    int32_t n_splits;
    int32_t m_tiles;
    size_t workspace_bytes;
};
AttnPlan attn_bf16_plan(const AttnProblem& p);
hipError_t attn_bf16_launch(const AttnProblem& p, const AttnPlan& plan, void* workspace,
                            hipStream_t stream);
hipError_t attn_f32_launch(const AttnProblem& p, hipStream_t stream);

hipError_t frame_keys_launch(const void* k, int n_frames, int tokens_per_frame, int d_prime,
                             int dtype, float* frame_keys, hipStream_t stream);

struct RetrieveArgs {
    const float* frame_keys;
    int64_t frame_keys_stride;
    int32_t n_frames;
    const void* q_question;
    int32_t n_questions, n_q_tokens, k;
    int32_t n_q_heads, n_kv_heads, head_dim, dtype;
    int32_t* idx;
    int32_t* n_sel;
    float* scores;   // [n_questions, n_frames], never NULL here (workspace if the caller gave none)
    float* q_vec;    // [n_questions, D'] workspace: pooled question vectors
    // External retrieval (Eq. 2 on given embeddings): q_question == NULL, q_vec_given holds the
    // question embeddings, dim their length; scores are divided by tau.
    const float* q_vec_given;
    int32_t dim;     // vector length; 0 = Hkv * D
    float inv_tau;   // 1 for internal retrieval
};
hipError_t retrieve_launch(const RetrieveArgs& a, hipStream_t stream);

hipError_t block_keys_launch(const float* frame_keys, int n_frames, int b, int d_prime, float* block_keys,
                             hipStream_t stream);
hipError_t expand_blocks_launch(const int32_t* block_idx, int n_questions, int k_blocks, int b, int n_frames,
                                int32_t* frame_idx, int32_t* n_sel, hipStream_t stream);

hipError_t gather_launch(const void* src_k, const void* src_v, int n_src_frames, const int32_t* idx,
                         int n_blocks, size_t frame_bytes, void* dst_k, void* dst_v,
                         hipStream_t stream);

constexpr int MAX_GATHER_LAYERS = 64;
hipError_t gather_layers_launch(const void* const* src_k, const void* const* src_v, int n_layers, int n_src_frames,
                                const int32_t* idx, int blocks_per_layer, size_t frame_bytes, void* dst_k, void* dst_v,
                                hipStream_t stream);

// Position policy of the retrieved keys (gather.hip): new position of gathered token j of a
// question = pos_offset (+ j unless is_static); cached keys carry no rotation, or (src_rotated)
// the rotation of their stream position src_pos_offset + token index.
struct RopeArgs {
    double log2_base;
    int64_t pos_offset, src_pos_offset;
    int32_t is_static, src_rotated, interleaved;
};
hipError_t gather_rope_launch(const void* src_k, const void* src_v, int n_src_frames, const int32_t* idx,
                              int n_questions, int k_slots, int n_f, int n_kv_heads, int d, int dtype,
                              void* dst_k, void* dst_v, const RopeArgs& ra, hipStream_t stream);

// Measurement probes (probe.hip).
hipError_t launch_probe_copy(void* dst, const void* src, int64_t n_bytes, hipStream_t stream);
hipError_t launch_probe_mfma(float* sink, int32_t n_workgroups, int32_t n_iters, hipStream_t stream);
double probe_mfma_flop(int32_t n_workgroups, int32_t n_iters);

}  // namespace rekv
