/*
 * rekv.h - C ABI of the ReKV hot path for AMD MI355X (gfx950).
 *
 * ReKV ("Streaming Video Question-Answering with In-context Video KV-Cache
 * Retrieval") changes only the attention of a decoder Video-LLM:
 *   - the video stream is encoded chunk by chunk with sliding-window attention
 *     (method section, Eq. 1),
 *   - each frame keeps the mean of its key vectors as a representative vector, a
 *     question is pooled the same way, frames are ranked by cosine similarity
 *     (Eq. 2 with tau = 1) and the r best frames' KV is reloaded onto the GPU
 *     (internal video KV-cache retrieval),
 *   - the question tokens attend to the retrieved KV and to themselves (Eq. 3).
 * This library is those steps for one attention layer on one GPU.  The Q/K/V
 * projections, RoPE and the rest of the model stay with the caller.
 *
 * Conventions shared by every call
 *   - Pointers are DEVICE pointers unless a parameter says "host".
 *   - Layout is token-major and dense: Q and O are [tokens, Hq, D]; K and V are
 *     [tokens, Hkv, D]; the element type is the context's dtype (fp32 or bf16).
 *     Query head h uses KV head h / (Hq / Hkv).
 *   - The caller owns every buffer.  The library never frees or keeps a caller
 *     pointer after the call's work has completed on the stream.  The context owns
 *     a private workspace (split-KV partial results, pooled question vectors,
 *     scores), one side stream and two events.
 *   - The workspace grows on demand: a call whose shapes need more than any call
 *     before it on this context frees the old block and allocates a larger one
 *     (hipFree + hipMalloc: the device is synchronised, and the call is not legal
 *     under stream capture).  Run each shape once before capturing a graph or
 *     entering a loop that must not allocate; rekv_decode_attention_noalloc never
 *     allocates.  The workspace is shared by all calls on the context, so a context
 *     serves one stream at a time.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     are asynchronous on it, except where a parameter says otherwise.
 *   - Every call returns a rekv_status.  Arguments are checked before anything is
 *     launched (the one exception, host path 1 of rekv_gather_kv, says so there);
 *     rekv_last_error() describes the argument that was refused.  A context may be
 *     used by one host thread at a time.
 */
#ifndef REKV_H
#define REKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rekv_ctx rekv_ctx; /* opaque */

typedef enum {
    REKV_OK = 0,
    REKV_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, Hq % Hkv != 0, ... */
    REKV_ERR_UNSUPPORTED = 2, /* a shape the kernels do not cover (see rekv_create) */
    REKV_ERR_NOMEM = 3,       /* the context's workspace could not be grown */
    REKV_ERR_HIP = 4          /* a HIP runtime call failed; message holds hipGetErrorString */
} rekv_status;

typedef enum { REKV_F32 = 0, REKV_BF16 = 1 } rekv_dtype;

typedef struct {
    int32_t n_q_heads;        /* Hq */
    int32_t n_kv_heads;       /* Hkv, divides Hq */
    int32_t head_dim;         /* D: 64 or 128 for bf16; a multiple of 4 up to 256 for fp32 */
    int32_t tokens_per_frame; /* N_f > 0 */
    int32_t dtype;            /* rekv_dtype of Q/K/V/O */
    float softmax_scale;      /* 0 means 1/sqrt(D) */
} rekv_shape;

/* Creates a context for one layer shape on the current HIP device.  Host call; allocates
 * the side stream and events.  *out is NULL on failure. */
rekv_status rekv_create(const rekv_shape* shape, rekv_ctx** out);

/* Waits for the side stream, frees the workspace.  NULL is accepted. */
void rekv_destroy(rekv_ctx* ctx);

/* Message of the last failed call on this context (empty string if none).  With a NULL
 * context, the message of the last failed rekv_create on this thread. */
const char* rekv_last_error(const rekv_ctx* ctx);

/*
 * Video stream encoding with sliding-window attention, Eq. 1.
 *
 * Encodes n_chunks >= 1 consecutive chunks of l_x tokens.  Chunk c starts at stream
 * token t0 = first_token + c * l_x.  Each of its tokens attends to the local window
 * L = the last min(l_l, t0) tokens before t0 (the same L for the whole chunk, as Eq. 1
 * defines it) and, causally, to the chunk's tokens up to itself.  Several chunks in one
 * call give exactly the result of one call per chunk, because the keys and values are
 * inputs.
 *
 *   q        [n_chunks * l_x, Hq, D]   queries of the chunks' tokens
 *   k_cache  [>= first_token + n_chunks * l_x, Hkv, D]  the stream's keys indexed by
 *   v_cache  same shape                stream token, already holding the chunks' own K/V
 *   out      [n_chunks * l_x, Hq, D]
 *   l_l      window length in tokens (>= 0)
 */
rekv_status rekv_encode_chunk(rekv_ctx* ctx, const void* q, const void* k_cache,
                              const void* v_cache, int64_t first_token, int32_t l_x,
                              int32_t n_chunks, int32_t l_l, void* out, void* stream);

/*
 * Representative frame vectors (internal retrieval): for each frame the mean of its
 * N_f key vectors, KV heads concatenated to D' = Hkv * D.
 *
 *   k           [n_frames * N_f, Hkv, D]   keys of n_frames whole frames
 *   frame_keys  [n_frames, D'] fp32 (always fp32, accumulated in fp32)
 */
rekv_status rekv_frame_keys(rekv_ctx* ctx, const void* k, int32_t n_frames, float* frame_keys,
                            void* stream);

/*
 * Internal retrieval: pooled question vector, Eq. 2 cosine scores (tau = 1), top-k.
 *
 * For each of n_questions questions: the question vector is the mean of its N_q query
 * vectors, the G query heads of a KV group averaged so that it has D' entries; the score
 * of frame f < n_frames is the cosine between that vector and frame_keys[f] (0 when either
 * norm is 0); the k best-scoring frames are selected, ties going to the lower frame index.
 * n_frames is the number of frames visible to the question (its timestamp cut-off).
 *
 *   frame_keys          [n_frames, D'] fp32 per table
 *   frame_keys_stride   elements between the tables of consecutive questions; 0 = all
 *                       questions share one table (many questions on one stream); a
 *                       per-layer table per "question" gives per-layer retrieval
 *   q_question          [n_questions, N_q, Hq, D] in the context dtype
 *   idx                 [n_questions, k] int32: the selected frames in ascending frame
 *                       order; entries past n_sel are -1
 *   n_sel               [n_questions] int32: min(k, n_frames); may be NULL
 *   scores              [n_questions, n_frames] fp32, may be NULL
 * Limits: 1 <= k <= 4096, n_frames >= 1, (Hq / Hkv) * D <= 4096; q_question 16-byte aligned.
 */
rekv_status rekv_retrieve_topk(rekv_ctx* ctx, const float* frame_keys, int64_t frame_keys_stride,
                               int32_t n_frames, const void* q_question, int32_t n_questions,
                               int32_t n_q_tokens, int32_t k, int32_t* idx, int32_t* n_sel,
                               float* scores, void* stream);

/*
 * External retrieval scoring (external video KV-cache retrieval, Eq. 2 with its temperature):
 * the same cosine ranking on embeddings the caller computed elsewhere (the paper uses a
 * CLIP-like encoder pair, which is not part of this library).
 *   Sim(v, q) = v.q / (tau |v| |q|); a zero-norm vector scores 0; selection as in
 *   rekv_retrieve_topk (ties to the lower index, ascending output, -1 padding).
 *
 *   frame_emb  [n_frames, dim] fp32, 16-byte aligned, dim a multiple of 4, one
 *              table shared by all questions
 *   q_emb      [n_questions, dim] fp32, 16-byte aligned
 *   tau        > 0 (a positive tau does not change the ranking, only the reported scores)
 *   idx, n_sel, scores   as in rekv_retrieve_topk
 */
rekv_status rekv_retrieve_external(rekv_ctx* ctx, const float* frame_emb, int32_t n_frames, int32_t dim,
                                   const float* q_emb, int32_t n_questions, float tau, int32_t k,
                                   int32_t* idx, int32_t* n_sel, float* scores, void* stream);

/*
 * Block-level retrieval (retrieval section and the block-size ablation): b consecutive
 * frames form a block whose vector is the average of their frame vectors; blocks are scored
 * and selected like frames, ceil(r / b) of them, and all their frames are retrieved.
 * The paper leaves the case b not dividing the frame count open; here the last block holds
 * the remaining frames.
 *
 * rekv_block_keys: block_keys[j] = mean of frame_keys[j*b .. min((j+1)*b, n_frames) - 1].
 *   frame_keys  [n_frames, D'] fp32, 16-byte aligned;  block_keys  [ceil(n_frames / b), D'] fp32
 *   A caller that scores blocks keeps this table up to date as frames arrive (re-running the
 *   call on the last, still growing block) and passes it to rekv_retrieve_topk with
 *   n_frames = the number of blocks and k = ceil(r / b).
 * rekv_expand_blocks: turns the selected blocks into the frame list rekv_gather_kv takes.
 *   block_idx   [n_questions, k_blocks] int32, ascending, -1 padded (rekv_retrieve_topk's idx)
 *   frame_idx   [n_questions, k_blocks * b] int32: the blocks' frames in order; slots past the
 *               end of the stream (the short last block) or of the selection hold -1, always
 *               at the tail
 *   n_sel       [n_questions] int32: frames listed per question; may be NULL
 */
rekv_status rekv_block_keys(rekv_ctx* ctx, const float* frame_keys, int32_t n_frames, int32_t b,
                            float* block_keys, void* stream);
rekv_status rekv_expand_blocks(rekv_ctx* ctx, const int32_t* block_idx, int32_t n_questions,
                               int32_t k_blocks, int32_t b, int32_t n_frames, int32_t* frame_idx,
                               int32_t* n_sel, void* stream);

/*
 * Reload of the retrieved KV (overview figure, panel (c), and the text after Eq. 2: the
 * key-value vectors of the r selected frames are brought back onto the GPU to serve as the
 * context of question answering): copies the selected frames' key and value blocks into one
 * dense buffer per question, in the order idx gives them (ascending frame index).
 *
 *   src_k, src_v  [n_src_frames * N_f, Hkv, D] in HBM (src_on_host = 0) or in pinned host
 *                 memory (src_on_host = 1 or 2, host pointers; memory from hipHostMalloc)
 *   idx           [n_questions, k] int32 on the device; the destination block of an entry
 *                 < 0 (the -1 padding of a short selection) is zero-filled; so is that of an
 *                 entry >= n_src_frames on the device path and host path 2, while host
 *                 path 1 reports such an entry as an error.  Pass the selection's n_sel to
 *                 the attention call so that the zero-filled blocks are not attended to.
 *   dst_k, dst_v  [n_questions, k * N_f, Hkv, D] in HBM
 * Host path 1 (copy engine): idx is copied to the host (the call blocks until `stream`
 * reaches it, and that copy has run even if an entry is then refused), then one async copy
 * per run of consecutive frames and tensor goes to the context's side stream; `stream` waits
 * on an event for their completion, so later work on `stream` sees the data.
 * Host path 2 (zero-copy): the gather kernel itself reads the pinned arrays over the host
 * link, on the side stream, ordered after `stream` and joined back into it; the host does not
 * block and idx never leaves the device.  Out-of-range entries are skipped as on the device path.
 */
rekv_status rekv_gather_kv(rekv_ctx* ctx, const void* src_k, const void* src_v,
                           int32_t src_on_host, int32_t n_src_frames, const int32_t* idx,
                           int32_t n_questions, int32_t k, void* dst_k, void* dst_v, void* stream);

/*
 * rekv_gather_kv for several layers in one launch.  In the method every layer retrieves its own
 * frames ("Internal Video KV-Cache Retrieval": retrieval runs inside each attention layer, on
 * that layer's keys), so a whole model reloads n_layers independent selections from n_layers
 * pairs of arenas; here they are one grid instead of n_layers small ones.
 *
 *   src_k, src_v  HOST arrays of n_layers device pointers, each [n_src_frames * N_f, Hkv, D]
 *                 in HBM (1 <= n_layers <= 64); the arrays are read during the call only
 *   idx           [n_layers, n_questions, k] int32 on the device, as in rekv_gather_kv
 *   dst_k, dst_v  [n_layers, n_questions, k * N_f, Hkv, D] in HBM
 * Entries of idx outside [0, n_src_frames) zero-fill their block.
 */
rekv_status rekv_gather_kv_layers(rekv_ctx* ctx, const void* const* src_k, const void* const* src_v,
                                  int32_t n_layers, int32_t n_src_frames, const int32_t* idx,
                                  int32_t n_questions, int32_t k, void* dst_k, void* dst_v, void* stream);

/*
 * Reload of the retrieved KV with the position policy of the "Positional Encoding" paragraph:
 * for question answering the original stream positions of the retrieved tokens are dropped
 * and the gathered tokens are numbered one after the other, like ordinary text; the static
 * variant gives all of them one position.  Values are copied as by rekv_gather_kv; keys are rotated (rotary position
 * embedding: pair i of a head vector turns by position * base^(-2i/D)) to
 *   pos_mode 0 (consecutive): position pos_offset + j for gathered token j of the question,
 *   pos_mode 1 (static):      position pos_offset for every token.
 * The cache may hold keys without positions (src_rotated = 0) or keys already rotated at
 * their stream position src_pos_offset + token index (src_rotated = 1); those are turned by
 * the difference.  rope_layout 0 pairs dims (i, i + D/2), 1 pairs dims (2i, 2i + 1).
 * Angles are formed and range-reduced in double precision.
 *
 *   src_k, src_v, idx, dst_k, dst_v, n_src_frames, n_questions, k   as in rekv_gather_kv;
 *                 entries of idx outside the arena zero-fill their block
 *   src_on_host   0: the arenas are in HBM; 1: they are pinned host memory (host pointers, from
 *                 hipHostMalloc) - offloaded KV - and the kernels read them over the host link on
 *                 the context's side stream, ordered after `stream` and joined back into it, as
 *                 host path 2 of rekv_gather_kv does
 *   rope_base     > 1 (10000 in RoFormer)
 *   D             a multiple of 16 (bf16) or 8 (fp32), at most 256
 */
rekv_status rekv_gather_kv_rope(rekv_ctx* ctx, const void* src_k, const void* src_v, int32_t src_on_host,
                                int32_t n_src_frames, const int32_t* idx, int32_t n_questions, int32_t k,
                                void* dst_k, void* dst_v, double rope_base, int32_t rope_layout, int32_t pos_mode,
                                int64_t pos_offset, int32_t src_rotated, int64_t src_pos_offset, void* stream);

/*
 * Question answering over the retrieved KV, Eq. 3 with X = the question tokens: every
 * question token attends to all n_ret_tokens retrieved tokens and, causally, to the
 * question tokens up to itself.
 *
 *   q, out          [n_questions, N_q, Hq, D]
 *   k_ret, v_ret    [n_questions, n_ret_tokens, Hkv, D]   (n_ret_tokens may be 0)
 *   n_sel           device int32 [n_questions] or NULL: frames actually retrieved for each
 *                   question (the n_sel of rekv_retrieve_topk / rekv_expand_blocks).  Question
 *                   i attends to its first min(n_sel[i] * N_f, n_ret_tokens) retrieved tokens
 *                   only, so the padding of a selection shorter than k (young stream, ragged
 *                   last block) stays out of the softmax.  NULL: all n_ret_tokens are valid.
 *   k_self, v_self  [n_questions, N_q, Hkv, D]
 */
rekv_status rekv_qa_attention(rekv_ctx* ctx, const void* q, const void* k_ret, const void* v_ret,
                              int32_t n_ret_tokens, const int32_t* n_sel, const void* k_self,
                              const void* v_self, int32_t n_questions, int32_t n_q_tokens, void* out,
                              void* stream);

/*
 * Answer decoding over the retrieved KV, Eq. 3 with X = the token(s) being decoded: the
 * context is the retrieved KV followed by the text KV so far (question and generated
 * tokens).  The caller has already appended the new tokens' own K/V, so they are the last
 * n_new_tokens of the n_text_tokens valid text rows; new token i attends to every retrieved
 * token and to text rows j <= n_text_tokens - n_new_tokens + i.  rekv_qa_attention is the
 * case n_new_tokens = n_text_tokens = text_stride = N_q.
 *
 *   q, out          [n_questions, n_new_tokens, Hq, D]
 *   k_ret, v_ret    [n_questions, n_ret_tokens, Hkv, D]   (n_ret_tokens may be 0)
 *   n_sel           as in rekv_qa_attention (device int32 [n_questions] or NULL)
 *   k_text, v_text  [n_questions, text_stride, Hkv, D], the first n_text_tokens rows of each
 *                   question valid (text_stride >= n_text_tokens >= n_new_tokens >= 1)
 */
rekv_status rekv_decode_attention(rekv_ctx* ctx, const void* q, const void* k_ret, const void* v_ret,
                                  int32_t n_ret_tokens, const int32_t* n_sel, const void* k_text,
                                  const void* v_text, int64_t text_stride, int32_t n_text_tokens,
                                  int32_t n_questions, int32_t n_new_tokens, void* out, void* stream);

/*
 * rekv_decode_attention for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops that decode token after token, harnesses that forbid hipMalloc.
 * Same arguments, same kernels, same result.  The split-KV partial results go to a static
 * device array of 33 MiB inside the library (one copy per GPU, held until the process ends)
 * instead of the context's growable workspace, so the call never allocates, frees or
 * synchronises.  A launch that would need more scratch than that is refused with
 * REKV_ERR_UNSUPPORTED (fp32 contexts use no scratch at all).  Every call on a GPU shares that
 * GPU's array: calls that overlap in time on one GPU - other streams, other contexts - race;
 * calls ordered on one stream are safe.  Nothing in the array needs to start at zero: a launch
 * writes every partial result it later reads.
 */
rekv_status rekv_decode_attention_noalloc(rekv_ctx* ctx, const void* q, const void* k_ret,
                                          const void* v_ret, int32_t n_ret_tokens, const int32_t* n_sel,
                                          const void* k_text, const void* v_text, int64_t text_stride,
                                          int32_t n_text_tokens, int32_t n_questions,
                                          int32_t n_new_tokens, void* out, void* stream);

/*
 * Eq. 3 straight from the KV arena: the same attention as rekv_decode_attention (hence as
 * rekv_qa_attention, which is its case n_new_tokens = n_text_tokens), but the retrieved KV is
 * read in place through the frame list that retrieval produced, so the gathered copy is
 * neither written nor read back.  The retrieved context of question i is the frames
 * idx[i][0 .. n_ret_frames), in that order.
 *
 *   q, out          [n_questions, n_new_tokens, Hq, D]
 *   k_src, v_src    [n_src_frames * N_f, Hkv, D] in HBM, each below 4 GiB
 *   idx             [n_questions, idx_stride] int32 on the device, idx_stride >= n_ret_frames;
 *                   the first min(n_ret_frames, n_sel[i]) entries of row i must be frames of
 *                   the arena (entries outside [0, n_src_frames) are clamped into it, never
 *                   followed out of bounds); 1 <= n_ret_frames <= 1024
 *   n_sel           device int32 [n_questions] or NULL: entries of each row that are real
 *                   selections (rekv_retrieve_topk's n_sel); the -1 padding after them is
 *                   neither read nor attended to.  NULL: all n_ret_frames entries are used.
 *   k_text, v_text, text_stride, n_text_tokens, n_new_tokens   as in rekv_decode_attention
 */
rekv_status rekv_attention_indexed(rekv_ctx* ctx, const void* q, const void* k_src, const void* v_src,
                                   int32_t n_src_frames, const int32_t* idx, int64_t idx_stride,
                                   int32_t n_ret_frames, const int32_t* n_sel, const void* k_text, const void* v_text,
                                   int64_t text_stride, int32_t n_text_tokens, int32_t n_questions,
                                   int32_t n_new_tokens, void* out, void* stream);

/*
 * rekv_attention_indexed with the position policy of the "Positional Encoding" paragraph: the
 * retrieved frames' VALUES are read in place through the frame list, their KEYS are first turned
 * to the positions they take in the question-answering context (a pre-pass over the frame list
 * that writes the re-positioned keys to k_pos; values carry no position), then Eq. 3 runs on
 * those keys.  Against gather-with-positions followed by attention this saves writing and
 * re-reading the values.  Position arguments as in rekv_gather_kv_rope (pos_mode 0: gathered
 * token j of a question gets position pos_offset + j; 1: pos_offset for all); attention
 * arguments as in rekv_attention_indexed, with idx_stride == n_ret_frames.
 *
 *   k_pos   [n_questions, n_ret_frames * N_f, Hkv, D] in HBM, caller-owned scratch that receives
 *           the re-positioned keys (its contents after the call are those keys; blocks of
 *           entries outside the arena are zero)
 *   k_src, v_src   in HBM, the V arena below 4 GiB
 */
rekv_status rekv_attention_indexed_rope(rekv_ctx* ctx, const void* q, const void* k_src, const void* v_src,
                                        int32_t n_src_frames, const int32_t* idx, int64_t idx_stride,
                                        int32_t n_ret_frames, const int32_t* n_sel, void* k_pos,
                                        double rope_base, int32_t rope_layout, int32_t pos_mode,
                                        int64_t pos_offset, int32_t src_rotated, int64_t src_pos_offset,
                                        const void* k_text, const void* v_text, int64_t text_stride,
                                        int32_t n_text_tokens, int32_t n_questions, int32_t n_new_tokens,
                                        void* out, void* stream);

/*
 * Offload of encoded KV to RAM (the paragraph after Eq. 1: every frame's KV is kept, and what
 * leaves the local window moves off the GPU; appendix "Multi-processing Serving": the encoder
 * process hands the stream's KV to the answering processes through host memory).  Copies
 * n_frames whole frames of K and V, starting at frame first_frame of the device arrays, to the
 * same frame positions of the pinned host arrays.
 * The copies run on the context's side stream after everything queued on `stream` so far;
 * `stream` does not wait for them.  rekv_offload_wait() blocks the host until all offloads
 * issued on this context have landed; rekv_offload_join() instead makes `stream` wait for them
 * on the device (the host does not block), so that work queued on `stream` afterwards may
 * overwrite the device arrays - the slots of evicted frames - while the host copies stay intact.
 *
 *   dev_k, dev_v    [>= (first_frame + n_frames) * N_f, Hkv, D] in HBM
 *   host_k, host_v  same indexing, pinned host memory (host pointers)
 */
rekv_status rekv_offload_kv(rekv_ctx* ctx, const void* dev_k, const void* dev_v, void* host_k,
                            void* host_v, int64_t first_frame, int32_t n_frames, void* stream);
rekv_status rekv_offload_wait(rekv_ctx* ctx);
rekv_status rekv_offload_join(rekv_ctx* ctx, void* stream);

/*
 * Measurement probes.  They are not operations of the method: they show what this GPU
 * sustains on the two resources the path is priced against, so that a kernel's rate can be
 * read against the machine it ran on as well as against the published peaks.
 *
 * rekv_probe_copy: plain streaming copy of n_bytes (a multiple of 16; both pointers 16-byte
 *   aligned, device memory, not overlapping).  Moves n_bytes in and n_bytes out of HBM; it
 *   is also the kernel of known size that the HBM byte counters are calibrated on.
 * rekv_probe_mfma: n_workgroups workgroups of 4 wavefronts, each wavefront issuing
 *   4 * n_iters (n_iters rounded up to a multiple of 8) bf16 32x32x16 MFMAs on four independent
 *   accumulators, cycling through 8 operand fragment pairs held in registers.  sink receives
 *   n_workgroups * 256 floats (so the work is not optimised away); *flop (host pointer, may
 *   be NULL) receives the floating-point operations of the launch.
 */
rekv_status rekv_probe_copy(rekv_ctx* ctx, void* dst, const void* src, int64_t n_bytes, void* stream);
rekv_status rekv_probe_mfma(rekv_ctx* ctx, float* sink, int32_t n_workgroups, int32_t n_iters,
                            double* flop, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* REKV_H */
