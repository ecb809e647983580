// The C ABI of librekv: argument validation, the context (workspace, side stream, events)
// and dispatch to the kernels.  No arithmetic of the method happens in this file.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>

#include "common.h"

struct rekv_ctx {
    rekv_shape shape;
    float scale;
    int device;
    void* ws;             // workspace: split-KV partials, or pooled questions + scores
    size_t ws_bytes;
    void* scratch;        // this device's copy of the static scratch array
    hipStream_t side;     // host<->device copies of offloaded KV
    hipEvent_t ev_main;   // recorded on the caller's stream, waited on by the side stream
    hipEvent_t ev_side;   // recorded on the side stream, waited on by the caller's stream
    int32_t* idx_host;    // pinned staging for the index list of the host gather
    size_t idx_host_cap;  // entries
    char err[512];
};

// Scratch of the allocation-free entry point (rekv_decode_attention_noalloc): the split-KV
// partial results of one launch.  One copy per GPU, held until the process ends; every call on a
// GPU shares it.  The bf16 plan never asks for more: at most 512 workgroups x 128 rows x
// (D + 2) floats when the key range is split.
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)33 << 20;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

namespace {

thread_local char g_create_err[512] = "";

// Device address of `scratch` on each GPU (the array's name is only a host-side handle).
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

// Looks the address up once per device; that device must be current.
hipError_t scratch_address(int device, void** out) {
    *out = nullptr;
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

rekv_status fail(rekv_ctx* ctx, rekv_status code, const char* fmt, ...) {
    char* dst = ctx ? ctx->err : g_create_err;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 512, fmt, ap);
    va_end(ap);
    return code;
}

rekv_status fail_hip(rekv_ctx* ctx, const char* what, hipError_t e) {
    return fail(ctx, REKV_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

size_t elem_size(const rekv_ctx* c) { return c->shape.dtype == REKV_BF16 ? 2 : 4; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Grows the context's workspace.  Freeing the old block waits for the device, so work that
// still reads it has finished.
rekv_status reserve(rekv_ctx* c, size_t bytes) {
    if (bytes <= c->ws_bytes) return REKV_OK;
    if (c->ws) {
        hipError_t e = hipFree(c->ws);
        c->ws = nullptr;
        c->ws_bytes = 0;
        if (e != hipSuccess) return fail_hip(c, "hipFree(workspace)", e);
    }
    bytes = (bytes + (size_t(1) << 20) - 1) & ~((size_t(1) << 20) - 1);
    hipError_t e = hipMalloc(&c->ws, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        c->ws = nullptr;
        return fail(c, REKV_ERR_NOMEM, "workspace of %zu bytes: %s", bytes, hipGetErrorString(e));
    }
    c->ws_bytes = bytes;
    return REKV_OK;
}

// fixed_ws != NULL: the launch may use only that buffer of fixed_ws_bytes (no allocation);
// otherwise the context's workspace grows as needed.
rekv_status run_attention(rekv_ctx* c, const rekv::AttnProblem& p, hipStream_t stream, void* fixed_ws = nullptr,
                          size_t fixed_ws_bytes = 0) {
    if (c->shape.dtype == REKV_F32) {
        if (p.n_items > 65535)
            return fail(c, REKV_ERR_UNSUPPORTED, "fp32 attention takes at most 65535 chunks/questions per call");
        hipError_t e = rekv::attn_f32_launch(p, stream);
        return e == hipSuccess ? REKV_OK : fail_hip(c, "fp32 attention launch", e);
    }
    const rekv::AttnPlan plan = rekv::attn_bf16_plan(p);
    const int64_t blocks = (int64_t)p.n_items * p.n_kv_heads * plan.m_tiles * plan.n_splits;
    if (blocks > 0x7FFFFFFF) return fail(c, REKV_ERR_UNSUPPORTED, "attention grid of %lld workgroups", (long long)blocks);
    void* ws = fixed_ws;
    if (fixed_ws) {
        if (plan.workspace_bytes > fixed_ws_bytes)
            return fail(c, REKV_ERR_UNSUPPORTED, "this launch needs %zu bytes of scratch, the static buffer holds %zu",
                        plan.workspace_bytes, fixed_ws_bytes);
    } else {
        rekv_status s = reserve(c, plan.workspace_bytes);
        if (s != REKV_OK) return s;
        ws = c->ws;
    }
    hipError_t e = rekv::attn_bf16_launch(p, plan, ws, stream);
    return e == hipSuccess ? REKV_OK : fail_hip(c, "bf16 attention launch", e);
}

}  // namespace

extern "C" {

rekv_status rekv_create(const rekv_shape* shape, rekv_ctx** out) {
    if (out) *out = nullptr;
    if (!shape || !out) return fail(nullptr, REKV_ERR_INVALID_ARG, "rekv_create: null argument");
    if (shape->n_q_heads <= 0 || shape->n_kv_heads <= 0 || shape->n_q_heads % shape->n_kv_heads != 0)
        return fail(nullptr, REKV_ERR_INVALID_ARG, "n_q_heads=%d must be a positive multiple of n_kv_heads=%d",
                    shape->n_q_heads, shape->n_kv_heads);
    if (shape->tokens_per_frame <= 0)
        return fail(nullptr, REKV_ERR_INVALID_ARG, "tokens_per_frame=%d must be positive", shape->tokens_per_frame);
    if (!(shape->softmax_scale >= 0.f) || shape->softmax_scale > 1e30f)
        return fail(nullptr, REKV_ERR_INVALID_ARG, "softmax_scale must be finite and >= 0 (0 selects 1/sqrt(D))");
    if (shape->dtype == REKV_BF16) {
        if (shape->head_dim != 64 && shape->head_dim != 128)
            return fail(nullptr, REKV_ERR_UNSUPPORTED, "bf16 kernels cover head_dim 64 and 128, not %d", shape->head_dim);
    } else if (shape->dtype == REKV_F32) {
        if (shape->head_dim <= 0 || shape->head_dim > 256 || shape->head_dim % 4 != 0)
            return fail(nullptr, REKV_ERR_UNSUPPORTED, "fp32 kernels cover head_dim a multiple of 4 up to 256, not %d", shape->head_dim);
    } else {
        return fail(nullptr, REKV_ERR_INVALID_ARG, "dtype=%d is neither REKV_F32 nor REKV_BF16", shape->dtype);
    }
    rekv_ctx* c = new (std::nothrow) rekv_ctx;
    if (!c) return fail(nullptr, REKV_ERR_NOMEM, "host allocation of the context failed");
    memset(c, 0, sizeof(*c));
    c->shape = *shape;
    c->scale = shape->softmax_scale > 0.f ? shape->softmax_scale : 1.0f / sqrtf((float)shape->head_dim);
    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) e = scratch_address(c->device, &c->scratch);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_main, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_side, hipEventDisableTiming);
    if (e != hipSuccess) {
        rekv_status s = fail_hip(nullptr, "rekv_create", e);
        rekv_destroy(c);
        return s;
    }
    *out = c;
    return REKV_OK;
}

void rekv_destroy(rekv_ctx* c) {
    if (!c) return;
    if (c->side) {
        (void)hipStreamSynchronize(c->side);
        (void)hipStreamDestroy(c->side);
    }
    if (c->ev_main) (void)hipEventDestroy(c->ev_main);
    if (c->ev_side) (void)hipEventDestroy(c->ev_side);
    if (c->ws) (void)hipFree(c->ws);
    if (c->idx_host) (void)hipHostFree(c->idx_host);
    delete c;
}

const char* rekv_last_error(const rekv_ctx* c) { return c ? c->err : g_create_err; }

rekv_status rekv_encode_chunk(rekv_ctx* c, const void* q, const void* k_cache, const void* v_cache,
                              int64_t first_token, int32_t l_x, int32_t n_chunks, int32_t l_l,
                              void* out, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!q || !k_cache || !v_cache || !out) return fail(c, REKV_ERR_INVALID_ARG, "rekv_encode_chunk: null pointer");
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_encode_chunk: pointers must be 16-byte aligned");
    if (first_token < 0 || l_x <= 0 || n_chunks <= 0 || l_l < 0)
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_encode_chunk: first_token=%lld l_x=%d n_chunks=%d l_l=%d",
                    (long long)first_token, l_x, n_chunks, l_l);
    if ((int64_t)l_x * (c->shape.n_q_heads / c->shape.n_kv_heads) > 0x3FFFFFFF)
        return fail(c, REKV_ERR_UNSUPPORTED, "rekv_encode_chunk: chunk of %d tokens is too long", l_x);
    rekv::AttnProblem p;
    memset(&p, 0, sizeof(p));
    p.q = q; p.out = out;
    p.k_a = k_cache; p.v_a = v_cache; p.k_b = k_cache; p.v_b = v_cache;
    p.first_token = first_token; p.l_l = l_l; p.len_a = 0; p.len_b = l_x; p.len_q = l_x; p.b_stride = 0;
    p.n_items = n_chunks; p.is_encode = 1;
    p.n_q_heads = c->shape.n_q_heads; p.n_kv_heads = c->shape.n_kv_heads; p.head_dim = c->shape.head_dim;
    p.scale = c->scale;
    return run_attention(c, p, static_cast<hipStream_t>(stream));
}

rekv_status rekv_qa_attention(rekv_ctx* c, const void* q, const void* k_ret, const void* v_ret,
                              int32_t n_ret_tokens, const int32_t* n_sel, const void* k_self, const void* v_self,
                              int32_t n_questions, int32_t n_q_tokens, void* out, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!q || !k_self || !v_self || !out || (n_ret_tokens > 0 && (!k_ret || !v_ret)))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_qa_attention: null pointer");
    if (!aligned16(q) || !aligned16(k_ret) || !aligned16(v_ret) || !aligned16(k_self) || !aligned16(v_self) || !aligned16(out))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_qa_attention: pointers must be 16-byte aligned");
    if (n_ret_tokens < 0 || n_questions <= 0 || n_q_tokens <= 0)
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_qa_attention: n_ret_tokens=%d n_questions=%d n_q_tokens=%d",
                    n_ret_tokens, n_questions, n_q_tokens);
    if ((int64_t)n_q_tokens * (c->shape.n_q_heads / c->shape.n_kv_heads) > 0x3FFFFFFF)
        return fail(c, REKV_ERR_UNSUPPORTED, "rekv_qa_attention: question of %d tokens is too long", n_q_tokens);
    rekv::AttnProblem p;
    memset(&p, 0, sizeof(p));
    p.q = q; p.out = out;
    p.k_a = k_ret ? k_ret : k_self; p.v_a = v_ret ? v_ret : v_self; p.k_b = k_self; p.v_b = v_self;
    p.first_token = 0; p.l_l = 0; p.len_a = n_ret_tokens; p.len_b = n_q_tokens; p.len_q = n_q_tokens;
    p.b_stride = n_q_tokens;
    p.a_valid_frames = n_sel; p.n_f = c->shape.tokens_per_frame;
    p.n_items = n_questions; p.is_encode = 0;
    p.n_q_heads = c->shape.n_q_heads; p.n_kv_heads = c->shape.n_kv_heads; p.head_dim = c->shape.head_dim;
    p.scale = c->scale;
    return run_attention(c, p, static_cast<hipStream_t>(stream));
}

// Shared body of rekv_decode_attention and its allocation-free variant.
static rekv_status decode_attention(rekv_ctx* c, const char* fn, bool no_alloc, const void* q, const void* k_ret,
                                    const void* v_ret, int32_t n_ret_tokens, const int32_t* n_sel,
                                    const void* k_text, const void* v_text, int64_t text_stride,
                                    int32_t n_text_tokens, int32_t n_questions, int32_t n_new_tokens, void* out,
                                    void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!q || !k_text || !v_text || !out || (n_ret_tokens > 0 && (!k_ret || !v_ret)))
        return fail(c, REKV_ERR_INVALID_ARG, "%s: null pointer", fn);
    if (!aligned16(q) || !aligned16(k_ret) || !aligned16(v_ret) || !aligned16(k_text) || !aligned16(v_text) || !aligned16(out))
        return fail(c, REKV_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", fn);
    if (n_ret_tokens < 0 || n_questions <= 0 || n_new_tokens <= 0 || n_text_tokens < n_new_tokens ||
        text_stride < n_text_tokens)
        return fail(c, REKV_ERR_INVALID_ARG,
                    "%s: n_ret_tokens=%d n_questions=%d n_new_tokens=%d n_text_tokens=%d text_stride=%lld", fn,
                    n_ret_tokens, n_questions, n_new_tokens, n_text_tokens, (long long)text_stride);
    if ((int64_t)n_new_tokens * (c->shape.n_q_heads / c->shape.n_kv_heads) > 0x3FFFFFFF)
        return fail(c, REKV_ERR_UNSUPPORTED, "%s: %d new tokens are too many", fn, n_new_tokens);
    rekv::AttnProblem p;
    memset(&p, 0, sizeof(p));
    p.q = q; p.out = out;
    p.k_a = k_ret ? k_ret : k_text; p.v_a = v_ret ? v_ret : v_text; p.k_b = k_text; p.v_b = v_text;
    p.first_token = 0; p.l_l = 0; p.len_a = n_ret_tokens; p.len_b = n_text_tokens; p.len_q = n_new_tokens;
    p.b_stride = text_stride;
    p.a_valid_frames = n_sel; p.n_f = c->shape.tokens_per_frame;
    p.n_items = n_questions; p.is_encode = 0;
    p.n_q_heads = c->shape.n_q_heads; p.n_kv_heads = c->shape.n_kv_heads; p.head_dim = c->shape.head_dim;
    p.scale = c->scale;
    if (no_alloc) return run_attention(c, p, static_cast<hipStream_t>(stream), c->scratch, NOALLOC_SCRATCH_BYTES);
    return run_attention(c, p, static_cast<hipStream_t>(stream));
}

rekv_status rekv_decode_attention(rekv_ctx* c, const void* q, const void* k_ret, const void* v_ret,
                                  int32_t n_ret_tokens, const int32_t* n_sel, const void* k_text,
                                  const void* v_text, int64_t text_stride, int32_t n_text_tokens,
                                  int32_t n_questions, int32_t n_new_tokens, void* out, void* stream) {
    return decode_attention(c, "rekv_decode_attention", false, q, k_ret, v_ret, n_ret_tokens, n_sel, k_text, v_text,
                            text_stride, n_text_tokens, n_questions, n_new_tokens, out, stream);
}

rekv_status rekv_decode_attention_noalloc(rekv_ctx* c, const void* q, const void* k_ret, const void* v_ret,
                                          int32_t n_ret_tokens, const int32_t* n_sel, const void* k_text,
                                          const void* v_text, int64_t text_stride, int32_t n_text_tokens,
                                          int32_t n_questions, int32_t n_new_tokens, void* out, void* stream) {
    return decode_attention(c, "rekv_decode_attention_noalloc", true, q, k_ret, v_ret, n_ret_tokens, n_sel, k_text,
                            v_text, text_stride, n_text_tokens, n_questions, n_new_tokens, out, stream);
}

rekv_status rekv_attention_indexed(rekv_ctx* c, const void* q, const void* k_src, const void* v_src,
                                   int32_t n_src_frames, const int32_t* idx, int64_t idx_stride,
                                   int32_t n_ret_frames, const int32_t* n_sel, const void* k_text, const void* v_text,
                                   int64_t text_stride, int32_t n_text_tokens, int32_t n_questions,
                                   int32_t n_new_tokens, void* out, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!q || !k_src || !v_src || !idx || !k_text || !v_text || !out)
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_attention_indexed: null pointer");
    if (!aligned16(q) || !aligned16(k_src) || !aligned16(v_src) || !aligned16(k_text) || !aligned16(v_text) || !aligned16(out))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_attention_indexed: pointers must be 16-byte aligned");
    if (n_src_frames <= 0 || n_ret_frames <= 0 || idx_stride < n_ret_frames || n_questions <= 0 ||
        n_new_tokens <= 0 || n_text_tokens < n_new_tokens || text_stride < n_text_tokens)
        return fail(c, REKV_ERR_INVALID_ARG,
                    "rekv_attention_indexed: n_src_frames=%d n_ret_frames=%d idx_stride=%lld n_questions=%d n_new_tokens=%d "
                    "n_text_tokens=%d text_stride=%lld", n_src_frames, n_ret_frames, (long long)idx_stride, n_questions,
                    n_new_tokens, n_text_tokens, (long long)text_stride);
    const int64_t n_f = c->shape.tokens_per_frame;
    const int64_t row_bytes = (int64_t)c->shape.n_kv_heads * c->shape.head_dim * (int64_t)elem_size(c);
    if (n_ret_frames > 1024 || n_ret_frames * n_f >= (1 << 23))
        return fail(c, REKV_ERR_UNSUPPORTED, "rekv_attention_indexed: at most 1024 frames and 2^23 - 1 tokens per question (got %d frames)",
                    n_ret_frames);
    if ((int64_t)n_src_frames * n_f * row_bytes > 0xFFF00000LL)
        return fail(c, REKV_ERR_UNSUPPORTED, "rekv_attention_indexed: the K (and V) arena must stay below 4 GiB (%d frames of %lld bytes)",
                    n_src_frames, (long long)(n_f * row_bytes));
    if ((int64_t)n_new_tokens * (c->shape.n_q_heads / c->shape.n_kv_heads) > 0x3FFFFFFF)
        return fail(c, REKV_ERR_UNSUPPORTED, "rekv_attention_indexed: %d new tokens are too many", n_new_tokens);
    rekv::AttnProblem p;
    memset(&p, 0, sizeof(p));
    p.q = q; p.out = out;
    p.k_a = k_src; p.v_a = v_src; p.k_b = k_text; p.v_b = v_text;
    p.len_a = (int32_t)(n_ret_frames * n_f); p.len_b = n_text_tokens; p.len_q = n_new_tokens;
    p.b_stride = text_stride;
    p.n_items = n_questions; p.is_encode = 0;
    p.n_q_heads = c->shape.n_q_heads; p.n_kv_heads = c->shape.n_kv_heads; p.head_dim = c->shape.head_dim;
    p.scale = c->scale;
    p.a_index = idx; p.a_index_stride = idx_stride; p.n_f = (int32_t)n_f; p.n_src_frames = n_src_frames;
    p.a_valid_frames = n_sel;
    return run_attention(c, p, static_cast<hipStream_t>(stream));
}

rekv_status rekv_frame_keys(rekv_ctx* c, const void* k, int32_t n_frames, float* frame_keys, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!k || !frame_keys) return fail(c, REKV_ERR_INVALID_ARG, "rekv_frame_keys: null pointer");
    if (!aligned16(k)) return fail(c, REKV_ERR_INVALID_ARG, "rekv_frame_keys: k must be 16-byte aligned");
    if (n_frames <= 0) return fail(c, REKV_ERR_INVALID_ARG, "rekv_frame_keys: n_frames=%d", n_frames);
    hipError_t e = rekv::frame_keys_launch(k, n_frames, c->shape.tokens_per_frame,
                                           c->shape.n_kv_heads * c->shape.head_dim, c->shape.dtype,
                                           frame_keys, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? REKV_OK : fail_hip(c, "frame_keys launch", e);
}

rekv_status rekv_retrieve_topk(rekv_ctx* c, const float* frame_keys, int64_t frame_keys_stride,
                               int32_t n_frames, const void* q_question, int32_t n_questions,
                               int32_t n_q_tokens, int32_t k, int32_t* idx, int32_t* n_sel,
                               float* scores, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!frame_keys || !q_question || !idx) return fail(c, REKV_ERR_INVALID_ARG, "rekv_retrieve_topk: null pointer");
    if (!aligned16(frame_keys) || !aligned16(q_question) || frame_keys_stride < 0 || frame_keys_stride % 4 != 0)
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_retrieve_topk: frame_keys and q_question must be 16-byte aligned, the stride a non-negative multiple of 4");
    if (n_frames <= 0 || n_questions <= 0 || n_q_tokens <= 0 || k <= 0 || k > 4096)
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_retrieve_topk: n_frames=%d n_questions=%d n_q_tokens=%d k=%d (1..4096)",
                    n_frames, n_questions, n_q_tokens, k);
    const int d_prime = c->shape.n_kv_heads * c->shape.head_dim;
    if ((c->shape.n_q_heads / c->shape.n_kv_heads) * c->shape.head_dim > 4096)
        return fail(c, REKV_ERR_UNSUPPORTED, "rekv_retrieve_topk: (Hq/Hkv)*D=%d exceeds 4096",
                    (c->shape.n_q_heads / c->shape.n_kv_heads) * c->shape.head_dim);
    if (n_questions > 65535) return fail(c, REKV_ERR_UNSUPPORTED, "rekv_retrieve_topk: at most 65535 questions per call");
    const size_t qv_bytes = ((size_t)n_questions * d_prime * sizeof(float) + 255) & ~size_t(255);
    const size_t sc_bytes = scores ? 0 : (size_t)n_questions * n_frames * sizeof(float);
    rekv_status s = reserve(c, qv_bytes + sc_bytes);
    if (s != REKV_OK) return s;
    rekv::RetrieveArgs a;
    a.frame_keys = frame_keys; a.frame_keys_stride = frame_keys_stride; a.n_frames = n_frames;
    a.q_question = q_question; a.n_questions = n_questions; a.n_q_tokens = n_q_tokens; a.k = k;
    a.n_q_heads = c->shape.n_q_heads; a.n_kv_heads = c->shape.n_kv_heads; a.head_dim = c->shape.head_dim;
    a.dtype = c->shape.dtype;
    a.idx = idx; a.n_sel = n_sel;
    a.q_vec = static_cast<float*>(c->ws);
    a.scores = scores ? scores : reinterpret_cast<float*>(static_cast<char*>(c->ws) + qv_bytes);
    a.q_vec_given = nullptr; a.dim = 0; a.inv_tau = 1.f;
    hipError_t e = rekv::retrieve_launch(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? REKV_OK : fail_hip(c, "retrieval launch", e);
}

rekv_status rekv_retrieve_external(rekv_ctx* c, const float* frame_emb, int32_t n_frames, int32_t dim,
                                   const float* q_emb, int32_t n_questions, float tau, int32_t k,
                                   int32_t* idx, int32_t* n_sel, float* scores, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!frame_emb || !q_emb || !idx) return fail(c, REKV_ERR_INVALID_ARG, "rekv_retrieve_external: null pointer");
    if (!aligned16(frame_emb) || !aligned16(q_emb))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_retrieve_external: embeddings must be 16-byte aligned");
    if (n_frames <= 0 || n_questions <= 0 || k <= 0 || k > 4096 || dim <= 0 || dim % 4 != 0 || !(tau > 0.f))
        return fail(c, REKV_ERR_INVALID_ARG,
                    "rekv_retrieve_external: n_frames=%d n_questions=%d k=%d (1..4096) dim=%d (multiple of 4) tau=%g (> 0)",
                    n_frames, n_questions, k, dim, (double)tau);
    if (n_questions > 65535) return fail(c, REKV_ERR_UNSUPPORTED, "rekv_retrieve_external: at most 65535 questions per call");
    if (!scores) {
        rekv_status s = reserve(c, (size_t)n_questions * n_frames * sizeof(float));
        if (s != REKV_OK) return s;
    }
    rekv::RetrieveArgs a;
    memset(&a, 0, sizeof(a));
    a.frame_keys = frame_emb; a.frame_keys_stride = 0; a.n_frames = n_frames;
    a.n_questions = n_questions; a.k = k;
    a.idx = idx; a.n_sel = n_sel;
    a.scores = scores ? scores : static_cast<float*>(c->ws);
    a.q_vec_given = q_emb; a.dim = dim; a.inv_tau = 1.f / tau;
    hipError_t e = rekv::retrieve_launch(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? REKV_OK : fail_hip(c, "external retrieval launch", e);
}

rekv_status rekv_block_keys(rekv_ctx* c, const float* frame_keys, int32_t n_frames, int32_t b,
                            float* block_keys, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!frame_keys || !block_keys) return fail(c, REKV_ERR_INVALID_ARG, "rekv_block_keys: null pointer");
    if (!aligned16(frame_keys)) return fail(c, REKV_ERR_INVALID_ARG, "rekv_block_keys: frame_keys must be 16-byte aligned");
    if (n_frames <= 0 || b <= 0) return fail(c, REKV_ERR_INVALID_ARG, "rekv_block_keys: n_frames=%d b=%d", n_frames, b);
    const int d_prime = c->shape.n_kv_heads * c->shape.head_dim;
    hipError_t e = rekv::block_keys_launch(frame_keys, n_frames, b, d_prime, block_keys, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? REKV_OK : fail_hip(c, "block_keys launch", e);
}

rekv_status rekv_expand_blocks(rekv_ctx* c, const int32_t* block_idx, int32_t n_questions, int32_t k_blocks,
                               int32_t b, int32_t n_frames, int32_t* frame_idx, int32_t* n_sel, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!block_idx || !frame_idx) return fail(c, REKV_ERR_INVALID_ARG, "rekv_expand_blocks: null pointer");
    if (n_questions <= 0 || k_blocks <= 0 || b <= 0 || n_frames <= 0 || (int64_t)k_blocks * b > (1 << 20))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_expand_blocks: n_questions=%d k_blocks=%d b=%d n_frames=%d (k_blocks*b <= 2^20)",
                    n_questions, k_blocks, b, n_frames);
    hipError_t e = rekv::expand_blocks_launch(block_idx, n_questions, k_blocks, b, n_frames, frame_idx, n_sel,
                                              static_cast<hipStream_t>(stream));
    return e == hipSuccess ? REKV_OK : fail_hip(c, "expand_blocks launch", e);
}

rekv_status rekv_gather_kv(rekv_ctx* c, const void* src_k, const void* src_v, int32_t src_on_host,
                           int32_t n_src_frames, const int32_t* idx, int32_t n_questions, int32_t k,
                           void* dst_k, void* dst_v, void* stream_) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!src_k || !src_v || !idx || !dst_k || !dst_v) return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv: null pointer");
    if (!aligned16(src_k) || !aligned16(src_v) || !aligned16(dst_k) || !aligned16(dst_v))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv: pointers must be 16-byte aligned");
    if (n_src_frames <= 0 || n_questions <= 0 || k <= 0 || src_on_host < 0 || src_on_host > 2)
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv: n_src_frames=%d n_questions=%d k=%d src_on_host=%d",
                    n_src_frames, n_questions, k, src_on_host);
    const int64_t n_blocks = (int64_t)n_questions * k;
    if (n_blocks > 0x7FFFFFFF) return fail(c, REKV_ERR_UNSUPPORTED, "rekv_gather_kv: %lld blocks", (long long)n_blocks);
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const size_t frame_bytes = (size_t)c->shape.tokens_per_frame * c->shape.n_kv_heads * c->shape.head_dim * elem_size(c);
    if (frame_bytes % 16 != 0) return fail(c, REKV_ERR_UNSUPPORTED, "rekv_gather_kv: frame of %zu bytes is not a multiple of 16", frame_bytes);

    if (!src_on_host) {
        hipError_t e = rekv::gather_launch(src_k, src_v, n_src_frames, idx, (int)n_blocks, frame_bytes,
                                           dst_k, dst_v, stream);
        return e == hipSuccess ? REKV_OK : fail_hip(c, "gather launch", e);
    }

    if (src_on_host == 2) {
        // Zero-copy host path: the gather kernel reads the pinned host arrays over the host link.
        // It runs on the side stream after everything queued on `stream` (the index list is
        // produced there); `stream` then waits for it.  No host synchronisation.
        void *dk = nullptr, *dv = nullptr;
        hipError_t e = hipHostGetDevicePointer(&dk, const_cast<void*>(src_k), 0);
        if (e == hipSuccess) e = hipHostGetDevicePointer(&dv, const_cast<void*>(src_v), 0);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv: src is not pinned host memory (%s)", hipGetErrorString(e));
        }
        e = hipEventRecord(c->ev_main, stream);
        if (e == hipSuccess) e = hipStreamWaitEvent(c->side, c->ev_main, 0);
        if (e == hipSuccess)
            e = rekv::gather_launch(dk, dv, n_src_frames, idx, (int)n_blocks, frame_bytes, dst_k, dst_v, c->side);
        if (e == hipSuccess) e = hipEventRecord(c->ev_side, c->side);
        if (e == hipSuccess) e = hipStreamWaitEvent(stream, c->ev_side, 0);
        return e == hipSuccess ? REKV_OK : fail_hip(c, "rekv_gather_kv: zero-copy gather", e);
    }

    // Host path: bring the index list to the host, then one async copy per frame and tensor
    // on the side stream, ordered after `stream` (the destination may still be in use there)
    // and joined back into it.
    if ((size_t)n_blocks > c->idx_host_cap) {
        if (c->idx_host) (void)hipHostFree(c->idx_host);
        c->idx_host = nullptr;
        c->idx_host_cap = 0;
        hipError_t e = hipHostMalloc(reinterpret_cast<void**>(&c->idx_host), (size_t)n_blocks * sizeof(int32_t), hipHostMallocDefault);
        if (e != hipSuccess) { (void)hipGetLastError(); return fail(c, REKV_ERR_NOMEM, "pinned index staging: %s", hipGetErrorString(e)); }
        c->idx_host_cap = (size_t)n_blocks;
    }
    hipError_t e = hipMemcpyAsync(c->idx_host, idx, (size_t)n_blocks * sizeof(int32_t), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipEventRecord(c->ev_main, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail_hip(c, "rekv_gather_kv: index copy", e);
    for (int64_t b = 0; b < n_blocks; ++b)
        if (c->idx_host[b] >= n_src_frames)
            return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv: idx[%lld]=%d is not below n_src_frames=%d",
                        (long long)b, c->idx_host[b], n_src_frames);
    e = hipStreamWaitEvent(c->side, c->ev_main, 0);
    for (int64_t b = 0; b < n_blocks && e == hipSuccess; ++b) {
        const int32_t f = c->idx_host[b];
        char* dk = static_cast<char*>(dst_k) + (size_t)b * frame_bytes;
        char* dv = static_cast<char*>(dst_v) + (size_t)b * frame_bytes;
        if (f < 0) {
            e = hipMemsetAsync(dk, 0, frame_bytes, c->side);
            if (e == hipSuccess) e = hipMemsetAsync(dv, 0, frame_bytes, c->side);
            continue;
        }
        // runs of consecutive frames in consecutive slots move as one copy
        int64_t run = 1;
        while (b + run < n_blocks && c->idx_host[b + run] == f + run) ++run;
        e = hipMemcpyAsync(dk, static_cast<const char*>(src_k) + (size_t)f * frame_bytes, run * frame_bytes, hipMemcpyHostToDevice, c->side);
        if (e == hipSuccess)
            e = hipMemcpyAsync(dv, static_cast<const char*>(src_v) + (size_t)f * frame_bytes, run * frame_bytes, hipMemcpyHostToDevice, c->side);
        b += run - 1;
    }
    if (e == hipSuccess) e = hipEventRecord(c->ev_side, c->side);
    if (e == hipSuccess) e = hipStreamWaitEvent(stream, c->ev_side, 0);
    return e == hipSuccess ? REKV_OK : fail_hip(c, "rekv_gather_kv: host copies", e);
}

rekv_status rekv_gather_kv_layers(rekv_ctx* c, const void* const* src_k, const void* const* src_v, int32_t n_layers,
                                  int32_t n_src_frames, const int32_t* idx, int32_t n_questions, int32_t k,
                                  void* dst_k, void* dst_v, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!src_k || !src_v || !idx || !dst_k || !dst_v) return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv_layers: null pointer");
    if (n_layers <= 0 || n_layers > rekv::MAX_GATHER_LAYERS)
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv_layers: n_layers=%d (1..%d)", n_layers, rekv::MAX_GATHER_LAYERS);
    if (!aligned16(dst_k) || !aligned16(dst_v))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv_layers: pointers must be 16-byte aligned");
    for (int i = 0; i < n_layers; ++i)
        if (!src_k[i] || !src_v[i] || !aligned16(src_k[i]) || !aligned16(src_v[i]))
            return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv_layers: arena %d is null or not 16-byte aligned", i);
    if (n_src_frames <= 0 || n_questions <= 0 || k <= 0)
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv_layers: n_src_frames=%d n_questions=%d k=%d", n_src_frames, n_questions, k);
    const int64_t per_layer = (int64_t)n_questions * k;
    if (per_layer * n_layers > 0x7FFFFFFF) return fail(c, REKV_ERR_UNSUPPORTED, "rekv_gather_kv_layers: %lld blocks", (long long)(per_layer * n_layers));
    const size_t frame_bytes = (size_t)c->shape.tokens_per_frame * c->shape.n_kv_heads * c->shape.head_dim * elem_size(c);
    if (frame_bytes % 16 != 0) return fail(c, REKV_ERR_UNSUPPORTED, "rekv_gather_kv_layers: frame of %zu bytes is not a multiple of 16", frame_bytes);
    hipError_t e = rekv::gather_layers_launch(src_k, src_v, n_layers, n_src_frames, idx, (int)per_layer, frame_bytes, dst_k,
                                              dst_v, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? REKV_OK : fail_hip(c, "gather_layers launch", e);
}

// Argument checks and RopeArgs shared by the calls that re-position keys.
static rekv_status rope_args(rekv_ctx* c, const char* fn, double rope_base, int32_t rope_layout, int32_t pos_mode,
                             int64_t pos_offset, int32_t src_rotated, int64_t src_pos_offset, rekv::RopeArgs* ra) {
    if (!(rope_base > 1.0) || !(rope_base < 1e30) || (rope_layout != 0 && rope_layout != 1) ||
        (pos_mode != 0 && pos_mode != 1) || (src_rotated != 0 && src_rotated != 1))
        return fail(c, REKV_ERR_INVALID_ARG, "%s: rope_base=%g (> 1) rope_layout=%d pos_mode=%d src_rotated=%d (each 0 or 1)", fn,
                    rope_base, rope_layout, pos_mode, src_rotated);
    const int d = c->shape.head_dim, epc = c->shape.dtype == REKV_BF16 ? 8 : 4;
    if (d > 256 || d % (2 * epc) != 0)
        return fail(c, REKV_ERR_UNSUPPORTED, "%s: head_dim=%d must be a multiple of %d, at most 256", fn, d, 2 * epc);
    const int64_t span = (int64_t)1 << 40;     // positions far below 2^53 keep the double-precision angle exact
    if (pos_offset < -span || pos_offset > span || src_pos_offset < -span || src_pos_offset > span)
        return fail(c, REKV_ERR_INVALID_ARG, "%s: position offsets must lie within +-2^40", fn);
    ra->log2_base = log2(rope_base);
    ra->pos_offset = pos_offset; ra->src_pos_offset = src_pos_offset;
    ra->is_static = pos_mode; ra->src_rotated = src_rotated; ra->interleaved = rope_layout;
    return REKV_OK;
}

rekv_status rekv_gather_kv_rope(rekv_ctx* c, const void* src_k, const void* src_v, int32_t src_on_host,
                                int32_t n_src_frames, const int32_t* idx, int32_t n_questions, int32_t k,
                                void* dst_k, void* dst_v, double rope_base, int32_t rope_layout, int32_t pos_mode,
                                int64_t pos_offset, int32_t src_rotated, int64_t src_pos_offset, void* stream_) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!src_k || !src_v || !idx || !dst_k || !dst_v) return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv_rope: null pointer");
    if (!aligned16(src_k) || !aligned16(src_v) || !aligned16(dst_k) || !aligned16(dst_v))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv_rope: pointers must be 16-byte aligned");
    if (n_src_frames <= 0 || n_questions <= 0 || k <= 0 || (int64_t)n_questions * k > 0x7FFFFFFF ||
        (src_on_host != 0 && src_on_host != 1))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv_rope: n_src_frames=%d n_questions=%d k=%d src_on_host=%d (0 or 1)",
                    n_src_frames, n_questions, k, src_on_host);
    rekv::RopeArgs ra;
    rekv_status st = rope_args(c, "rekv_gather_kv_rope", rope_base, rope_layout, pos_mode, pos_offset, src_rotated,
                               src_pos_offset, &ra);
    if (st != REKV_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (!src_on_host) {
        hipError_t e = rekv::gather_rope_launch(src_k, src_v, n_src_frames, idx, n_questions, k, c->shape.tokens_per_frame,
                                                c->shape.n_kv_heads, c->shape.head_dim, c->shape.dtype, dst_k, dst_v, ra, stream);
        return e == hipSuccess ? REKV_OK : fail_hip(c, "gather_kv_rope launch", e);
    }
    // Pinned host source: the kernels read the host arrays over the host link, on the side stream,
    // ordered after `stream` (which produced idx) and joined back into it.
    void *dk = nullptr, *dv = nullptr;
    hipError_t e = hipHostGetDevicePointer(&dk, const_cast<void*>(src_k), 0);
    if (e == hipSuccess) e = hipHostGetDevicePointer(&dv, const_cast<void*>(src_v), 0);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_gather_kv_rope: src is not pinned host memory (%s)", hipGetErrorString(e));
    }
    e = hipEventRecord(c->ev_main, stream);
    if (e == hipSuccess) e = hipStreamWaitEvent(c->side, c->ev_main, 0);
    if (e == hipSuccess)
        e = rekv::gather_rope_launch(dk, dv, n_src_frames, idx, n_questions, k, c->shape.tokens_per_frame, c->shape.n_kv_heads,
                                     c->shape.head_dim, c->shape.dtype, dst_k, dst_v, ra, c->side);
    if (e == hipSuccess) e = hipEventRecord(c->ev_side, c->side);
    if (e == hipSuccess) e = hipStreamWaitEvent(stream, c->ev_side, 0);
    return e == hipSuccess ? REKV_OK : fail_hip(c, "rekv_gather_kv_rope: host-source gather", e);
}

rekv_status rekv_attention_indexed_rope(rekv_ctx* c, const void* q, const void* k_src, const void* v_src,
                                        int32_t n_src_frames, const int32_t* idx, int64_t idx_stride,
                                        int32_t n_ret_frames, const int32_t* n_sel, void* k_pos, double rope_base,
                                        int32_t rope_layout, int32_t pos_mode, int64_t pos_offset, int32_t src_rotated,
                                        int64_t src_pos_offset, const void* k_text, const void* v_text,
                                        int64_t text_stride, int32_t n_text_tokens, int32_t n_questions,
                                        int32_t n_new_tokens, void* out, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!q || !k_src || !v_src || !idx || !k_pos || !k_text || !v_text || !out)
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_attention_indexed_rope: null pointer");
    if (!aligned16(q) || !aligned16(k_src) || !aligned16(v_src) || !aligned16(k_pos) || !aligned16(k_text) ||
        !aligned16(v_text) || !aligned16(out))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_attention_indexed_rope: pointers must be 16-byte aligned");
    if (n_src_frames <= 0 || n_ret_frames <= 0 || idx_stride != n_ret_frames || n_questions <= 0 ||
        n_new_tokens <= 0 || n_text_tokens < n_new_tokens || text_stride < n_text_tokens)
        return fail(c, REKV_ERR_INVALID_ARG,
                    "rekv_attention_indexed_rope: n_src_frames=%d n_ret_frames=%d idx_stride=%lld (must equal n_ret_frames) "
                    "n_questions=%d n_new_tokens=%d n_text_tokens=%d text_stride=%lld", n_src_frames, n_ret_frames,
                    (long long)idx_stride, n_questions, n_new_tokens, n_text_tokens, (long long)text_stride);
    const int64_t n_f = c->shape.tokens_per_frame;
    const int64_t row_bytes = (int64_t)c->shape.n_kv_heads * c->shape.head_dim * (int64_t)elem_size(c);
    if (n_ret_frames > 1024 || n_ret_frames * n_f >= (1 << 23))
        return fail(c, REKV_ERR_UNSUPPORTED, "rekv_attention_indexed_rope: at most 1024 frames and 2^23 - 1 tokens per question (got %d frames)",
                    n_ret_frames);
    if ((int64_t)n_src_frames * n_f * row_bytes > 0xFFF00000LL)
        return fail(c, REKV_ERR_UNSUPPORTED, "rekv_attention_indexed_rope: the V arena must stay below 4 GiB (%d frames of %lld bytes)",
                    n_src_frames, (long long)(n_f * row_bytes));
    if ((int64_t)n_questions * n_ret_frames > 0x7FFFFFFF ||
        (int64_t)n_new_tokens * (c->shape.n_q_heads / c->shape.n_kv_heads) > 0x3FFFFFFF)
        return fail(c, REKV_ERR_UNSUPPORTED, "rekv_attention_indexed_rope: too many frames or new tokens");
    rekv::RopeArgs ra;
    rekv_status st = rope_args(c, "rekv_attention_indexed_rope", rope_base, rope_layout, pos_mode, pos_offset, src_rotated,
                               src_pos_offset, &ra);
    if (st != REKV_OK) return st;
    // pre-pass over the index list: the selected frames' keys, turned to their new positions, into k_pos
    hipError_t e = rekv::gather_rope_launch(k_src, v_src, n_src_frames, idx, n_questions, n_ret_frames, (int)n_f,
                                            c->shape.n_kv_heads, c->shape.head_dim, c->shape.dtype, k_pos, nullptr, ra,
                                            static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(c, "rekv_attention_indexed_rope: key pre-pass", e);
    rekv::AttnProblem p;
    memset(&p, 0, sizeof(p));
    p.q = q; p.out = out;
    p.k_a = k_pos; p.v_a = v_src; p.k_b = k_text; p.v_b = v_text;
    p.len_a = (int32_t)(n_ret_frames * n_f); p.len_b = n_text_tokens; p.len_q = n_new_tokens;
    p.b_stride = text_stride;
    p.n_items = n_questions; p.is_encode = 0;
    p.n_q_heads = c->shape.n_q_heads; p.n_kv_heads = c->shape.n_kv_heads; p.head_dim = c->shape.head_dim;
    p.scale = c->scale;
    p.a_index = idx; p.a_index_stride = idx_stride; p.n_f = (int32_t)n_f; p.n_src_frames = n_src_frames;
    p.a_valid_frames = n_sel; p.a_k_dense = 1;
    return run_attention(c, p, static_cast<hipStream_t>(stream));
}

rekv_status rekv_offload_kv(rekv_ctx* c, const void* dev_k, const void* dev_v, void* host_k, void* host_v,
                            int64_t first_frame, int32_t n_frames, void* stream_) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!dev_k || !dev_v || !host_k || !host_v) return fail(c, REKV_ERR_INVALID_ARG, "rekv_offload_kv: null pointer");
    if (first_frame < 0 || n_frames <= 0)
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_offload_kv: first_frame=%lld n_frames=%d", (long long)first_frame, n_frames);
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const size_t frame_bytes = (size_t)c->shape.tokens_per_frame * c->shape.n_kv_heads * c->shape.head_dim * elem_size(c);
    const size_t off = (size_t)first_frame * frame_bytes, bytes = (size_t)n_frames * frame_bytes;
    hipError_t e = hipEventRecord(c->ev_main, stream);
    if (e == hipSuccess) e = hipStreamWaitEvent(c->side, c->ev_main, 0);
    if (e == hipSuccess)
        e = hipMemcpyAsync(static_cast<char*>(host_k) + off, static_cast<const char*>(dev_k) + off, bytes, hipMemcpyDeviceToHost, c->side);
    if (e == hipSuccess)
        e = hipMemcpyAsync(static_cast<char*>(host_v) + off, static_cast<const char*>(dev_v) + off, bytes, hipMemcpyDeviceToHost, c->side);
    return e == hipSuccess ? REKV_OK : fail_hip(c, "rekv_offload_kv", e);
}

rekv_status rekv_offload_wait(rekv_ctx* c) {
    if (!c) return REKV_ERR_INVALID_ARG;
    hipError_t e = hipStreamSynchronize(c->side);
    return e == hipSuccess ? REKV_OK : fail_hip(c, "rekv_offload_wait", e);
}

rekv_status rekv_offload_join(rekv_ctx* c, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    hipError_t e = hipEventRecord(c->ev_side, c->side);
    if (e == hipSuccess) e = hipStreamWaitEvent(static_cast<hipStream_t>(stream), c->ev_side, 0);
    return e == hipSuccess ? REKV_OK : fail_hip(c, "rekv_offload_join", e);
}

rekv_status rekv_probe_copy(rekv_ctx* c, void* dst, const void* src, int64_t n_bytes, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!dst || !src) return fail(c, REKV_ERR_INVALID_ARG, "rekv_probe_copy: null pointer");
    if (n_bytes <= 0 || n_bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) % 16 != 0)
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_probe_copy: n_bytes=%lld and both pointers must be multiples of 16",
                    (long long)n_bytes);
    hipError_t e = rekv::launch_probe_copy(dst, src, n_bytes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? REKV_OK : fail_hip(c, "rekv_probe_copy", e);
}

rekv_status rekv_probe_mfma(rekv_ctx* c, float* sink, int32_t n_workgroups, int32_t n_iters, double* flop, void* stream) {
    if (!c) return REKV_ERR_INVALID_ARG;
    if (!sink) return fail(c, REKV_ERR_INVALID_ARG, "rekv_probe_mfma: null pointer");
    if (n_workgroups <= 0 || n_workgroups > (1 << 20) || n_iters <= 0 || n_iters > (1 << 24))
        return fail(c, REKV_ERR_INVALID_ARG, "rekv_probe_mfma: n_workgroups=%d n_iters=%d", n_workgroups, n_iters);
    if (flop) *flop = rekv::probe_mfma_flop(n_workgroups, n_iters);
    hipError_t e = rekv::launch_probe_mfma(sink, n_workgroups, n_iters, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? REKV_OK : fail_hip(c, "rekv_probe_mfma", e);
}

}  // extern "C"
