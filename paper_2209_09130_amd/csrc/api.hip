// C ABI of libsamp: argument checking, weight packing at create time, workspace carving and the
// per-layer kernel sequence of Section 3.2 (seven kernels per layer plus entry / exit handling).
#include "../../include/samp.h"
#include "samp_common.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

using namespace samp;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                               \
    do {                                                                                            \
        hipError_t e_ = (expr);                                                                     \
        if (e_ != hipSuccess) return fail(SAMP_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));    \
    } while (0)

constexpr size_t ALIGN = 256;
size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
bool good_scale(float s) { return std::isfinite(s) && s > 0.0f; }
// An int8 score is at most 64 * 127 * 127 in magnitude, so with the multiplier bounded like this the argument of
// the softmax exponential stays above -2^30, the range its integer exponent arithmetic is good for.
constexpr float MAX_SCORE_MULTIPLIER = 256.0f;
bool good_score_multiplier(float m) { return m > 0.0f && m <= MAX_SCORE_MULTIPLIER; }

struct Layer {
    int mode;
    samp_layer_scales_t s;
    // INT8 blocks: int8 weights and folded epilogue tables; FP16 blocks: fp16 weights
    void *w_qkv, *w_o, *w_f1, *w_f2;
    float *m_qkv, *bq_qkv, *m_o, *m_f1, *m_f2;
    float *b_qkv, *b_o, *b_f1, *b_f2, *g1, *be1, *g2, *be2;
    float m_sc, inv_sp, m_ctx;                      // attention multipliers of an INT8 MHA block
    GeluTable gelu;                                 // FFN1 epilogue's threshold table (entries == nullptr: none for this step)
};

struct Carver {                                     // hands out aligned pieces of a device buffer
    char *base; size_t off;
    template <class T> T *take(size_t count) { T *p = reinterpret_cast<T *>(base + off); off += up(count * sizeof(T)); return p; }
};

size_t staging_bytes(const samp_config_t &c)
{
    const size_t big = (size_t)std::max(3 * c.hidden, c.ffn) * c.hidden;    // largest matrix, elements
    return up(big * 2) + up((size_t)std::max(3 * c.hidden, c.ffn) * sizeof(float));
}

// bit 0: MHA INT8, bit 1: FFN INT8; only with bit 0, and not both: bit 2 unsigned softmax codes, bit 3 binary16 softmax output
bool valid_mode(int m)
{
    if (m < 0 || m > 15) return false;
    const int p = m & (SAMP_P_UNSIGNED | SAMP_P_FP16);
    return !p || ((m & SAMP_MHA_INT8) && p != (SAMP_P_UNSIGNED | SAMP_P_FP16));
}

int check_config(const samp_config_t *c)
{
    if (!c) return fail(SAMP_ERR_ARG, "config is NULL");
    if (c->layers < 1 || c->heads < 1 || c->max_batch < 1) return fail(SAMP_ERR_SHAPE, "layers, heads, max_batch must be >= 1");
    if (c->max_batch > SAMP_MAX_BATCH) return fail(SAMP_ERR_SHAPE, "max_batch must not exceed %d sequences", SAMP_MAX_BATCH);
    if (c->hidden != c->heads * 64) return fail(SAMP_ERR_SHAPE, "head size hidden/heads must be 64 (hidden=%d heads=%d)", c->hidden, c->heads);
    if (c->hidden % 128 || c->hidden > 2048) return fail(SAMP_ERR_SHAPE, "hidden must be a multiple of 128, at most 2048");
    if (c->ffn < 128 || c->ffn % 128) return fail(SAMP_ERR_SHAPE, "ffn must be a positive multiple of 128");
    if (c->max_seq < 1 || c->max_seq > SAMP_MAX_SEQ) return fail(SAMP_ERR_SHAPE, "max_seq must be in [1, %d]", SAMP_MAX_SEQ);
    if ((long long)c->max_batch * c->max_seq > SAMP_MAX_TOKENS)
        return fail(SAMP_ERR_SHAPE, "max_batch * max_seq must not exceed %d tokens", SAMP_MAX_TOKENS);
    if (!(c->ln_eps >= 0.0f) || !std::isfinite(c->ln_eps)) return fail(SAMP_ERR_ARG, "ln_eps must be finite and >= 0");
    return SAMP_OK;
}

size_t layer_arena_bytes(const samp_config_t &c, int mode)
{
    const size_t H = c.hidden, F = c.ffn;
    size_t n = 0;
    const size_t e_mha = (mode & 1) ? 1 : 2, e_ffn = (mode & 2) ? 1 : 2;
    n += up(3 * H * H * e_mha) + up(H * H * e_mha) + up(F * H * e_ffn) + up(H * F * e_ffn);
    n += 2 * up(3 * H * 4) + up(H * 4) + up(F * 4) + up(H * 4);             // m_qkv, bq_qkv, m_o, m_f1, m_f2
    n += up(3 * H * 4) + up(F * 4) + 6 * up(H * 4);                         // biases and LayerNorm vectors
    if (mode & 2) n += up((size_t)GELU_TABLE_MAX_BINS * 8);                 // FFN1 epilogue's threshold table
    return n;
}

constexpr int MAX_EVENTS = 4096;

}  // namespace

// Workspace of samp_encoder_forward_noalloc: one array per GPU, living in the library's own device image for as
// long as the process runs.  In host code the array's name is only a handle for hipGetSymbolAddress: the address
// kernels can use is looked up once per device (noalloc_scratch) and used everywhere after that.
static __device__ __align__(256) unsigned char scratch[SAMP_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];

// Device address of `scratch` on the current device (looked up on the first call per device; concurrent first
// calls look it up twice and store the same value).
int noalloc_scratch(void **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(SAMP_ERR_ARG, "device index %d is outside [0, %d)", dev, MAX_DEVICES);
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || !aligned(p, ALIGN)) return fail(SAMP_ERR_HIP, "the scratch array has no usable device address");
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return SAMP_OK;
}

}  // namespace

constexpr int MAX_GROUPS = 4;

struct samp_encoder {
    samp_config_t cfg;
    std::vector<Layer> L;
    bool all_fp16;
    int prof_which = SAMP_PROF_OFF;
    int fusion_wanted = 0;                          // QKV GEMM + attention in one kernel: 0 by size, 1 never, 2 whenever the shape allows
    std::vector<Timing> events;                     // pool, created on first use
    int events_used = 0;
    // batch-group concurrency: sequences are independent, so a batch is cut into groups that run on side
    // streams at the same time (one chain's kernels leave the chip idle while they start up and drain)
    int groups_wanted = 0;                          // 0 = choose by size
    hipStream_t side[MAX_GROUPS - 1] = {};
    hipEvent_t fork = nullptr, join[MAX_GROUPS - 1] = {};
    bool streams_ready = false;
    // whole-forward HIP graphs, one per distinct argument set (the forward is launch-bound: a few
    // hundred kernels of 5..30 microseconds); captured on an internal stream, replayed on the caller's
    struct Graph { const void *hidden, *mask, *out, *ws; int B, S, G; int seen; hipGraphExec_t exec; const void *seg; samp_embedding_t emb; int tuning; };
    std::vector<Graph> graphs;
    bool graphs_enabled = true;
    hipStream_t cap = nullptr;
};

namespace {

const Timing *timing(samp_encoder *e, int which)
{
    if (e->prof_which != which || e->events_used >= MAX_EVENTS) return nullptr;
    if ((int)e->events.size() <= e->events_used) {
        Timing t;
        if (hipEventCreate(&t.start) != hipSuccess || hipEventCreate(&t.stop) != hipSuccess) return nullptr;
        e->events.push_back(t);
    }
    return &e->events[e->events_used++];
}

int choose_groups(const samp_encoder *e, int B, int S)
{
    int g = e->groups_wanted;
    // measured (BERT-base, 128 tokens): below about 2560 token rows one chain is faster (batch 16: 0.68 against 0.74 ms),
    // from there on two are, at every size (batch 32: 0.83 against 0.97 ms, 128 x 512: -1.4 to -5 %, batch 256: -10 %);
    // three or four never beat two
    if (g <= 0) g = ((long)B * S >= 2560) ? 2 : 1;
    if (g > MAX_GROUPS) g = MAX_GROUPS;
    if (g > B) g = B;
    return g;
}

struct Workspace {
    int *cu, *row_map;
    void *x, *qkv, *ctx, *ao, *h1, *f1, *f2, *y;
    float *absmax;                                  // [layers*10], calibration only
    size_t bytes;
};

Workspace carve(const samp_config_t &c, int B, int S, void *base)
{
    const size_t T = (size_t)B * S, H = c.hidden, F = c.ffn;
    Carver cv{static_cast<char *>(base), 0};
    Workspace w;
    w.cu = cv.take<int>(B + 1);
    w.row_map = cv.take<int>(T);
    w.absmax = cv.take<float>((size_t)c.layers * 10);
    w.x = cv.take<__half>(T * H);
    w.qkv = cv.take<__half>(T * 3 * H);
    w.ctx = cv.take<__half>(T * H);
    w.ao = cv.take<__half>(T * H);
    w.h1 = cv.take<__half>(T * H);
    w.f1 = cv.take<__half>(T * F);
    w.f2 = cv.take<__half>(T * H);
    w.y = cv.take<__half>(T * H);
    w.bytes = cv.off;
    return w;
}

// input of a forward that starts from ids: the Embedding kernel produces layer 0's input
struct Ids { samp_embedding_t emb; const int32_t *token_ids, *segment_ids; };

int check_forward_args(const samp_encoder_t *enc, const void *hidden, int B, int S, const void *workspace, size_t ws_bytes)
{
    if (!enc || !hidden || !workspace) return fail(SAMP_ERR_ARG, "encoder, input or workspace is NULL");
    if (B < 1 || S < 1) return fail(SAMP_ERR_SHAPE, "B and S must be >= 1");
    if (B > enc->cfg.max_batch || S > enc->cfg.max_seq)
        return fail(SAMP_ERR_SHAPE, "B=%d S=%d exceed max_batch=%d max_seq=%d", B, S, enc->cfg.max_batch, enc->cfg.max_seq);
    if (!aligned(workspace, ALIGN)) return fail(SAMP_ERR_SPACE, "workspace must be 256-byte aligned");
    const size_t need = samp_encoder_workspace_bytes(enc, B, S);
    if (ws_bytes < need) return fail(SAMP_ERR_SPACE, "workspace has %zu bytes, %zu needed", ws_bytes, need);
    return SAMP_OK;
}

// The kernel sequence.  calib: FP16-only run that also records each tensor's absmax.
int run(samp_encoder_t *enc, const void *hidden, const Ids *ids, const int32_t *mask, int B, int S, void *out, void *workspace,
        hipStream_t st, bool calib)
{
    const samp_config_t &c = enc->cfg;
    const int H = c.hidden, F = c.ffn, heads = c.heads, Lc = c.layers;
    Workspace w = carve(c, B, S, workspace);
    const int Tmax = B * S;
    const bool packed = mask != nullptr;
    const int *cu = nullptr, *row_map = nullptr;
    Rows rows{Tmax, nullptr};
    const void *x = nullptr;
    const bool first8 = (enc->L[0].mode & 1) != 0;

    if (calib) HIP_TRY(launch_fill_f32(w.absmax, Lc * 10, 0.0f, st));

    // entry: padding removal and, if layer 0's attention block is INT8, quantisation by its producer
    if (ids) {                                      // the Embedding kernel is layer 0's producer
        if (packed) {
            HIP_TRY(launch_seq_offsets(mask, B, S, w.cu, st));
            cu = w.cu; row_map = w.row_map; rows.dev_rows = w.cu + B;
        }
        const samp_embedding_t &e = ids->emb;
        EmbedArgs ea{ids->token_ids, ids->segment_ids, (const __half *)e.token_table, (const __half *)e.segment_table,
                     (const __half *)e.position_table, e.vocab, e.segments, e.positions, e.gamma, e.beta, e.ln_eps,
                     packed ? w.cu : nullptr, B, S, H, w.x, first8, first8 ? enc->L[0].s.x : 1.0f,
                     packed ? w.row_map : nullptr, packed ? (__half *)out : nullptr};
        HIP_TRY(launch_embed_ln(ea, st, timing(enc, SAMP_PROF_ENTRY)));
        x = w.x;
    } else if (packed) {
        HIP_TRY(launch_seq_offsets(mask, B, S, w.cu, st));
        HIP_TRY(launch_pack_rows((const __half *)hidden, w.cu, B, S, H, first8 ? enc->L[0].s.x : 0.0f, w.x, w.row_map,
                                 (__half *)out, st, timing(enc, SAMP_PROF_ENTRY)));
        cu = w.cu; row_map = w.row_map; rows.dev_rows = w.cu + B;
        x = w.x;
    } else if (first8) {
        HIP_TRY(launch_quantize_rows((const __half *)hidden, (size_t)Tmax * H, enc->L[0].s.x, (int8_t *)w.x, st,
                                     timing(enc, SAMP_PROF_ENTRY)));
        x = w.x;
    } else {
        x = hidden;                                 // fp16 input consumed in place
    }
    void *ybuf[2] = {w.y, w.x};                     // layer outputs alternate; w.x is free after layer 0's LN-1
    int yi = 0;

    for (int l = 0; l < Lc; l++) {
        const Layer &Y = enc->L[l];
        const bool mha8 = Y.mode & 1, ffn8 = Y.mode & 2, last = (l == Lc - 1);
        const bool next8 = !last && (enc->L[l + 1].mode & 1);
        float *am = calib ? w.absmax + l * 10 : nullptr;

        if (mha8) {
            // sequences of at most 128 tokens: the QKV tile of a (sequence, head) is one block tile and all that head's
            // attention needs, so one kernel does both.  It pays from about 128 such blocks per launch (BERT-base, 128
            // tokens: batch 4 +12 %, 8 +-0, 16 -1.6 %, 32 -4.9 %, 256 -6.8 % on the forward).  The 256-token flavour
            // (one block per CU, a wave's 64 queries one after the other) loses against the two kernels, whose exact
            // exponentials run four blocks to a CU (BERT-large 32 x 256: +6 %); it runs only when forced.
            const bool can_fuse = S <= (enc->fusion_wanted == 2 ? 256 : 128) && !(Y.mode & SAMP_P_FP16);
            if (can_fuse && (enc->fusion_wanted == 2 || (enc->fusion_wanted == 0 && B * heads >= 128)))
                HIP_TRY(launch_qkv_attention_i8((const int8_t *)x, (const int8_t *)Y.w_qkv, Y.m_qkv, Y.bq_qkv, cu, B, S, H, Y.m_sc,
                                                Y.inv_sp, Y.m_ctx, (Y.mode & SAMP_P_UNSIGNED) != 0, (int8_t *)w.ctx, st,
                                                timing(enc, SAMP_PROF_QKV_ATTN)));
            else {
                HIP_TRY(launch_gemm_i8(EPI_REQUANT, (const int8_t *)x, (const int8_t *)Y.w_qkv, w.qkv, Y.m_qkv, Y.bq_qkv, 0.f,
                                       nullptr, rows, 3 * H, H, st, timing(enc, SAMP_PROF_QKV)));
                if (Y.mode & SAMP_P_FP16)
                    HIP_TRY(launch_attention_i8_p16((const int8_t *)w.qkv, cu, B, S, H, heads, Y.m_sc, Y.m_ctx, (int8_t *)w.ctx,
                                                    st, timing(enc, SAMP_PROF_ATTN)));
                else
                    HIP_TRY(launch_attention_i8((const int8_t *)w.qkv, cu, B, S, H, heads, Y.m_sc, Y.inv_sp, Y.m_ctx,
                                                (Y.mode & SAMP_P_UNSIGNED) != 0, (int8_t *)w.ctx, nullptr, st,
                                                timing(enc, SAMP_PROF_ATTN)));
            }
            HIP_TRY(launch_gemm_i8(EPI_REQUANT, (const int8_t *)w.ctx, (const int8_t *)Y.w_o, w.ao, Y.m_o, nullptr, 0.f,
                                   nullptr, rows, H, H, st, timing(enc, SAMP_PROF_ATTN_OUT)));
        } else {
            if (am) HIP_TRY(launch_absmax_f16((const __half *)x, rows, H, H, am + 0, st));
            // (calibration taps q, k, v and the softmax output, so it keeps the two kernels; with binary32 exponentials
            //  the 256-token flavour pays as well: BERT-large 32 x 256 with FP16 attention blocks -12.7 %)
            if (!am && S <= 256 && (enc->fusion_wanted == 2 || (enc->fusion_wanted == 0 && B * heads >= 128))) {
                HIP_TRY(launch_qkv_attention_f16((const __half *)x, (const __half *)Y.w_qkv, Y.b_qkv, cu, B, S, H, 0.125f,
                                                 (__half *)w.ctx, st, timing(enc, SAMP_PROF_QKV_ATTN)));
            } else {
                HIP_TRY(launch_gemm_f16((const __half *)x, (const __half *)Y.w_qkv, Y.b_qkv, false, (__half *)w.qkv, rows,
                                        3 * H, H, st, timing(enc, SAMP_PROF_QKV)));
                if (am)
                    for (int part = 0; part < 3; part++)
                        HIP_TRY(launch_absmax_f16((const __half *)w.qkv + part * H, rows, H, 3 * H, am + 1 + part, st));
                HIP_TRY(launch_attention_f16((const __half *)w.qkv, cu, B, S, H, heads, 0.125f, (__half *)w.ctx,
                                             am ? am + 4 : nullptr, st, timing(enc, SAMP_PROF_ATTN)));
            }
            if (am) HIP_TRY(launch_absmax_f16((const __half *)w.ctx, rows, H, H, am + 5, st));
            HIP_TRY(launch_gemm_f16((const __half *)w.ctx, (const __half *)Y.w_o, nullptr, false, (__half *)w.ao, rows, H, H,
                                    st, timing(enc, SAMP_PROF_ATTN_OUT)));
            if (am) HIP_TRY(launch_absmax_f16((const __half *)w.ao, rows, H, H, am + 6, st));
        }
        {   // bias + residual + LayerNorm (+ quantise for an INT8 FFN); residual = the block's own input tensor
            AddLnArgs a{w.ao, mha8, Y.s.attn_out, Y.b_o, x, mha8, Y.s.x, Y.g1, Y.be1, c.ln_eps,
                        w.h1, ffn8, Y.s.ffn_in, nullptr, am ? am + 7 : nullptr, rows, H};
            HIP_TRY(launch_add_ln(a, st, timing(enc, SAMP_PROF_LN1)));
        }
        if (ffn8) {
            HIP_TRY(launch_gemm_i8(EPI_GELU_QUANT, (const int8_t *)w.h1, (const int8_t *)Y.w_f1, w.f1, Y.m_f1, Y.b_f1,
                                   1.0f / Y.s.ffn_mid, &Y.gelu, rows, F, H, st, timing(enc, SAMP_PROF_FFN1)));
            HIP_TRY(launch_gemm_i8(EPI_REQUANT, (const int8_t *)w.f1, (const int8_t *)Y.w_f2, w.f2, Y.m_f2, nullptr, 0.f,
                                   nullptr, rows, H, F, st, timing(enc, SAMP_PROF_FFN2)));
        } else {
            HIP_TRY(launch_gemm_f16((const __half *)w.h1, (const __half *)Y.w_f1, Y.b_f1, true, (__half *)w.f1, rows, F, H,
                                    st, timing(enc, SAMP_PROF_FFN1)));
            if (am) HIP_TRY(launch_absmax_f16((const __half *)w.f1, rows, F, F, am + 8, st));
            HIP_TRY(launch_gemm_f16((const __half *)w.f1, (const __half *)Y.w_f2, nullptr, false, (__half *)w.f2, rows, H, F,
                                    st, timing(enc, SAMP_PROF_FFN2)));
            if (am) HIP_TRY(launch_absmax_f16((const __half *)w.f2, rows, H, H, am + 9, st));
        }
        {   // second fused step; the last layer always leaves fp16, scattered back to [B,S,H]
            void *dst = last ? (calib ? ybuf[yi] : out) : ybuf[yi];
            AddLnArgs a{w.f2, ffn8, Y.s.ffn_out, Y.b_f2, w.h1, ffn8, Y.s.ffn_in, Y.g2, Y.be2, c.ln_eps,
                        dst, next8, next8 ? enc->L[l + 1].s.x : 1.0f, (last && !calib) ? row_map : nullptr, nullptr, rows, H};
            HIP_TRY(launch_add_ln(a, st, timing(enc, SAMP_PROF_LN2)));
            x = dst;
            yi ^= 1;
        }
    }
    return SAMP_OK;
}

}  // namespace

extern "C" {

const char *samp_last_error(void) { return g_err; }

size_t samp_encoder_arena_bytes(const samp_config_t *cfg, const uint8_t *modes)
{
    if (check_config(cfg) != SAMP_OK) return 0;
    if (!modes) { fail(SAMP_ERR_ARG, "modes is NULL"); return 0; }
    size_t n = 0;
    for (int l = 0; l < cfg->layers; l++) {
        if (!valid_mode(modes[l])) { fail(SAMP_ERR_ARG, "unknown mode %d for layer %d", modes[l], l); return 0; }
        n += layer_arena_bytes(*cfg, modes[l]);
    }
    return n + staging_bytes(*cfg);
}

int samp_encoder_create(const samp_config_t *cfg, const uint8_t *modes, const samp_layer_weights_t *weights,
                        const samp_layer_scales_t *scales, void *dev_arena, size_t arena_bytes, void *stream,
                        samp_encoder_t **out)
{
    if (int rc = check_config(cfg)) return rc;
    if (!modes || !weights || !dev_arena || !out) return fail(SAMP_ERR_ARG, "modes, weights, dev_arena or out is NULL");
    *out = nullptr;
    bool any8 = false;
    for (int l = 0; l < cfg->layers; l++) {
        if (!valid_mode(modes[l])) return fail(SAMP_ERR_ARG, "unknown mode %d for layer %d", modes[l], l);
        any8 |= modes[l] != 0;
        const samp_layer_weights_t &w = weights[l];
        if (!w.w_qkv || !w.w_o || !w.w_ffn1 || !w.w_ffn2 || !w.b_qkv || !w.b_o || !w.b_ffn1 || !w.b_ffn2 || !w.ln1_g ||
            !w.ln1_b || !w.ln2_g || !w.ln2_b)
            return fail(SAMP_ERR_ARG, "layer %d has a NULL weight pointer", l);
    }
    if (any8 && !scales) return fail(SAMP_ERR_ARG, "scales is NULL but a layer has an INT8 block");
    for (int l = 0; l < cfg->layers && any8; l++) {
        const samp_layer_scales_t &s = scales[l];
        const bool need_x = (modes[l] & 1);
        if (need_x && !(good_scale(s.x) && good_scale(s.q) && good_scale(s.k) && good_scale(s.v) &&
                        ((modes[l] & SAMP_P_FP16) || good_scale(s.p)) && good_scale(s.ctx) && good_scale(s.attn_out)))
            return fail(SAMP_ERR_SCALE, "layer %d: an attention-block scale is not finite and positive", l);
        if ((modes[l] & 2) && !(good_scale(s.ffn_in) && good_scale(s.ffn_mid) && good_scale(s.ffn_out)))
            return fail(SAMP_ERR_SCALE, "layer %d: a feed-forward-block scale is not finite and positive", l);
    }
    if (!aligned(dev_arena, ALIGN)) return fail(SAMP_ERR_SPACE, "arena must be 256-byte aligned");
    const size_t need = samp_encoder_arena_bytes(cfg, modes);
    if (arena_bytes < need) return fail(SAMP_ERR_SPACE, "arena has %zu bytes, %zu needed", arena_bytes, need);

    hipStream_t st = static_cast<hipStream_t>(stream);
    samp_encoder *E = new (std::nothrow) samp_encoder();
    if (!E) return fail(SAMP_ERR_ARG, "out of host memory");
    E->cfg = *cfg;
    E->all_fp16 = !any8;
    E->L.resize(cfg->layers);
    const size_t H = cfg->hidden, F = cfg->ffn;
    Carver cv{static_cast<char *>(dev_arena), 0};
    const size_t big = std::max(3 * H, F);
    __half *stage = cv.take<__half>(big * H);
    float *s_w = cv.take<float>(big);

    std::vector<std::vector<uint32_t>> gelu_host;                // staging of the tables until the stream has copied them
    auto body = [&]() -> int {
        for (int l = 0; l < cfg->layers; l++) {
            Layer &Y = E->L[l];
            const samp_layer_weights_t &w = weights[l];
            Y.mode = modes[l];
            if (scales) Y.s = scales[l]; else memset(&Y.s, 0, sizeof(Y.s));
            const bool mha8 = Y.mode & 1, ffn8 = Y.mode & 2;
            auto vec = [&](const float *src, size_t n, float **dst) -> int {
                *dst = cv.take<float>(n);
                HIP_TRY(hipMemcpyAsync(*dst, src, n * sizeof(float), hipMemcpyHostToDevice, st));
                return SAMP_OK;
            };
            if (int rc = vec(w.b_qkv, 3 * H, &Y.b_qkv)) return rc;
            if (int rc = vec(w.b_o, H, &Y.b_o)) return rc;
            if (int rc = vec(w.b_ffn1, F, &Y.b_f1)) return rc;
            if (int rc = vec(w.b_ffn2, H, &Y.b_f2)) return rc;
            if (int rc = vec(w.ln1_g, H, &Y.g1)) return rc;
            if (int rc = vec(w.ln1_b, H, &Y.be1)) return rc;
            if (int rc = vec(w.ln2_g, H, &Y.g2)) return rc;
            if (int rc = vec(w.ln2_b, H, &Y.be2)) return rc;
            Y.m_qkv = cv.take<float>(3 * H); Y.bq_qkv = cv.take<float>(3 * H);
            Y.m_o = cv.take<float>(H); Y.m_f1 = cv.take<float>(F); Y.m_f2 = cv.take<float>(H);

            // fp16 matrix -> either kept as fp16 or quantised per output channel into int8
            auto matrix = [&](const uint16_t *src, size_t N, size_t K, bool q8, void **dst) -> int {
                if (!q8) {
                    *dst = cv.take<__half>(N * K);
                    HIP_TRY(hipMemcpyAsync(*dst, src, N * K * 2, hipMemcpyHostToDevice, st));
                } else {
                    *dst = cv.take<int8_t>(N * K);
                    HIP_TRY(hipMemcpyAsync(stage, src, N * K * 2, hipMemcpyHostToDevice, st));
                    HIP_TRY(launch_quantize_weight(stage, (int)N, (int)K, (int8_t *)*dst, s_w, st));
                }
                return SAMP_OK;
            };
            if (int rc = matrix(w.w_qkv, 3 * H, H, mha8, &Y.w_qkv)) return rc;
            if (mha8) {
                const float so[3] = {Y.s.q, Y.s.k, Y.s.v};
                for (int part = 0; part < 3; part++)
                    HIP_TRY(launch_fold(nullptr, Y.s.x, s_w + part * H, Y.b_qkv + part * H, so[part], (int)H,
                                        Y.m_qkv + part * H, Y.bq_qkv + part * H, st));
                Y.m_sc = (float)((double)Y.s.q * (double)Y.s.k / std::sqrt(64.0));
                if (!good_score_multiplier(Y.m_sc))
                    return fail(SAMP_ERR_SCALE, "layer %d: s_q * s_k / 8 must not exceed %g", l, (double)MAX_SCORE_MULTIPLIER);
                Y.inv_sp = 1.0f / Y.s.p;
                Y.m_ctx = (Y.mode & SAMP_P_FP16) ? (float)((double)Y.s.v / (double)Y.s.ctx)
                                                 : (float)((double)Y.s.p * (double)Y.s.v / (double)Y.s.ctx);
            }
            if (int rc = matrix(w.w_o, H, H, mha8, &Y.w_o)) return rc;
            if (mha8) HIP_TRY(launch_fold(nullptr, Y.s.ctx, s_w, nullptr, Y.s.attn_out, (int)H, Y.m_o, nullptr, st));
            if (int rc = matrix(w.w_ffn1, F, H, ffn8, &Y.w_f1)) return rc;
            if (ffn8) HIP_TRY(launch_fold(nullptr, Y.s.ffn_in, s_w, nullptr, 1.0f, (int)F, Y.m_f1, nullptr, st));
            Y.gelu = GeluTable{{0.f, 0.f, 0.f, 0}, nullptr};
            if (ffn8) {
                // built on the host from the binary64 definition; a step too fine for a table of this size keeps the
                // per-element evaluation
                uint32_t *dev_entries = cv.take<uint32_t>((size_t)GELU_TABLE_MAX_BINS * 2);
                gelu_host.emplace_back((size_t)GELU_TABLE_MAX_BINS * 2);
                if (gelu_table_build(1.0f / Y.s.ffn_mid, &Y.gelu.spec, gelu_host.back().data())) {
                    HIP_TRY(hipMemcpyAsync(dev_entries, gelu_host.back().data(), (size_t)Y.gelu.spec.bins * 8, hipMemcpyHostToDevice, st));
                    Y.gelu.entries = dev_entries;
                }
            }
            if (int rc = matrix(w.w_ffn2, H, F, ffn8, &Y.w_f2)) return rc;
            if (ffn8) HIP_TRY(launch_fold(nullptr, Y.s.ffn_mid, s_w, nullptr, Y.s.ffn_out, (int)H, Y.m_f2, nullptr, st));
        }
        HIP_TRY(hipStreamSynchronize(st));
        return SAMP_OK;
    };
    const int rc = body();
    if (rc != SAMP_OK) { delete E; return rc; }
    *out = E;
    return SAMP_OK;
}

size_t samp_encoder_workspace_bytes(const samp_encoder_t *enc, int32_t B, int32_t S)
{
    if (!enc || B < 1 || S < 1) { fail(SAMP_ERR_ARG, "encoder is NULL or B, S < 1"); return 0; }
    // enough for the whole batch in one piece and for any split into up to MAX_GROUPS groups
    size_t need = carve(enc->cfg, B, S, nullptr).bytes;
    for (int g = 2; g <= MAX_GROUPS && g <= B; g++) {
        const size_t split = (size_t)g * carve(enc->cfg, (B + g - 1) / g, S, nullptr).bytes;
        if (split > need) need = split;
    }
    return need;
}

int samp_encoder_set_groups(samp_encoder_t *enc, int32_t groups)
{
    if (!enc) return fail(SAMP_ERR_ARG, "encoder is NULL");
    if (groups < 0 || groups > MAX_GROUPS) return fail(SAMP_ERR_ARG, "groups must be in [0, %d]", MAX_GROUPS);
    enc->groups_wanted = groups;
    return SAMP_OK;
}

int samp_encoder_set_qkv_fusion(samp_encoder_t *enc, int32_t mode)
{
    if (!enc) return fail(SAMP_ERR_ARG, "encoder is NULL");
    if (mode < 0 || mode > 2) return fail(SAMP_ERR_ARG, "mode must be 0 (by size), 1 (never) or 2 (whenever the shape allows)");
    enc->fusion_wanted = mode;
    return SAMP_OK;
}

static int forward_eager(samp_encoder_t *enc, const void *hidden, const Ids *ids, const int32_t *mask, int32_t B, int32_t S,
                         void *out, void *workspace, hipStream_t st)
{
    const int G = choose_groups(enc, B, S);
    if (G == 1) return run(enc, hidden, ids, mask, B, S, out, workspace, st, false);
    if (!enc->streams_ready) {
        for (int i = 0; i < MAX_GROUPS - 1; i++) {
            HIP_TRY(hipStreamCreateWithFlags(&enc->side[i], hipStreamNonBlocking));
            HIP_TRY(hipEventCreateWithFlags(&enc->join[i], hipEventDisableTiming));
        }
        HIP_TRY(hipEventCreateWithFlags(&enc->fork, hipEventDisableTiming));
        enc->streams_ready = true;
    }
    // group g owns sequences [g*Bg, ...): its slice of hidden / mask / out and its own workspace piece
    const int Bg = (B + G - 1) / G;
    const size_t piece = carve(enc->cfg, Bg, S, nullptr).bytes;
    const size_t seq_elems = (size_t)S * enc->cfg.hidden;
    // while a kernel is being timed the groups run one after another on the caller's stream, so that
    // each timed launch has the device to itself (same launch shapes, no overlap in the figures)
    const bool serial = enc->prof_which != SAMP_PROF_OFF;
    if (!serial) HIP_TRY(hipEventRecord(enc->fork, st));
    for (int g = 0; g < G; g++) {
        const int b0 = g * Bg, nb = std::min(Bg, B - b0);
        if (nb <= 0) break;
        hipStream_t gs = (g == 0 || serial) ? st : enc->side[g - 1];
        if (g > 0 && !serial) HIP_TRY(hipStreamWaitEvent(gs, enc->fork, 0));
        Ids part;
        if (ids) part = Ids{ids->emb, ids->token_ids + (size_t)b0 * S, ids->segment_ids ? ids->segment_ids + (size_t)b0 * S : nullptr};
        const int rc = run(enc, ids ? nullptr : (const __half *)hidden + b0 * seq_elems, ids ? &part : nullptr,
                           mask ? mask + (size_t)b0 * S : nullptr, nb, S,
                           (__half *)out + b0 * seq_elems, (char *)workspace + g * piece, gs, false);
        if (rc != SAMP_OK) return rc;
        if (g > 0 && !serial) {
            HIP_TRY(hipEventRecord(enc->join[g - 1], gs));
            HIP_TRY(hipStreamWaitEvent(st, enc->join[g - 1], 0));
        }
    }
    return SAMP_OK;
}

// forward from a hidden state (ids == nullptr) or from ids (hidden == nullptr), with the graph cache
static int forward_common(samp_encoder_t *enc, const void *hidden, const Ids *ids, const int32_t *mask, int32_t B, int32_t S,
                          void *out, void *workspace, hipStream_t st);

int samp_encoder_forward(samp_encoder_t *enc, const void *hidden, const int32_t *mask, int32_t B, int32_t S, void *out,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (int rc = check_forward_args(enc, hidden, B, S, workspace, workspace_bytes)) return rc;
    if (!aligned(hidden, 16)) return fail(SAMP_ERR_ARG, "hidden must be 16-byte aligned");
    if (!out) return fail(SAMP_ERR_ARG, "out is NULL");
    if (out == hidden) return fail(SAMP_ERR_ARG, "out must not alias hidden");
    if (!aligned(out, 16)) return fail(SAMP_ERR_ARG, "out must be 16-byte aligned");
    return forward_common(enc, hidden, nullptr, mask, B, S, out, workspace, static_cast<hipStream_t>(stream));
}

int samp_encoder_forward_noalloc(samp_encoder_t *enc, const void *hidden, const int32_t *mask, int32_t B, int32_t S, void *out,
                                 void *stream)
{
    if (!enc || !hidden || !out) return fail(SAMP_ERR_ARG, "encoder, input or output is NULL");
    if (B < 1 || S < 1) return fail(SAMP_ERR_SHAPE, "B and S must be >= 1");
    if (B > enc->cfg.max_batch || S > enc->cfg.max_seq)
        return fail(SAMP_ERR_SHAPE, "B=%d S=%d exceed max_batch=%d max_seq=%d", B, S, enc->cfg.max_batch, enc->cfg.max_seq);
    if (!aligned(hidden, 16) || !aligned(out, 16)) return fail(SAMP_ERR_ARG, "hidden and out must be 16-byte aligned");
    if (out == hidden) return fail(SAMP_ERR_ARG, "out must not alias hidden");
    if (enc->prof_which != SAMP_PROF_OFF) return fail(SAMP_ERR_ARG, "kernel timing is on: it creates events, which this entry point must not");
    const size_t need = carve(enc->cfg, B, S, nullptr).bytes;
    if (need > (size_t)SAMP_NOALLOC_SCRATCH_BYTES)
        return fail(SAMP_ERR_SPACE, "B=%d S=%d need %zu bytes of workspace, the built-in scratch array holds %d: use samp_encoder_forward",
                    B, S, need, SAMP_NOALLOC_SCRATCH_BYTES);
    void *ws = nullptr;
    if (int rc = noalloc_scratch(&ws)) return rc;
    // one group, plain launches on the caller's stream: no side streams, events or graphs are created on this path
    return run(enc, hidden, nullptr, mask, B, S, out, ws, static_cast<hipStream_t>(stream), false);
}

static int check_embedding(const samp_embedding_t *e, int H, int S)
{
    if (!e) return fail(SAMP_ERR_ARG, "embedding is NULL");
    if (!e->token_table || !e->segment_table || !e->position_table || !e->gamma || !e->beta)
        return fail(SAMP_ERR_ARG, "an embedding table or LayerNorm vector is NULL");
    if (!aligned(e->token_table, 16) || !aligned(e->segment_table, 16) || !aligned(e->position_table, 16) ||
        !aligned(e->gamma, 16) || !aligned(e->beta, 16))
        return fail(SAMP_ERR_ARG, "embedding tables and LayerNorm vectors must be 16-byte aligned");
    if (e->vocab < 1 || e->segments < 1) return fail(SAMP_ERR_SHAPE, "vocab and segments must be >= 1");
    if (e->positions < S) return fail(SAMP_ERR_SHAPE, "position table has %d rows, S=%d needed", e->positions, S);
    if (!(e->ln_eps >= 0.0f) || !std::isfinite(e->ln_eps)) return fail(SAMP_ERR_ARG, "ln_eps must be finite and >= 0");
    if (H < 16 || H % 16 || H > 2048) return fail(SAMP_ERR_SHAPE, "H %% 16 == 0 and H <= 2048 required");
    return SAMP_OK;
}

int samp_encoder_forward_ids(samp_encoder_t *enc, const samp_embedding_t *emb, const int32_t *token_ids,
                             const int32_t *segment_ids, const int32_t *mask, int32_t B, int32_t S, void *out,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    if (int rc = check_forward_args(enc, token_ids, B, S, workspace, workspace_bytes)) return rc;
    if (int rc = check_embedding(emb, enc->cfg.hidden, S)) return rc;
    if (!out) return fail(SAMP_ERR_ARG, "out is NULL");
    if (!aligned(out, 16)) return fail(SAMP_ERR_ARG, "out must be 16-byte aligned");
    const Ids ids{*emb, token_ids, segment_ids};
    return forward_common(enc, nullptr, &ids, mask, B, S, out, workspace, static_cast<hipStream_t>(stream));
}

int samp_embed_ln(const samp_embedding_t *emb, const int32_t *token_ids, const int32_t *segment_ids, int32_t B, int32_t S,
                  int32_t H, void *out, int32_t out_i8, float s_out, void *stream)
{
    if (!token_ids || !out) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (B < 1 || S < 1) return fail(SAMP_ERR_SHAPE, "B and S must be >= 1");
    if (int rc = check_embedding(emb, H, S)) return rc;
    if (out_i8 && !good_scale(s_out)) return fail(SAMP_ERR_SCALE, "the output step is not finite and positive");
    if (!aligned(out, 16)) return fail(SAMP_ERR_ARG, "out must be 16-byte aligned");
    EmbedArgs ea{token_ids, segment_ids, (const __half *)emb->token_table, (const __half *)emb->segment_table,
                 (const __half *)emb->position_table, emb->vocab, emb->segments, emb->positions, emb->gamma, emb->beta,
                 emb->ln_eps, nullptr, B, S, H, out, out_i8 != 0, out_i8 ? s_out : 1.0f, nullptr, nullptr};
    HIP_TRY(launch_embed_ln(ea, (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

static int forward_common(samp_encoder_t *enc, const void *hidden, const Ids *ids, const int32_t *mask, int32_t B, int32_t S,
                          void *out, void *workspace, hipStream_t st)
{
    const void *key = ids ? (const void *)ids->token_ids : hidden;
    const void *key_seg = ids ? (const void *)ids->segment_ids : nullptr;
    samp_embedding_t key_emb;
    std::memset(&key_emb, 0, sizeof(key_emb));
    if (ids) key_emb = ids->emb;
    if (!enc->graphs_enabled || enc->prof_which != SAMP_PROF_OFF) return forward_eager(enc, hidden, ids, mask, B, S, out, workspace, st);

    const int G = choose_groups(enc, B, S);
    // a recorded graph holds the tile configurations in force when it was captured: the process-wide tuning
    // override and the encoder's fusion switch are part of the key, so that a changed override records anew instead of replaying the old choice
    const int tuning = (gemm_config_override.load(std::memory_order_relaxed) + 1) | (enc->fusion_wanted << 8);
    samp_encoder::Graph *g = nullptr;
    for (auto &e : enc->graphs)
        if (e.hidden == key && e.seg == key_seg && std::memcmp(&e.emb, &key_emb, sizeof(key_emb)) == 0 && e.mask == mask && e.out == out && e.ws == workspace &&
            e.B == B && e.S == S && e.G == G && e.tuning == tuning) g = &e;
    if (g && g->exec) { HIP_TRY(hipGraphLaunch(g->exec, st)); return SAMP_OK; }
    if (!g) {                                       // first sight of these arguments: run eagerly (one-off set-up happens here)
        if (enc->graphs.size() >= 8) {
            if (enc->graphs.front().exec) (void)hipGraphExecDestroy(enc->graphs.front().exec);
            enc->graphs.erase(enc->graphs.begin());
        }
        enc->graphs.push_back({key, mask, out, workspace, B, S, G, 1, nullptr, key_seg, key_emb, tuning});
        return forward_eager(enc, hidden, ids, mask, B, S, out, workspace, st);
    }
    // second sight: record the same launches into a graph on an internal stream, then replay it
    if (!enc->cap) HIP_TRY(hipStreamCreateWithFlags(&enc->cap, hipStreamNonBlocking));
    hipGraph_t graph = nullptr;
    hipError_t e = hipStreamBeginCapture(enc->cap, hipStreamCaptureModeRelaxed);
    int rc = SAMP_OK;
    if (e == hipSuccess) {
        rc = forward_eager(enc, hidden, ids, mask, B, S, out, workspace, enc->cap);
        e = hipStreamEndCapture(enc->cap, &graph);
    }
    if (e == hipSuccess && rc == SAMP_OK) e = hipGraphInstantiate(&g->exec, graph, nullptr, nullptr, 0);
    if (graph) (void)hipGraphDestroy(graph);
    if (e != hipSuccess || rc != SAMP_OK || !g->exec) {  // capture not possible here: stay with plain launches
        (void)hipGetLastError();
        g->exec = nullptr;
        enc->graphs_enabled = false;
        return forward_eager(enc, hidden, ids, mask, B, S, out, workspace, st);
    }
    HIP_TRY(hipGraphLaunch(g->exec, st));
    return SAMP_OK;
}

int samp_encoder_set_graph(samp_encoder_t *enc, int32_t enabled)
{
    if (!enc) return fail(SAMP_ERR_ARG, "encoder is NULL");
    enc->graphs_enabled = enabled != 0;
    return SAMP_OK;
}

int samp_encoder_calibrate(samp_encoder_t *enc, const void *hidden, const int32_t *mask, int32_t B, int32_t S,
                           void *workspace, size_t workspace_bytes, void *stream, samp_layer_scales_t *scales_out)
{
    if (int rc = check_forward_args(enc, hidden, B, S, workspace, workspace_bytes)) return rc;
    if (!scales_out) return fail(SAMP_ERR_ARG, "scales_out is NULL");
    if (!aligned(hidden, 16)) return fail(SAMP_ERR_ARG, "hidden must be 16-byte aligned");
    if (!enc->all_fp16) return fail(SAMP_ERR_ARG, "calibration needs an encoder whose layers are all SAMP_FP16");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (int rc = run(enc, hidden, nullptr, mask, B, S, nullptr, workspace, st, true)) return rc;
    const int n = enc->cfg.layers * 10;
    std::vector<float> am(n);
    Workspace w = carve(enc->cfg, B, S, workspace);
    HIP_TRY(hipMemcpyAsync(am.data(), w.absmax, n * sizeof(float), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    float *dst = reinterpret_cast<float *>(scales_out);
    for (int i = 0; i < n; i++) dst[i] = am[i] / 127.0f;
    return SAMP_OK;
}

int samp_encoder_destroy(samp_encoder_t *enc)
{
    if (!enc) return SAMP_OK;
    for (Timing &t : enc->events) { (void)hipEventDestroy(t.start); (void)hipEventDestroy(t.stop); }
    if (enc->streams_ready) {
        for (int i = 0; i < MAX_GROUPS - 1; i++) { (void)hipStreamDestroy(enc->side[i]); (void)hipEventDestroy(enc->join[i]); }
        (void)hipEventDestroy(enc->fork);
    }
    for (auto &g : enc->graphs) if (g.exec) (void)hipGraphExecDestroy(g.exec);
    if (enc->cap) (void)hipStreamDestroy(enc->cap);
    delete enc;
    return SAMP_OK;
}

int samp_encoder_profile(samp_encoder_t *enc, int which)
{
    if (!enc) return fail(SAMP_ERR_ARG, "encoder is NULL");
    if (which < SAMP_PROF_OFF || which > SAMP_PROF_QKV_ATTN) return fail(SAMP_ERR_ARG, "unknown kernel class %d", which);
    enc->prof_which = which;
    return SAMP_OK;
}

int samp_encoder_profile_read(samp_encoder_t *enc, double *mean_ms, int64_t *launches)
{
    if (!enc || !mean_ms || !launches) return fail(SAMP_ERR_ARG, "NULL argument");
    double total = 0.0;
    for (int i = 0; i < enc->events_used; i++) {
        HIP_TRY(hipEventSynchronize(enc->events[i].stop));
        float ms = 0.0f;
        HIP_TRY(hipEventElapsedTime(&ms, enc->events[i].start, enc->events[i].stop));
        total += ms;
    }
    *launches = enc->events_used;
    *mean_ms = enc->events_used ? total / enc->events_used : 0.0;
    enc->events_used = 0;
    return SAMP_OK;
}

// ---- single steps --------------------------------------------------------------------------------

static int check_gemm(const void *A, const void *W, const void *out, int M, int N, int K, int kmul)
{
    if (!A || !W || !out) return fail(SAMP_ERR_ARG, "NULL matrix pointer");
    if (M < 1 || N < 128 || N % 128 || K < kmul || K % kmul)
        return fail(SAMP_ERR_SHAPE, "GEMM needs M >= 1, N %% 128 == 0, K %% %d == 0 (M=%d N=%d K=%d)", kmul, M, N, K);
    if (!aligned(A, 16) || !aligned(W, 16) || !aligned(out, 16)) return fail(SAMP_ERR_ARG, "matrices must be 16-byte aligned");
    return SAMP_OK;
}

int samp_gemm_i8_i32(const int8_t *A, const int8_t *W, int32_t *C, int32_t M, int32_t N, int32_t K, void *stream)
{
    if (int rc = check_gemm(A, W, C, M, N, K, 64)) return rc;
    HIP_TRY(launch_gemm_i8(EPI_RAW_I32, A, W, C, nullptr, nullptr, 0.f, nullptr, Rows{M, nullptr}, N, K, (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

int samp_gemm_i8_requant(const int8_t *A, const int8_t *W, const float *m, const float *b, int8_t *out, int32_t M,
                         int32_t N, int32_t K, void *stream)
{
    if (int rc = check_gemm(A, W, out, M, N, K, 64)) return rc;
    if (!m) return fail(SAMP_ERR_ARG, "multiplier table is NULL");
    HIP_TRY(launch_gemm_i8(EPI_REQUANT, A, W, out, m, b, 0.f, nullptr, Rows{M, nullptr}, N, K, (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

int samp_gemm_i8_gelu_quant(const int8_t *A, const int8_t *W, const float *m, const float *bias, float s_out,
                            const samp_gelu_table_t *table, const void *table_entries, int8_t *out, int32_t M, int32_t N,
                            int32_t K, void *stream)
{
    if (int rc = check_gemm(A, W, out, M, N, K, 64)) return rc;
    if (!m || !bias) return fail(SAMP_ERR_ARG, "multiplier or bias table is NULL");
    if (!good_scale(s_out)) return fail(SAMP_ERR_SCALE, "s_out must be finite and positive");
    GeluTable gt{{0.f, 0.f, 0.f, 0}, nullptr};
    if (table || table_entries) {
        if (!table || !table_entries) return fail(SAMP_ERR_ARG, "a threshold table needs both its description and its entries");
        if (!aligned(table_entries, 8)) return fail(SAMP_ERR_ARG, "table_entries must be 8-byte aligned");
        if (table->bins < 2 || table->bins > GELU_TABLE_MAX_BINS || table->t_max != 8388608.0f + (float)(table->bins - 1) ||
            !(table->rate > 0.0f) || !std::isfinite(table->rate) || !std::isfinite(table->offset))
            return fail(SAMP_ERR_ARG, "the threshold table's description is not one samp_gelu_table_build wrote");
        gt = GeluTable{{table->rate, table->offset, table->t_max, table->bins}, static_cast<const uint32_t *>(table_entries)};
    }
    HIP_TRY(launch_gemm_i8(EPI_GELU_QUANT, A, W, out, m, bias, 1.0f / s_out, gt.entries ? &gt : nullptr, Rows{M, nullptr}, N, K,
                           (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

int samp_gelu_table_build(float s_out, samp_gelu_table_t *table, void *host_entries, size_t entries_bytes)
{
    if (!table || !host_entries) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (!good_scale(s_out)) return fail(SAMP_ERR_SCALE, "s_out must be finite and positive");
    if (entries_bytes < SAMP_GELU_TABLE_BYTES)
        return fail(SAMP_ERR_SPACE, "entries buffer has %zu bytes, %d needed", entries_bytes, SAMP_GELU_TABLE_BYTES);
    GeluTableSpec sp;
    if (!gelu_table_build(1.0f / s_out, &sp, static_cast<uint32_t *>(host_entries)))
        return fail(SAMP_ERR_SCALE, "the step %g needs more than %d bins", (double)s_out, GELU_TABLE_MAX_BINS);
    table->rate = sp.rate; table->offset = sp.offset; table->t_max = sp.t_max; table->bins = sp.bins;
    return SAMP_OK;
}

int samp_gemm_f16(const uint16_t *A, const uint16_t *W, const float *bias, int32_t gelu, uint16_t *out, int32_t M, int32_t N,
                  int32_t K, void *stream)
{
    if (int rc = check_gemm(A, W, out, M, N, K, 32)) return rc;
    HIP_TRY(launch_gemm_f16((const __half *)A, (const __half *)W, bias, gelu != 0, (__half *)out, Rows{M, nullptr}, N, K,
                            (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

static int check_attention(const void *qkv, const int32_t *cu, int B, int max_len, int hidden, int heads, const void *ctx)
{
    (void)cu;                                                     // NULL: B sequences of exactly max_len rows
    if (!qkv || !ctx) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (B < 1 || max_len < 1 || max_len > SAMP_MAX_SEQ) return fail(SAMP_ERR_SHAPE, "B >= 1 and 1 <= max_len <= %d required", SAMP_MAX_SEQ);
    if (heads < 1 || hidden != heads * 64) return fail(SAMP_ERR_SHAPE, "head size must be 64");
    if (!aligned(qkv, 16) || !aligned(ctx, 16)) return fail(SAMP_ERR_ARG, "tensors must be 16-byte aligned");
    return SAMP_OK;
}

int samp_attention_i8(const int8_t *qkv, const int32_t *cu, int32_t B, int32_t max_len, int32_t hidden, int32_t heads,
                      float s_q, float s_k, float s_v, float s_p, float s_ctx, int32_t p_kind, int8_t *ctx,
                      uint64_t *p_hist, void *stream)
{
    if (int rc = check_attention(qkv, cu, B, max_len, hidden, heads, ctx)) return rc;
    if (p_kind < 0 || p_kind > 2) return fail(SAMP_ERR_ARG, "p_kind must be 0, 1 or 2");
    if (!(good_scale(s_q) && good_scale(s_k) && good_scale(s_v) && (p_kind == 2 || good_scale(s_p)) && good_scale(s_ctx)))
        return fail(SAMP_ERR_SCALE, "attention scales must be finite and positive");
    const float m_sc = (float)((double)s_q * (double)s_k / std::sqrt(64.0));
    if (!good_score_multiplier(m_sc)) return fail(SAMP_ERR_SCALE, "s_q * s_k / 8 must not exceed %g", (double)MAX_SCORE_MULTIPLIER);
    if (p_kind == 2) {
        if (p_hist) return fail(SAMP_ERR_ARG, "a binary16 softmax output has no code histogram");
        HIP_TRY(launch_attention_i8_p16(qkv, cu, B, max_len, hidden, heads, m_sc, (float)((double)s_v / (double)s_ctx), ctx,
                                        (hipStream_t)stream, nullptr));
        return SAMP_OK;
    }
    const float m_ctx = (float)((double)s_p * (double)s_v / (double)s_ctx);
    HIP_TRY(launch_attention_i8(qkv, cu, B, max_len, hidden, heads, m_sc, 1.0f / s_p, m_ctx, p_kind == 1, ctx,
                                reinterpret_cast<unsigned long long *>(p_hist), (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

int samp_qkv_attention_i8(const int8_t *x, const int8_t *w_qkv, const float *m, const float *b, const int32_t *cu, int32_t B,
                          int32_t max_len, int32_t hidden, int32_t heads, float s_q, float s_k, float s_v, float s_p,
                          float s_ctx, int32_t p_kind, int8_t *ctx, void *stream)
{
    if (p_kind < 0 || p_kind > 1) return fail(SAMP_ERR_ARG, "p_kind must be 0 or 1");
    if (!x || !w_qkv || !m || !ctx) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (B < 1 || max_len < 1 || max_len > 256) return fail(SAMP_ERR_SHAPE, "B >= 1 and 1 <= max_len <= 256 required");
    if (heads < 1 || hidden != heads * 64) return fail(SAMP_ERR_SHAPE, "head size must be 64");
    if (!aligned(x, 16) || !aligned(w_qkv, 16) || !aligned(ctx, 16) || !aligned(m, 16) || (b && !aligned(b, 16)))
        return fail(SAMP_ERR_ARG, "tensors must be 16-byte aligned");
    if (!(good_scale(s_q) && good_scale(s_k) && good_scale(s_v) && good_scale(s_p) && good_scale(s_ctx)))
        return fail(SAMP_ERR_SCALE, "attention scales must be finite and positive");
    const float m_sc = (float)((double)s_q * (double)s_k / std::sqrt(64.0));
    if (!good_score_multiplier(m_sc)) return fail(SAMP_ERR_SCALE, "s_q * s_k / 8 must not exceed %g", (double)MAX_SCORE_MULTIPLIER);
    const float m_ctx = (float)((double)s_p * (double)s_v / (double)s_ctx);
    HIP_TRY(launch_qkv_attention_i8(x, w_qkv, m, b, cu, B, max_len, hidden, m_sc, 1.0f / s_p, m_ctx, p_kind == 1, ctx,
                                    (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

int samp_qkv_attention_f16(const uint16_t *x, const uint16_t *w_qkv, const float *bias, const int32_t *cu, int32_t B,
                           int32_t max_len, int32_t hidden, int32_t heads, uint16_t *ctx, void *stream)
{
    if (!x || !w_qkv || !ctx) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (B < 1 || max_len < 1 || max_len > 256) return fail(SAMP_ERR_SHAPE, "B >= 1 and 1 <= max_len <= 256 required");
    if (heads < 1 || hidden != heads * 64) return fail(SAMP_ERR_SHAPE, "head size must be 64");
    if (!aligned(x, 16) || !aligned(w_qkv, 16) || !aligned(ctx, 16)) return fail(SAMP_ERR_ARG, "tensors must be 16-byte aligned");
    HIP_TRY(launch_qkv_attention_f16((const __half *)x, (const __half *)w_qkv, bias, cu, B, max_len, hidden, 0.125f, (__half *)ctx,
                                     (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

int samp_attention_f16(const uint16_t *qkv, const int32_t *cu, int32_t B, int32_t max_len, int32_t hidden, int32_t heads,
                       uint16_t *ctx, void *stream)
{
    if (int rc = check_attention(qkv, cu, B, max_len, hidden, heads, ctx)) return rc;
    HIP_TRY(launch_attention_f16((const __half *)qkv, cu, B, max_len, hidden, heads, 0.125f, (__half *)ctx, nullptr,
                                 (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

int samp_add_ln(const void *in, int32_t in_i8, float s_in, const float *bias, const void *res, int32_t res_i8, float s_res,
                const float *gamma, const float *beta, float eps, void *out, int32_t out_i8, float s_out, int32_t M, int32_t H,
                void *stream)
{
    if (!in || !bias || !res || !gamma || !beta || !out) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (M < 1 || H < 16 || H % 16 || H > 2048) return fail(SAMP_ERR_SHAPE, "M >= 1, H %% 16 == 0, H <= 2048 required");
    if ((in_i8 && !good_scale(s_in)) || (res_i8 && !good_scale(s_res)) || (out_i8 && !good_scale(s_out)))
        return fail(SAMP_ERR_SCALE, "a step of an int8 operand is not finite and positive");
    AddLnArgs a{in, in_i8 != 0, s_in, bias, res, res_i8 != 0, s_res, gamma, beta, eps, out, out_i8 != 0, s_out,
                nullptr, nullptr, Rows{M, nullptr}, H};
    HIP_TRY(launch_add_ln(a, (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

int samp_gelu_quant(const float *y, int64_t n, float s_out, int8_t *codes, float *fast, void *stream)
{
    if (!y || !codes) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (n < 1) return fail(SAMP_ERR_SHAPE, "n >= 1 required");
    if (!good_scale(s_out)) return fail(SAMP_ERR_SCALE, "s_out must be finite and positive");
    HIP_TRY(launch_gelu_quant(y, (size_t)n, 1.0f / s_out, codes, fast, (hipStream_t)stream));
    return SAMP_OK;
}

int samp_quantize_f16_i8(const uint16_t *x, int64_t n, float s_x, int8_t *out, void *stream)
{
    if (!x || !out) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (n < 8 || n % 8) return fail(SAMP_ERR_SHAPE, "n must be a positive multiple of 8");
    if (!good_scale(s_x)) return fail(SAMP_ERR_SCALE, "s_x must be finite and positive");
    if (!aligned(x, 16) || !aligned(out, 8)) return fail(SAMP_ERR_ARG, "x must be 16-byte and out 8-byte aligned");
    HIP_TRY(launch_quantize_rows((const __half *)x, (size_t)n, s_x, out, (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

int samp_quantize_weight(const uint16_t *W, int32_t N, int32_t K, int8_t *Wq, float *s_w, void *stream)
{
    if (!W || !Wq || !s_w) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (N < 1 || K < 1) return fail(SAMP_ERR_SHAPE, "N, K >= 1 required");
    HIP_TRY(launch_quantize_weight((const __half *)W, N, K, Wq, s_w, (hipStream_t)stream));
    return SAMP_OK;
}

static int check_curves(const double *accuracy, const double *latency, int32_t n)
{
    if (!accuracy || !latency) return fail(SAMP_ERR_ARG, "accuracy or latency is NULL");
    if (n < 1 || n > 64) return fail(SAMP_ERR_SHAPE, "n must be in [1, 64]");
    for (int i = 0; i < n; i++) {
        if (!std::isfinite(accuracy[i]) || !std::isfinite(latency[i])) return fail(SAMP_ERR_ARG, "setting %d: accuracy and latency must be finite", i);
        if (!(latency[i] > 0.0)) return fail(SAMP_ERR_ARG, "setting %d: latency must be positive", i);
    }
    return SAMP_OK;
}

int samp_allocate_decay_aware(const double *accuracy, const double *latency, int32_t n, int32_t *setting_out)
{
    if (int rc = check_curves(accuracy, latency, n)) return rc;
    if (!setting_out) return fail(SAMP_ERR_ARG, "setting_out is NULL");
    *setting_out = allocate_decay_aware(accuracy, latency, n);
    return SAMP_OK;
}

int samp_recommend(const double *accuracy, const double *latency, int32_t n, double max_latency, double min_accuracy,
                   int32_t *settings_out, int32_t capacity, int32_t *count_out)
{
    if (int rc = check_curves(accuracy, latency, n)) return rc;
    if (!settings_out || !count_out) return fail(SAMP_ERR_ARG, "settings_out or count_out is NULL");
    if (capacity < 1) return fail(SAMP_ERR_ARG, "capacity must be >= 1");
    if (std::isinf(max_latency) || std::isinf(min_accuracy)) return fail(SAMP_ERR_ARG, "thresholds must be finite or NaN (unset)");
    *count_out = recommend_settings(accuracy, latency, n, max_latency, min_accuracy, settings_out, capacity);
    return SAMP_OK;
}

int samp_classify(const uint16_t *hidden, int32_t B, int32_t S, int32_t H, const uint16_t *w_pool, const float *b_pool,
                  const uint16_t *w_cls, const float *b_cls, int32_t classes, float *logits, void *stream)
{
    if (!hidden || !w_pool || !b_pool || !w_cls || !b_cls || !logits) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (B < 1 || S < 1 || classes < 1) return fail(SAMP_ERR_SHAPE, "B, S and classes must be >= 1");
    if (H < 8 || H % 8 || H > 4096) return fail(SAMP_ERR_SHAPE, "H %% 8 == 0 and H <= 4096 required");
    if (!aligned(hidden, 16) || !aligned(w_pool, 16) || !aligned(w_cls, 16))
        return fail(SAMP_ERR_ARG, "hidden and the weight matrices must be 16-byte aligned");
    HIP_TRY(launch_classify((const __half *)hidden, B, S, H, (const __half *)w_pool, b_pool, (const __half *)w_cls, b_cls,
                            classes, logits, (hipStream_t)stream));
    return SAMP_OK;
}

int samp_probe_mfma_rate(int32_t fp16, int32_t random_operands, int32_t iters, void *dev_sink, void *stream, double *ops_per_s)
{
    if (!dev_sink || !ops_per_s) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (iters < 1 || iters > (1 << 20)) return fail(SAMP_ERR_ARG, "iters must be in [1, 2^20]");
    HIP_TRY(probe_mfma_rate(fp16 != 0, random_operands != 0, iters, (int *)dev_sink, (hipStream_t)stream, ops_per_s));
    return SAMP_OK;
}

int samp_probe_copy_rate(const void *src, void *dst, size_t bytes, int32_t reps, void *stream, double *bytes_per_s)
{
    if (!src || !dst || !bytes_per_s) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (bytes < 16 || bytes % 16 || reps < 1) return fail(SAMP_ERR_SHAPE, "bytes must be a positive multiple of 16, reps >= 1");
    if (!aligned(src, 16) || !aligned(dst, 16)) return fail(SAMP_ERR_ARG, "buffers must be 16-byte aligned");
    HIP_TRY(probe_copy_rate(src, dst, bytes, reps, (hipStream_t)stream, bytes_per_s));
    return SAMP_OK;
}

int samp_probe_feed_rate(const void *operands, size_t bytes, int32_t rows, int32_t N, int32_t kbytes, int32_t reps,
                         void *dev_sink, void *stream, double *bytes_per_s)
{
    if (!operands || !dev_sink || !bytes_per_s) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (rows < 128 || rows % 128 || N < 128 || N % 128 || kbytes < 128 || kbytes % 128 || reps < 1)
        return fail(SAMP_ERR_SHAPE, "rows, N and kbytes must be positive multiples of 128, reps >= 1");
    if ((long long)(rows / 128) * (N / 128) > (1 << 20)) return fail(SAMP_ERR_SHAPE, "too many tiles");
    const size_t a_bytes = (size_t)rows * kbytes, w_bytes = (size_t)N * kbytes;
    if (bytes < a_bytes + w_bytes) return fail(SAMP_ERR_SPACE, "the operand buffer must hold (rows + N) * kbytes bytes");
    if (!aligned(operands, 16)) return fail(SAMP_ERR_ARG, "the operand buffer must be 16-byte aligned");
    HIP_TRY(probe_feed_rate(operands, (const char *)operands + a_bytes, rows, N, kbytes, reps, (int *)dev_sink,
                            (hipStream_t)stream, bytes_per_s));
    return SAMP_OK;
}

int samp_code_histogram(const int8_t *codes, size_t n, uint64_t *hist, void *stream)
{
    if (!codes || !hist) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (n < 1) return fail(SAMP_ERR_SHAPE, "n must be >= 1");
    HIP_TRY(launch_code_histogram(codes, n, reinterpret_cast<unsigned long long *>(hist), (hipStream_t)stream));
    return SAMP_OK;
}

int samp_set_gemm_config(int32_t config)
{
    if (config < -1 || config > 7) return fail(SAMP_ERR_ARG, "config must be in [-1, 7]");
    gemm_config_override = config;
    return SAMP_OK;
}

int samp_pack_rows(const uint16_t *hidden, const int32_t *mask, int32_t B, int32_t S, int32_t H, float s_x, void *packed,
                   int32_t *cu, int32_t *row_map, void *stream)
{
    if (!hidden || !mask || !packed || !cu || !row_map) return fail(SAMP_ERR_ARG, "NULL pointer");
    if (B < 1 || S < 1 || H < 8 || H % 8) return fail(SAMP_ERR_SHAPE, "B, S >= 1 and H %% 8 == 0 required");
    if (B > SAMP_MAX_BATCH) return fail(SAMP_ERR_SHAPE, "B must not exceed %d sequences", SAMP_MAX_BATCH);
    HIP_TRY(launch_seq_offsets(mask, B, S, cu, (hipStream_t)stream));
    HIP_TRY(launch_pack_rows((const __half *)hidden, cu, B, S, H, s_x, packed, row_map, nullptr, (hipStream_t)stream, nullptr));
    return SAMP_OK;
}

}  // extern "C"
