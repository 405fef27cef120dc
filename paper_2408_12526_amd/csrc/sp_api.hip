// C ABI of libsp_mi355x.so: argument checks, weight upload, workspace carve-up
// and the order in which the kernels of one forward pass are enqueued.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <mutex>
#include <thread>
#include <vector>

#include "sp_dispatch.h"
#include "sp_internal.h"

namespace sp {

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static bool config_ok(const sp_config* c)
{
    if (!c) return false;
    if (c->K < 1 || c->layers < 1 || c->hidden < 1 || c->heads < 1 || c->ffn < 1 || c->vocab < 1 || c->max_pos < 1 ||
        c->classes < 1)
        return false;
    if (c->dtype != SP_DTYPE_FP32 && c->dtype != SP_DTYPE_BF16 && c->dtype != SP_DTYPE_FP8) return false;
    if (!(c->ln_eps >= 0.f)) return false;
    return true;
}

// what the kernels support
static bool config_supported(const sp_config& c)
{
    if (c.hidden % c.heads || c.hidden / c.heads != 64) return false;
    if (c.classes > 16 || c.hidden > 1024 || c.K > 64) return false;
    if (c.hidden % 128 || c.ffn % 128) return false;   // reduction depth of every projection: whole 64-wide k-tiles, at least two
    return true;
}

ArenaLayout make_arena_layout(const sp_config& c)
{
    const size_t H = c.hidden, F = c.ffn, C = c.classes;
    const size_t wb = bf16_path(c) ? 2 : 4;  // bytes per matrix / table element
    const size_t q8 = c.dtype == SP_DTYPE_FP8 ? 1 : 0;     // fp8 copies of three matrices
    ArenaLayout L{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    L.tok = take((size_t)c.vocab * H * wb);
    L.pos = take((size_t)c.max_pos * H * wb);
    L.emb_g = take(H * 4);
    L.emb_b = take(H * 4);
    L.layer0 = o;
    {
        size_t base = o;
        L.wqkv = take(3 * H * H * wb) - base;
        L.bqkv = take(3 * H * 4) - base;
        L.wo = take(H * H * wb) - base;
        L.bo = take(H * 4) - base;
        L.ln1g = take(H * 4) - base;
        L.ln1b = take(H * 4) - base;
        L.w1 = take(F * H * wb) - base;
        L.b1 = take(F * 4) - base;
        L.w2 = take(H * F * wb) - base;
        L.b2 = take(H * 4) - base;
        L.ln2g = take(H * 4) - base;
        L.ln2b = take(H * 4) - base;
        L.wk_io = take(H * H * wb) - base;
        if (q8) {
            L.wqkv8 = take(3 * H * H) - base;
            L.sqkv = take(3 * H * 4) - base;
            L.wo8 = take(H * H) - base;
            L.so = take(H * 4) - base;
            L.w18 = take(F * H) - base;
            L.s1 = take(F * 4) - base;
            L.w28 = take(H * F) - base;
            L.s2 = take(H * 4) - base;
        }
        L.layer_stride = o - base;
        o = base + L.layer_stride * (size_t)c.layers;
    }
    L.wp = take(H * H * wb);
    L.wp_t = take(H * H * wb);
    L.bp = take(H * 4);
    L.wc = take(C * H * wb);
    L.bc = take(C * 4);
    L.student_stride = align_up(o, 4096);
    return L;
}

WsLayout make_ws_layout(const sp_config& c, int total_tokens, int batch)
{
    WsLayout W{};
    const size_t ab = bf16_path(c) ? 2 : 4;
    const size_t rows = align_up((size_t)total_tokens, kRowPad);
    const size_t K = c.K, H = c.hidden, F = c.ffn;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes, 256); return at; };
    W.x = take(K * rows * H * ab);
    W.qkv = take(K * rows * 3 * H * ab);
    W.vt = take(K * rows * H * ab);
    W.att = take(K * rows * H * ab);
    W.u = take(K * rows * H * ab);
    W.x1 = take(K * rows * H * ab);
    W.g = take(K * rows * F * ab);
    W.z = take(K * (size_t)batch * c.classes * 4);
    W.zpart = take(K * (size_t)(H / 64) * batch * c.classes * 4);
    // compact buffers for the first-token rows of the last layer (never used by calls of fewer than
    // kFirstOnlyMinTokens tokens: those get none)
    const size_t crows = total_tokens >= kFirstOnlyMinTokens ? align_up((size_t)batch, kRowPad) : 0;
    W.cx = take(K * crows * H * ab);
    W.cq = take(K * crows * H * ab);
    W.catt = take(K * crows * H * ab);
    W.cu_ = take(K * crows * H * ab);
    W.cx1 = take(K * crows * H * ab);
    W.cg = take(K * crows * F * ab);
    W.cqt = take(K * crows * (size_t)c.heads * H * ab);
    W.cxb = take(K * crows * (size_t)c.heads * H * ab);
    W.part = take(K * (size_t)kSplitMax * kSplitRows * H * 4);
    W.lpart = take(2 * (size_t)batch * c.classes * 4);
    if (c.dtype == SP_DTYPE_FP8 && rows >= (size_t)kFp8MinRows) {
        W.xq = take(K * rows * H);
        W.x1q = take(K * rows * H);
        W.attq = take(K * rows * H);
        W.gq = take(K * rows * F);
    }
    W.crows = (int)crows;
    W.end = o;
    W.rows = (int)rows;
    W.act_bytes = (int)ab;
    return W;
}

static size_t student_blob_floats(const sp_config& c)
{
    const size_t H = c.hidden, F = c.ffn, C = c.classes;
    const size_t layer = 4 * (H * H + H) + 2 * H + (H * F + F) + (F * H + H) + 2 * H;
    return (size_t)c.vocab * H + (size_t)c.max_pos * H + 2 * H + (size_t)c.layers * layer + H * H + H + H * C + C;
}

// ---- host-side conversion into the arena image --------------------------------

static inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// OCP e4m3 (4 exponent bits, bias 7, 3 mantissa bits, no infinities, largest finite value 448): round to nearest
// even, saturating.
static inline uint8_t f32_to_e4m3(float f)
{
    const uint8_t sign = std::signbit(f) ? 0x80 : 0;
    const float a = std::fabs(f);
    if (a != a) return (uint8_t)(sign | 0x7f);
    if (a >= 448.f) return (uint8_t)(sign | 0x7e);
    if (a < 0.015625f) {                                   // below 2^-6: multiples of 2^-9
        const int q = (int)std::nearbyint(a * 512.f);     // 0..8 (8 = the smallest normal number)
        return (uint8_t)(sign | q);
    }
    int e;
    const float mant = std::frexp(a, &e);                  // a = mant * 2^e, mant in [0.5, 1)
    int q = (int)std::nearbyint((mant * 2.f - 1.f) * 8.f); // 0..8
    int ex = e - 1;                                        // a = (1 + q / 8) * 2^ex
    if (q == 8) { q = 0; ++ex; }
    const int code = ((ex + 7) << 3) | q;
    return (uint8_t)(sign | (code > 0x7e ? 0x7e : code));
}

// dst8[o][i] = e4m3(src[i][o] / scale[o]), scale[o] = max_i |src[i][o]| / 448 (1 for an all-zero column);
// src is [n_in][n_out]
static void quantize_transposed(uint8_t* dst8, float* scale, const float* src, size_t n_in, size_t n_out)
{
    std::vector<float> amax(n_out, 0.f);
    for (size_t i = 0; i < n_in; ++i)
        for (size_t o = 0; o < n_out; ++o) {
            const float a = std::fabs(src[i * n_out + o]);
            if (a > amax[o]) amax[o] = a;
        }
    for (size_t o = 0; o < n_out; ++o) scale[o] = amax[o] > 0.f ? amax[o] / 448.f : 1.f;
    const size_t T = 32;
    for (size_t i0 = 0; i0 < n_in; i0 += T)
        for (size_t o0 = 0; o0 < n_out; o0 += T) {
            const size_t i1 = i0 + T < n_in ? i0 + T : n_in, o1 = o0 + T < n_out ? o0 + T : n_out;
            for (size_t o = o0; o < o1; ++o)
                for (size_t i = i0; i < i1; ++i) dst8[o * n_in + i] = f32_to_e4m3(src[i * n_out + o] / scale[o]);
        }
}

struct Writer {
    bool bf16;
    // copy n values as the arena's matrix element type
    void copy(char* dst, const float* src, size_t n) const
    {
        if (bf16) {
            uint16_t* d = (uint16_t*)dst;
            for (size_t i = 0; i < n; ++i) d[i] = f32_to_bf16_rne(src[i]);
        } else {
            memcpy(dst, src, n * 4);
        }
    }
    // dst[o][i] = src[i][o]; src is [n_in][n_out]; dst row stride n_in
    void transpose(char* dst, const float* src, size_t n_in, size_t n_out) const
    {
        const size_t T = 32;
        for (size_t i0 = 0; i0 < n_in; i0 += T)
            for (size_t o0 = 0; o0 < n_out; o0 += T) {
                const size_t i1 = i0 + T < n_in ? i0 + T : n_in, o1 = o0 + T < n_out ? o0 + T : n_out;
                for (size_t o = o0; o < o1; ++o)
                    for (size_t i = i0; i < i1; ++i) {
                        const float v = src[i * n_out + o];
                        if (bf16) ((uint16_t*)dst)[o * n_in + i] = f32_to_bf16_rne(v);
                        else ((float*)dst)[o * n_in + i] = v;
                    }
            }
    }
};

static void fill_student(const sp_config& c, const ArenaLayout& L, const float* src, char* dst)
{
    const size_t H = c.hidden, F = c.ffn, C = c.classes, wb = bf16_path(c) ? 2 : 4;
    const bool q8 = c.dtype == SP_DTYPE_FP8;
    Writer w{bf16_path(c)};
    const float* p = src;
    w.copy(dst + L.tok, p, (size_t)c.vocab * H); p += (size_t)c.vocab * H;
    w.copy(dst + L.pos, p, (size_t)c.max_pos * H); p += (size_t)c.max_pos * H;
    memcpy(dst + L.emb_g, p, H * 4); p += H;
    memcpy(dst + L.emb_b, p, H * 4); p += H;
    for (int l = 0; l < c.layers; ++l) {
        char* lb = dst + L.layer0 + (size_t)l * L.layer_stride;
        for (int part = 0; part < 3; ++part) {  // Wq bq Wk bk Wv bv -> rows [part*H, part*H+H) of the fused matrix
            if (part == 1) w.copy(lb + L.wk_io, p, H * H);
            if (q8) quantize_transposed((uint8_t*)(lb + L.wqkv8) + (size_t)part * H * H, (float*)(lb + L.sqkv) + part * H, p, H, H);
            w.transpose(lb + L.wqkv + (size_t)part * H * H * wb, p, H, H); p += H * H;
            memcpy(lb + L.bqkv + (size_t)part * H * 4, p, H * 4); p += H;
        }
        if (q8) quantize_transposed((uint8_t*)(lb + L.wo8), (float*)(lb + L.so), p, H, H);
        w.transpose(lb + L.wo, p, H, H); p += H * H;
        memcpy(lb + L.bo, p, H * 4); p += H;
        memcpy(lb + L.ln1g, p, H * 4); p += H;
        memcpy(lb + L.ln1b, p, H * 4); p += H;
        if (q8) quantize_transposed((uint8_t*)(lb + L.w18), (float*)(lb + L.s1), p, H, F);
        w.transpose(lb + L.w1, p, H, F); p += H * F;
        memcpy(lb + L.b1, p, F * 4); p += F;
        if (q8) quantize_transposed((uint8_t*)(lb + L.w28), (float*)(lb + L.s2), p, F, H);
        w.transpose(lb + L.w2, p, F, H); p += F * H;
        memcpy(lb + L.b2, p, H * 4); p += H;
        memcpy(lb + L.ln2g, p, H * 4); p += H;
        memcpy(lb + L.ln2b, p, H * 4); p += H;
    }
    w.copy(dst + L.wp, p, H * H);
    w.transpose(dst + L.wp_t, p, H, H); p += H * H;
    memcpy(dst + L.bp, p, H * 4); p += H;
    w.copy(dst + L.wc, p, H * C); p += H * C;
    memcpy(dst + L.bc, p, C * 4); p += C;
}

// Optional per-phase timing: an event is recorded after every launch and tagged with its phase.
struct PhaseTimer {
    std::vector<hipEvent_t> ev;      // grows with the launch count (a dozen per layer)
    std::vector<int> phase;
    int n = 0;
    bool ok = true;
    void mark(int ph, hipStream_t s)
    {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) { ok = false; return; }
        try { ev.push_back(e); phase.push_back(ph); } catch (...) { (void)hipEventDestroy(e); ok = false; return; }
        ++n;
        if (hipEventRecord(e, s) != hipSuccess) ok = false;
    }
    void release() { for (int i = 0; i < n; ++i) (void)hipEventDestroy(ev[i]); ev.clear(); phase.clear(); n = 0; }
};

// The forward of students [m0, m0 + k) of the model (k >= 1), all of it enqueued on stream s.  Every buffer of the
// workspace is sliced per student, so groups of students can run side by side on different streams.  With
// with_head the group's z rows are written; logits (the group's own sum, in student order) only if non-null.
static int run_students(const sp_model* M0, const WsLayout& W, const int32_t* ids, const int32_t* cu, int B, int T,
                        int max_seqlen, int m0, int k, int stop_layers, bool with_head, char* w, float* logits,
                        hipStream_t s, PhaseTimer* pt)
{
    const sp_config& c = M0->cfg;
    sp_model shifted = *M0;                 // launchers address student i of the group as arena + i * stride
    shifted.arena = M0->arena + (size_t)m0 * M0->L.student_stride;
    const sp_model* M = &shifted;
    const int H = c.hidden, F = c.ffn, rows = W.rows;
    // rows actually computed: the packed tokens rounded up to the token tile the GEMMs will use
    const int mtile = T > 256 ? 256 : (T > 64 ? 128 : 64);
    const int mrows = (T + mtile - 1) / mtile * mtile;
    const size_t ab = W.act_bytes;
    const size_t sH = (size_t)rows * H * ab, s3H = 3 * sH, sF = (size_t)rows * F * ab;
    char *x = w + W.x + m0 * sH, *qkv = w + W.qkv + m0 * s3H, *vt = w + W.vt + m0 * sH, *att = w + W.att + m0 * sH;
    char *u = w + W.u + m0 * sH, *x1 = w + W.x1 + m0 * sH, *g = w + W.g + m0 * sF;
    float* z = (float*)(w + W.z) + (size_t)m0 * B * c.classes;
    float* zpart = (float*)(w + W.zpart) + (size_t)m0 * (H / 64) * B * c.classes;
    const ArenaLayout& L = M->L;

#define SP_TRY(expr) do { if ((expr) != hipSuccess) return SP_EHIP; } while (0)
#define SP_MARK(ph) do { if (pt) pt->mark(ph, s); } while (0)
    // quantised students: the three large projections of the all-token layers on fp8 operands (large calls only)
    // (the fp8 kernel has one tile size, 256 x 256: widths that are not multiples of it stay on the bf16 path)
    const bool fp8 = c.dtype == SP_DTYPE_FP8 && mrows % 256 == 0 && mrows >= kFp8MinRows && W.xq && H % 256 == 0 &&
                     F % 256 == 0;
    const size_t qH = (size_t)rows * H, qF = (size_t)rows * F;       // bytes per student of the fp8 buffers
    char *xq = fp8 ? w + W.xq + m0 * qH : nullptr, *x1q = fp8 ? w + W.x1q + m0 * qH : nullptr;
    char *gq = fp8 ? w + W.gq + m0 * qF : nullptr, *attq = fp8 ? w + W.attq + m0 * qH : nullptr;
    SP_MARK(-1);
    SP_TRY(launch_embed_ln(M, ids, cu, B, T, rows, mrows, k, x, att, s, xq, kActQuantScale, attq));
    SP_MARK(SP_PHASE_EMBED);
    // Last layer on the first-token rows only (see sp_config.last_layer_all_tokens).  Not used by the partial
    // forwards of the tests unless they stop before the last layer.
    const bool first_only = !c.last_layer_all_tokens && with_head && T >= kFirstOnlyMinTokens &&
                            attention_first_fold_supported(c, max_seqlen);
    const int crows = W.crows;
    const int ctile = B > 256 ? 256 : (B > 64 ? 128 : 64);
    const int cmrows = (B + ctile - 1) / ctile * ctile;
    const int nh = c.heads;
    const size_t cH = (size_t)crows * H * ab, cF = (size_t)crows * F * ab, cHH = (size_t)crows * nh * H;   // cHH: elements
    char *cx = w + W.cx + m0 * cH, *cq = w + W.cq + m0 * cH, *catt = w + W.catt + m0 * cH, *cu2 = w + W.cu_ + m0 * cH;
    char *cx1 = w + W.cx1 + m0 * cH, *cg = w + W.cg + m0 * cF;
    char *cqt = w + W.cqt + m0 * cHH * ab, *cxb = w + W.cxb + m0 * cHH * ab;
    bool compact_final = false, small_head = false, first_tail = false;
    size_t small_head_lo = 0;
    int small_head_splits = 1;
    // Calls of a few dozen tokens: split the reduction range of the two projections that are followed by a LayerNorm
    // (largest slice count that leaves every slice at least two 64-wide k-tiles).
    const size_t slice = (size_t)kSplitRows * H;
    float* part = (float*)(w + W.part) + (size_t)m0 * kSplitMax * slice;
    int split_o = 1, split_d = 1;
    if (bf16_path(c) && mrows <= kSplitRows) {
        for (int sp = kSplitMax; sp > 1; --sp) {
            if (split_o == 1 && (H / 64) % sp == 0 && H / 64 / sp >= 2) split_o = sp;
            if (split_d == 1 && (F / 64) % sp == 0 && F / 64 / sp >= 2) split_d = sp;
        }
    }
    // the same for the first-token rows of the last layer when they are few (a batch of up to 128 sequences)
    int csplit_o = 1, csplit_d = 1;
    if (first_only && cmrows <= kSplitRows) {
        for (int sp = kSplitMax; sp > 1; --sp) {
            if (csplit_o == 1 && (H / 64) % sp == 0 && H / 64 / sp >= 2) csplit_o = sp;
            if (csplit_d == 1 && (F / 64) % sp == 0 && F / 64 / sp >= 2) csplit_d = sp;
        }
    }
    for (int l = 0; l < stop_layers; ++l) {
        const size_t lo = L.layer0 + (size_t)l * L.layer_stride;
        if (first_only && l == c.layers - 1) {
            SP_TRY(launch_gather_first(M, x, cu, B, T, rows, cx, catt, crows, cmrows, k, s));
            SP_MARK(SP_PHASE_LAST_FIRST);
            // queries of the first tokens, folded through the key projection: qt[b][h] = Wk[:, h] q[b][h]
            SP_TRY(launch_gemm(M, cx, H, lo + L.wqkv, lo + L.bqkv, cq, H, nullptr, 0, cmrows, H, H, k, EPI_BIAS, cH, cH, 0,
                               s));
            SP_TRY(launch_head_gemm(M, cq, (size_t)crows * H, 64, H, lo + L.wk_io, 64, H, 0, 0, false, cqt, cHH, H, nh * H,
                                    cmrows, H, 64, k, s));
            SP_MARK(SP_PHASE_LAST_FIRST);
            // p-weighted mean of the token rows per (sequence, head), then the value projection of those rows
            SP_TRY(launch_attention_first_fold(M, x, cqt, cxb, cu, B, T, max_seqlen, rows, crows, cmrows, k, s));
            SP_TRY(launch_head_gemm(M, cxb, cHH, H, nh * H, lo + L.wqkv + (size_t)2 * H * H * ab, (size_t)64 * H, H,
                                    lo + L.bqkv + (size_t)2 * H * 4, 64, true, catt, (size_t)crows * H, 64, H, cmrows, 64, H,
                                    k, s));
            SP_MARK(SP_PHASE_LAST_FIRST);
            if (csplit_o > 1) {
                // few rows: a 64-row tile walking the whole reduction range is a long serial chain; split it over
                // workgroups and add the slices together with bias, residual and LayerNorm
                SP_TRY(launch_gemm_splitk(M, catt, H, lo + L.wo, part, cmrows, H, H, k, csplit_o, cH, slice, s));
                SP_MARK(SP_PHASE_LAST_FIRST);
                SP_TRY(launch_ln_reduce(M, part, csplit_o, slice, lo + L.bo, cx, cx1, crows, cmrows, k, lo + L.ln1g,
                                        lo + L.ln1b, s));
            } else {
                SP_TRY(launch_gemm(M, catt, H, lo + L.wo, lo + L.bo, cu2, H, cx, H, cmrows, H, H, k, EPI_BIAS_RESIDUAL, cH,
                                   cH, cH, s));
                SP_MARK(SP_PHASE_LAST_FIRST);
                SP_TRY(launch_layernorm(M, cu2, cx1, crows, cmrows, k, lo + L.ln1g, lo + L.ln1b, s));
            }
            SP_MARK(SP_PHASE_LAST_FIRST);
            SP_TRY(launch_gemm(M, cx1, H, lo + L.w1, lo + L.b1, cg, F, nullptr, 0, cmrows, F, H, k, EPI_BIAS_GELU, cH, cF, 0,
                               s));
            SP_MARK(SP_PHASE_LAST_FIRST);
            if (csplit_d > 1) {
                SP_TRY(launch_gemm_splitk(M, cg, F, lo + L.w2, part, cmrows, H, F, k, csplit_d, cF, slice, s));
                SP_MARK(SP_PHASE_LAST_FIRST);
                SP_TRY(launch_ln_reduce(M, part, csplit_d, slice, lo + L.b2, cx1, cx, crows, cmrows, k, lo + L.ln2g,
                                        lo + L.ln2b, s));
            } else {
                SP_TRY(launch_gemm(M, cg, F, lo + L.w2, lo + L.b2, cu2, H, cx1, H, cmrows, H, F, k, EPI_BIAS_RESIDUAL, cF,
                                   cH, cH, s));
                SP_MARK(SP_PHASE_LAST_FIRST);
                SP_TRY(launch_layernorm(M, cu2, cx, crows, cmrows, k, lo + L.ln2g, lo + L.ln2b, s));
            }
            SP_MARK(SP_PHASE_LAST_FIRST);
            compact_final = true;
            continue;
        }
        if (fp8)
            SP_TRY(launch_gemm_fp8(M, xq, H, lo + L.wqkv8, lo + L.sqkv, lo + L.bqkv, kActQuantScale, qkv, 3 * H, nullptr, 0,
                                   mrows, 3 * H, H, k, EPI_QKV, qH, s3H, 0, s, vt, 2 * H, rows, sH, 1.f));
        else if (bf16_path(c))
            SP_TRY(launch_gemm(M, x, H, lo + L.wqkv, lo + L.bqkv, qkv, 3 * H, nullptr, 0, mrows, 3 * H, H, k, EPI_QKV,
                               sH, s3H, 0, s, vt, 2 * H, rows, sH));
        else
            SP_TRY(launch_gemm(M, x, H, lo + L.wqkv, lo + L.bqkv, qkv, 3 * H, nullptr, 0, mrows, 3 * H, H, k, EPI_BIAS,
                               sH, s3H, 0, s));
        SP_MARK(SP_PHASE_QKV);
        // (quantised students: the output projection reads the fp8 copy only, so a whole forward skips the bf16 one;
        // the partial forwards of the tests keep it)
        SP_TRY(launch_attention(M, qkv, vt, fp8 && with_head ? nullptr : att, cu, B, T, max_seqlen, rows, k, s, attq,
                                kActQuantScale));
        SP_MARK(SP_PHASE_ATTENTION);
        if (with_head && !c.last_layer_all_tokens && l == c.layers - 1 && m0 == 0 && first_rows_tail_supported(c, B)) {
            // last layer of a whole forward of a few sequences: from here on only their first-token rows are needed,
            // and those go through per-feature dot products instead of 64-row tiles.  Calls of up to 128 tokens: the
            // small-call head takes over from the raw down-projection (one slice); longer ones: pooler by dot
            // products as well, then the classifier kernel (the pooled rows sit behind the scratch).
            float* ut = part + (size_t)k * slice;           // behind the slice the head reads
            if (split_o > 1 && split_d > 1) {
                SP_TRY(launch_first_rows_tail(M, lo, att, x, x1, g, ut, part, slice, nullptr, cu, B, T, rows, k, s));
                small_head = true;
                small_head_lo = lo;
                small_head_splits = 1;
            } else {
                SP_TRY(launch_first_rows_tail(M, lo, att, x, x1, g, ut, nullptr, 0, ut + first_rows_tail_scratch_floats(c, k),
                                              cu, B, T, rows, k, s));
                first_tail = true;
            }
            SP_MARK(SP_PHASE_LAST_FIRST);
            continue;
        }
        if (split_o > 1) {
            // few tokens: the reduction range is split over workgroups, and the slices are added together with the
            // bias, the residual and the LayerNorm
            SP_TRY(launch_gemm_splitk(M, att, H, lo + L.wo, part, mrows, H, H, k, split_o, sH, slice, s));
            SP_MARK(SP_PHASE_OPROJ);
            SP_TRY(launch_ln_reduce(M, part, split_o, slice, lo + L.bo, x, x1, rows, mrows, k, lo + L.ln1g, lo + L.ln1b, s));
            SP_MARK(SP_PHASE_LAYERNORM);
        } else {
            if (fp8)
                SP_TRY(launch_gemm_fp8(M, attq, H, lo + L.wo8, lo + L.so, lo + L.bo, kActQuantScale, u, H, x, H, mrows, H, H,
                                       k, EPI_BIAS_RESIDUAL, qH, sH, sH, s, nullptr, 0, 0, 0, 1.f));
            else
                SP_TRY(launch_gemm(M, att, H, lo + L.wo, lo + L.bo, u, H, x, H, mrows, H, H, k, EPI_BIAS_RESIDUAL, sH, sH,
                                   sH, s));
            SP_MARK(SP_PHASE_OPROJ);
            SP_TRY(launch_layernorm(M, u, x1, rows, mrows, k, lo + L.ln1g, lo + L.ln1b, s, x1q, kActQuantScale));
            SP_MARK(SP_PHASE_LAYERNORM);
        }
        if (fp8)
            SP_TRY(launch_gemm_fp8(M, x1q, H, lo + L.w18, lo + L.s1, lo + L.b1, kActQuantScale, gq, F, nullptr, 0, mrows, F,
                                   H, k, EPI_BIAS_GELU, qH, qF, 0, s, nullptr, 0, 0, 0, kActQuantScale));
        else
            SP_TRY(launch_gemm(M, x1, H, lo + L.w1, lo + L.b1, g, F, nullptr, 0, mrows, F, H, k, EPI_BIAS_GELU, sH, sF, 0,
                               s));
        SP_MARK(SP_PHASE_FFN_UP);
        if (split_d > 1) {
            SP_TRY(launch_gemm_splitk(M, g, F, lo + L.w2, part, mrows, H, F, k, split_d, sF, slice, s));
            SP_MARK(SP_PHASE_FFN_DOWN);
            if (with_head && l == c.layers - 1 && m0 == 0) {
                // last layer of a whole forward: only the first-token rows go on, and the head rebuilds them from the
                // slices itself
                small_head = true;
                small_head_lo = lo;
                small_head_splits = split_d;
            } else {
                SP_TRY(launch_ln_reduce(M, part, split_d, slice, lo + L.b2, x1, x, rows, mrows, k, lo + L.ln2g, lo + L.ln2b, s));
                SP_MARK(SP_PHASE_LAYERNORM);
            }
        } else {
            if (fp8)
                SP_TRY(launch_gemm_fp8(M, gq, F, lo + L.w28, lo + L.s2, lo + L.b2, kActQuantScale, u, H, x1, H, mrows, H, F,
                                       k, EPI_BIAS_RESIDUAL, qF, sH, sH, s, nullptr, 0, 0, 0, 1.f));
            else
                SP_TRY(launch_gemm(M, g, F, lo + L.w2, lo + L.b2, u, H, x1, H, mrows, H, F, k, EPI_BIAS_RESIDUAL, sF, sH,
                                   sH, s));
            SP_MARK(SP_PHASE_FFN_DOWN);
            SP_TRY(launch_layernorm(M, u, x, rows, mrows, k, lo + L.ln2g, lo + L.ln2b, s, xq, kActQuantScale));
            SP_MARK(SP_PHASE_LAYERNORM);
        }
    }
    if (with_head) {
        if (compact_final) {
            // pooler as one more student-grouped projection (tanh epilogue) on the first-token rows, then the classifier
            // (into the pre-LayerNorm scratch rows, which are free by now: the queries and the attention output of the
            // first tokens stay readable after the call)
            SP_TRY(launch_gemm(M, cx, H, L.wp_t, L.bp, cu2, H, nullptr, 0, cmrows, H, H, k, EPI_BIAS_TANH, cH, cH, 0, s));
            SP_TRY(launch_head_classify(M, cu2, B, crows, k, z, logits, s));
        } else if (first_tail)
            SP_TRY(launch_head_classify(M, part + (size_t)k * slice + first_rows_tail_scratch_floats(c, k), B,
                                        first_rows_tail_pooled_rows(), k, z, logits, s, true));
        else if (small_head)
            SP_TRY(launch_head_small(M, part, small_head_splits, slice, small_head_lo + L.b2, x1, small_head_lo + L.ln2g,
                                     small_head_lo + L.ln2b, cu, B, T, rows, k, z, zpart, logits, s));
        else
            SP_TRY(launch_head(M, x, cu, B, T, rows, k, z, zpart, logits, s));
        SP_MARK(SP_PHASE_HEAD);
    }
#undef SP_MARK
#undef SP_TRY
    return SP_OK;
}

// Whole call: argument checks, then either all active students on the caller's stream, or, for large calls, two
// halves of them side by side: the first on the caller's stream, the second on the model's auxiliary stream (forked
// and joined with events, so the call stays asynchronous and capturable).  The matrix-core phases run at the
// package power limit while the bandwidth-bound phases leave most of it unused; two groups of students drift out
// of phase and fill each other's gaps (measured about 3 % on the burst workload; starting the second group late,
// after the first group's first projection, measured no better).  The logits are summed over all
// students in ascending order after the join, so the result does not depend on the grouping.
static int two_groups_min_tokens()
{
    static const int v = [] { const char* e = getenv("SP_TWO_GROUPS_MIN_TOKENS"); return e ? atoi(e) : 8192; }();
    return v;
}

static int run_forward(const sp_model* M, const int32_t* ids, const int32_t* cu, int B, int T, int max_seqlen, int k,
                       int stop_layers, bool with_head, void* ws, size_t ws_bytes, float* logits, hipStream_t s,
                       PhaseTimer* pt = nullptr)
{
    if (!M || !ids || !cu || !ws || (with_head && !logits)) return SP_EINVAL;
    if (((uintptr_t)ws & 255) || ((uintptr_t)ids & 3) || ((uintptr_t)cu & 3) || ((uintptr_t)logits & 3)) return SP_EINVAL;
    const sp_config& c = M->cfg;
    if (B < 1 || T < B || max_seqlen < 1 || max_seqlen > c.max_pos || (int64_t)B * max_seqlen < T) return SP_ESHAPE;
    if (k < 1 || k > c.K) return SP_EKACTIVE;
    if (stop_layers < 0 || stop_layers > c.layers) return SP_EINVAL;
    const WsLayout W = make_ws_layout(c, T, B);
    if (ws_bytes < W.end) return SP_ENOMEM;
    char* w = (char*)ws;

    const bool two_groups = with_head && !pt && k >= 2 && T >= two_groups_min_tokens() && !c.single_stream && M->aux;
    if (!two_groups)
        return run_students(M, W, ids, cu, B, T, max_seqlen, 0, k, stop_layers, with_head, w, logits, s, pt);

    const int ka = (k + 1) / 2;
    float* lpart = (float*)(w + W.lpart);
    const size_t n = (size_t)B * c.classes;
    std::lock_guard<std::mutex> hold(*M->mu);       // one fork/join at a time on the model's stream and events
    if (hipEventRecord(M->ev_fork, s) != hipSuccess || hipStreamWaitEvent(M->aux, M->ev_fork, 0) != hipSuccess)
        return SP_EHIP;
    int rc = run_students(M, W, ids, cu, B, T, max_seqlen, 0, ka, stop_layers, true, w, lpart, s, nullptr);
    const int rc2 = run_students(M, W, ids, cu, B, T, max_seqlen, ka, k - ka, stop_layers, true, w, lpart + n, M->aux,
                                 nullptr);
    // join even after an error, so that the auxiliary stream never runs on beyond the call
    if (hipEventRecord(M->ev_join, M->aux) != hipSuccess || hipStreamWaitEvent(s, M->ev_join, 0) != hipSuccess)
        return SP_EHIP;
    if (rc == SP_OK) rc = rc2;
    if (rc != SP_OK) return rc;
    if (launch_sum_students((const float*)(w + W.z), (int)n, k, logits, s) != hipSuccess) return SP_EHIP;
    return SP_OK;
}

// ---- workspace for callers that cannot allocate ---------------------------------------------------
// One array per GPU, part of the library's device image: every GPU the library runs on holds it until the process
// ends.  In host code the array's name is only a stand-in for the symbol; the device address is looked up once per
// device and everything on the host (kernel arguments included) goes through that pointer.
constexpr size_t kStaticScratchBytes = (size_t)SP_STATIC_SCRATCH_MIB << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::mutex scratch_mu;
static void* scratch_ptr[kMaxDevices];      // per device; null until looked up

// The current device's copy of the array (looked up on the first request for that device).
static int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SP_EHIP;
    if (dev < 0 || dev >= kMaxDevices) return SP_EINVAL;
    std::lock_guard<std::mutex> hold(scratch_mu);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SP_EHIP;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return SP_OK;
}

}  // namespace sp

using namespace sp;

extern "C" {

size_t sp_blob_floats(const sp_config* cfg)
{
    if (!config_ok(cfg)) return 0;
    return (size_t)cfg->K * student_blob_floats(*cfg);
}

size_t sp_arena_bytes(const sp_config* cfg)
{
    if (!config_ok(cfg)) return 0;
    return make_arena_layout(*cfg).student_stride * (size_t)cfg->K;
}

size_t sp_workspace_bytes(const sp_config* cfg, int32_t max_tokens, int32_t max_batch)
{
    if (!config_ok(cfg) || max_tokens < 1 || max_batch < 1) return 0;
    return make_ws_layout(*cfg, max_tokens, max_batch).end;
}

int sp_workspace_layout(const sp_config* cfg, int32_t total_tokens, int32_t batch, sp_ws_layout* out)
{
    if (!config_ok(cfg) || !out) return SP_EINVAL;
    if (total_tokens < 1 || batch < 1) return SP_ESHAPE;
    const WsLayout W = make_ws_layout(*cfg, total_tokens, batch);
    out->x = W.x; out->qkv = W.qkv; out->vt = W.vt; out->att = W.att; out->x1 = W.x1; out->g = W.g; out->z = W.z;
    out->rows = W.rows; out->act_bytes = W.act_bytes;
    out->first_q = W.cq; out->first_att = W.catt; out->first_rows = W.crows;
    out->xq = W.xq; out->x1q = W.x1q; out->gq = W.gq; out->attq = W.attq;
    return SP_OK;
}

int sp_load_students(const sp_config* cfg, const float* host_weights, size_t nfloats, void* device_arena,
                     size_t arena_bytes, void* hip_stream, sp_model** out)
{
    if (!config_ok(cfg) || !host_weights || !device_arena || !out) return SP_EINVAL;
    if ((uintptr_t)device_arena & 255) return SP_EINVAL;
    if (!config_supported(*cfg)) return SP_ESHAPE;
    const size_t per = student_blob_floats(*cfg);
    if (nfloats < per * (size_t)cfg->K) return SP_ENOMEM;
    const ArenaLayout L = make_arena_layout(*cfg);
    if (arena_bytes < L.student_stride * (size_t)cfg->K) return SP_ENOMEM;

    sp_model* m = new (std::nothrow) sp_model;
    if (!m) return SP_ENOMEM;
    m->cfg = *cfg; m->arena = (char*)device_arena; m->L = L;

    // Build the arena image on the host, a few students at a time, then upload.
    const int K = cfg->K;
    const int group = K < 4 ? K : 4;
    char* stage = (char*)calloc((size_t)group, L.student_stride);
    if (!stage) { delete m; return SP_ENOMEM; }
    hipStream_t s = (hipStream_t)hip_stream;
    int rc = SP_OK;
    for (int m0 = 0; m0 < K && rc == SP_OK; m0 += group) {
        const int n = m0 + group <= K ? group : K - m0;
        std::thread th[4];                  // (group <= 4); a thread that cannot be started is replaced by a plain call
        for (int i = 0; i < n; ++i) {
            try {
                th[i] = std::thread(fill_student, std::cref(*cfg), std::cref(L), host_weights + (size_t)(m0 + i) * per,
                                    stage + (size_t)i * L.student_stride);
            } catch (...) {
                fill_student(*cfg, L, host_weights + (size_t)(m0 + i) * per, stage + (size_t)i * L.student_stride);
            }
        }
        for (int i = 0; i < n; ++i)
            if (th[i].joinable()) th[i].join();
        if (hipMemcpyAsync((char*)device_arena + (size_t)m0 * L.student_stride, stage, (size_t)n * L.student_stride,
                           hipMemcpyHostToDevice, s) != hipSuccess || hipStreamSynchronize(s) != hipSuccess)
            rc = SP_EHIP;
    }
    free(stage);
    if (rc != SP_OK) { delete m; return rc; }
    // Auxiliary stream (default priority) and events for calls that run two groups of students side by side; without
    // them every call stays on the caller's stream.
    m->mu = new (std::nothrow) std::mutex;
    if (m->mu && hipStreamCreateWithFlags(&m->aux, hipStreamNonBlocking) == hipSuccess) {
        if (hipEventCreateWithFlags(&m->ev_fork, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&m->ev_join, hipEventDisableTiming) != hipSuccess) {
            if (m->ev_fork) (void)hipEventDestroy(m->ev_fork);
            (void)hipStreamDestroy(m->aux);
            m->aux = nullptr; m->ev_fork = m->ev_join = nullptr;
        }
    } else {
        m->aux = nullptr;
    }
    // this device's copy of the static workspace (sp_forward_static): looked up now, with the device current, so
    // that the calls themselves do nothing but enqueue kernels
    void* unused = nullptr;
    (void)static_scratch(&unused);
    *out = m;
    return SP_OK;
}

size_t sp_static_scratch_bytes(void) { return kStaticScratchBytes; }

int sp_forward_static(const sp_model* model, const int32_t* token_ids, const int32_t* cu_seqlens, int32_t batch,
                      int32_t total_tokens, int32_t max_seqlen, int32_t k_active, float* logits_out, void* hip_stream)
{
    if (!model) return SP_EINVAL;
    if (batch < 1 || total_tokens < batch) return SP_ESHAPE;
    // too large for the static array: refuse before anything is enqueued
    if (make_ws_layout(model->cfg, total_tokens, batch).end > kStaticScratchBytes) return SP_ETOOBIG;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != SP_OK) return rc;
    return run_forward(model, token_ids, cu_seqlens, batch, total_tokens, max_seqlen, k_active, model->cfg.layers,
                       true, ws, kStaticScratchBytes, logits_out, (hipStream_t)hip_stream);
}

int sp_forward(const sp_model* model, const int32_t* token_ids, const int32_t* cu_seqlens, int32_t batch,
               int32_t total_tokens, int32_t max_seqlen, int32_t k_active, void* workspace, size_t workspace_bytes,
               float* logits_out, void* hip_stream)
{
    if (!model) return SP_EINVAL;
    return run_forward(model, token_ids, cu_seqlens, batch, total_tokens, max_seqlen, k_active, model->cfg.layers,
                       true, workspace, workspace_bytes, logits_out, (hipStream_t)hip_stream);
}

int sp_forward_partial(const sp_model* model, const int32_t* token_ids, const int32_t* cu_seqlens, int32_t batch,
                       int32_t total_tokens, int32_t max_seqlen, int32_t k_active, int32_t stop_after_layers,
                       void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!model) return SP_EINVAL;
    return run_forward(model, token_ids, cu_seqlens, batch, total_tokens, max_seqlen, k_active, stop_after_layers,
                       false, workspace, workspace_bytes, nullptr, (hipStream_t)hip_stream);
}

int sp_forward_profiled(const sp_model* model, const int32_t* token_ids, const int32_t* cu_seqlens, int32_t batch,
                        int32_t total_tokens, int32_t max_seqlen, int32_t k_active, void* workspace,
                        size_t workspace_bytes, float* logits_out, void* hip_stream, float* phase_ms_host)
{
    if (!model || !phase_ms_host) return SP_EINVAL;
    PhaseTimer pt;
    hipStream_t s = (hipStream_t)hip_stream;
    int rc = run_forward(model, token_ids, cu_seqlens, batch, total_tokens, max_seqlen, k_active, model->cfg.layers,
                         true, workspace, workspace_bytes, logits_out, s, &pt);
    if (hipStreamSynchronize(s) != hipSuccess || !pt.ok) rc = rc == SP_OK ? SP_EHIP : rc;
    for (int i = 0; i < SP_PHASE_COUNT; ++i) phase_ms_host[i] = 0.f;
    if (rc == SP_OK)
        for (int i = 1; i < pt.n; ++i) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, pt.ev[i - 1], pt.ev[i]) != hipSuccess) { rc = SP_EHIP; break; }
            phase_ms_host[pt.phase[i]] += ms;
        }
    pt.release();
    return rc;
}

int sp_probe_e4m3(const float* x_host, int64_t n, uint8_t* codes_host)
{
    if (!x_host || !codes_host) return SP_EINVAL;
    if (n < 0) return SP_ESHAPE;
    for (int64_t i = 0; i < n; ++i) codes_host[i] = f32_to_e4m3(x_host[i]);
    return SP_OK;
}

int sp_probe_gelu(const float* x_device, float* y_device, int64_t n, void* hip_stream)
{
    if (!x_device || !y_device) return SP_EINVAL;
    if (n < 1 || n > ((int64_t)1 << 31)) return SP_ESHAPE;
    return launch_gelu_probe(x_device, y_device, (long)n, (hipStream_t)hip_stream) == hipSuccess ? SP_OK : SP_EHIP;
}

int sp_probe_gelu_fp8(const float* x_device, float* y_device, int64_t n, void* hip_stream)
{
    if (!x_device || !y_device) return SP_EINVAL;
    if (n < 1 || n > ((int64_t)1 << 31)) return SP_ESHAPE;
    return launch_gelu_q8_probe(x_device, y_device, (long)n, (hipStream_t)hip_stream) == hipSuccess ? SP_OK : SP_EHIP;
}

void sp_free(sp_model* model)
{
    if (!model) return;
    if (model->aux) {
        (void)hipStreamSynchronize(model->aux);
        (void)hipEventDestroy(model->ev_fork);
        (void)hipEventDestroy(model->ev_join);
        (void)hipStreamDestroy(model->aux);
    }
    delete model->mu;
    delete model;
}

const char* sp_strerror(int code)
{
    switch (code) {
        case SP_OK: return "ok";
        case SP_EINVAL: return "invalid argument (null or misaligned pointer, malformed config)";
        case SP_ESHAPE: return "unsupported or inconsistent shape";
        case SP_EKACTIVE: return "k_active outside 1..K";
        case SP_ENOMEM: return "buffer smaller than required";
        case SP_EHIP: return "HIP runtime error";
        case SP_ETOOBIG: return "call too large for the library's static workspace (use sp_forward with a workspace of your own)";
        case SP_EFULL: return "length-aware buffer storage full";
        case SP_EEMPTY: return "length-aware buffer empty";
        default: return "unknown error code";
    }
}

int sp_check_inputs(const sp_model* model, const int32_t* token_ids, const int32_t* cu_seqlens, int32_t batch,
                    int32_t total_tokens, int32_t max_seqlen, void* scratch, void* hip_stream, int32_t* problems_host)
{
    if (!model || !token_ids || !cu_seqlens || !scratch || !problems_host || ((uintptr_t)scratch & 3)) return SP_EINVAL;
    if (batch < 1 || total_tokens < batch || max_seqlen < 1 || max_seqlen > model->cfg.max_pos) return SP_ESHAPE;
    hipStream_t s = (hipStream_t)hip_stream;
    if (sp::launch_check_inputs(token_ids, cu_seqlens, batch, total_tokens, max_seqlen, model->cfg.vocab,
                                (unsigned*)scratch, s) != hipSuccess)
        return SP_EHIP;
    unsigned flags = 0;
    if (hipMemcpyAsync(&flags, scratch, sizeof flags, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return SP_EHIP;
    *problems_host = (int32_t)flags;
    return SP_OK;
}

int sp_pack(const int32_t* lengths_host, int32_t batch, int32_t* cu_seqlens_host)
{
    if (!lengths_host || !cu_seqlens_host) return SP_EINVAL;
    if (batch < 1) return SP_ESHAPE;
    int64_t acc = 0;
    cu_seqlens_host[0] = 0;
    for (int32_t i = 0; i < batch; ++i) {
        if (lengths_host[i] < 1) return SP_ESHAPE;
        acc += lengths_host[i];
        if (acc > INT32_MAX) return SP_ESHAPE;
        cu_seqlens_host[i + 1] = (int32_t)acc;
    }
    return SP_OK;
}

}  // extern "C"
