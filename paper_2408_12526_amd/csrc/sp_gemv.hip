// Last layer of a call of a few sequences, after its attention: only the first token of each sequence feeds the head
// (the pooled representation of Section 3.1), so the attention-output projection, the FFN and their LayerNorms are
// needed for one row per sequence.  A 64-row projection tile would compute 63 dead rows per sequence and walk the
// reduction range as a serial chain of k-tiles in a few dozen workgroups; here every output feature of those rows is a
// dot product of its own: one wave per few features reads its weight rows in one round trip (weights are stored
// [out][in], the reduction index contiguous), all waves of the chip at once.  Three launches:
//   first_o_kernel:     u[b]  = att[first token of b] . Wo^T + bo + x[first token of b]                (fp32)
//   first_up_kernel:    x1[b] = LN(u[b]; ln1) (each wave normalises the rows for itself: 768 values), written once as
//                       bf16 into the x1 row of the first token; g[b] = gelu(x1[b] . W1^T + b1)              (bf16)
//   first_down_kernel:  g[b] . W2^T, raw, into slice 0 of the split-reduction buffer at the first token's row: the
//                       small-call head (head_small_kernel) adds bias and residual, normalises, pools and classifies
//                       (calls of up to 128 tokens, whose other layers use that buffer and that head anyway);
//                       or, for longer calls, u2[b] = g[b] . W2^T + b2 + x1[b] (fp32), followed by
//   first_pool_kernel:  pooled[b] = tanh(LN(u2[b]; ln2) . Wp^T + bp) (fp32), the classifier kernel's input.
// Rounding points are those of the small-call path: operands bf16, accumulation fp32, x1, g and the final hidden state
// rounded to bf16.
#include "sp_internal.h"

namespace sp {

namespace {

constexpr int kFirstMaxSeqs = 4;

__device__ inline void unpack8(const bf16x8 v, float (&f)[8])
{
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = (float)v[e];
}

__device__ inline int first_row(const int32_t* cu, int b, int Tn)
{
    const int r = cu[b];
    return r < 0 ? 0 : (r >= Tn ? Tn - 1 : r);
}

// acc[f][b] = sum over this lane's chunks of W[n0 + f][chunk] . a[b][chunk]; lane l owns the 8-element chunks
// l + 64 i, i < MAXCH, of the reduction range.  Every weight chunk of the wave is requested before the first is used.
template <int NPW, int MAXCH, int NB>
__device__ inline void dot_rows(const bf16* __restrict__ W, int ldw, int n0, int nch, int lane, int B,
                                const bf16x8 (&a)[NB][MAXCH], float (&acc)[NPW][NB])
{
    bf16x8 w[NPW][MAXCH];
#pragma unroll
    for (int f = 0; f < NPW; ++f)
#pragma unroll
        for (int i = 0; i < MAXCH; ++i) {
            const int c = lane + 64 * i;
            if (c < nch) w[f][i] = *(const bf16x8*)(W + (size_t)(n0 + f) * ldw + c * 8);
        }
#pragma unroll
    for (int f = 0; f < NPW; ++f)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[f][b] = 0.f;
#pragma unroll
    for (int f = 0; f < NPW; ++f)
#pragma unroll
        for (int i = 0; i < MAXCH; ++i) {
            if (lane + 64 * i < nch) {
                float wf[8];
                unpack8(w[f][i], wf);
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    if (b < B) {
                        float af[8];
                        unpack8(a[b][i], af);
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[f][b] = __builtin_fmaf(wf[e], af[e], acc[f][b]);
                    }
            }
        }
#pragma unroll
    for (int f = 0; f < NPW; ++f)
#pragma unroll
        for (int b = 0; b < NB; ++b)
            if (b < B) acc[f][b] = wave_sum(acc[f][b]);
}

// rows of a bf16 activation buffer, one per sequence: row index first_row(b) (token rows) or b (compact rows)
template <int MAXCH, int NB>
__device__ inline void load_rows(const bf16* __restrict__ src, int ld, const int32_t* cu, int B, int Tn, bool token_rows,
                                 int nch, int lane, bf16x8 (&a)[NB][MAXCH])
{
#pragma unroll
    for (int b = 0; b < NB; ++b)
        if (b < B) {
            const bf16* row = src + (size_t)(token_rows ? first_row(cu, b, Tn) : b) * ld;
#pragma unroll
            for (int i = 0; i < MAXCH; ++i) {
                const int c = lane + 64 * i;
                if (c < nch) a[b][i] = *(const bf16x8*)(row + c * 8);
            }
        }
}

constexpr int kNpwO = 2, kNpwUp = 4, kNpwDown = 1, kNpwPool = 2;   // output features per wave

// a[b] = bf16(LN(u[b]; gamma, beta)) for this lane's chunks of the rows u[b] (fp32, H values each).  Every wave does this
// for itself: a row is 768-1024 values, the statistics are two wave reductions.
template <int NB>
__device__ inline void layernorm_rows(const float* __restrict__ u, const float* __restrict__ gam,
                                      const float* __restrict__ bet, float eps, int H, int B, int lane,
                                      bf16x8 (&a)[NB][2])
{
    const int nch = H >> 3;
    const float inv_h = __builtin_amdgcn_rcpf((float)H);
#pragma unroll
    for (int b = 0; b < NB; ++b)
        if (b < B) {
            const float* row = u + (size_t)b * H;
            float v[2][8];
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int c = lane + 64 * i;
#pragma unroll
                for (int e = 0; e < 8; ++e) v[i][e] = 0.f;
                if (c < nch) {
                    const f32x4 lo = *(const f32x4*)(row + c * 8), hi = *(const f32x4*)(row + c * 8 + 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) { v[i][e] = lo[e]; v[i][4 + e] = hi[e]; }
#pragma unroll
                    for (int e = 0; e < 8; ++e) s += v[i][e];
                }
            }
            const float mean = wave_sum(s) * inv_h;
            float q = 0.f;
#pragma unroll
            for (int i = 0; i < 2; ++i)
                if (lane + 64 * i < nch)
#pragma unroll
                    for (int e = 0; e < 8; ++e) { const float d = v[i][e] - mean; q += d * d; }
            const float inv = __builtin_amdgcn_rsqf(wave_sum(q) * inv_h + eps);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int c = lane + 64 * i;
                if (c < nch) {
                    const f32x4 g0 = *(const f32x4*)(gam + c * 8), g1 = *(const f32x4*)(gam + c * 8 + 4);
                    const f32x4 b0 = *(const f32x4*)(bet + c * 8), b1 = *(const f32x4*)(bet + c * 8 + 4);
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        a[b][i][e] = (bf16)((e < 4 ? g0[e] : g1[e - 4]) * ((v[i][e] - mean) * inv) + (e < 4 ? b0[e] : b1[e - 4]));
                }
            }
        }
}


// (NB: the most sequences an instance handles, 1 or kFirstMaxSeqs; a call of one sequence keeps a quarter of the rows in
// registers and runs at a higher occupancy)
// u[m][b][n] = att[m][first token of b] . Wo[n] + bo[n] + x[m][first token of b][n]
template <int NB>
__global__ __launch_bounds__(256) void first_o_kernel(const char* __restrict__ arena, size_t student_stride, size_t w_off,
                                                      size_t b_off, const bf16* __restrict__ att,
                                                      const bf16* __restrict__ x, int rows,
                                                      const int32_t* __restrict__ cu, int B, int Tn, int H,
                                                      float* __restrict__ u)
{
    const int m = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n0 = (blockIdx.x * 4 + wave) * kNpwO;
    if (n0 >= H) return;
    const char* sb = arena + (size_t)m * student_stride;
    bf16x8 a[NB][2];
    load_rows<2, NB>(att + (size_t)m * rows * H, H, cu, B, Tn, true, H >> 3, lane, a);
    float acc[kNpwO][NB];
    dot_rows<kNpwO, 2, NB>((const bf16*)(sb + w_off), H, n0, H >> 3, lane, B, a, acc);
    if (lane < kNpwO * NB) {
        const int f = lane / NB, b = lane % NB;
        if (b < B) {
            float v = 0.f;
#pragma unroll
            for (int ff = 0; ff < kNpwO; ++ff)
#pragma unroll
                for (int bb = 0; bb < NB; ++bb)
                    if (ff == f && bb == b) v = acc[ff][bb];
            const int n = n0 + f;
            v += ((const float*)(sb + b_off))[n] + (float)x[((size_t)m * rows + first_row(cu, b, Tn)) * H + n];
            u[((size_t)m * kFirstMaxSeqs + b) * H + n] = v;
        }
    }
}

// x1[m][first token of b] = LN(u[m][b]) (bf16); g[m][b][n] = gelu(x1 . W1[n] + b1[n]) (bf16)
template <int NB>
__global__ __launch_bounds__(256) void first_up_kernel(const char* __restrict__ arena, size_t student_stride, size_t w_off,
                                                       size_t b_off, size_t g_off, size_t beta_off, float eps,
                                                       const float* __restrict__ u, bf16* __restrict__ x1, int rows,
                                                       const int32_t* __restrict__ cu, int B, int Tn, int H, int F,
                                                       bf16* __restrict__ g, int ldg)
{
    const int m = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n0 = (blockIdx.x * 4 + wave) * kNpwUp;
    if (n0 >= F) return;
    const char* sb = arena + (size_t)m * student_stride;
    const int nch = H >> 3;
    const float* gam = (const float*)(sb + g_off);
    const float* bet = (const float*)(sb + beta_off);
    bf16x8 a[NB][2];
    layernorm_rows<NB>(u + (size_t)m * kFirstMaxSeqs * H, gam, bet, eps, H, B, lane, a);
    // the rows once more for what adds them as the residual of the down-projection
    if (blockIdx.x == 0 && wave == 0) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
            if (b < B)
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    if (lane + 64 * i < nch)
                        *(bf16x8*)(x1 + ((size_t)m * rows + first_row(cu, b, Tn)) * H + (lane + 64 * i) * 8) = a[b][i];
    }
    float acc[kNpwUp][NB];
    dot_rows<kNpwUp, 2, NB>((const bf16*)(sb + w_off), H, n0, nch, lane, B, a, acc);
    if (lane < kNpwUp * NB) {
        const int f = lane / NB, b = lane % NB;
        if (b < B) {
            float v = 0.f;
#pragma unroll
            for (int ff = 0; ff < kNpwUp; ++ff)
#pragma unroll
                for (int bb = 0; bb < NB; ++bb)
                    if (ff == f && bb == b) v = acc[ff][bb];
            const int n = n0 + f;
            g[((size_t)m * rows + b) * ldg + n] = (bf16)gelu_erf_fast(v + ((const float*)(sb + b_off))[n]);
        }
    }
}

// RAW:  part[m][first token of b][n] = g[m][b] . W2[n]                 (the small-call head adds bias and residual)
// else: u2[m][b][n] = g[m][b] . W2[n] + b2[n] + x1[m][first token of b][n]     (out = u2, out_ss = kFirstMaxSeqs * H)
template <int NB, bool RAW>
__global__ __launch_bounds__(256) void first_down_kernel(const char* __restrict__ arena, size_t student_stride,
                                                         size_t w_off, size_t b_off, const bf16* __restrict__ g, int ldg,
                                                         const bf16* __restrict__ x1, int rows,
                                                         const int32_t* __restrict__ cu, int B, int Tn, int H, int F,
                                                         float* __restrict__ out, size_t out_ss)
{
    const int m = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n0 = (blockIdx.x * 4 + wave) * kNpwDown;
    if (n0 >= H) return;
    const char* sb = arena + (size_t)m * student_stride;
    bf16x8 a[NB][8];
    load_rows<8, NB>(g + (size_t)m * rows * ldg, ldg, cu, B, Tn, false, F >> 3, lane, a);
    float acc[kNpwDown][NB];
    dot_rows<kNpwDown, 8, NB>((const bf16*)(sb + w_off), F, n0, F >> 3, lane, B, a, acc);
    if (lane < NB && lane < B) {
        float v = 0.f;
#pragma unroll
        for (int bb = 0; bb < NB; ++bb)
            if (bb == lane) v = acc[0][bb];
        const int r = first_row(cu, lane, Tn);
        if (RAW)
            out[(size_t)m * out_ss + (size_t)r * H + n0] = v;
        else
            out[(size_t)m * out_ss + (size_t)lane * H + n0] =
                v + ((const float*)(sb + b_off))[n0] + (float)x1[((size_t)m * rows + r) * H + n0];
    }
}

// pooled[m][b][n] = tanh(LN(u2[m][b]; ln2) . Wp[n] + bp[n])   (fp32 [k][kFirstMaxSeqs][H], as the small-call head keeps it)
template <int NB>
__global__ __launch_bounds__(256) void first_pool_kernel(const char* __restrict__ arena, size_t student_stride,
                                                         size_t w_off, size_t b_off, size_t g_off, size_t beta_off,
                                                         float eps, const float* __restrict__ u2, int B, int H,
                                                         float* __restrict__ pooled)
{
    const int m = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n0 = (blockIdx.x * 4 + wave) * kNpwPool;
    if (n0 >= H) return;
    const char* sb = arena + (size_t)m * student_stride;
    bf16x8 a[NB][2];
    layernorm_rows<NB>(u2 + (size_t)m * kFirstMaxSeqs * H, (const float*)(sb + g_off), (const float*)(sb + beta_off), eps,
                       H, B, lane, a);
    float acc[kNpwPool][NB];
    dot_rows<kNpwPool, 2, NB>((const bf16*)(sb + w_off), H, n0, H >> 3, lane, B, a, acc);
    if (lane < kNpwPool * NB) {
        const int f = lane / NB, b = lane % NB;
        if (b < B) {
            float v = 0.f;
#pragma unroll
            for (int ff = 0; ff < kNpwPool; ++ff)
#pragma unroll
                for (int bb = 0; bb < NB; ++bb)
                    if (ff == f && bb == b) v = acc[ff][bb];
            const int n = n0 + f;
            pooled[((size_t)m * kFirstMaxSeqs + b) * H + n] = tanhf(v + ((const float*)(sb + b_off))[n]);
        }
    }
}

}  // namespace

bool first_rows_tail_supported(const sp_config& c, int B)
{
    return bf16_path(c) && B >= 1 && B <= kFirstMaxSeqs && c.hidden % 8 == 0 && c.hidden <= 1024 && c.ffn % 8 == 0 &&
           c.ffn <= 4096 && c.hidden % kNpwO == 0 && c.ffn % kNpwUp == 0 && c.hidden % kNpwPool == 0;
}

size_t first_rows_tail_scratch_floats(const sp_config& c, int k) { return (size_t)2 * k * kFirstMaxSeqs * c.hidden; }
int first_rows_tail_pooled_rows() { return kFirstMaxSeqs; }

hipError_t launch_first_rows_tail(const sp_model* M, size_t lo, const void* att, const void* x, void* x1, void* g,
                                  float* scratch, float* part, size_t part_ss, float* pooled, const int32_t* cu, int B,
                                  int T, int rows, int k, hipStream_t s)
{
    const sp_config& c = M->cfg;
    const ArenaLayout& L = M->L;
    if (!first_rows_tail_supported(c, B) || rows < kFirstMaxSeqs || (part == nullptr) == (pooled == nullptr))
        return hipErrorInvalidValue;
    const int H = c.hidden, F = c.ffn;
    float* u = scratch;
    float* u2 = scratch + (size_t)k * kFirstMaxSeqs * H;
#define SP_LAUNCH(KERN, NPW, N, ...)                                                                                \
    do {                                                                                                            \
        hipLaunchKernelGGL(KERN, dim3((unsigned)(((N) / (NPW) + 3) / 4), (unsigned)k), dim3(256), 0, s, M->arena,   \
                           L.student_stride, __VA_ARGS__);                                                          \
        const hipError_t e = hipGetLastError();                                                                     \
        if (e != hipSuccess) return e;                                                                              \
    } while (0)
#define SP_FIRST_TAIL(NB)                                                                                           \
    do {                                                                                                            \
        SP_LAUNCH(first_o_kernel<NB>, kNpwO, H, lo + L.wo, lo + L.bo, (const bf16*)att, (const bf16*)x, rows, cu, B, \
                  T, H, u);                                                                                         \
        SP_LAUNCH(first_up_kernel<NB>, kNpwUp, F, lo + L.w1, lo + L.b1, lo + L.ln1g, lo + L.ln1b, c.ln_eps,          \
                  (const float*)u, (bf16*)x1, rows, cu, B, T, H, F, (bf16*)g, F);                                   \
        if (part) {                                                                                                 \
            SP_LAUNCH((first_down_kernel<NB, true>), kNpwDown, H, lo + L.w2, lo + L.b2, (const bf16*)g, F,           \
                      (const bf16*)x1, rows, cu, B, T, H, F, part, part_ss);                                        \
        } else {                                                                                                    \
            SP_LAUNCH((first_down_kernel<NB, false>), kNpwDown, H, lo + L.w2, lo + L.b2, (const bf16*)g, F,          \
                      (const bf16*)x1, rows, cu, B, T, H, F, u2, (size_t)kFirstMaxSeqs * H);                        \
            SP_LAUNCH(first_pool_kernel<NB>, kNpwPool, H, L.wp_t, L.bp, lo + L.ln2g, lo + L.ln2b, c.ln_eps,          \
                      (const float*)u2, B, H, pooled);                                                 \
        }                                                                                                           \
    } while (0)
    if (B == 1) SP_FIRST_TAIL(1);
    else SP_FIRST_TAIL(kFirstMaxSeqs);
#undef SP_FIRST_TAIL
#undef SP_LAUNCH
    return hipSuccess;
}

}  // namespace sp
