// Internal declarations shared by the translation units of libsp_mi355x.so.
// Nothing here is part of the C ABI (that is include/sp.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "sp.h"

namespace sp {

// SP_DTYPE_FP8 is the bf16 path with fp8 copies of the four projection matrices: everything that asks "bf16 or fp32
// storage" treats the two alike.
inline bool bf16_path(const sp_config& c) { return c.dtype != SP_DTYPE_FP32; }

typedef __bf16 bf16;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#if defined(__HIPCC__)
// ---- device helpers shared by the projection kernels ---------------------------------------------
// GELU (erf form) for outputs that are rounded to bf16 afterwards, written with the complementary error function:
//   gelu(x) = x (1 + erf(x / sqrt 2)) / 2 = max(x, 0) - |x| erfc(|x| / sqrt 2) / 2,
//   log2 erfc(z) = z Q(z) on [0, 4.3], Q a degree-5 minimax fit (weighted for the absolute error of gelu);
//   erfc(4.3) = 1.2e-9, so |x| is clamped at 4.3 sqrt 2 (in the erfc term only: beyond it the term stays below 4e-9
//   instead of growing with |x|).
// Evaluated in fp32 the result is within 3.2e-7 of the exact function for every x (0.03 bf16 ulp at most where
// |gelu| > 1e-3).  One quarter-rate instruction (exp2) and nine full-rate ones: the epilogue of the FFN
// up-projection is bound by these vector instructions while the matrix cores wait (libm's erff costs several times
// more; the rational-exponential formula 7.1.26 of Abramowitz & Stegun needs a reciprocal as well).  To get there:
//   * the polynomial is in a = |x| directly (coefficient i carries 2^(-(i + 1) / 2)), so z is never formed, and the
//     halving of erfc rides in the exponent: |x| erfc / 2 = a 2^(a Q'(a) - 1), the -1 being the addend of the
//     multiply-add that forms the exponent;
//   * clamps are median-of-three instructions (one each for the clamp of x and for max(x, 0), the latter with the
//     largest finite float as its upper bound: fminf / fmaxf, and a median with an infinite bound, which the
//     compiler rewrites as one of them, cost a second instruction that quiets signalling NaNs first); |.| is an
//     operand modifier.
__device__ inline float gelu_erf_fast(float x)
{
    const float a = __builtin_fabsf(__builtin_amdgcn_fmed3f(x, -6.0811f, 6.0811f));
    float q = __builtin_fmaf(2.992383634e-05f, a, -7.398715825e-04f);
    q = __builtin_fmaf(q, a, 7.977455854e-03f);
    q = __builtin_fmaf(q, a, -5.323817581e-02f);
    q = __builtin_fmaf(q, a, -4.589156806e-01f);
    q = __builtin_fmaf(q, a, -1.151147127e+00f);
    const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(q, a, -1.0f));
    return __builtin_fmaf(-a, e, __builtin_amdgcn_fmed3f(x, 0.0f, 3.402823466e+38f));
}

// The same function where the result is stored as an e4m3 code (three mantissa bits: steps of 2^-4 relative): the
// exponent is a cubic, log2(erfc(a / sqrt 2) / 2) ~ -1 + a (c0 + a (c1 + a c2)), fitted (minimax in the error of
// the function value) on [0, 4.5]; all three coefficients are negative, so it keeps falling beyond the fitted range and
// needs no clamp.  Within 8.6e-5 of the erf form everywhere, a thirtieth of the e4m3 step at the function's minimum
// (-0.17): four multiply-adds, one median and the exponential.
// The scaled form returns s gelu(y / s) for y = s x, with the coefficients divided by s, s^2, s^3 by the caller
// (gelu_q8_coefficients): the scale of the quantised output then costs no instruction per value.
constexpr float kGeluQ8C0 = -1.140919014e+00f, kGeluQ8C1 = -4.882554528e-01f, kGeluQ8C2 = -2.763128887e-02f;
__device__ inline float gelu_erf_q8_scaled(float y, float k0, float k1, float k2)
{
    const float a = __builtin_fabsf(y);
    float q = __builtin_fmaf(k2, a, k1);
    q = __builtin_fmaf(q, a, k0);
    const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(q, a, -1.0f));
    return __builtin_fmaf(-a, e, __builtin_amdgcn_fmed3f(y, 0.0f, 3.402823466e+38f));
}
__device__ inline float gelu_erf_q8(float x) { return gelu_erf_q8_scaled(x, kGeluQ8C0, kGeluQ8C1, kGeluQ8C2); }

// ---- reductions over the 64 lanes of a wave, result in every lane -------------------------------------------------
// Inside a row of 16 lanes the second operand of each step comes through the data-parallel-primitive path of the
// instruction itself (neighbour in the pair, other pair of the quad, mirror image in the half row, mirror image in the
// row: after each step every lane of the growing group holds the group's result); rows 0|1 and 2|3, then the two halves
// of the wave, are exchanged by the row / half swap instructions (both operands hold the value; afterwards one has the
// even rows' (lower half's) data in every row (half), the other the odd rows' (upper half's)).  Eight instructions
// where six general lane permutations through LDS (`__shfl_xor`) take about forty, and no LDS round trips on the
// critical path.  Every lane of the wave must be active.  (The swaps are inline assembly with the two idle issue slots
// the hardware wants after a vector write of their operands: this toolchain's builtins return their first result
// twice.)
template <int CTRL>
__device__ inline float dpp_moved(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ inline void swap_rows(float& a, float& b)       // odd rows of a <-> even rows of b
{
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ inline void swap_halves(float& a, float& b)     // lanes 32-63 of a <-> lanes 0-31 of b
{
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
constexpr int kDppPair = 0xB1, kDppQuad = 0x4E, kDppHalfRowMirror = 0x141, kDppRowMirror = 0x140;
__device__ inline float wave_sum(float v)
{
    v += dpp_moved<kDppPair>(v);           // quad_perm [1, 0, 3, 2]
    v += dpp_moved<kDppQuad>(v);           // quad_perm [2, 3, 0, 1]
    v += dpp_moved<kDppHalfRowMirror>(v);
    v += dpp_moved<kDppRowMirror>(v);
    float a = v, b = v;
    swap_rows(a, b);
    v = a + b;
    a = v;
    b = v;
    swap_halves(a, b);
    return a + b;
}
__device__ inline float wave_max(float v)
{
    v = __builtin_fmaxf(v, dpp_moved<kDppPair>(v));
    v = __builtin_fmaxf(v, dpp_moved<kDppQuad>(v));
    v = __builtin_fmaxf(v, dpp_moved<kDppHalfRowMirror>(v));
    v = __builtin_fmaxf(v, dpp_moved<kDppRowMirror>(v));
    float a = v, b = v;
    swap_rows(a, b);
    v = __builtin_fmaxf(a, b);
    a = v;
    b = v;
    swap_halves(a, b);
    return __builtin_fmaxf(a, b);
}

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_void;

template <int N>
__device__ inline void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// Workgroup barrier that waits for this wave's LDS traffic only.  (__syncthreads() also waits for every
// outstanding global load, which would serialise the loads that are deliberately left in flight across it.)
__device__ inline void barrier_lds()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

#endif  // __HIPCC__

constexpr int kRowPad = 256;  // activation rows per student are padded to a multiple of this
constexpr int kSplitMax = 8;  // slices of a split reduction (small calls only)
constexpr int kSplitRows = 128;   // most token rows a call may compute and still take the split path
constexpr int kFirstOnlyMinTokens = 1024;   // smallest call whose last layer runs on the first-token rows only
// fp8 projections: activations are quantised as e4m3(value * kActQuantScale) by the kernel that produces them
// (LayerNorm outputs and GELU outputs are of order one: 448 / 16 = 28 before saturation, 2^-6 / 16 = 1e-3 before the
// subnormal range), and only calls that compute at least kFp8MinRows rows use them
constexpr float kActQuantScale = 16.f;
constexpr int kFp8MinRows = 2048;

// Byte offsets of every tensor inside one student's slab of the weight arena.
// The encoder matrices are stored transposed with respect to the host blob,
// [out][in], so that the reduction index is contiguous for both GEMM operands;
// the pooler and classifier matrices keep the blob's [in][out] order.
struct ArenaLayout {
    size_t tok, pos, emb_g, emb_b;
    size_t layer0, layer_stride;
    // relative to the start of a layer
    size_t wqkv, bqkv, wo, bo, ln1g, ln1b, w1, b1, w2, b2, ln2g, ln2b;
    size_t wk_io;                  // the key projection once more, [in][out] as in the host blob (folded first-token queries)
    // SP_DTYPE_FP8 only (0 otherwise), relative to the start of a layer: the fused q|k|v, attention-output, FFN-up and
    // FFN-down matrices once more as e4m3 codes, [out][in] bytes, and their per-output-feature scales (fp32)
    size_t wqkv8, sqkv, wo8, so, w18, s1, w28, s2;
    size_t wp, wp_t, bp, wc, bc;   // wp: [in][out] (column-parallel head kernel); wp_t: [out][in] (GEMM operand)
    size_t student_stride;
};

ArenaLayout make_arena_layout(const sp_config& c);

// Workspace carve-up for one call.
struct WsLayout {
    size_t x, qkv, vt, att, u, x1, g, z, zpart, end;
    size_t cx, cq, catt, cu_, cx1, cg;   // first-token rows only: [K][crows][H] (cg: [F]), last layer
    size_t cqt, cxb;                     // folded queries / weighted mean rows: [K][crows][heads][H]
    size_t part;                         // fp32 partial sums of split reductions: [K][kSplitMax][kSplitRows][H]
    size_t lpart;                        // per-group logit sums when two groups of students run side by side: [2][B][C]
    size_t xq, x1q, attq, gq;            // SP_DTYPE_FP8 only: fp8 copies of x, x1 and att ([K][rows][H] bytes), fp8 g ([K][rows][F])
    int rows, crows;
    int act_bytes;
};
WsLayout make_ws_layout(const sp_config& c, int total_tokens, int batch);

}  // namespace sp

struct sp_model {
    sp_config cfg;
    char* arena;
    sp::ArenaLayout L;
    // for calls that run two groups of students side by side (null: never)
    hipStream_t aux = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    std::mutex* mu = nullptr;
};

namespace sp {

// ---- launchers (each returns the hipError_t of its launch) ------------------

// X[m][row][:] = LN(tok[id[row]] + pos[row - cu[seq(row)]]) for row < T; zero rows up to `rows`.
// Rows T..mrows of x and of att are zeroed.
// xq (may be null): the rows once more as fp8 (e4m3) codes of value * qscale, [m][rows][H] bytes; attq (may be
// null): fp8 attention output buffer of the same shape, whose rows T..mrows are zeroed like those of att.
hipError_t launch_embed_ln(const sp_model* M, const int32_t* ids, const int32_t* cu, int B, int T, int rows,
                           int mrows, int k, void* x, void* att, hipStream_t s, void* xq = nullptr, float qscale = 1.f,
                           void* attq = nullptr);

// out[m][row][:] = LN(u[m][row][:]; g, b); g/b are byte offsets into the student slab.
hipError_t launch_layernorm(const sp_model* M, const void* u, void* out, int rows, int mrows, int k, size_t g_off,
                            size_t b_off, hipStream_t s, void* outq = nullptr, float qscale = 1.f);

// EPI_QKV (bf16 path only): bias; output columns >= n_split (the value projection) are written transposed,
// out2[m][column - n_split][row], so that attention reads key-contiguous value tiles.
enum Epilogue { EPI_BIAS = 0, EPI_BIAS_GELU = 1, EPI_BIAS_RESIDUAL = 2, EPI_QKV = 3, EPI_BIAS_TANH = 4, EPI_PARTIAL = 5 };

// out[m][row][0..N) = epi(A[m][row][0..Kd) . W^T + bias), W stored [N][Kd] at w_off of each student.
// lda / ldo / ldr are row strides in elements; residual may be null unless EPI_BIAS_RESIDUAL;
// mrows (a multiple of 64, <= the padded row count) is how many rows are computed.
hipError_t launch_gemm(const sp_model* M, const void* A, int lda, size_t w_off, size_t b_off, void* out, int ldo,
                       const void* residual, int ldr, int mrows, int N, int Kd, int k, Epilogue epi,
                       size_t a_student_stride, size_t o_student_stride, size_t r_student_stride, hipStream_t s,
                       void* out2 = nullptr, int n_split = 0, int ld2 = 0, size_t o2_student_stride = 0);

// The same projection on fp8 operands (SP_DTYPE_FP8; 256 x 256 tile only: mrows and N multiples of 256, Kd of 128).
// A8: e4m3 codes of activation * a_qscale, [m][row][lda] bytes; weights at w_off (e4m3, [N][Kd] bytes) with fp32
// scales at s_off; epi is EPI_QKV (bf16 out, value third transposed into out2), EPI_BIAS_GELU (out: e4m3 codes of
// gelu(.) * out_qscale, ldo bytes per row) or EPI_BIAS_RESIDUAL (bf16 out).  Student strides in bytes.
hipError_t launch_gemm_fp8(const sp_model* M, const void* A8, int lda, size_t w_off, size_t s_off, size_t b_off,
                           float a_qscale, void* out, int ldo, const void* residual, int ldr, int mrows, int N, int Kd,
                           int k, Epilogue epi, size_t a_student_stride, size_t o_student_stride,
                           size_t r_student_stride, hipStream_t s, void* out2, int n_split, int ld2,
                           size_t o2_student_stride, float out_qscale);

// y[i] = GELU as the bf16 FFN up-projection's epilogue evaluates it, in fp32 (i < n).  Test aid.
// Last layer after its attention for the first-token rows of a call of a few sequences (see sp_gemv.hip): scratch is
// fp32 memory of first_rows_tail_scratch_floats elements, g the FFN activation buffer (its first rows are used), x1 the
// buffer whose first-token rows receive LN(u).  Exactly one of part and pooled is given: part, the split-reduction
// buffer whose slice 0 receives the raw down-projection at the first tokens' rows (student stride part_ss elements;
// launch_head_small with one slice finishes the call), or pooled, fp32 [k][first_rows_tail_pooled_rows][H], whose rows
// b receive the pooled rows (launch_head_classify with pooled_f32 finishes the call).
bool first_rows_tail_supported(const sp_config& c, int B);
size_t first_rows_tail_scratch_floats(const sp_config& c, int k);
int first_rows_tail_pooled_rows();
hipError_t launch_first_rows_tail(const sp_model* M, size_t lo, const void* att, const void* x, void* x1, void* g,
                                  float* scratch, float* part, size_t part_ss, float* pooled, const int32_t* cu, int B,
                                  int T, int rows, int k, hipStream_t s);
hipError_t launch_gelu_probe(const float* x, float* y, long n, hipStream_t s);
hipError_t launch_gelu_q8_probe(const float* x, float* y, long n, hipStream_t s);

// Split reduction for calls of a few dozen tokens, where one workgroup per 64x64 output tile walking the whole
// reduction range is a long serial chain: partials[m][s][row][0..N) = A[m][row][s*Kd/splits ..) . W^T (fp32, no bias),
// s < splits; slice_elems = elements between consecutive slices (>= mrows * N).  bf16 path only.
hipError_t launch_gemm_splitk(const sp_model* M, const void* A, int lda, size_t w_off, float* partials, int mrows, int N,
                              int Kd, int k, int splits, size_t a_student_stride, size_t slice_elems, hipStream_t s);

// out[m][row][:] = LN(sum_s partials[m][s][row][:] + bias + residual[m][row][:]; g, b): the reduction of
// launch_gemm_splitk fused with the bias, the residual add and the LayerNorm that follow the projection.
hipError_t launch_ln_reduce(const sp_model* M, const float* partials, int splits, size_t slice_elems, size_t bias_off,
                            const void* residual, void* out, int rows, int mrows, int k, size_t g_off, size_t b_off,
                            hipStream_t s);

// att[m][t][h*64..] = softmax(q k^T / 8) v inside each sequence; qkv rows are [q | k | v] of width 3H.
// bf16 path: the values are read from vt[m][H][rows] (transposed) instead of the third slice of qkv.
// attq (may be null, bf16 path only): the output once more as e4m3 codes of value * qscale, [m][rows][H] bytes.
hipError_t launch_attention(const sp_model* M, const void* qkv, const void* vt, void* att, const int32_t* cu, int B,
                            int T, int max_seqlen, int rows, int k, hipStream_t s, void* attq = nullptr,
                            float qscale = 1.f);

// First-token rows of every sequence: xc[m][b][:] = x[m][cu[b]][:] (b < B), zero rows up to cmrows; the same
// rows of attc are zeroed.
hipError_t launch_gather_first(const sp_model* M, const void* x, const int32_t* cu, int B, int T, int rows, void* xc,
                               void* attc, int crows, int cmrows, int k, hipStream_t s);

// Per-head small products on the matrix cores: out[m][r][h][n] = sum_k A[m][r][h][k] W[m][h][n][k] (+ bias[m][h][n])
// for r < mrows, n < N, k < Kd, every head h and student m < k.  Strides (_ss per student, _hs per head, ld per
// row) are in elements; w_off / b_off are byte offsets into the student slab (bias: fp32).
hipError_t launch_head_gemm(const sp_model* M, const void* A, size_t a_ss, size_t a_hs, int lda, size_t w_off,
                            size_t w_hs, int ldw, size_t b_off, size_t b_hs, bool has_bias, void* out, size_t o_ss,
                            size_t o_hs, int ldo, int mrows, int N, int Kd, int k, hipStream_t s);

// Attention of the first token of each sequence with folded queries: for sequence b and head h,
// p = softmax_t(qt[m][b][h] . x[m][t] / 8) over the tokens t of the sequence and xbar[m][b][h][:] = sum_t p_t x[m][t][:].
// qt and xbar are [m][crows][heads][H]; rows b in [B, cmrows) of xbar are zeroed.
bool attention_first_fold_supported(const sp_config& c, int max_seqlen);
hipError_t launch_attention_first_fold(const sp_model* M, const void* x, const void* qt, void* xbar, const int32_t* cu,
                                       int B, int T, int max_seqlen, int rows, int crows, int cmrows, int k,
                                       hipStream_t s);

// Head on pooled rows: z[m][b][c] = pooled[m][b] . Wc + bc; logits[b][c] = sum_{m<k} z[m][b][c] (m ascending).
hipError_t launch_head_classify(const sp_model* M, const void* pooled, int B, int crows, int k, float* z, float* logits,
                                hipStream_t s, bool pooled_f32 = false);   // pooled rows bf16, or fp32 if pooled_f32

// flags[0] |= SP_BAD_* bits for the inputs of a forward (flags[0] is cleared first, on the same stream).
hipError_t launch_check_inputs(const int32_t* ids, const int32_t* cu, int B, int T, int max_seqlen, int vocab,
                               unsigned* flags, hipStream_t s);

// logits[i] = sum_{m<k} z[m][i], m ascending (i < n).
hipError_t launch_sum_students(const float* z, int n, int k, float* logits, hipStream_t s);

// z[m][b][c] = tanh(x[m][cu[b]] Wp + bp) Wc + bc (row b itself if cu is null) ; logits[b][c] = sum_{m<k} z[m][b][c] (m ascending).
hipError_t launch_head(const sp_model* M, const void* x, const int32_t* cu, int B, int T, int rows, int k, float* z,
                       float* zpart, float* logits, hipStream_t s);

// The same head for calls of a few dozen tokens: stage 1 rebuilds the first-token rows from the slices of the last split
// reduction (+ bias + residual + LayerNorm: what launch_ln_reduce would have written), so that launch is not needed
// for the last layer of a whole forward.  bf16 only.
hipError_t launch_head_small(const sp_model* M, const float* partials, int splits, size_t slice_elems, size_t bias_off,
                             const void* residual, size_t g_off, size_t b_off, const int32_t* cu, int B, int T, int rows,
                             int k, float* z, float* zpart, float* logits, hipStream_t s);

}  // namespace sp
