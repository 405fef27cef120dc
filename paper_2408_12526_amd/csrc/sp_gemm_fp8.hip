// Student-grouped projections on fp8 (e4m3) operands for large calls of quantised students:
//   out[m] = epilogue((A8[m] . W8[m]^T) * (sw[m][n] / qa) + bias[m][n])
// A8 are activations quantised by their producer as e4m3(value * qa) (one power-of-two scale per tensor), W8 the
// weights quantised at load per output feature n as e4m3(W[n][:] / sw[n]); the products are accumulated in fp32
// by v_mfma_f32_32x32x64_f8f6f4 (both block scales 1).
//
// Tile 256 tokens x 256 features, 256 threads = 2 x 2 waves of 128 x 128, one workgroup per compute unit.  A row of
// a k-tile is 128 bytes (128 reduction elements), so the LDS geometry ([row][8 slots of 16 B], slot = chunk ^
// ((row >> 1) & 7)), the direct-to-LDS wave-loads (8 rows x 128 B) and the bytes moved per matrix-core cycle are
// those of the bf16 kernel; a matrix instruction consumes 64 reduction elements: 32 bytes per lane, two 16-byte
// chunks of a row (chunks 4 s + 2 g and 4 s + 2 g + 1 in k-step s for lane half g; both operands use the same map,
// so the order inside the reduction is immaterial).
//
// Two stages of 64 KB.  One iteration (k-tile kt, first k-step's fragments already in registers):
//   read the second k-step's fragments; 16 matrix instructions of the first k-step;
//   wait for this wave's share of k-tile kt + 1, barrier (stage of kt is free, kt + 1 is visible);
//   read the first k-step's fragments of kt + 1; 16 matrix instructions of the second k-step, with the 16
//   wave-loads of k-tile kt + 2 (into the freed stage) issued one per instruction.
#include <atomic>
#include <type_traits>

#include "sp_internal.h"

namespace sp {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));

constexpr int F8_BM = 256, F8_BN = 256, F8_KB = 128;        // tile; bytes (= elements) of a row per k-tile
constexpr int F8_STAGE = (F8_BM + F8_BN) * 8;               // 16-byte units per stage
constexpr size_t F8_SMEM = (size_t)2 * F8_STAGE * 16;       // 128 KB

template <int EPI>
__global__ __launch_bounds__(256, 1) void gemm_fp8_kernel(const unsigned char* __restrict__ A, int lda, size_t a_ss,
                                                          const char* __restrict__ arena, size_t student_stride,
                                                          size_t w_off, size_t s_off, size_t b_off, float inv_qa,
                                                          void* __restrict__ outv, int ldo, size_t o_ss,
                                                          const bf16* __restrict__ res, int ldr, size_t r_ss, int Kd,
                                                          int mtiles, int ntiles, int total, bf16* __restrict__ out2,
                                                          int n_split, int ld2, size_t o2_ss, int mb, float q_out)
{
    constexpr int BM = F8_BM, KB = F8_KB, STAGE = F8_STAGE;
    constexpr int TM = 4, TN = 4, WT = 128;
    extern __shared__ uint4 smem[];

    const int chunk = (total + 7) >> 3;
    const int lin = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);
    if (lin >= total) return;
    const int tiles = ntiles * mtiles, tl = lin % tiles, m = lin / tiles;
    const int gi = tl / (mb * ntiles), rb = tl - gi * mb * ntiles;
    const int mbe = mtiles - gi * mb < mb ? mtiles - gi * mb : mb;
    const int nt = rb / mbe, mt = gi * mb + rb % mbe;
    const int m0 = mt * BM, n0 = nt * F8_BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const char* sb = arena + (size_t)m * student_stride;
    const unsigned char* Ag = A + (size_t)m * a_ss + (size_t)m0 * lda;
    const unsigned char* Wg = (const unsigned char*)(sb + w_off) + (size_t)n0 * Kd;

    // loader: lane -> (row lane / 8 of the wave-load, LDS slot lane % 8); it fetches chunk slot ^ key(row)
    const int lrow = lane >> 3, lslot = lane & 7;
    const int lchunk = lslot ^ ((4 * wave + (lrow >> 1)) & 7);
    // (uniform base + 32-bit lane offset: the loads can take their base from scalar registers, and no per-load
    // address has to be kept in vector registers across the main loop)
    const unsigned a_lane = (unsigned)((wave * 8 + lrow) * lda + lchunk * 16);
    const unsigned w_lane = (unsigned)((wave * 8 + lrow) * Kd + lchunk * 16);
    auto issue_a = [&](int i, int kb, int stage) {           // i-th of the 8 wave-loads of an activation tile
        __builtin_amdgcn_global_load_lds((gbl_void*)(Ag + ((size_t)i * 32 * lda + kb) + a_lane),
                                         (lds_void*)(smem + stage * STAGE + (wave + i * 4) * 64), 16, 0, 0);
    };
    auto issue_w = [&](int i, int kb, int stage) {           // ... of a weight tile
        __builtin_amdgcn_global_load_lds((gbl_void*)(Wg + ((size_t)i * 32 * Kd + kb) + w_lane),
                                         (lds_void*)(smem + stage * STAGE + BM * 8 + (wave + i * 4) * 64), 16, 0, 0);
    };

    const int j31 = lane & 31, g = lane >> 5;
    const int nk = Kd / KB;
    const float* scl = (const float*)(sb + s_off) + n0 + wn * WT + 4 * g;
    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < 8; ++i) issue_a(i, 0, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) issue_w(i, 0, 0);
    {
        // the accumulators start from bias / (sw / qa), so that the epilogue's multiplication restores the bias
        const float* bias = (const float*)(sb + b_off) + n0 + wn * WT + 4 * g;
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const f32x4 b4 = *(const f32x4*)(bias + i * 32 + 8 * v4), s4 = *(const f32x4*)(scl + i * 32 + 8 * v4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float seed = b4[e] / (s4[e] * inv_qa);
#pragma unroll
                    for (int j = 0; j < TM; ++j) acc[i][j][4 * v4 + e] = seed;
                }
            }
    }

    int woff[TN], xoff[TM], wkey[TN], xkey[TM];
#pragma unroll
    for (int i = 0; i < TN; ++i) { const int r = wn * WT + i * 32 + j31; woff[i] = BM * 8 + r * 8; wkey[i] = (r >> 1) & 7; }
#pragma unroll
    for (int j = 0; j < TM; ++j) { const int r = wm * WT + j * 32 + j31; xoff[j] = r * 8; xkey[j] = (r >> 1) & 7; }
    auto frag = [&](const uint4* st, int off, int key, int s) {
        const int c0 = 4 * s + 2 * g;
        const uint4 lo = st[off + (c0 ^ key)], hi = st[off + ((c0 + 1) ^ key)];
        return v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
    };
    auto read_frags = [&](const uint4* st, int s, v8i (&fw)[TN], v8i (&fx)[TM]) {
#pragma unroll
        for (int i = 0; i < TN; ++i) fw[i] = frag(st, woff[i], wkey[i], s);
#pragma unroll
        for (int j = 0; j < TM; ++j) fx[j] = frag(st, xoff[j], xkey[j], s);
    };
    // sixteen matrix instructions; with LOADS, the sixteen wave-loads of k-tile lkt (into `lstage`) go one in front
    // of each
    auto multiply = [&](const v8i (&fw)[TN], const v8i (&fx)[TM], auto loads_c, int lkt, int lstage) {
        constexpr bool LOADS = decltype(loads_c)::value;
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const int idx = i * TM + j;
                if (LOADS) {
                    if (idx < 8) issue_a(idx, lkt * KB, lstage); else issue_w(idx - 8, lkt * KB, lstage);
                }
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fw[i], fx[j], acc[i][j], 0, 0, 0, 0x7f7f7f7f,
                                                                            0, 0x7f7f7f7f);
                __builtin_amdgcn_sched_barrier(0);
            }
    };

    v8i fw0[TN], fx0[TM], fw1[TN], fx1[TM];
    f32x4 f4[TN][4];                                        // sw / qa of the lane's features
    wait_vmcnt<0>();
    barrier_lds();
    if (nk > 1) {
#pragma unroll
        for (int i = 0; i < 8; ++i) issue_a(i, KB, 1);
#pragma unroll
        for (int i = 0; i < 8; ++i) issue_w(i, KB, 1);
    }
    read_frags(smem, 0, fw0, fx0);
    // NEXT: k-tile kt + 1 exists; LOADS: k-tile kt + 2 exists (the steady state has both and no branch)
    auto ktile = [&](int kt, auto next_c, auto loads_c) {
        constexpr bool NEXT = decltype(next_c)::value;
        const int st = kt & 1;
        __builtin_amdgcn_s_waitcnt(0xc07f);                 // lgkmcnt(0): the first k-step's fragments are here
        __builtin_amdgcn_sched_barrier(0);
        read_frags(smem + st * STAGE, 1, fw1, fx1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fw0, fx0, std::false_type{}, 0, 0);
        if (NEXT) wait_vmcnt<0>();                          // this wave's share of k-tile kt + 1 (requested a k-tile ago)
        __builtin_amdgcn_s_waitcnt(0xc07f);                 // lgkmcnt(0): the second k-step's fragments are here
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (NEXT) read_frags(smem + (st ^ 1) * STAGE, 0, fw0, fx0);
        __builtin_amdgcn_sched_barrier(0);
        multiply(fw1, fx1, loads_c, kt + 2, st);
    };
    {
        int kt = 0;
        for (; kt + 2 < nk; ++kt) ktile(kt, std::true_type{}, std::true_type{});
        if (kt + 1 < nk) { ktile(kt, std::true_type{}, std::false_type{}); ++kt; }
        ktile(kt, std::false_type{}, std::false_type{});
    }
    // the epilogue's per-feature factors sw / qa (fetched here and not earlier: the main loop has no registers to
    // spare for them)
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) f4[i][v4] = *(const f32x4*)(scl + i * 32 + 8 * v4) * inv_qa;

    // ---- epilogue.  Accumulator element v of lane l in block (i, j): token = l % 32,
    // feature = 8 * (v / 4) + 4 * (l / 32) + v % 4 inside the 32x32 block.  After the barrier of the last
    // iteration nobody reads the ring: each wave stages its 128 x 128 sub-tile in its own slice of it.
    const size_t row0 = (size_t)m0 + wm * WT;
    const int col0 = n0 + wn * WT;

    if (EPI == EPI_BIAS_GELU) {
        // fp8 output, e4m3(gelu(.) * q_out): staged [128 tokens][128 bytes], chunk (feature / 16) ^ (token & 7)
        char* slice = (char*)smem + (size_t)wave * (WT * WT);
#pragma unroll
        for (int jj = 0; jj < TM; ++jj)
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const int f = i * 32 + 8 * v4 + 4 * g, t = jj * 32 + j31;
                    float r[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) r[e] = gelu_erf_fast(acc[i][jj][4 * v4 + e] * f4[i][v4][e]) * q_out;
                    int w = 0;
                    w = __builtin_amdgcn_cvt_pk_fp8_f32(r[0], r[1], w, false);
                    w = __builtin_amdgcn_cvt_pk_fp8_f32(r[2], r[3], w, true);
                    *(int*)(slice + t * 128 + (((f >> 4) ^ (t & 7)) << 4) + (f & 15)) = w;
                }
        unsigned char* dst = (unsigned char*)outv + (size_t)m * o_ss + row0 * ldo + col0;
        const int rr = lane >> 3, cc = lane & 7;
#pragma unroll 4
        for (int q = 0; q < 16; ++q) {
            const int t = q * 8 + rr;
            *(uint4*)(dst + (size_t)t * ldo + ((cc ^ (t & 7)) << 4)) = *(const uint4*)(slice + t * 128 + (cc << 4));
        }
        return;
    }

    char* slice = (char*)smem + (size_t)wave * (WT * WT * 2);
    bf16* out = (bf16*)outv;
    const bool transposed = EPI == EPI_QKV && n0 >= n_split;
    const int rr = lane >> 4, cc = lane & 15;
    if (EPI == EPI_QKV && transposed) {
        // staged [128 features][128 tokens]: 256-byte rows, chunk (token / 8) ^ (feature & 15)
#pragma unroll
        for (int jj = 0; jj < TM; ++jj)
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int f = i * 32 + 8 * (e >> 2) + 4 * g + (e & 3), t = jj * 32 + j31;
                    *(bf16*)(slice + f * 256 + (((t >> 3) ^ (f & 15)) << 4) + (t & 7) * 2) =
                        (bf16)(acc[i][jj][e] * f4[i][e >> 2][e & 3]);
                }
        bf16* dst = out2 + (size_t)m * o2_ss + (size_t)(col0 - n_split) * ld2 + row0;
#pragma unroll 4
        for (int q = 0; q < 32; ++q) {
            const int f = q * 4 + rr;
            *(uint4*)(dst + (size_t)f * ld2 + ((cc ^ (f & 15)) << 3)) = *(const uint4*)(slice + f * 256 + (cc << 4));
        }
        return;
    }

    // staged [128 tokens][128 features]: 256-byte rows, chunk (feature / 8) ^ (token & 15)
    if (EPI == EPI_BIAS_RESIDUAL) {
        const bf16* rb = res + (size_t)m * r_ss + row0 * ldr + col0;
#pragma unroll 8
        for (int q = 0; q < 32; ++q) {
            const int t = q * 4 + rr;
            __builtin_amdgcn_global_load_lds((gbl_void*)(rb + (size_t)t * ldr + ((cc ^ (t & 15)) << 3)),
                                             (lds_void*)(slice + q * 1024), 16, 0, 0);
        }
        wait_vmcnt<0>();
    }
#pragma unroll
    for (int jj = 0; jj < TM; ++jj)
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int f = i * 32 + 8 * v4 + 4 * g, t = jj * 32 + j31;
                char* c = slice + t * 256 + (((f >> 3) ^ (t & 15)) << 4) + (f & 7) * 2;
                float r[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = acc[i][jj][4 * v4 + e] * f4[i][v4][e];
                if (EPI == EPI_BIAS_RESIDUAL) {
                    const bf16x4 x4 = *(const bf16x4*)c;
#pragma unroll
                    for (int e = 0; e < 4; ++e) r[e] += (float)x4[e];
                }
                bf16x4 o4;
#pragma unroll
                for (int e = 0; e < 4; ++e) o4[e] = (bf16)r[e];
                *(bf16x4*)c = o4;
            }
    bf16* dst = out + (size_t)m * o_ss + row0 * ldo + col0;
#pragma unroll 4
    for (int q = 0; q < 32; ++q) {
        const int t = q * 4 + rr;
        *(uint4*)(dst + (size_t)t * ldo + ((cc ^ (t & 15)) << 3)) = *(const uint4*)(slice + t * 256 + (cc << 4));
    }
}

template <int EPI>
hipError_t launch_fp8_tile(const sp_model* M, const void* A8, int lda, size_t w_off, size_t s_off, size_t b_off,
                           float inv_qa, void* out, int ldo, const void* residual, int ldr, int mrows, int N, int Kd,
                           int k, size_t a_ss, size_t o_ss, size_t r_ss, hipStream_t s, void* out2, int n_split, int ld2,
                           size_t o2_ss, float q_out)
{
    auto kern = gemm_fp8_kernel<EPI>;
    static std::atomic<bool> raised{false};   // per instantiation; the attribute is sticky for the process
    if (!raised.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)F8_SMEM);
        if (e != hipSuccess) return e;
        raised.store(true, std::memory_order_release);
    }
    const int mtiles = mrows / F8_BM, ntiles = N / F8_BN, total = k * mtiles * ntiles;
    const int grid = ((total + 7) / 8) * 8;
    const int mb = ntiles >= 6 ? 5 : 1;                     // token-tile blocking, as for the bf16 tile of this size
    // a_ss: bytes (= elements); o_ss: bytes per student of the output (fp8: elements; bf16: 2 per element)
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), F8_SMEM, s, (const unsigned char*)A8, lda, a_ss, M->arena,
                       M->L.student_stride, w_off, s_off, b_off, inv_qa, out, ldo, EPI == EPI_BIAS_GELU ? o_ss : o_ss / 2,
                       (const bf16*)residual, ldr, r_ss / 2, Kd, mtiles, ntiles, total, (bf16*)out2, n_split, ld2,
                       o2_ss / 2, mb, q_out);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_fp8(const sp_model* M, const void* A8, int lda, size_t w_off, size_t s_off, size_t b_off,
                           float a_qscale, void* out, int ldo, const void* residual, int ldr, int mrows, int N, int Kd,
                           int k, Epilogue epi, size_t a_student_stride, size_t o_student_stride,
                           size_t r_student_stride, hipStream_t s, void* out2, int n_split, int ld2,
                           size_t o2_student_stride, float out_qscale)
{
    if (M->cfg.dtype != SP_DTYPE_FP8 || mrows % 256 || N % 256 || Kd % 128 || Kd < 128 || lda % 16 || !(a_qscale > 0.f))
        return hipErrorInvalidValue;
    if (epi == EPI_BIAS_RESIDUAL && !residual) return hipErrorInvalidValue;
    if (epi == EPI_QKV && (!out2 || n_split % 256 || ld2 % 8)) return hipErrorInvalidValue;
    const float inv_qa = 1.0f / a_qscale;
#define SP_ARGS M, A8, lda, w_off, s_off, b_off, inv_qa, out, ldo, residual, ldr, mrows, N, Kd, k, a_student_stride, \
                o_student_stride, r_student_stride, s
    switch (epi) {
        case EPI_QKV: return launch_fp8_tile<EPI_QKV>(SP_ARGS, out2, n_split, ld2, o2_student_stride, 1.f);
        case EPI_BIAS_GELU: return launch_fp8_tile<EPI_BIAS_GELU>(SP_ARGS, nullptr, 0, 0, 0, out_qscale);
        case EPI_BIAS_RESIDUAL: return launch_fp8_tile<EPI_BIAS_RESIDUAL>(SP_ARGS, nullptr, 0, 0, 0, 1.f);
        default: return hipErrorInvalidValue;
    }
#undef SP_ARGS
}

}  // namespace sp
