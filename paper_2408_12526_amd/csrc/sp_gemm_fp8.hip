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
// Five slots of one operand tile each (256 rows x 128 B = 32 KB; the whole LDS), as in the bf16 kernel of this tile
// size: k-tile t keeps its activations in slot 2 t mod 5 and its weights in slot (2 t + 1) mod 5.  A k-tile is two
// k-steps of sixteen matrix instructions; each instruction pair carries one wave-load and one fragment read (the
// fragments of the next k-step go into the second register set), so that the load path sees one request per 128
// matrix-core cycles all the time and a load has more than a thousand cycles to land:
//   k-step 0 of k-tile j: activations of k-tile j + 2 -> slot of the weights of k-tile j - 1 (free since the barrier
//                         of k-tile j - 1); fragments of k-step 1;
//   barrier (every wave holds its last fragments of k-tile j; k-tile j + 1 has landed and is visible to all);
//   k-step 1:             weights of k-tile j + 2 -> slot of the activations of k-tile j; fragments of k-step 0 of
//                         k-tile j + 1.
#include <atomic>
#include <type_traits>

#include "sp_internal.h"

namespace sp {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int F8_BM = 256, F8_BN = 256, F8_KB = 128;        // tile; bytes (= elements) of a row per k-tile
constexpr int F8_SLOT = 256 * 8;                            // 16-byte units per slot (one operand tile)
constexpr size_t F8_SMEM = (size_t)5 * F8_SLOT * 16;        // 160 KB
static_assert(F8_BM == 256 && F8_BN == 256, "a slot holds one 256-row operand tile");

template <int EPI>
__global__ __launch_bounds__(256, 1) void gemm_fp8_kernel(const unsigned char* __restrict__ A, int lda, size_t a_ss,
                                                          const char* __restrict__ arena, size_t student_stride,
                                                          size_t w_off, size_t s_off, size_t b_off, float inv_qa,
                                                          void* __restrict__ outv, int ldo, size_t o_ss,
                                                          const bf16* __restrict__ res, int ldr, size_t r_ss, int Kd,
                                                          int mtiles, int ntiles, int total, bf16* __restrict__ out2,
                                                          int n_split, int ld2, size_t o2_ss, int mb, float q_out)
{
    constexpr int BM = F8_BM, KB = F8_KB, SLOT = F8_SLOT;
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
    auto issue_a = [&](int i, int kb, int slot) {            // i-th of the 8 wave-loads of an activation tile
        __builtin_amdgcn_global_load_lds((gbl_void*)(Ag + ((size_t)i * 32 * lda + kb) + a_lane),
                                         (lds_void*)(smem + slot * SLOT + (wave + i * 4) * 64), 16, 0, 0);
    };
    auto issue_w = [&](int i, int kb, int slot) {            // ... of a weight tile
        __builtin_amdgcn_global_load_lds((gbl_void*)(Wg + ((size_t)i * 32 * Kd + kb) + w_lane),
                                         (lds_void*)(smem + slot * SLOT + (wave + i * 4) * 64), 16, 0, 0);
    };

    const int j31 = lane & 31, g = lane >> 5;
    const int nk = Kd / KB;
    const float* scl = (const float*)(sb + s_off) + n0 + wn * WT + 4 * g;
    f32x16 acc[TN][TM];
    // The accumulators start from bias / (sw / qa), so that the epilogue's multiplication by sw / qa restores the
    // bias.  Bias and scales of the wave's 128 features come in by one direct-to-LDS load as well, the oldest in
    // flight (lanes 0-31: bias, lanes 32-63: scales), into the part of slot 4 that only this wave's own first load
    // of the activation tile of k-tile 2 overwrites later.  (Fetched into registers instead, their use would make
    // the compiler wait for every direct-to-LDS load issued after them.)
    float* seed_lds = (float*)(smem + 4 * SLOT + wave * 64);
    {
        const float* src = (lane < 32 ? (const float*)(sb + b_off) : (const float*)(sb + s_off)) + n0 + wn * WT + 4 * (lane & 31);
        __builtin_amdgcn_global_load_lds((gbl_void*)src, (lds_void*)seed_lds, 16, 0, 0);
    }
    // start: both tiles of k-tiles 0 and 1
#pragma unroll
    for (int i = 0; i < 8; ++i) issue_a(i, 0, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) issue_w(i, 0, 1);
    if (nk > 1) {
#pragma unroll
        for (int i = 0; i < 8; ++i) issue_a(i, KB, 2);
#pragma unroll
        for (int i = 0; i < 8; ++i) issue_w(i, KB, 3);
    }

    // Fragment addresses.  Rows of the wave's blocks are 32 apart and the wave tiles start at multiples of 128, so
    // one swizzle key ((row >> 1) & 7 = (lane % 32 >> 1) & 7) serves every fragment of both operands; per operand
    // and chunk (two k-steps x two chunks) one lane offset, the block (32 rows = 4096 bytes) an immediate.
    const int key = (j31 >> 1) & 7;
    int wch[2][2], xch[2][2];                               // [k-step][chunk]: 16-byte unit inside a slot, block 0
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int c = (4 * st + 2 * g + h) ^ key;
            wch[st][h] = (wn * WT + j31) * 8 + c;
            xch[st][h] = (wm * WT + j31) * 8 + c;
        }
    auto frag = [&](int slot, const int (&ch)[2][2], int blk, int st) {
        // (read as vector types, not as the four members of a uint4: the compiler keeps type-based alias information
        // on such loads, and without it it makes every LDS read wait for all direct-to-LDS loads in flight)
        const v4i* base = (const v4i*)(smem + slot * SLOT + blk * (32 * 8));
        const v4i lo = base[ch[st][0]], hi = base[ch[st][1]];
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // residual rows of this wave's 128 x 128 sub-tile -> its staging slice, [128 tokens][256 bytes] with chunk
    // (feature / 8) ^ (token & 15); 32 wave-loads of four rows each
    const size_t row0 = (size_t)m0 + wm * WT;
    const int col0 = n0 + wn * WT;
    char* slice = (char*)smem + (size_t)wave * (WT * WT * 2);
    // (wave-load q covers tokens 4 q + lane / 16; the swizzle repeats every 16 tokens, so four lane offsets serve
    // all of them and the rest of the address is uniform)
    unsigned roff[4];
#pragma unroll
    for (int qq = 0; qq < 4; ++qq) {
        const int t = qq * 4 + (lane >> 4), cc = lane & 15;
        roff[qq] = EPI == EPI_BIAS_RESIDUAL ? (unsigned)(t * ldr + ((cc ^ t) << 3)) * 2u : 0u;
    }
    const char* rbase = (const char*)(res + (size_t)m * r_ss + row0 * ldr + col0);
    auto issue_residual = [&](int q) {
        __builtin_amdgcn_global_load_lds((gbl_void*)(rbase + (size_t)(q >> 2) * 16 * ldr * 2 + roff[q & 3]),
                                         (lds_void*)(slice + q * 1024), 16, 0, 0);
    };

    v8i fw[2][TN], fx[2][TM];
    f32x4 f4[TN][4];                                        // sw / qa of the lane's features
    if (nk > 1) wait_vmcnt<16>(); else wait_vmcnt<0>();   // bias, scales and k-tile 0
    barrier_lds();
    {
        // (all reads first, one wait: with direct-to-LDS loads in flight the compiler waits for the whole LDS queue
        // at every first use of a read's result)
        f32x4 b4[TN][4], s4[TN][4];
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                b4[i][v4] = *(const f32x4*)(seed_lds + i * 32 + 8 * v4 + 4 * g);
                s4[i][v4] = *(const f32x4*)(seed_lds + 128 + i * 32 + 8 * v4 + 4 * g);
            }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float seed = b4[i][v4][e] * __builtin_amdgcn_rcpf(s4[i][v4][e] * inv_qa);
#pragma unroll
                    for (int j = 0; j < TM; ++j) acc[i][j][4 * v4 + e] = seed;
                }
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);                     // lgkmcnt(0): the seeds are read before slot 4 is refilled
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < TN; ++i) fw[0][i] = frag(1, wch, i, 0);
#pragma unroll
    for (int j = 0; j < TM; ++j) fx[0][j] = frag(0, xch, j, 0);

    int sa = 0;                                             // activation slot of k-tile j
    // One k-tile; the flags are compile-time, so no variant has a branch in its body.
    //   L0 / L1: the loads of k-step 0 / 1 exist (k-tile j + 2 exists);  NEXT: k-tile j + 1 exists;
    //   RES: k-step 1 carries the residual loads (last k-tile: the whole ring is free after its barrier).
    auto ktile = [&](int j, auto l0_c, auto l1_c, auto next_c, auto res_c) {
        constexpr bool L0 = decltype(l0_c)::value, L1 = decltype(l1_c)::value, NEXT = decltype(next_c)::value;
        constexpr bool RES = decltype(res_c)::value;
        auto rot = [](int s0, int d) { const int t = s0 + d; return t >= 5 ? t - 5 : t; };
        const int s1 = rot(sa, 1), s2 = rot(sa, 2), s3 = rot(sa, 3), s4 = rot(sa, 4);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (s == 1) {
                // k-tile j + 1 has landed; the only younger loads are the eight of k-step 0
                if (L1) wait_vmcnt<8>(); else if (NEXT) wait_vmcnt<0>();
                barrier_lds();
            }
            __builtin_amdgcn_sched_barrier(0);
            const int xslot = s == 0 ? sa : s2, wslot = s == 0 ? s1 : s3, fstep = s == 0 ? 1 : 0;
#pragma unroll
            for (int q = 0; q < 8; ++q) {                   // one load, one fragment, two matrix instructions
                if (s == 0 && L0) issue_a(q, (j + 2) * KB, s4);
                if (s == 1 && L1) issue_w(q, (j + 2) * KB, sa);
                if (s == 1 && RES) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) issue_residual(4 * q + r);
                }
                if (s == 0 || NEXT) {
                    if (q < TN) fw[(s + 1) & 1][q] = frag(wslot, wch, q, fstep);
                    else fx[(s + 1) & 1][q - TN] = frag(xslot, xch, q - TN, fstep);
                }
#pragma unroll
                for (int idx = 2 * q; idx < 2 * q + 2; ++idx) {
                    const int i = idx / TM, jj = idx % TM;
                    acc[i][jj] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fw[s & 1][i], fx[s & 1][jj], acc[i][jj], 0,
                                                                                 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        sa = s2;
    };
    {
        constexpr std::true_type Y{};
        constexpr std::false_type N{};
        constexpr std::integral_constant<bool, EPI == EPI_BIAS_RESIDUAL> R{};
        if (nk >= 3) {
            // (the first k-tile stays outside the loop: its matrix instructions take the seeds from vector registers
            // and leave their results in accumulation registers, which is where the loop then keeps them)
            ktile(0, Y, Y, Y, N);
            for (int jt = 1; jt < nk - 2; ++jt) ktile(jt, Y, Y, Y, N);
            ktile(nk - 2, N, N, Y, N);
            ktile(nk - 1, N, N, N, R);
        } else if (nk == 2) {
            ktile(0, N, N, Y, N);
            ktile(1, N, N, N, R);
        } else {
            ktile(0, N, N, N, R);
        }
    }
    // the epilogue's per-feature factors sw / qa (fetched here and not earlier: the main loop has no registers to
    // spare for them)
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4)                     // (GELU: the output scale rides in the factors, see below)
            f4[i][v4] = *(const f32x4*)(scl + i * 32 + 8 * v4) * (EPI == EPI_BIAS_GELU ? inv_qa * q_out : inv_qa);

    // ---- epilogue.  Accumulator element v of lane l in block (i, j): token = l % 32,
    // feature = 8 * (v / 4) + 4 * (l / 32) + v % 4 inside the 32x32 block.  After the barrier of the last
    // iteration nobody reads the ring: each wave stages its 128 x 128 sub-tile in its own slice of it.
    if (EPI == EPI_BIAS_GELU) {
        // fp8 output, e4m3(gelu(.) * q_out): staged [128 tokens][128 bytes], chunk (feature / 16) ^ (token & 7).
        // The values arrive scaled by q_out, and the fit's coefficients are scaled to match.
        const float iq = 1.0f / q_out;
        const float k0 = kGeluQ8C0 * iq, k1 = kGeluQ8C1 * iq * iq, k2 = kGeluQ8C2 * iq * iq * iq;
        char* slice8 = (char*)smem + (size_t)wave * (WT * WT);
#pragma unroll
        for (int jj = 0; jj < TM; ++jj)
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const int f = i * 32 + 8 * v4 + 4 * g, t = jj * 32 + j31;
                    float r[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) r[e] = gelu_erf_q8_scaled(acc[i][jj][4 * v4 + e] * f4[i][v4][e], k0, k1, k2);
                    int w = 0;
                    w = __builtin_amdgcn_cvt_pk_fp8_f32(r[0], r[1], w, false);
                    w = __builtin_amdgcn_cvt_pk_fp8_f32(r[2], r[3], w, true);
                    *(int*)(slice8 + t * 128 + (((f >> 4) ^ (t & 7)) << 4) + (f & 15)) = w;
                }
        unsigned char* dst = (unsigned char*)outv + (size_t)m * o_ss + row0 * ldo + col0;
        const int rr = lane >> 3, cc = lane & 7;
#pragma unroll 4
        for (int q = 0; q < 16; ++q) {
            const int t = q * 8 + rr;
            *(uint4*)(dst + (size_t)t * ldo + ((cc ^ (t & 7)) << 4)) = *(const uint4*)(slice8 + t * 128 + (cc << 4));
        }
        return;
    }

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
    if (EPI == EPI_BIAS_RESIDUAL) wait_vmcnt<0>();          // the residual rows, requested during the last k-step
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

// y[i] = the GELU of the fp8 epilogue evaluated on x[i], before the scaling and the rounding to e4m3 (test aid)
__global__ void gelu_q8_probe_kernel(const float* __restrict__ x, float* __restrict__ y, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) y[i] = gelu_erf_q8(x[i]);
}

}  // namespace

hipError_t launch_gelu_q8_probe(const float* x, float* y, long n, hipStream_t s)
{
    if (n < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gelu_q8_probe_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, x, y, n);
    return hipGetLastError();
}

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
