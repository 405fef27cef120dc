// Student-grouped projections: out[m] = epilogue(A[m] . W[m]^T + bias[m]) for every active
// student m.  The bf16 kernel runs on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32
// accumulate) with both operands staged through LDS; the fp32 kernel is a plain FMA tile
// kernel used by the fp32 path.
#include <atomic>
#include <type_traits>

#include "sp_internal.h"

namespace sp {

namespace {

__device__ inline float gelu_erf(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f)); }

// -------------------------------------------------------------------------------------
// bf16 MFMA kernel (v_mfma_f32_32x32x16_bf16), 256 threads = 2 x 2 waves, tile BM tokens x BN features.
//
// Operand roles are swapped with respect to the textbook picture: the weight tile is the MFMA "A" operand
// (rows = output features) and the activation tile the "B" operand (columns = tokens), so a lane of the
// 32x32 accumulator owns one token and runs of four consecutive features.
//
// Data movement
//   * global -> LDS with direct-to-LDS loads (no register staging).  A wave-load moves 8 rows x 128 bytes
//     (64 reduction elements) and lands as 1 KB of contiguous LDS.
//   * LDS tile = [row][8 slots of 16 B]; slot s of row r holds k-chunk s ^ ((r >> 1) & 7).  The 16 lanes that
//     a ds_read_b128 serves per cycle then hit 16 distinct 16-byte bank groups (no bank conflicts), and the
//     global side still reads whole 128-byte rows.
//   * ring of two stages (128 x 128 tile) or three (64 x 64) over the reduction dimension.  The loads that refill
//     a stage are spread over the MFMAs of two k-steps (a burst of loads stalls the issuing wave behind the
//     address unit's queue), and the fragments of k-step s + 1 are read while step s multiplies.  One barrier per 64-wide k-tile, placed where
//     every wave already holds its last fragments of the tile in registers.
//   * 256 x 256 tile: a wave stalls on its direct-to-LDS loads once more than about four of them per k-step are
//     issued (the address unit's queue), and two stages force sixteen loads per k-tile into the two k-steps that
//     leave them time to land.  Five slots of one operand tile each allow four loads in every k-step: the weight
//     tile of k-tile j + 2 is requested when k-tile j is finished (into its activation slot), the activation tile
//     of k-tile j + 2 already during k-tile j (into the weight slot of k-tile j - 1).
//   * epilogue through LDS: each wave stages its sub-tile in its own slice of the ring, so that global writes are
//     whole 16-byte-per-lane row segments.  Staged rows are unpadded and their 16-byte chunks XOR-swizzled by row,
//     which lets the residual rows arrive by the same direct-to-LDS loads: half of them are requested before the
//     last k-tile (into the ring stage that is already idle), the rest while the first half is being processed.
//   * the accumulators start from the bias values (sixteen dependent global loads in the epilogue cost several
//     microseconds per tile, and so the adds disappear as well); they come in through LDS by the first
//     direct-to-LDS load of the kernel (see request_bias).
// -------------------------------------------------------------------------------------
template <int BM, int BN>
struct GemmTile {
    static constexpr int BK = 64, STEPS = 4, LSPREAD = 2;
    // ring depth: three stages for the 64 x 64 tile (measured, 64 rows x 8 students: FFN down, depth 3072, 26.4 -> 17.5 us;
    // FFN up 11.2 -> 10.2 us; four stages no better; one student: no change, a lone workgroup per compute unit is
    // bound by that unit's load path at about 28 B per cycle either way), two for the 128 x 128 tile
    static constexpr int NS = BM == 64 ? 3 : 2;
    static constexpr int WTM = BM / 2, WTN = BN / 2;        // wave tile
    // The 256 x 256 tile keeps a ring of five operand tiles (256 rows x 64 reduction elements, 32 KB each: the whole
    // LDS) instead of two stages of an activation and a weight tile; the smaller tiles use the two-stage ring.
    static constexpr bool RING5 = BM == 256 && BN == 256;
    static constexpr size_t ring_bytes = RING5 ? (size_t)5 * 256 * 8 * 16 : (size_t)NS * (BM + BN) * 8 * 16;
    // epilogue staging: wave w keeps rows [h * WTM / 2, (h + 1) * WTM / 2) of its sub-tile, WTN * 2 bytes each, in
    // one half of the staging area (= one stage of the two-stage ring, two slots of the five-slot ring)
    static constexpr size_t half_bytes = (size_t)(BM + BN) * 8 * 16;
    static_assert(NS >= 2 && (size_t)4 * (WTM / 2) * WTN * 2 <= half_bytes, "staging halves must fit the ring stages");
    // (the smaller tiles keep the waves' bias values behind the ring, one kilobyte per wave)
    static constexpr size_t smem_bytes = ring_bytes + (RING5 ? 0 : 4 * 1024);
};

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256, 1) void gemm_bf16_kernel(const bf16* __restrict__ A, int lda, size_t a_ss,
                                                           const char* __restrict__ arena, size_t student_stride,
                                                           size_t w_off, size_t b_off, bf16* __restrict__ out, int ldo,
                                                           size_t o_ss, const bf16* __restrict__ res, int ldr,
                                                           size_t r_ss, int Kd, int mtiles, int ntiles, int total,
                                                           bf16* __restrict__ out2, int n_split, int ld2, size_t o2_ss,
                                                           int ksplit, int ldw, int mb)
{
    using G = GemmTile<BM, BN>;
    constexpr int BK = G::BK, NS = G::NS, STEPS = G::STEPS, LSPREAD = G::LSPREAD;
    constexpr int LA = BM / 32, LW = BN / 32;               // wave-loads (8 rows each) per wave per stage
    constexpr int LPW = LA + LW, LPS = LPW / LSPREAD;
    constexpr int TM = BM / 64, TN = BN / 64;               // 32x32 blocks per wave: tokens, features
    constexpr int STAGE = (BM + BN) * 8;                    // 16-byte units per stage
    static_assert(LPW % LSPREAD == 0, "loads must split evenly over the steps that carry them");
    extern __shared__ uint4 smem[];

    // XCD-aware tile order: consecutive workgroup ids go to different XCDs, so each XCD gets a contiguous run of
    // (student, token tile, feature tile) triples; neighbours share the activation tile and the student's
    // weights in that XCD's L2.
    const int chunk = (total + 7) >> 3;
    const int lin = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);
    if (lin >= total) return;
    // (student, slice of the reduction range, token tile, feature tile); ksplit > 1 only with EPI_PARTIAL, where a
    // workgroup reduces over Kd elements starting at sp * Kd and the slices are added by a later kernel
    const int tiles = ntiles * mtiles, tl = lin % tiles, sp = (lin / tiles) % ksplit;
    const int m = lin / (tiles * ksplit);
    // inside a student: blocks of mb token tiles; inside a block the feature tile is the slow index, so the
    // workgroups resident at one time share mb activation tiles (which then stay in the L2) and stream the weights
    const int gi = tl / (mb * ntiles), rb = tl - gi * mb * ntiles;
    const int mbe = mtiles - gi * mb < mb ? mtiles - gi * mb : mb;
    const int nt = rb / mbe, mt = gi * mb + rb % mbe;
    const int m0 = mt * BM, n0 = nt * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const bf16* Ag = A + (size_t)m * a_ss + (size_t)m0 * lda + (size_t)sp * Kd;
    const bf16* Wg = (const bf16*)(arena + (size_t)m * student_stride + w_off) + (size_t)n0 * ldw + (size_t)sp * Kd;

    // loader: lane -> (row lane / 8 of the wave-load, LDS slot lane % 8); it fetches k-chunk slot ^ key(row)
    const int lrow = lane >> 3, lslot = lane & 7;
    const int lchunk = lslot ^ ((4 * wave + (lrow >> 1)) & 7);
    const bf16* a_src = Ag + (size_t)(wave * 8 + lrow) * lda + lchunk * 8;
    const bf16* w_src = Wg + (size_t)(wave * 8 + lrow) * ldw + lchunk * 8;
    auto issue1 = [&](int i, int k0, int stage) {           // i-th wave-load of a stage (activation rows first)
        if (i < LA)
            __builtin_amdgcn_global_load_lds((gbl_void*)(a_src + (size_t)i * 32 * lda + k0),
                                             (lds_void*)(smem + stage * STAGE + (wave + i * 4) * 64), 16, 0, 0);
        else
            __builtin_amdgcn_global_load_lds((gbl_void*)(w_src + (size_t)(i - LA) * 32 * ldw + k0),
                                             (lds_void*)(smem + stage * STAGE + BM * 8 + (wave + (i - LA) * 4) * 64),
                                             16, 0, 0);
    };

    // The accumulators start from the lane's bias values.  They come in through LDS, by one direct-to-LDS wave-load
    // per wave issued before the operand tiles (lane l fetches features 4 (l mod WTN / 4) .. + 3 of the wave's WTN, so
    // the first WTN floats of the wave's kilobyte are its bias): fetched into registers instead, their first use would
    // make the compiler wait for every direct-to-LDS load issued after them, i.e. for the whole ring instead of the
    // first k-tile.
    const int j31 = lane & 31, g = lane >> 5;
    f32x4 b4[TN][4];
    auto request_bias = [&](float* seed_lds) {
        if (EPI == EPI_PARTIAL) return;
        const float* bias_w = (const float*)(arena + (size_t)m * student_stride + b_off) + n0 + wn * G::WTN;
        __builtin_amdgcn_global_load_lds((gbl_void*)(bias_w + 4 * (lane % (G::WTN / 4))), (lds_void*)seed_lds, 16, 0, 0);
    };
    auto read_bias = [&](const float* seed_lds) {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4)
                b4[i][v4] = EPI == EPI_PARTIAL ? f32x4{0.f, 0.f, 0.f, 0.f} : *(const f32x4*)(seed_lds + 4 * g + i * 32 + 8 * v4);
        __builtin_amdgcn_sched_barrier(0);
    };

    // Epilogue staging geometry (used early by the residual prefetch).
    constexpr int WTM = G::WTM, WTN = G::WTN;
    constexpr int ROWB = WTN * 2;                           // bytes per staged row
    constexpr int CPR = WTN / 8;                            // 16-byte chunks per staged row
    constexpr int RPI = 64 / CPR;                           // rows per row-wise instruction
    constexpr int KSH = CPR == 16 ? 0 : (CPR == 8 ? 1 : 2); // rows that share a swizzle key: 256 bytes of LDS
    constexpr int HR = WTM / 2;                             // rows per staging half
    const int rr = lane / CPR, cc = lane % CPR;
    const size_t row0 = (size_t)m0 + wm * WTM;
    const int col0 = n0 + wn * WTN;
    // staging half 0 sits in a ring stage that is idle during the last k-tile (the one after it in ring order), half 1
    // in the next one (for a two-stage ring: the last k-tile's own stage, free once the loop is over)
    const int ha = (Kd / BK) % NS, hb1 = (Kd / BK + 1) % NS;
    // five-slot ring: the last k-tile sits in slots sl, sl + 1 (mod 5).  Staging half 0 is a pair of adjacent slots
    // among the other three (idle during the last k-tile), half 1 a pair among the rest (free once the loop is over).
    const int sl = (2 * (Kd / BK - 1)) % 5;
    const int hs0 = sl == 0 ? 2 : (sl == 1 ? 3 : (sl == 4 ? 1 : 0)), hs1 = sl <= 1 ? 0 : (sl == 4 ? 3 : 2);
    auto half_ptr = [&](int h) {
        const size_t hb = G::RING5 ? (size_t)(h ? hs1 : hs0) * (256 * 8 * 16) : (size_t)(h ? hb1 : ha) * G::half_bytes;
        return (char*)smem + hb + (size_t)wave * HR * ROWB;
    };
    auto swz = [](int r, int chunk) { return chunk ^ ((r >> KSH) & (CPR - 1)); };
    // Row-wise instructions (residual loads, output stores) move RPI whole staged rows each; the swizzle repeats
    // every 16 rows, so NQ per-lane offsets serve every 16-row period and the rest of the address is uniform.
    constexpr int NQ = 16 / RPI;
    unsigned soff[NQ], xch[NQ];                             // LDS byte offset inside a period; swizzled chunk
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        xch[q] = (unsigned)swz(q * RPI + rr, cc);
        soff[q] = (unsigned)((q * RPI + rr) * ROWB) + (xch[q] << 4);
    }
    // residual rows of staging half h -> LDS (asynchronous; this wave's own slice)
    auto issue_residual = [&](int h) {
        const char* rb = (const char*)(res + (size_t)m * r_ss + (row0 + (size_t)h * HR) * ldr + col0);
        char* base = half_ptr(h);
#pragma unroll
        for (int pr = 0; pr < HR / 16; ++pr)
#pragma unroll
            for (int q = 0; q < NQ; ++q)
                __builtin_amdgcn_global_load_lds(
                    (gbl_void*)(rb + (size_t)pr * 32 * ldr + (unsigned)((q * RPI + rr) * ldr * 2 + (xch[q] << 4))),
                    (lds_void*)(base + (pr * 16 + q * RPI) * ROWB), 16, 0, 0);
    };

    int woff[TN], xoff[TM], wkey[TN], xkey[TM];
#pragma unroll
    for (int i = 0; i < TN; ++i) { const int r = wn * G::WTN + i * 32 + j31; woff[i] = (G::RING5 ? 0 : BM * 8) + r * 8; wkey[i] = (r >> 1) & 7; }
#pragma unroll
    for (int j = 0; j < TM; ++j) { const int r = wm * G::WTM + j * 32 + j31; xoff[j] = r * 8; xkey[j] = (r >> 1) & 7; }
    bf16x8 fw[2][TN], fx[2][TM];

    const int nk = Kd / BK;
    f32x16 acc[TN][TM];
    if constexpr (G::RING5) {
        constexpr int SLOT = 256 * 8;                       // 16-byte units per slot
        auto issue_a = [&](int i, int k0, int slot) {       // i-th of the 8 wave-loads of an activation tile
            __builtin_amdgcn_global_load_lds((gbl_void*)(a_src + (size_t)i * 32 * lda + k0),
                                             (lds_void*)(smem + slot * SLOT + (wave + i * 4) * 64), 16, 0, 0);
        };
        auto issue_w = [&](int i, int k0, int slot) {       // ... of a weight tile
            __builtin_amdgcn_global_load_lds((gbl_void*)(w_src + (size_t)i * 32 * ldw + k0),
                                             (lds_void*)(smem + slot * SLOT + (wave + i * 4) * 64), 16, 0, 0);
        };
        // k-tile t: activations in slot 2 t mod 5, weights in slot (2 t + 1) mod 5.  Start: the wave's 128 bias values
        // (one wave-load, both lane halves fetch the same 512 bytes, into the part of slot 4 that only this wave's own
        // first load of the activation tile of k-tile 2 overwrites later), then both tiles of k-tiles 0 and 1 (the reduction depth is
        // at least 256: four k-tiles or more).
        float* seed_lds = (float*)(smem + 4 * SLOT + wave * 64);
        request_bias(seed_lds);
#pragma unroll
        for (int i = 0; i < 8; ++i) issue_a(i, 0, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) issue_w(i, 0, 1);
#pragma unroll
        for (int i = 0; i < 8; ++i) issue_a(i, BK, 2);
#pragma unroll
        for (int i = 0; i < 8; ++i) issue_w(i, BK, 3);
        wait_vmcnt<16>();                                   // bias and k-tile 0
        barrier_lds();
        read_bias(seed_lds);
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = b4[i][e >> 2][e & 3];
        __builtin_amdgcn_s_waitcnt(0xc07f);                 // lgkmcnt(0): the bias is read before slot 4 is refilled
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TN; ++i) fw[0][i] = __builtin_bit_cast(bf16x8, smem[SLOT + woff[i] + (g ^ wkey[i])]);
#pragma unroll
        for (int j = 0; j < TM; ++j) fx[0][j] = __builtin_bit_cast(bf16x8, smem[xoff[j] + (g ^ xkey[j])]);

        int sa = 0;                                         // activation slot of k-tile j
        // One k-tile.  Loads, four per k-step (one per quarter-step):
        //   step 0: second half of the weight tile of k-tile j + 1 -> slot sa + 3 (activations of k-tile j - 1)
        //   steps 1, 2: activation tile of k-tile j + 2            -> slot sa + 4 (weights of k-tile j - 1)
        //   step 3, after the barrier: first half of the weight tile of k-tile j + 2 -> slot sa (idle from here on)
        // The barrier of step 3 needs k-tile j + 1 complete; the only younger loads are the eight of the activation
        // tile of k-tile j + 2.
        // The variants (first k-tile, steady state, last two) are compile-time instances: none has a branch in its body,
        // and the scheduling fences fix the interleaving of loads, LDS reads and MFMAs in all of them.
        //   L0: the loads of step 0 exist (j >= 1 and k-tile j + 1 exists);  L2: those of steps 1 to 3 (k-tile j + 2 exists);
        //   NEXT: k-tile j + 1 exists.
        auto ktile = [&](int j, auto l0_c, auto l2_c, auto next_c) {
            constexpr bool L0 = decltype(l0_c)::value, L2 = decltype(l2_c)::value, NEXT = decltype(next_c)::value;
            auto rot = [](int s0, int d) { const int t = s0 + d; return t >= 5 ? t - 5 : t; };
            const int s1 = rot(sa, 1), s2 = rot(sa, 2), s3 = rot(sa, 3), s4 = rot(sa, 4);
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                if (s == STEPS - 1) {
                    if (L2) wait_vmcnt<8>(); else if (NEXT) wait_vmcnt<0>();
                    barrier_lds();
                }
                __builtin_amdgcn_sched_barrier(0);
                const bool do_loads = s == 0 ? L0 : L2;
                const bool do_frags = s + 1 < STEPS || NEXT;
                const int xslot = s + 1 < STEPS ? sa : s2, wslot = s + 1 < STEPS ? s1 : s3;
                const int kg = 2 * (s + 1 < STEPS ? s + 1 : 0) + g;
                constexpr int NF = TM + TN, NM = TM * TN;
#pragma unroll
                for (int q = 0; q < 4; ++q) {               // quarter-steps: one load, two fragment reads, four MFMAs
                    if (do_loads) {
                        if (s == 0) issue_w(4 + q, (j + 1) * BK, s3);
                        else if (s == 1) issue_a(q, (j + 2) * BK, s4);
                        else if (s == 2) issue_a(4 + q, (j + 2) * BK, s4);
                        else issue_w(q, (j + 2) * BK, sa);
                    }
                    if (do_frags) {
#pragma unroll
                        for (int f = q * NF / 4; f < (q + 1) * NF / 4; ++f) {
                            if (f < TN)
                                fw[(s + 1) & 1][f] = __builtin_bit_cast(bf16x8, smem[wslot * SLOT + woff[f] + (kg ^ wkey[f])]);
                            else
                                fx[(s + 1) & 1][f - TN] =
                                    __builtin_bit_cast(bf16x8, smem[xslot * SLOT + xoff[f - TN] + (kg ^ xkey[f - TN])]);
                        }
                    }
#pragma unroll
                    for (int idx = q * NM / 4; idx < (q + 1) * NM / 4; ++idx) {
                        const int i = idx / TM, jj = idx % TM;
                        acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[s & 1][i], fx[s & 1][jj], acc[i][jj], 0, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            sa = s2;
        };
        {
            constexpr std::true_type Y{};
            constexpr std::false_type N{};
            // (the launcher gives this tile only reduction depths of at least 256: four k-tiles or more)
            ktile(0, N, Y, Y);
            for (int jt = 1; jt < nk - 2; ++jt) ktile(jt, Y, Y, Y);
            ktile(nk - 2, Y, N, Y);
            // from here on only the two slots of the last k-tile are read: the first half of the residual rows goes
            // into two of the others
            if (EPI == EPI_BIAS_RESIDUAL) issue_residual(0);
            ktile(nk - 1, N, N, N);
        }
    } else {
        float* seed_lds = (float*)((char*)smem + G::ring_bytes) + wave * 256;   // one kilobyte per wave behind the ring
        request_bias(seed_lds);
#pragma unroll
        for (int t = 0; t < NS; ++t)
            if (t < nk)
#pragma unroll
                for (int i = 0; i < LPW; ++i) issue1(i, t * BK, t);
        if (nk >= NS) wait_vmcnt<(NS - 1) * LPW>(); else wait_vmcnt<0>();   // bias and k-tile 0
        barrier_lds();
        read_bias(seed_lds);
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = b4[i][e >> 2][e & 3];
#pragma unroll
        for (int i = 0; i < TN; ++i) fw[0][i] = __builtin_bit_cast(bf16x8, smem[woff[i] + (g ^ wkey[i])]);
#pragma unroll
        for (int j = 0; j < TM; ++j) fx[0][j] = __builtin_bit_cast(bf16x8, smem[xoff[j] + (g ^ xkey[j])]);

        int stage = 0, pstage = NS - 1;                         // stage of k-tile j, of k-tile j - 1
        // One k-tile.  STEADY: every load / prefetch condition is known to hold, so the body has no branches and
        // the scheduling fences below fix the interleaving of loads, LDS reads and MFMAs.
        auto ktile = [&](int j, auto steady_c) {
            constexpr bool STEADY = decltype(steady_c)::value;
            const int nstage = stage + 1 == NS ? 0 : stage + 1;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                if (s == STEPS - 1) {
                    // every wave holds (or has requested) its last fragments of k-tile j: after the barrier nobody reads
                    // this stage any more, and k-tile j + 1 (waited for here) is visible to all
                    // (the last k-tile has no successor to wait for; residual rows may be in flight there)
                    if (STEADY || j + NS <= nk) wait_vmcnt<(NS - 2) * LPW>(); else if (j + 1 < nk) wait_vmcnt<0>();
                    barrier_lds();
                }
                __builtin_amdgcn_sched_barrier(0);
                // refill: k-tile j + NS -> this stage (from the last step on), k-tile j - 1 + NS -> previous stage
                const int lt = s == STEPS - 1 ? j + NS : j - 1 + NS;
                const int lstage = s == STEPS - 1 ? stage : pstage;
                const bool do_loads = ((s + 1) % STEPS) < LSPREAD && (STEADY || ((s == STEPS - 1 || j >= 1) && lt < nk));
                const bool do_frags = s + 1 < STEPS || STEADY || j + 1 < nk;
                const int fstage = s + 1 < STEPS ? stage : nstage, fstep = s + 1 < STEPS ? s + 1 : 0;
                const int kg = 2 * fstep + g;
                constexpr int NF = TM + TN, NM = TM * TN;
#pragma unroll
                for (int q = 0; q < 4; ++q) {                   // quarter-steps: a share of loads, fragment reads, MFMAs
                    if (do_loads) {
#pragma unroll
                        for (int i = q * LPS / 4; i < (q + 1) * LPS / 4; ++i)
                            issue1(((s + 1) % STEPS) * LPS + i, lt * BK, lstage);
                    }
                    if (do_frags) {
#pragma unroll
                        for (int f = q * NF / 4; f < (q + 1) * NF / 4; ++f) {
                            if (f < TN)
                                fw[(s + 1) & 1][f] = __builtin_bit_cast(bf16x8, smem[fstage * STAGE + woff[f] + (kg ^ wkey[f])]);
                            else
                                fx[(s + 1) & 1][f - TN] =
                                    __builtin_bit_cast(bf16x8, smem[fstage * STAGE + xoff[f - TN] + (kg ^ xkey[f - TN])]);
                        }
                    }
#pragma unroll
                    for (int idx = q * NM / 4; idx < (q + 1) * NM / 4; ++idx) {
                        const int i = idx / TM, jj = idx % TM;
                        acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[s & 1][i], fx[s & 1][jj], acc[i][jj], 0, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            pstage = stage;
            stage = nstage;
        };
        int jt = 0;
        ktile(jt++, std::false_type{});
        for (; jt < nk - NS; ++jt) ktile(jt, std::true_type{});
        for (; jt < nk; ++jt) {
            // from here on the stage of k-tile nk - 2 is read by nobody: the first half of the residual rows goes there
            if (EPI == EPI_BIAS_RESIDUAL && jt == nk - 1) issue_residual(0);
            ktile(jt, std::false_type{});
        }

    }

    // ---- epilogue.  Accumulator element v of lane l in block (i, j): token = l % 32,
    // feature = 8 * (v / 4) + 4 * (l / 32) + v % 4 inside the 32x32 block.
    // The barrier in the last step of the last k-tile already separates every fragment read from what follows:
    // the ring is free.
    if (EPI == EPI_PARTIAL) {
        // fp32 partial sums of this slice of the reduction range: out[(m * ksplit + sp)][row][feature], no bias
        float* po = (float*)out + ((size_t)m * ksplit + sp) * o_ss + (row0 + j31) * ldo + col0 + 4 * g;
#pragma unroll
        for (int jj = 0; jj < TM; ++jj)
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4)
                    *(f32x4*)(po + (size_t)jj * 32 * ldo + i * 32 + 8 * v4) =
                        f32x4{acc[i][jj][4 * v4], acc[i][jj][4 * v4 + 1], acc[i][jj][4 * v4 + 2], acc[i][jj][4 * v4 + 3]};
        return;
    }
    if (EPI == EPI_BIAS_RESIDUAL) issue_residual(1);
    // EPI_QKV: feature tiles at or beyond n_split (the value projection) are staged feature-major and written
    // transposed, out2[feature - n_split][token]; the choice is uniform over the workgroup.
    const bool transposed = EPI == EPI_QKV && n0 >= n_split;
    // staged cell of (row r of the wave tile, 2-byte column c): half r / HR, chunk c / 8 swizzled by the row
    auto cell = [&](int r, int c) {
        const int h = r / HR, rh = r % HR;
        return half_ptr(h) + rh * ROWB + (swz(rh, c >> 3) << 4) + (c & 7) * 2;
    };
    char* dst = (char*)(EPI == EPI_QKV && transposed ? out2 + (size_t)m * o2_ss + (size_t)(col0 - n_split) * ld2 + row0
                                                     : out + (size_t)m * o_ss + row0 * ldo + col0);
    const unsigned dpitch = 2u * (unsigned)(EPI == EPI_QKV && transposed ? ld2 : ldo);   // bytes
    unsigned doff[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) doff[q] = (unsigned)(q * RPI + rr) * dpitch + (unsigned)cc * 16u;
    // accumulators of token blocks [j0, j1) -> staging (bias is already in them)
    auto stage_blocks = [&](int j0, int j1) {
#pragma unroll
        for (int jj = j0; jj < j1; ++jj)
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const int f = i * 32 + 8 * v4 + 4 * g;
                    float r[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) r[e] = acc[i][jj][4 * v4 + e];
                    if (EPI == EPI_BIAS_GELU) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) r[e] = gelu_erf_fast(r[e]);
                    }
                    if (EPI == EPI_BIAS_TANH) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) r[e] = tanhf(r[e]);
                    }
                    if (EPI == EPI_QKV && transposed) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) *(bf16*)cell(f + e, jj * 32 + j31) = (bf16)r[e];
                    } else {
                        char* c = cell(jj * 32 + j31, f);
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
                }
    };
    // staged rows of half h -> global memory, 16 bytes per lane, whole row segments (rows are tokens, or features
    // if transposed)
    auto store_half = [&](int h) {
        const char* base = half_ptr(h);
        char* db = dst + (size_t)h * HR * dpitch;
#pragma unroll 2
        for (int pr = 0; pr < HR / 16; ++pr)
#pragma unroll
            for (int q = 0; q < NQ; ++q)
                *(uint4*)(db + (size_t)pr * 16 * dpitch + doff[q]) = *(const uint4*)(base + pr * 16 * ROWB + soff[q]);
    };
    constexpr int NRL = HR / RPI;                           // residual loads, and row stores, per half
    if (TM >= 2 && !(EPI == EPI_QKV && transposed)) {
        // token blocks [0, TM / 2) live in half 0: the second half of the residual rows arrives while the first
        // is computed, and the stores of the first half drain while the second is computed.  The waits are for
        // this wave's own loads (no barrier); they come before any store is issued, because the counter orders
        // loads among loads only.
        if (EPI == EPI_BIAS_RESIDUAL) wait_vmcnt<NRL>();
        stage_blocks(0, TM / 2);
        if (EPI == EPI_BIAS_RESIDUAL) wait_vmcnt<0>();
        store_half(0);
        stage_blocks(TM / 2, TM);
        store_half(1);
    } else {
        // one token block spans both halves, or staged rows are features: stage everything first
        if (EPI == EPI_BIAS_RESIDUAL) wait_vmcnt<0>();
        stage_blocks(0, TM);
        store_half(0);
        store_half(1);
    }
}

// -------------------------------------------------------------------------------------
// fp32 kernel: square tile of 16 TS rows x 16 TS features (TS = 4: 64 x 64, TS = 2: 32 x 32 for calls whose larger
// tiles would leave most compute units idle), 16 x 16 threads with TS x TS outputs each, FMA only, the reduction index
// ascending for every output.  Slabs of 64 along the reduction: the next slab's rows are requested (into registers)
// before the current one is multiplied, so a slab costs one memory round trip or its arithmetic, whichever is longer.
// -------------------------------------------------------------------------------------
template <int EPI, int TS>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int lda, size_t a_ss,
                                                       const char* __restrict__ arena, size_t student_stride,
                                                       size_t w_off, size_t b_off, float* __restrict__ out, int ldo,
                                                       size_t o_ss, const float* __restrict__ res, int ldr,
                                                       size_t r_ss, int Kd)
{
    constexpr int BT = 16 * TS, BK = 64, PITCH = BT + 4;
    constexpr int LPT = BT * BK / 4 / 256;                  // 16-byte loads per thread and operand: 16 rows apart
    typedef float fts __attribute__((ext_vector_type(TS)));
    __shared__ float As[BK][PITCH], Ws[BK][PITCH];
    const int m = blockIdx.z, m0 = blockIdx.y * BT, n0 = blockIdx.x * BT;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const float* Ag = A + (size_t)m * a_ss + (size_t)m0 * lda;
    const float* Wg = (const float*)(arena + (size_t)m * student_stride + w_off) + (size_t)n0 * Kd;
    const int lr = tid >> 4, lk = (tid & 15) * 4;           // loader: row lr + 16 i of the tile, reduction elements lk .. lk + 3
    f32x4 pa[LPT], pw[LPT];
    auto request = [&](int k0) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            pa[i] = *(const f32x4*)(Ag + (size_t)(lr + 16 * i) * lda + k0 + lk);
            pw[i] = *(const f32x4*)(Wg + (size_t)(lr + 16 * i) * Kd + k0 + lk);
        }
    };
    float acc[TS][TS] = {};
    request(0);
    for (int k0 = 0; k0 < Kd; k0 += BK) {
#pragma unroll
        for (int i = 0; i < LPT; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) { As[lk + e][lr + 16 * i] = pa[i][e]; Ws[lk + e][lr + 16 * i] = pw[i][e]; }
        __syncthreads();
        if (k0 + BK < Kd) request(k0 + BK);
#pragma unroll 16
        for (int kk = 0; kk < BK; ++kk) {
            const fts a = *(const fts*)&As[kk][ty * TS];
            const fts w = *(const fts*)&Ws[kk][tx * TS];
#pragma unroll
            for (int i = 0; i < TS; ++i)
#pragma unroll
                for (int j = 0; j < TS; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
    const float* bias = (const float*)(arena + (size_t)m * student_stride + b_off);
    const fts bv = *(const fts*)(bias + n0 + tx * TS);
#pragma unroll
    for (int i = 0; i < TS; ++i) {
        const size_t row = (size_t)(m0 + ty * TS + i);
        fts r;
#pragma unroll
        for (int j = 0; j < TS; ++j) r[j] = acc[i][j] + bv[j];
        if (EPI == EPI_BIAS_GELU) {
#pragma unroll
            for (int j = 0; j < TS; ++j) r[j] = gelu_erf(r[j]);
        }
        if (EPI == EPI_BIAS_RESIDUAL) r += *(const fts*)(res + (size_t)m * r_ss + row * ldr + n0 + tx * TS);
        *(fts*)(out + (size_t)m * o_ss + row * ldo + n0 + tx * TS) = r;
    }
}

// The same product for deep reductions on small grids (the FFN down-projection of a call of a few dozen tokens): one
// 32 x 32 tile per workgroup, the reduction range split over its four waves (a quarter each, ascending inside it, 4 x 4
// outputs per lane, wave-private slabs of 32 along the reduction), the four partial tiles added in wave order through
// LDS.  A single chain over the whole depth costs one memory round trip per slab; here a wave has four slabs in flight
// at once and a quarter of the depth to walk.  Kd must be a multiple of 512 (a wave's quarter: whole groups of four slabs).
template <int EPI, int TS>
__global__ __launch_bounds__(256) void gemm_f32_ksplit_kernel(const float* __restrict__ A, int lda, size_t a_ss,
                                                              const char* __restrict__ arena, size_t student_stride,
                                                              size_t w_off, size_t b_off, float* __restrict__ out,
                                                              int ldo, size_t o_ss, const float* __restrict__ res,
                                                              int ldr, size_t r_ss, int Kd)
{
    // tile of 8 TS x 8 TS outputs (TS = 4: 32 x 32; TS = 2: 16 x 16, four times the workgroups, when even the 32 x 32
    // tiles would leave most of the chip idle); a lane owns TS x TS of them
    constexpr int BT = 8 * TS, BK = 32, PITCH = BT + 4, SLAB = BK * PITCH;
    typedef float fts __attribute__((ext_vector_type(TS)));
    __shared__ __attribute__((aligned(16))) float lds[4 * 2 * SLAB];   // per wave: activation slab, weight slab
    const int m = blockIdx.z, m0 = blockIdx.y * BT, n0 = blockIdx.x * BT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tx = lane & 7, ty = lane >> 3;                // this lane's outputs: rows TS ty .., features TS tx ..
    const int kw = Kd / 4, kb = wave * kw;
    const float* Ag = A + (size_t)m * a_ss + (size_t)m0 * lda + kb;
    const float* Wg = (const float*)(arena + (size_t)m * student_stride + w_off) + (size_t)n0 * Kd + kb;
    float* As = lds + wave * 2 * SLAB;
    float* Ws = As + SLAB;
    // A wave requests four slabs (128 of its reduction range: all of it at a depth of 512) before it uses the first, so
    // their memory round trips overlap; then slab after slab goes through the wave's LDS and is multiplied.
    constexpr int NSL = 4, LPT = BT * BK / 4 / 64;          // 16-byte loads per lane, slab and operand
    f32x4 pa[NSL][LPT], pw[NSL][LPT];
    float acc[TS][TS] = {};
    for (int kc0 = 0; kc0 < kw; kc0 += NSL * BK) {
#pragma unroll
        for (int sl = 0; sl < NSL; ++sl)
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                const int idx = lane + 64 * i, row = idx >> 3, kc = (idx & 7) * 4;
                pa[sl][i] = *(const f32x4*)(Ag + (size_t)row * lda + kc0 + sl * BK + kc);
                pw[sl][i] = *(const f32x4*)(Wg + (size_t)row * Kd + kc0 + sl * BK + kc);
            }
#pragma unroll
        for (int sl = 0; sl < NSL; ++sl) {
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                const int idx = lane + 64 * i, row = idx >> 3, kc = (idx & 7) * 4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    As[(kc + e) * PITCH + row] = pa[sl][i][e];
                    Ws[(kc + e) * PITCH + row] = pw[sl][i][e];
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll 8
            for (int kk = 0; kk < BK; ++kk) {
                const fts a = *(const fts*)&As[kk * PITCH + ty * TS];
                const fts w = *(const fts*)&Ws[kk * PITCH + tx * TS];
#pragma unroll
                for (int i = 0; i < TS; ++i)
#pragma unroll
                    for (int j = 0; j < TS; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();                // the slab is rewritten only after every lane has read it
        }
    }
    // partial tiles -> LDS (over the slabs, which nobody reads any more), then summed in wave order
    __syncthreads();
    float* red = lds;                                       // [wave][row][PITCH]
#pragma unroll
    for (int i = 0; i < TS; ++i)
#pragma unroll
        for (int jj = 0; jj < TS; ++jj) red[(wave * BT + ty * TS + i) * PITCH + tx * TS + jj] = acc[i][jj];
    __syncthreads();
    constexpr int OUTS = BT * BT / 256, TPR = BT / OUTS;    // outputs per thread (neighbours in a row); threads per row
    const int r = tid / TPR, c0 = (tid % TPR) * OUTS;
    const float* bias = (const float*)(arena + (size_t)m * student_stride + b_off);
    const size_t row = (size_t)(m0 + r);
#pragma unroll
    for (int o = 0; o < OUTS; ++o) {
        const int c = c0 + o;
        float v = red[r * PITCH + c];
#pragma unroll
        for (int wv = 1; wv < 4; ++wv) v += red[(wv * BT + r) * PITCH + c];
        v += bias[n0 + c];
        if (EPI == EPI_BIAS_GELU) v = gelu_erf(v);
        if (EPI == EPI_BIAS_RESIDUAL) v += res[(size_t)m * r_ss + row * ldr + n0 + c];
        out[(size_t)m * o_ss + row * ldo + n0 + c] = v;
    }
}

template <int BM, int BN, int EPI>
hipError_t launch_bf16_tile(const sp_model* M, const void* A, int lda, size_t w_off, size_t b_off, void* out, int ldo,
                            const void* residual, int ldr, int mrows, int N, int Kd, int k, size_t a_ss, size_t o_ss,
                            size_t r_ss, hipStream_t s, void* out2, int n_split, int ld2, size_t o2_ss, int ksplit = 1,
                            int ldw = 0)
{
    static_assert(BM == BN, "the transposed epilogue assumes a square wave tile");
    if (ldw == 0) ldw = Kd;
    constexpr size_t smem = GemmTile<BM, BN>::smem_bytes;
    auto kern = gemm_bf16_kernel<BM, BN, EPI>;
    if (smem > 48 * 1024) {
        static std::atomic<bool> raised{false};   // per instantiation; the attribute is sticky for the process
        if (!raised.load(std::memory_order_acquire)) {   // (threads that race here set the same value twice)
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return e;
            raised.store(true, std::memory_order_release);
        }
    }
    const int mtiles = mrows / BM, ntiles = N / BN, total = k * ksplit * mtiles * ntiles;
    const int grid = ((total + 7) / 8) * 8;
    // token-tile blocking of the tile order (see the kernel): with the large tile and many feature tiles, the 32
    // workgroups an XCD runs at a time then cover about 5 x 6 tiles and fetch 11 operand tiles instead of 15, and the
    // activation tiles are re-used from the L2 by the next feature tiles; measured 4-5 % faster for the
    // QKV and FFN up-projections, no gain or slower with three feature tiles
    const int mb = BM == 256 && ntiles >= 6 ? 5 : 1;
    // (o_ss: bytes per student for the bf16 epilogues, fp32 elements per slice for EPI_PARTIAL)
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), smem, s, (const bf16*)A, lda, a_ss / 2, M->arena,
                       M->L.student_stride, w_off, b_off, (bf16*)out, ldo, EPI == EPI_PARTIAL ? o_ss : o_ss / 2,
                       (const bf16*)residual, ldr, r_ss / 2, Kd, mtiles, ntiles, total, (bf16*)out2, n_split, ld2,
                       o2_ss / 2, ksplit, ldw, mb);
    return hipGetLastError();
}

// fewest 256 x 256 tiles a launch must have to use them (one per compute unit)
constexpr long kLargeTileMinWorkgroups = 256;

template <int EPI>
hipError_t launch_bf16(const sp_model* M, const void* A, int lda, size_t w_off, size_t b_off, void* out, int ldo,
                       const void* residual, int ldr, int mrows, int N, int Kd, int k, size_t a_ss, size_t o_ss,
                       size_t r_ss, hipStream_t s, void* out2, int n_split, int ld2, size_t o2_ss)
{
#define SP_ARGS M, A, lda, w_off, b_off, out, ldo, residual, ldr, mrows, N, Kd, k, a_ss, o_ss, r_ss, s, out2, n_split, ld2, o2_ss
    // a feature tile must lie entirely on one side of n_split
    // (a grid of fewer large tiles than compute units leaves part of the chip idle: smaller tiles then; measured on the
    // batch-32 workload, one student: 0.285 -> 0.236 ms per call)
    if (mrows % 256 == 0 && mrows >= 2048 && N % 256 == 0 && n_split % 256 == 0 && Kd >= 256 &&
        (long)k * (mrows / 256) * (N / 256) >= kLargeTileMinWorkgroups) {
        return launch_bf16_tile<256, 256, EPI>(SP_ARGS);
    }
    // (a grid of fewer 128x128 tiles than compute units would leave most of the chip idle: smaller tiles then)
    if (mrows % 128 == 0 && N % 128 == 0 && n_split % 128 == 0 && (long)k * (mrows / 128) * (N / 128) >= 256)
        return launch_bf16_tile<128, 128, EPI>(SP_ARGS);
    return launch_bf16_tile<64, 64, EPI>(SP_ARGS);
#undef SP_ARGS
}

template <int EPI>
hipError_t launch_f32(const sp_model* M, const void* A, int lda, size_t w_off, size_t b_off, void* out, int ldo,
                      const void* residual, int ldr, int mrows, int N, int Kd, int k, size_t a_ss, size_t o_ss,
                      size_t r_ss, hipStream_t s)
{
    // (rows and widths are multiples of 64 and the reduction depth of 128: the launcher's callers see to that)
    if (mrows % 64 || N % 64 || Kd % 64) return hipErrorInvalidValue;
    // 64 x 64 tiles when they give every compute unit a few workgroups; else 32 x 32 tiles, four times as many
    if ((long)(N / 64) * (mrows / 64) * k >= 1024) {
        hipLaunchKernelGGL((gemm_f32_kernel<EPI, 4>), dim3(N / 64, mrows / 64, k), dim3(256), 0, s, (const float*)A, lda,
                           a_ss / 4, M->arena, M->L.student_stride, w_off, b_off, (float*)out, ldo, o_ss / 4,
                           (const float*)residual, ldr, r_ss / 4, Kd);
    } else if (Kd >= 512 && Kd % 512 == 0 && (long)(N / 32) * (mrows / 32) * k <= 256) {
        // few tiles and a deep reduction: the reduction range over the four waves of a workgroup
        if ((long)(N / 32) * (mrows / 32) * k < 128)
            hipLaunchKernelGGL((gemm_f32_ksplit_kernel<EPI, 2>), dim3(N / 16, mrows / 16, k), dim3(256), 0, s,
                               (const float*)A, lda, a_ss / 4, M->arena, M->L.student_stride, w_off, b_off, (float*)out,
                               ldo, o_ss / 4, (const float*)residual, ldr, r_ss / 4, Kd);
        else
            hipLaunchKernelGGL((gemm_f32_ksplit_kernel<EPI, 4>), dim3(N / 32, mrows / 32, k), dim3(256), 0, s,
                               (const float*)A, lda, a_ss / 4, M->arena, M->L.student_stride, w_off, b_off, (float*)out,
                               ldo, o_ss / 4, (const float*)residual, ldr, r_ss / 4, Kd);
    } else {
        hipLaunchKernelGGL((gemm_f32_kernel<EPI, 2>), dim3(N / 32, mrows / 32, k), dim3(256), 0, s, (const float*)A, lda,
                           a_ss / 4, M->arena, M->L.student_stride, w_off, b_off, (float*)out, ldo, o_ss / 4,
                           (const float*)residual, ldr, r_ss / 4, Kd);
    }
    return hipGetLastError();
}

// y[i] = the GELU of the bf16 epilogue evaluated on x[i], before any rounding to bf16 (test aid)
__global__ void gelu_probe_kernel(const float* __restrict__ x, float* __restrict__ y, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) y[i] = gelu_erf_fast(x[i]);
}

}  // namespace

hipError_t launch_gelu_probe(const float* x, float* y, long n, hipStream_t s)
{
    if (n < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gelu_probe_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, x, y, n);
    return hipGetLastError();
}

hipError_t launch_gemm_splitk(const sp_model* M, const void* A, int lda, size_t w_off, float* partials, int mrows, int N,
                              int Kd, int k, int splits, size_t a_student_stride, size_t slice_elems, hipStream_t s)
{
    if (!bf16_path(M->cfg) || splits < 1 || mrows % 64 || N % 64 || Kd % (64 * splits) || Kd / splits < 128 ||
        slice_elems < (size_t)mrows * N)
        return hipErrorInvalidValue;
    return launch_bf16_tile<64, 64, EPI_PARTIAL>(M, A, lda, w_off, 0, partials, N, nullptr, 0, mrows, N, Kd / splits, k,
                                                 a_student_stride, slice_elems, 0, s, nullptr, 0, 0, 0, splits, Kd);
}

hipError_t launch_gemm(const sp_model* M, const void* A, int lda, size_t w_off, size_t b_off, void* out, int ldo,
                       const void* residual, int ldr, int mrows, int N, int Kd, int k, Epilogue epi,
                       size_t a_student_stride, size_t o_student_stride, size_t r_student_stride, hipStream_t s,
                       void* out2, int n_split, int ld2, size_t o2_student_stride)
{
    // shapes the kernels assume; config_supported() guarantees them for every model that loads
    if (mrows % 64 || N % 64 || Kd % 128 || (epi == EPI_BIAS_RESIDUAL && !residual)) return hipErrorInvalidValue;
    if (epi == EPI_QKV && (!bf16_path(M->cfg) || !out2 || n_split % 64 || ld2 % 8)) return hipErrorInvalidValue;
#define SP_ARGS M, A, lda, w_off, b_off, out, ldo, residual, ldr, mrows, N, Kd, k, a_student_stride, \
                o_student_stride, r_student_stride, s
    if (bf16_path(M->cfg)) {
        switch (epi) {
            case EPI_BIAS: return launch_bf16<EPI_BIAS>(SP_ARGS, nullptr, 0, 0, 0);
            case EPI_BIAS_GELU: return launch_bf16<EPI_BIAS_GELU>(SP_ARGS, nullptr, 0, 0, 0);
            case EPI_QKV: return launch_bf16<EPI_QKV>(SP_ARGS, out2, n_split, ld2, o2_student_stride);
            case EPI_BIAS_TANH: return launch_bf16<EPI_BIAS_TANH>(SP_ARGS, nullptr, 0, 0, 0);
            default: return launch_bf16<EPI_BIAS_RESIDUAL>(SP_ARGS, nullptr, 0, 0, 0);
        }
    }
    if (epi == EPI_QKV || epi == EPI_BIAS_TANH) return hipErrorInvalidValue;   // bf16 path only
    switch (epi) {
        case EPI_BIAS: return launch_f32<EPI_BIAS>(SP_ARGS);
        case EPI_BIAS_GELU: return launch_f32<EPI_BIAS_GELU>(SP_ARGS);
        default: return launch_f32<EPI_BIAS_RESIDUAL>(SP_ARGS);
    }
#undef SP_ARGS
}

}  // namespace sp
