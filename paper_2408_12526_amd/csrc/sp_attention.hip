// Multi-head self-attention over a packed batch: every sequence attends to itself only,
// over exactly its own tokens (cu_seqlens gives the boundaries); head width is 64.
#include <atomic>
#include <type_traits>

#include "sp_internal.h"

namespace sp {

namespace {

constexpr int kD = 64;          // head width
constexpr int kQPerWg = 256;    // queries per workgroup of the long-sequence body: 4 waves x 2 blocks of 32
constexpr int kKeyTile = 64;    // keys staged in LDS per step
constexpr int kKStride = kKeyTile + 1;   // 16-byte units per k-group of the key tile
constexpr int kVStride = 68;    // bf16 elements per row of the transposed value tile (136 B)
constexpr int kOutPitch = kD * 2 + 16;   // bytes per staged output row
constexpr int kLongKBytes = 8 * kKStride * 16, kLongVBytes = kD * kVStride * 2;
constexpr int kLongTileBytes = kLongKBytes + kLongVBytes;   // one buffer of the key/value tile
constexpr int kLongLdsBytes = 2 * kLongTileBytes;
static_assert(kLongTileBytes % 16 == 0 && 4 * 32 * kOutPitch <= kLongLdsBytes, "the output tiles reuse the key/value buffers");

// 2^x by the hardware instruction alone.  (exp2f() wraps it in a range test, a scaling and an ldexp so that results
// below 2^-126 come out as denormals: four more instructions per value, which a softmax numerator does not need;
// arguments here are <= 0, and what underflows is flushed to zero.)
__device__ inline float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }

// A query's keys sit in lanes l and l ^ 32: maximum and sum over the two (every lane active).
__device__ inline float max_across_halves(float x) { float lo = x, hi = x; swap_halves(lo, hi); return fmaxf(lo, hi); }
__device__ inline float sum_across_halves(float x) { float lo = x, hi = x; swap_halves(lo, hi); return lo + hi; }

// eight bf16 values (one 16-byte chunk of an output row) -> eight e4m3 codes of value * qscale
__device__ inline uint2 chunk_to_fp8(uint4 c, float qscale)
{
    const bf16x8 v = __builtin_bit_cast(bf16x8, c);
    int lo = 0, hi = 0;
    lo = __builtin_amdgcn_cvt_pk_fp8_f32((float)v[0] * qscale, (float)v[1] * qscale, lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32((float)v[2] * qscale, (float)v[3] * qscale, lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32((float)v[4] * qscale, (float)v[5] * qscale, hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32((float)v[6] * qscale, (float)v[7] * qscale, hi, true);
    return uint2{(unsigned)lo, (unsigned)hi};
}

// -------------------------------------------------------------------------------------
// bf16 body on the matrix cores for long sequences.  One workgroup = (student, sequence, head, block of 256
// queries); wave w owns queries q0 + 64 w .. + 63 as two blocks of 32, which share every key and value fragment
// it reads from LDS.  Per 64-key tile and query block:
//   S^T = K Q^T      (A operand: key rows from LDS, B operand: the block's queries, kept in
//                     registers for the whole kernel)
//   online softmax   per query = per lane column; a query's keys sit in 16 accumulator
//                    registers of two lanes (l and l + 32); the 1/sqrt(d) log2(e) factor rides in the
//                    fused multiply-add in front of the exponential
//   O^T += V^T P^T   (A operand: transposed value tile from LDS; B operand: the
//                     probabilities, which already sit in the B-operand register layout
//                     once the reduction slots of V^T are enumerated in the same key order)
// The key/value tiles are double-buffered in LDS and travel through registers: tile t + 2 is requested from
// memory and tile t + 1 written to the idle buffer while tile t is multiplied; one barrier per tile, which
// waits for LDS traffic only (the loads stay in flight across it).
// -------------------------------------------------------------------------------------
__device__ __forceinline__ void attention_long_body(char* lds, int bid, const bf16* __restrict__ qkv,
                                                    const bf16* __restrict__ vt, bf16* __restrict__ att,
                                                    const int32_t* __restrict__ cu, int B, int Tn, int rows, int H,
                                                    int heads, int max_seqlen, int nqc, int min_len,
                                                    unsigned char* __restrict__ attq, float qscale)
{
    const int m = blockIdx.y;
    // (sequence, head) pairs go round the XCDs one by one (the few long sequences of a serving batch are spread evenly:
    // a contiguous run of sequences per XCD left them unevenly loaded and was measured 1.5x slower), but the query
    // blocks of one pair stay on one XCD (workgroup id mod 8), so that its keys and values are fetched into one L2
    const int xcd = bid & 7, y = bid >> 3;
    const int qc = y % nqc, pair = (y / nqc) * 8 + xcd;
    if (pair >= B * heads) return;
    const int h = pair % heads;
    const int b = pair / heads;
    int t0 = cu[b], t1 = cu[b + 1];
    t0 = t0 < 0 ? 0 : (t0 > Tn - 1 ? Tn - 1 : t0);
    int L = t1 - t0;
    L = L < 1 ? 1 : L;
    L = L > max_seqlen ? max_seqlen : L;
    L = L > Tn - t0 ? Tn - t0 : L;
    const int q0 = qc * kQPerWg;
    if (q0 >= L || L <= min_len) return;            // whole workgroup leaves together

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, g = lane >> 5;
    const size_t ld = (size_t)3 * H;
    const bf16* base = qkv + ((size_t)m * rows + t0) * ld + h * kD;
    const int qw = q0 + wave * 64;                  // the wave's first query
    const int g4 = 4 * g;

    // queries: B operand of S^T = K Q^T, four k-steps of 16 over d
    bf16x8 qf[2][4];
    f32x16 o[2][2];
    float mrun[2], lrun[2];                         // running maximum (raw scores) and sum of a query's half of the keys
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int q = qw + 32 * qb + j;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint4 t = {0, 0, 0, 0};
            if (q < L) t = *(const uint4*)(base + (size_t)q * ld + 16 * s + 8 * g);
            qf[qb][s] = __builtin_bit_cast(bf16x8, t);
        }
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[qb][db][e] = 0.f;
        mrun[qb] = -INFINITY;
        lrun[qb] = 0.f;
    }
    const float sl2 = 0.125f * 1.44269504088896341f;   // 1/sqrt(64) * log2(e)

    // Key tiles start at a token index that is a multiple of 8, so that the transposed values (token-contiguous
    // rows) can be fetched 16 bytes at a time; tokens in front of the sequence are masked below.
    const int lead = t0 & 7;
    const bf16* vbase = vt + ((size_t)m * H + h * kD) * rows + (t0 - lead);
    const int lrow = tid >> 3, lc = tid & 7;
    uint4 kreg[2], vreg[2];
    auto fetch = [&](int kt0) {                     // what lies beyond the sequence is zero-filled
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int r = lrow + 32 * p;            // key of the tile, or head dimension
            kreg[p] = uint4{0, 0, 0, 0};
            vreg[p] = uint4{0, 0, 0, 0};
            if (kt0 + r >= 0 && kt0 + r < L) kreg[p] = *(const uint4*)(base + (ptrdiff_t)(kt0 + r) * (ptrdiff_t)ld + H + lc * 8);
            if (kt0 + lc * 8 < L) vreg[p] = *(const uint4*)(vbase + (size_t)r * rows + (kt0 + lead) + lc * 8);
        }
    };
    auto stage = [&](int buf) {                     // registers -> LDS buffer: keys [d-group of 8][key], values [d][key]
        uint4* sK = (uint4*)(lds + buf * kLongTileBytes);
        bf16* sVt = (bf16*)(lds + buf * kLongTileBytes + kLongKBytes);
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int r = lrow + 32 * p;
            sK[lc * kKStride + r] = kreg[p];
            uint2* vd = (uint2*)(sVt + r * kVStride + lc * 8);
            vd[0] = uint2{vreg[p].x, vreg[p].y};
            vd[1] = uint2{vreg[p].z, vreg[p].w};
        }
    };
    const bool act1 = qw + 32 < L;                  // the wave's second query block exists (wave-uniform)
    const bool act0 = qw < L;
    fetch(-lead);
    stage(0);
    if (-lead + kKeyTile < L) fetch(-lead + kKeyTile);
    barrier_lds();
    int buf = 0;
    for (int kt0 = -lead; kt0 < L; kt0 += kKeyTile, buf ^= 1) {
        const uint4* sK = (const uint4*)(lds + buf * kLongTileBytes);
        const bf16* sVt = (const bf16*)(lds + buf * kLongTileBytes + kLongKBytes);
        if (act0) {
            // scores of the wave's query blocks against the 64 keys: two 32x32 blocks each
            f32x16 sc[2][2];
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) sc[qb][kb][e] = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const bf16x8 kf = __builtin_bit_cast(bf16x8, sK[(2 * s + g) * kKStride + kb * 32 + j]);
                    sc[0][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[0][s], sc[0][kb], 0, 0, 0);
                    if (act1) sc[1][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[1][s], sc[1][kb], 0, 0, 0);
                }
            // accumulator register v of this lane is key 8*(v/4) + 4*g + v%4 of its block; only the first and the
            // last tile of a sequence have keys to mask
            const bool edge = kt0 < 0 || kt0 + kKeyTile > L;
            bf16x8 pf[2][2][2];
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                if (qb == 1 && !act1) continue;
                float mx = mrun[qb];
                if (edge) {
                    // key kt0 + c + 4 g with c = 32 kb + 8 (v / 4) + v % 4 is valid if 0 <= key < L: the upper bound is
                    // one comparison of the lane's 4 g with a uniform value; only the first four registers of block 0
                    // can lie in front of the sequence (kt0 >= -7)
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int c = kb * 32 + 8 * (v >> 2) + (v & 3);
                            bool ok = g4 < L - kt0 - c;
                            if (kb == 0 && v < 4) ok = ok && g4 >= -kt0 - c;
                            if (!ok) sc[qb][kb][v] = -INFINITY;
                        }
                }
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sc[qb][kb][v]);
                mx = max_across_halves(mx);                 // the other half of the query's keys
                const float alpha = exp2_raw((mrun[qb] - mx) * sl2);   // first tile: exp2(-inf) = 0
                mrun[qb] = mx;
                const float nm = -mx * sl2;
                float psum = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float p = exp2_raw(fmaf(sc[qb][kb][v], sl2, nm));
                        psum += p;
                        pf[qb][kb][v >> 3][v & 7] = (bf16)p;
                    }
                lrun[qb] = lrun[qb] * alpha + psum;
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int e = 0; e < 16; ++e) o[qb][db][e] *= alpha;
            }
            // O^T += V^T P^T.  Reduction slot e of k-step s2 in block kb is key
            // 32*kb + 16*s2 + 8*(e/4) + 4*g + e%4, the key held by register 8*s2 + e above.
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const int kbase = kb * 32 + 16 * s2 + 4 * g;
#pragma unroll
                    for (int db = 0; db < 2; ++db) {
                        const bf16* vr = sVt + (db * 32 + j) * kVStride + kbase;
                        const bf16x4 lo = *(const bf16x4*)vr, hi = *(const bf16x4*)(vr + 8);
                        const bf16x8 vf = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                        o[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[0][kb][s2], o[0][db], 0, 0, 0);
                        if (act1) o[1][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[1][kb][s2], o[1][db], 0, 0, 0);
                    }
                }
        }
        if (kt0 + kKeyTile < L) {
            stage(buf ^ 1);                         // (idle since the barrier of the previous tile)
            if (kt0 + 2 * kKeyTile < L) fetch(kt0 + 2 * kKeyTile);
        }
        barrier_lds();
    }

    // Each 32 x 64 output block leaves through a wave-private LDS tile (the key/value buffers are idle now) as whole
    // 128-byte rows.
    char* stg = lds + wave * (32 * kOutPitch);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int qs = qw + 32 * qb;                // first query of the block
        if (qs >= L) continue;
        const float inv = 1.0f / sum_across_halves(lrun[qb]);
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (bf16)(o[qb][db][4 * v4 + e] * inv);
                *(bf16x4*)(stg + j * kOutPitch + (db * 32 + 8 * v4 + 4 * g) * 2) = w;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const int orow = lane >> 3, oc = lane & 7;
        const size_t doff = ((size_t)m * rows + t0 + qs) * H + h * kD + oc * 8;
#pragma unroll
        for (int r0 = 0; r0 < 32; r0 += 8)
            if (qs + r0 + orow < L) {
                const uint4 c = *(const uint4*)(stg + (r0 + orow) * kOutPitch + oc * 16);
                if (att) *(uint4*)(att + doff + (size_t)(r0 + orow) * H) = c;   // (null: the fp8 copy alone)
                if (attq) *(uint2*)(attq + doff + (size_t)(r0 + orow) * H) = chunk_to_fp8(c, qscale);   // fp8 copy
            }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();            // the tile is rewritten by the next block
    }
}


// -------------------------------------------------------------------------------------
// bf16 kernel for short sequences (the common case of the serving workloads: tens of tokens).  One wave = one
// (student, sequence, head); the four waves of a workgroup take four heads of the same sequence and never
// synchronise with each other: each wave stages its 32-key tiles in a private slice of LDS.  Same arithmetic as
// the kernel above (S^T = K Q^T, online softmax per lane column, O^T += V^T P^T), 32 queries per pass; the next
// key tile is fetched into registers while the current one is multiplied.
// -------------------------------------------------------------------------------------
constexpr int kSKey = 32;                 // keys per tile
constexpr int kSKStride = kSKey + 1;      // 16-byte units per d-group of the key tile
constexpr int kSVStride = 36;             // bf16 elements per row of the transposed value tile (72 B)
static_assert(kD * kSVStride * 2 == 32 * (kSVStride * 4) && kSVStride * 4 >= kD * 2 + 16, "the value slice doubles as the 32 x 64 output staging tile");

// QB: blocks of 32 queries a wave carries through one pass over the keys.  Every pass re-reads the sequence's keys and
// values, and between the passes of a dozen waves per compute unit they do not survive in the L2 (measured: the bytes
// fetched from beyond the L2 are those of one read of the queries plus one read of keys and values PER PASS), so
// QB = 2 halves the passes of sequences of more than 32 tokens; it costs the registers of a second set of queries and
// output accumulators (two waves per SIMD instead of three).
constexpr int kShortKBytes = 8 * kSKStride * 16, kShortVBytes = kD * kSVStride * 2;   // per wave
constexpr int kShortLdsBytes = 4 * (kShortKBytes + kShortVBytes);

template <int QB>
__device__ __forceinline__ void attention_short_body(char* lds, int bid, const bf16* __restrict__ qkv,
                                                     const bf16* __restrict__ vt, bf16* __restrict__ att,
                                                     const int32_t* __restrict__ cu, int B, int Tn, int rows, int H,
                                                     int heads, int max_seqlen, int ngroups, int max_len,
                                                     unsigned char* __restrict__ attq, float qscale)
{
    const int m = blockIdx.y;
    // XCD-aware order (workgroup id mod 8 selects the XCD): each XCD takes a contiguous run of sequences, so that
    // the lines of the token-contiguous value rows which neighbouring sequences share are fetched into one L2
    const int total = B * ngroups, chunk = (total + 7) >> 3;
    const int lin = (bid & 7) * chunk + (bid >> 3);
    if ((bid >> 3) >= chunk || lin >= total) return;
    const int b = lin / ngroups, hg = lin % ngroups;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = hg * 4 + wave;
    int t0 = cu[b], t1 = cu[b + 1];
    t0 = t0 < 0 ? 0 : (t0 > Tn - 1 ? Tn - 1 : t0);
    int L = t1 - t0;
    L = L < 1 ? 1 : L;
    L = L > max_seqlen ? max_seqlen : L;
    L = L > Tn - t0 ? Tn - t0 : L;
    if (L > max_len || h >= heads) return;         // long sequences belong to the cooperative kernel
    uint4* sK = (uint4*)(lds + wave * kShortKBytes);
    bf16* sVt = (bf16*)(lds + 4 * kShortKBytes + wave * kShortVBytes);

    const int j = lane & 31, g = lane >> 5;
    const int g4 = 4 * g;
    const size_t ld = (size_t)3 * H;
    const bf16* base = qkv + ((size_t)m * rows + t0) * ld + h * kD;
    const float sl2 = 0.125f * 1.44269504088896341f;
    const int lkey = lane >> 3, lc = lane & 7;      // key loader: 8 keys x 8 sixteen-byte chunks per instruction
    const int vrow = lane >> 2, vc = lane & 3;      // value loader: 16 head dimensions x 4 chunks of 8 keys
    // key tiles start at a token index that is a multiple of 8 (16-byte fetches of the token-contiguous values);
    // tokens in front of the sequence are masked
    const int lead = t0 & 7;
    const bf16* vbase = vt + ((size_t)m * H + h * kD) * rows + (t0 - lead);

    for (int q0 = 0; q0 < L; q0 += 32 * QB) {
        // query block qb covers queries q0 + 32 qb .. + 31; it is skipped as a whole (wave-uniform) if it lies beyond
        // the sequence
        bf16x8 qf[QB][4];
        f32x16 o[QB][2];
        float mrun[QB], lrun[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int q = q0 + 32 * qb + j;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                uint4 t = {0, 0, 0, 0};
                if (q < L) t = *(const uint4*)(base + (size_t)q * ld + 16 * s + 8 * g);
                qf[qb][s] = __builtin_bit_cast(bf16x8, t);
            }
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[qb][db][e] = 0.f;
            mrun[qb] = -INFINITY;
            lrun[qb] = 0.f;
        }

        uint4 kreg[4], vreg[4];
        auto fetch = [&](int kt0) {                  // kt0: first key of the tile relative to the sequence start
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int key = kt0 + p * 8 + lkey;
                kreg[p] = uint4{0, 0, 0, 0};
                vreg[p] = uint4{0, 0, 0, 0};
                if (key >= 0 && key < L) kreg[p] = *(const uint4*)(base + (ptrdiff_t)key * (ptrdiff_t)ld + H + lc * 8);
                if (kt0 + vc * 8 < L) vreg[p] = *(const uint4*)(vbase + (size_t)(p * 16 + vrow) * rows + (kt0 + lead) + vc * 8);
            }
        };
        fetch(-lead);
        for (int kt0 = -lead; kt0 < L; kt0 += kSKey) {
            // registers -> this wave's LDS slice (what lies beyond the sequence was fetched as zeros)
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                sK[lc * kSKStride + p * 8 + lkey] = kreg[p];
                uint2* vd = (uint2*)(sVt + (p * 16 + vrow) * kSVStride + vc * 8);
                vd[0] = uint2{vreg[p].x, vreg[p].y};
                vd[1] = uint2{vreg[p].z, vreg[p].w};
            }
            if (kt0 + kSKey < L) fetch(kt0 + kSKey);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();

#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                if (qb > 0 && q0 + 32 * qb >= L) continue;
                f32x16 sc;
#pragma unroll
                for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const uint4 t = sK[(2 * s + g) * kSKStride + j];
                    sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, t), qf[qb][s], sc, 0, 0, 0);
                }
                float mx = mrun[qb];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    // key kt0 + c + 4 g, c = 8 (v / 4) + v % 4, is valid if 0 <= key < L: one comparison of the lane's
                    // 4 g with a uniform value; only the first four registers can lie in front of the sequence
                    const int c = 8 * (v >> 2) + (v & 3);
                    bool ok = g4 < L - kt0 - c;
                    if (v < 4) ok = ok && g4 >= -kt0 - c;
                    const float sv = ok ? sc[v] : -INFINITY;
                    sc[v] = sv;
                    mx = fmaxf(mx, sv);
                }
                mx = max_across_halves(mx);
                // (running maximum on the raw scores; the 1/sqrt(d) log2(e) factor rides in the multiply-add in front of
                // the exponential)
                const float alpha = exp2_raw((mrun[qb] - mx) * sl2);
                mrun[qb] = mx;
                const float nm = -mx * sl2;
                float psum = 0.f;
                bf16x8 pf[2];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = exp2_raw(fmaf(sc[v], sl2, nm));
                    psum += p;
                    pf[v >> 3][v & 7] = (bf16)p;
                }
                lrun[qb] = lrun[qb] * alpha + psum;
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int e = 0; e < 16; ++e) o[qb][db][e] *= alpha;
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const int kbase = 16 * s2 + 4 * g;
#pragma unroll
                    for (int db = 0; db < 2; ++db) {
                        const bf16* vr = sVt + (db * 32 + j) * kSVStride + kbase;
                        const bf16x4 lo = *(const bf16x4*)vr, hi = *(const bf16x4*)(vr + 8);
                        const bf16x8 vf = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                        o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[s2], o[qb][db], 0, 0, 0);
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();       // the slice is rewritten at the top of the next iteration
        }
        // A 32 x 64 output block leaves through this wave's (now idle) value slice, so that a store instruction
        // writes eight whole 128-byte rows (eight-byte pieces of 32 rows per instruction are several times slower
        // on the way to memory).
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int qs = q0 + 32 * qb;                    // first query of the block
            if (qb > 0 && qs >= L) continue;
            const float inv = 1.0f / sum_across_halves(lrun[qb]);
            char* stg = (char*)sVt;                         // 32 rows of 144 bytes = the whole slice
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    bf16x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (bf16)(o[qb][db][4 * v4 + e] * inv);
                    *(bf16x4*)(stg + j * (kSVStride * 4) + (db * 32 + 8 * v4 + 4 * g) * 2) = w;
                }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const int orow = lane >> 3, oc = lane & 7;
            const size_t doff = ((size_t)m * rows + t0 + qs) * H + h * kD + oc * 8;
#pragma unroll
            for (int r0 = 0; r0 < 32; r0 += 8)
                if (qs + r0 + orow < L) {
                    const uint4 c = *(const uint4*)(stg + (r0 + orow) * (kSVStride * 4) + oc * 16);
                    if (att) *(uint4*)(att + doff + (size_t)(r0 + orow) * H) = c;   // (null: the fp8 copy alone)
                    if (attq) *(uint2*)(attq + doff + (size_t)(r0 + orow) * H) = chunk_to_fp8(c, qscale);   // fp8 copy
                }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();                // the slice is rewritten by the next block / pass
        }
    }
}

template <int QB>
__global__ __launch_bounds__(256, QB == 1 ? 3 : 2) void attention_bf16_short_kernel(
    const bf16* __restrict__ qkv, const bf16* __restrict__ vt, bf16* __restrict__ att, const int32_t* __restrict__ cu,
    int B, int Tn, int rows, int H, int heads, int max_seqlen, int ngroups, int max_len,
    unsigned char* __restrict__ attq, float qscale)
{
    __shared__ __attribute__((aligned(16))) char lds[kShortLdsBytes];
    attention_short_body<QB>(lds, (int)blockIdx.x, qkv, vt, att, cu, B, Tn, rows, H, heads, max_seqlen, ngroups, max_len,
                             attq, qscale);
}

// Batches with sequences on both sides of the split: one launch.  The first nlong workgroup ids (a multiple of 8, so
// the id-to-XCD relation of both bodies is kept) are the cooperative kernel's (sequence, head, query block) items,
// most of which leave at once; the rest are the per-wave kernel's.  The few long items start first and run beside
// the many short ones instead of in a launch of their own that cannot fill the chip.
__global__ __launch_bounds__(256, 2) void attention_bf16_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ vt,
                                                                bf16* __restrict__ att, const int32_t* __restrict__ cu,
                                                                int B, int Tn, int rows, int H, int heads,
                                                                int max_seqlen, int nqc, int ngroups, int split_len,
                                                                int nlong, unsigned char* __restrict__ attq,
                                                                float qscale)
{
    constexpr int kBytes = kLongLdsBytes > kShortLdsBytes ? kLongLdsBytes : kShortLdsBytes;
    __shared__ __attribute__((aligned(16))) char lds[kBytes];
    const int bid = (int)blockIdx.x;
    if (bid < nlong)
        attention_long_body(lds, bid, qkv, vt, att, cu, B, Tn, rows, H, heads, max_seqlen, nqc, split_len, attq, qscale);
    else
        attention_short_body<2>(lds, bid - nlong, qkv, vt, att, cu, B, Tn, rows, H, heads, max_seqlen, ngroups,
                                split_len, attq, qscale);
}

// -------------------------------------------------------------------------------------
// Attention of one query per sequence (its first token), used when only the first-token rows of the last layer are
// needed.  With a single query q per (sequence, head) the key and value projections of the other tokens never
// have to be formed:
//     score_t = q . (Wk^T x_t + bk) = (Wk q) . x_t + q . bk        (q . bk is the same for every t: softmax drops it)
//     out     = sum_t p_t (Wv^T x_t + bv) = Wv^T (sum_t p_t x_t) + bv          (the p_t sum to one)
// so the layer needs q~ = Wk q (one small product per head), one pass over the token rows x that yields the
// p-weighted mean row x^ per head, and Wv^T x^ + bv (another small product per head).  That replaces a projection
// of every token onto 2 H features, and reading those back, by one read of x.
// -------------------------------------------------------------------------------------

// Per-head small products: out[m][r][h][n] = sum_k A[m][r][h][k] W[m][h][n][k] (+ bias[m][h][n]), r < 32 * mtiles,
// n < 32 * NT * nstrips, k < Kd.  One strip of 32 rows x (32 NT) outputs per wave (the strip shares the row operand and
// writes runs of 64 NT contiguous bytes), fragments read straight from global memory (the work is a few GFLOP per
// call).  Strides are in elements; the weights live in the arena at w_off (+ student stride).
template <int NT>
__global__ __launch_bounds__(256) void head_gemm_kernel(const bf16* __restrict__ A, size_t a_ss, size_t a_hs, int lda,
                                                        const char* __restrict__ arena, size_t student_stride,
                                                        size_t w_off, size_t w_hs, int ldw, size_t b_off, size_t b_hs,
                                                        int has_bias, bf16* __restrict__ out, size_t o_ss, size_t o_hs,
                                                        int ldo, int mtiles, int nstrips, int Kd, int heads, int total)
{
    // XCD-aware order: consecutive workgroup ids go to different XCDs; each XCD gets a contiguous run of (student,
    // head, group of four strips), so a head's weight slice is fetched into one L2 instead of all eight.
    const int chunk = (total + 7) >> 3;
    const int lin = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= chunk || lin >= total) return;
    const int per_head = (mtiles * nstrips + 3) / 4;
    const int m = lin / (per_head * heads), h = (lin / per_head) % heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int item = (lin % per_head) * 4 + wave;
    if (item >= mtiles * nstrips) return;
    const int ns = item % nstrips, mt = item / nstrips;
    const int j31 = lane & 31, g = lane >> 5;
    const bf16* a = A + (size_t)m * a_ss + (size_t)h * a_hs + (size_t)(mt * 32 + j31) * lda + 8 * g;
    const bf16* w = (const bf16*)(arena + (size_t)m * student_stride + w_off) + (size_t)h * w_hs +
                    (size_t)(ns * NT * 32 + j31) * ldw + 8 * g;
    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
#pragma unroll 8
    for (int k0 = 0; k0 < Kd; k0 += 16) {
        const bf16x8 fa = *(const bf16x8*)(a + k0);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const bf16x8 fw = *(const bf16x8*)(w + (size_t)t * 32 * ldw + k0);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw, fa, acc[t], 0, 0, 0);   // rows: output features, columns: r
        }
    }
    // lane: row r = j31 of the strip; output features 32 t + 8 (v / 4) + 4 g + v % 4.  The strip goes through a
    // wave-private LDS tile so that it leaves as whole 16-byte-per-lane row segments (eight-byte pieces scattered
    // over 32 rows per instruction are several times slower on the way to memory).
    constexpr int SW = NT * 32;                             // strip width (features)
    constexpr int PITCH = SW * 2 + 16;                      // bytes per staged row
    __shared__ __attribute__((aligned(16))) char stage_all[4][32 * PITCH];
    char* stg = stage_all[wave];
    const float* bias = (const float*)(arena + (size_t)m * student_stride + b_off) + (size_t)h * b_hs + ns * SW;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            const int f = 32 * t + 8 * v4 + 4 * g;
            bf16x4 r;
#pragma unroll
            for (int e = 0; e < 4; ++e) r[e] = (bf16)(acc[t][4 * v4 + e] + (has_bias ? bias[f + e] : 0.f));
            *(bf16x4*)(stg + j31 * PITCH + f * 2) = r;
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    constexpr int CPR = SW / 8, RPI = 64 / CPR;             // 16-byte chunks per row, rows per instruction
    const int rr = lane / CPR, cc = lane % CPR;
    bf16* o = out + (size_t)m * o_ss + (size_t)h * o_hs + (size_t)(mt * 32) * ldo + ns * SW + cc * 8;
#pragma unroll
    for (int r0 = 0; r0 < 32; r0 += RPI)
        *(uint4*)(o + (size_t)(r0 + rr) * ldo) = *(const uint4*)(stg + (r0 + rr) * PITCH + cc * 16);
}

// The same products when the reduction is long and the outputs are few (the value projection of the weighted mean rows:
// Kd = H, 64 outputs per head): one 32-row x 64-output item per workgroup, its four waves split the reduction range, and
// the partial tiles are added through LDS (waves in a fixed order), so that a wave's chain of dependent loads is a quarter
// as long and four times as many compute units take part.  Kd must be a multiple of 64.
__global__ __launch_bounds__(256) void head_gemm_ksplit_kernel(const bf16* __restrict__ A, size_t a_ss, size_t a_hs,
                                                               int lda, const char* __restrict__ arena,
                                                               size_t student_stride, size_t w_off, size_t w_hs,
                                                               int ldw, size_t b_off, size_t b_hs, int has_bias,
                                                               bf16* __restrict__ out, size_t o_ss, size_t o_hs, int ldo,
                                                               int mtiles, int nstrips, int Kd, int heads, int total)
{
    constexpr int NT = 2, SW = NT * 32, PP = 33;            // strip width; pitch of a feature's 32 rows (floats)
    __shared__ float part[4 * SW * PP];
    // XCD-aware order as in head_gemm_kernel: a head's weight slice is fetched into one L2
    const int chunk = (total + 7) >> 3;
    const int lin = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= chunk || lin >= total) return;
    const int per_head = mtiles * nstrips;
    const int m = lin / (per_head * heads), h = (lin / per_head) % heads, item = lin % per_head;
    const int ns = item % nstrips, mt = item / nstrips;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j31 = lane & 31, g = lane >> 5;
    const int kw = Kd / 4;                                  // this wave's share of the reduction range
    const bf16* a = A + (size_t)m * a_ss + (size_t)h * a_hs + (size_t)(mt * 32 + j31) * lda + wave * kw + 8 * g;
    const bf16* w = (const bf16*)(arena + (size_t)m * student_stride + w_off) + (size_t)h * w_hs +
                    (size_t)(ns * SW + j31) * ldw + wave * kw + 8 * g;
    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
#pragma unroll 12
    for (int k0 = 0; k0 < kw; k0 += 16) {
        const bf16x8 fa = *(const bf16x8*)(a + k0);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const bf16x8 fw = *(const bf16x8*)(w + (size_t)t * 32 * ldw + k0);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw, fa, acc[t], 0, 0, 0);   // rows: output features, columns: r
        }
    }
    // lane: row r = j31 of the strip; output features 32 t + 8 (v / 4) + 4 g + v % 4
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            part[(wave * SW + 32 * t + 8 * (v / 4) + 4 * g + v % 4) * PP + j31] = acc[t][v];
    __syncthreads();
    // thread: row r = tid % 32, eight neighbouring features: one 16-byte piece of the output row
    const int r = tid & 31, f0 = (tid >> 5) * 8;
    const float* bias = (const float*)(arena + (size_t)m * student_stride + b_off) + (size_t)h * b_hs + ns * SW + f0;
    bf16x8 o8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float sum = has_bias ? bias[i] : 0.f;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) sum += part[(wv * SW + f0 + i) * PP + r];
        o8[i] = (bf16)sum;
    }
    *(bf16x8*)(out + (size_t)m * o_ss + (size_t)h * o_hs + (size_t)(mt * 32 + r) * ldo + ns * SW + f0) = o8;
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Maximum / sum over the four lanes l % 16 + {0, 16, 32, 48} (every lane active).
__device__ inline float max_across_rows(float v)
{
    float a = v, b = v;
    swap_rows(a, b);
    v = fmaxf(a, b);
    a = v;
    b = v;
    swap_halves(a, b);
    return fmaxf(a, b);
}
__device__ inline float sum_across_rows(float v)
{
    float a = v, b = v;
    swap_rows(a, b);
    v = a + b;
    a = v;
    b = v;
    swap_halves(a, b);
    return a + b;
}

// One workgroup (eight waves) per (student, sequence); the sequence's token rows x are read from global memory once, in
// tiles of 32 tokens, and every wave touches only its own eighth of the features (FW = H / 8 of them):
//   scores: heads x tokens on the matrix cores (16 x 16 x 32 shape: two blocks of 16 tokens, FW / 32 steps of 32
//           features); the token rows arrive in registers in operand layout (lane: token l % 16, eight features); the
//           waves' partial tiles are added in a fixed order through LDS;
//   weighted rows: features x heads, reduction over the tile's 32 tokens in one instruction.  That operand wants eight
//           tokens of one feature per lane, so the wave writes its registers to its own LDS slab (16-byte chunks
//           XOR-swizzled by the token) and reads them back as 4-byte pieces (two neighbouring features) of eight
//           tokens, unzipped into two operands: row r of operand c is feature 2 r + c of a block of 32.  The softmax
//           is the running one (maximum and sum per head, accumulators rescaled when the maximum moves); every wave
//           keeps the statistics of all heads: lane l holds head l % 16 and tokens 8 (l / 16) ... + 8 of the tile.
// The next tile's rows are requested as soon as the current ones are in LDS.  Two workgroup barriers per tile; about
// 66 KB of LDS at hidden width 768 and at most 128 registers, so two workgroups share a compute unit and one's
// start-up and barrier waits are covered by the other.
//   qt   [m][b][head][H]   folded queries (row stride HEADS * H)
//   xbar [m][b][head][H]   output; rows b in [B, gridDim.x) are zeroed (they feed padded projections)
constexpr int kFoldWaves = 8;
template <int HEADS>
struct FoldLds {
    static constexpr int H = HEADS * kD, FW = H / kFoldWaves;   // features per wave
    static constexpr int SCP = 36;                          // pitch of a head's 32 scores (floats)
    static constexpr size_t slab_bytes = (size_t)32 * FW * 2;   // per wave: 32 tokens x FW features
    static constexpr size_t bytes = kFoldWaves * (slab_bytes + 16 * 32 * 4) + (size_t)16 * SCP * 4;
    static_assert(FW % 32 == 0 && HEADS <= 16 && bytes <= 160 * 1024, "whole reduction steps per wave, heads in one block");
};

template <int HEADS>
__global__ __launch_bounds__(512, HEADS == 16 ? 2 : 4) void attention_first_fold_kernel(const bf16* __restrict__ x,
                                                                      const bf16* __restrict__ qt,
                                                                      bf16* __restrict__ xbar,
                                                                      const int32_t* __restrict__ cu, int B, int Tn,
                                                                      int rows, int crows, int max_seqlen)
{
    using F = FoldLds<HEADS>;
    constexpr int H = F::H, FW = F::FW, SCP = F::SCP, NW = kFoldWaves;
    constexpr int KS = FW / 32;                             // 32-feature steps (scores) = 32-feature blocks (output)
    constexpr int PITCH = FW * 2;                           // slab row, bytes
    extern __shared__ uint4 fold_smem[];
    float* part = (float*)((char*)fold_smem + NW * F::slab_bytes);   // [waves][16][32] partial score tiles
    float* sc = part + NW * 16 * 32;                        // [16][SCP] scores of the current tile, log2 units
    const int m = blockIdx.y, b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    char* slab = (char*)fold_smem + wave * F::slab_bytes;   // this wave's features of the tile: [token][FW / 8 chunks]
    bf16* xb = xbar + ((size_t)m * crows + b) * HEADS * H;
    if (b >= B) {
        for (int c = tid; c < HEADS * H / 8; c += 64 * NW) ((uint4*)xb)[c] = make_uint4(0, 0, 0, 0);
        return;
    }
    int t0 = cu[b], t1 = cu[b + 1];
    t0 = t0 < 0 ? 0 : (t0 > Tn - 1 ? Tn - 1 : t0);
    int L = t1 - t0;
    L = L < 1 ? 1 : L;
    L = L > max_seqlen ? max_seqlen : L;
    L = L > Tn - t0 ? Tn - t0 : L;
    const int l16 = lane & 15, kg = lane >> 4;
    const bf16* xw = x + ((size_t)m * rows + t0) * H + wave * FW + 8 * kg;   // this lane's features of the first token
    const int nt = (L + 31) >> 5;

    // folded-query operands: row = head, the wave's features in steps of 32 (lane: eight of them)
    bf16x8 fq[KS];
    {
        const bf16* qr = qt + (((size_t)m * crows + b) * HEADS + (l16 < HEADS ? l16 : 0)) * H + wave * FW + 8 * kg;
#pragma unroll
        for (int st = 0; st < KS; ++st) {
            fq[st] = *(const bf16x8*)(qr + 32 * st);
            if (l16 >= HEADS) {
#pragma unroll
                for (int e = 0; e < 8; ++e) fq[st][e] = (bf16)0.f;
            }
        }
    }
    // token rows of a tile in operand layout: block nb holds tokens 16 nb + l16.  Rows beyond the sequence repeat its
    // last row (they get probability zero).
    bf16x8 xr[2][KS];
    auto load_tile = [&](int tile) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            int tok = tile * 32 + 16 * nb + l16;
            tok = tok < L ? tok : L - 1;
#pragma unroll
            for (int st = 0; st < KS; ++st) xr[nb][st] = *(const bf16x8*)(xw + (size_t)tok * H + 32 * st);
        }
    };
    load_tile(0);

    const float scale = 0.125f * 1.44269504088896341f;
    f32x4 acc[2 * KS];                                      // [block of 32 features][c]: feature 2 row + c, column = head
#pragma unroll
    for (int a = 0; a < 2 * KS; ++a) acc[a] = f32x4{0.f, 0.f, 0.f, 0.f};
    float mrun = -INFINITY, lrun = 0.f;
    for (int tile = 0; tile < nt; ++tile) {
        // partial scores[head][token] over this wave's features
        f32x4 sa[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int st = 0; st < KS; ++st)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
                sa[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fq[st], xr[nb][st], sa[nb], 0, 0, 0);   // rows: heads, columns: tokens
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 4; ++v) part[(wave * 16 + 4 * kg + v) * 32 + 16 * nb + l16] = sa[nb][v];
        // the rows into the wave's slab: chunk ch of token r sits in slot ch ^ ((r / 2) % 4).  (The wave's previous
        // reads of the slab are behind it: LDS accesses of one wave execute in order.)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int st = 0; st < KS; ++st)
                *(bf16x8*)(slab + (16 * nb + l16) * PITCH + (((4 * st + kg) ^ ((l16 >> 1) & 3)) << 4)) = xr[nb][st];
        __builtin_amdgcn_sched_barrier(0);                  // (the next rows take over the registers of these)
        if (tile + 1 < nt) load_tile(tile + 1);
        barrier_lds();
        {
            const int hh = tid >> 5, t = tid & 31;          // 16 x 32 sums, one per thread, waves in a fixed order
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) sum += part[(w * 16 + hh) * 32 + t];
            sc[hh * SCP + t] = tile * 32 + t < L ? sum * scale : -INFINITY;
        }
        barrier_lds();

        // xbar^T[feature][head] += sum_t x[t][feature] p[head][t]
        const float* sr = sc + (l16 < HEADS ? l16 : 0) * SCP + 8 * kg;
        const f32x4 s0 = *(const f32x4*)sr, s1 = *(const f32x4*)(sr + 4);
        float p[8];
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            p[e] = s0[e];
            p[4 + e] = s1[e];
            mx = fmaxf(mx, fmaxf(s0[e], s1[e]));
        }
        mx = fmaxf(mrun, max_across_rows(mx));              // finite: the tile has at least one token of the sequence
        const float alpha = exp2_raw(mrun - mx);            // first tile: exp2(-inf) = 0
        mrun = mx;
        float ls = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            p[e] = exp2_raw(p[e] - mx);
            ls += p[e];
        }
        lrun = fmaf(lrun, alpha, ls);
#pragma unroll
        for (int a = 0; a < 2 * KS; ++a) acc[a] *= alpha;
        bf16x8 fp;
#pragma unroll
        for (int e = 0; e < 8; ++e) fp[e] = (bf16)(l16 < HEADS ? p[e] : 0.f);
#pragma unroll
        for (int gq = 0; gq < KS; ++gq) {
            bf16x2 xv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e)                     // token 8 kg + e of the tile: (token / 2) % 4 = e / 2
                xv[e] = *(const bf16x2*)(slab + (8 * kg + e) * PITCH + (((4 * gq + (l16 >> 2)) ^ (e >> 1)) << 4) + (l16 & 3) * 4);
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                bf16x8 fx;
#pragma unroll
                for (int e = 0; e < 8; ++e) fx[e] = xv[e][c];
                acc[2 * gq + c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fx, fp, acc[2 * gq + c], 0, 0, 0);   // rows: features, columns: heads
            }
        }
    }
    const float inv = 1.0f / sum_across_rows(lrun);
    // lane: head l16; element v of acc[2 gq + c] is feature 32 gq + 2 (4 kg + v) + c of the wave's FW
    if (l16 < HEADS) {
#pragma unroll
        for (int gq = 0; gq < KS; ++gq) {
            bf16x8 r;
#pragma unroll
            for (int i = 0; i < 8; ++i) r[i] = (bf16)(acc[2 * gq + (i & 1)][i >> 1] * inv);
            *(bf16x8*)(xb + (size_t)l16 * H + wave * FW + 32 * gq + 8 * kg) = r;
        }
    }
}

// -------------------------------------------------------------------------------------
// fp32 kernel: one workgroup per (student, sequence, head, block of 64 queries); four neighbouring lanes share a query,
// sixteen of the head's 64 dimensions each (the score is summed over the quad, every lane rescales and accumulates its
// own sixteen output dimensions).  Keys and values come through LDS in chunks of 64 tokens; all lanes of a wave read
// the same key row (a broadcast).  Online softmax in registers, exact exponentials and division.
// -------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attention_f32_kernel(const float* __restrict__ qkv, float* __restrict__ att,
                                                            const int32_t* __restrict__ cu, int B, int Tn, int rows,
                                                            int H, int heads, int max_seqlen, int nqc)
{
    constexpr int KC = 64, DP = kD / 4;                     // keys per chunk; dimensions per lane
    __shared__ __attribute__((aligned(16))) float Ks[KC][kD], Vs[KC][kD];
    const int m = blockIdx.y;
    int idx = blockIdx.x;
    const int qc = idx % nqc; idx /= nqc;
    const int h = idx % heads;
    const int b = idx / heads;
    int t0 = cu[b], t1 = cu[b + 1];
    t0 = t0 < 0 ? 0 : (t0 > Tn - 1 ? Tn - 1 : t0);
    int L = t1 - t0;
    L = L < 1 ? 1 : L;
    L = L > max_seqlen ? max_seqlen : L;
    L = L > Tn - t0 ? Tn - t0 : L;
    if (qc * 64 >= L) return;                               // (uniform over the workgroup)
    const int tid = threadIdx.x, part = tid & 3, q = qc * 64 + (tid >> 2);
    const bool live = q < L;
    const size_t ld = (size_t)3 * H;
    const float* base = qkv + ((size_t)m * rows + t0) * ld + h * kD;
    float qv[DP], o[DP];
#pragma unroll
    for (int e4 = 0; e4 < DP; e4 += 4) {
        const f32x4 t = live ? *(const f32x4*)(base + (size_t)q * ld + DP * part + e4) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 4; ++e) { qv[e4 + e] = t[e]; o[e4 + e] = 0.f; }
    }
    float mrun = -INFINITY, lrun = 0.f;
    for (int kt0 = 0; kt0 < L; kt0 += KC) {
        const int nk = L - kt0 < KC ? L - kt0 : KC;
        __syncthreads();                                    // the previous chunk has been read by everybody
#pragma unroll
        for (int i = 0; i < KC * kD / 4 / 256; ++i) {
            const int c = tid + 256 * i, key = c >> 4, d = (c & 15) * 4;
            if (key < nk) {
                const float* kr = base + (size_t)(kt0 + key) * ld + H + d;
                *(f32x4*)&Ks[key][d] = *(const f32x4*)kr;
                *(f32x4*)&Vs[key][d] = *(const f32x4*)(kr + H);
            }
        }
        __syncthreads();
        for (int key = 0; key < nk; ++key) {
            float sdot = 0.f;
#pragma unroll
            for (int e4 = 0; e4 < DP; e4 += 4) {
                const f32x4 kv = *(const f32x4*)&Ks[key][DP * part + e4];
#pragma unroll
                for (int e = 0; e < 4; ++e) sdot = fmaf(qv[e4 + e], kv[e], sdot);
            }
            sdot += dpp_moved<kDppPair>(sdot);              // the four lanes of a query: every one ends with the whole sum
            sdot += dpp_moved<kDppQuad>(sdot);
            sdot *= 0.125f;
            const float mx = fmaxf(mrun, sdot);
            const float alpha = expf(mrun - mx), p = expf(sdot - mx);
            lrun = lrun * alpha + p;
#pragma unroll
            for (int e4 = 0; e4 < DP; e4 += 4) {
                const f32x4 vv = *(const f32x4*)&Vs[key][DP * part + e4];
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e4 + e] = o[e4 + e] * alpha + p * vv[e];
            }
            mrun = mx;
        }
    }
    if (live) {
        float* dst = att + ((size_t)m * rows + t0 + q) * H + h * kD + DP * part;
#pragma unroll
        for (int e4 = 0; e4 < DP; e4 += 4)
            *(f32x4*)(dst + e4) = f32x4{o[e4] / lrun, o[e4 + 1] / lrun, o[e4 + 2] / lrun, o[e4 + 3] / lrun};
    }
}

}  // namespace

hipError_t launch_attention(const sp_model* M, const void* qkv, const void* vt, void* att, const int32_t* cu, int B,
                            int T, int max_seqlen, int rows, int k, hipStream_t s, void* attq, float qscale)
{
    const sp_config& c = M->cfg;
    if (c.hidden / c.heads != kD) return hipErrorInvalidValue;
    if (!att && !(attq && bf16_path(c))) return hipErrorInvalidValue;   // (no bf16 output: the fp8 copy alone)
    if (bf16_path(c)) {
        // Sequences of up to 128 tokens: one wave per (sequence, head); longer ones: one workgroup per (sequence,
        // head, 128 queries) sharing the key/value tiles.  Each kernel skips the other's sequences.  (Giving the long
        // sequences of a serving batch to the per-wave kernel as well was measured slower: a 256-token sequence is 72
        // tile iterations in one wave, a long tail behind the ~5 of a typical one.)
        const int kShortLen = 128;
        const int ngroups = (c.heads + 3) / 4;
        const unsigned nshort = (unsigned)((B * ngroups + 7) / 8 * 8);
        if (max_seqlen > kShortLen) {
            const int nqc = (max_seqlen + kQPerWg - 1) / kQPerWg;
            const unsigned nlong = (unsigned)((B * c.heads + 7) / 8 * 8 * nqc);
            hipLaunchKernelGGL(attention_bf16_kernel, dim3(nlong + nshort, k), dim3(256), 0, s, (const bf16*)qkv,
                               (const bf16*)vt, (bf16*)att, cu, B, T, rows, c.hidden, c.heads, max_seqlen, nqc, ngroups,
                               kShortLen, (int)nlong, (unsigned char*)attq, qscale);
        } else if (max_seqlen > 32) {
            // two query blocks per pass wherever a sequence can have more than one (burst workload: 0.330 -> 0.280 ms
            // for the attention phase; four blocks, one wave per SIMD: 0.353 ms)
            hipLaunchKernelGGL(attention_bf16_short_kernel<2>, dim3(nshort, k), dim3(256), 0, s, (const bf16*)qkv,
                               (const bf16*)vt, (bf16*)att, cu, B, T, rows, c.hidden, c.heads, max_seqlen, ngroups,
                               kShortLen, (unsigned char*)attq, qscale);
        } else {
            hipLaunchKernelGGL(attention_bf16_short_kernel<1>, dim3(nshort, k), dim3(256), 0, s, (const bf16*)qkv,
                               (const bf16*)vt, (bf16*)att, cu, B, T, rows, c.hidden, c.heads, max_seqlen, ngroups,
                               kShortLen, (unsigned char*)attq, qscale);
        }
    } else {
        const int nqc = (max_seqlen + 63) / 64;
        dim3 grid((unsigned)(B * c.heads * nqc), k);
        hipLaunchKernelGGL(attention_f32_kernel, grid, dim3(256), 0, s, (const float*)qkv, (float*)att, cu, B, T, rows,
                           c.hidden, c.heads, max_seqlen, nqc);
    }
    return hipGetLastError();
}

hipError_t launch_head_gemm(const sp_model* M, const void* A, size_t a_ss, size_t a_hs, int lda, size_t w_off,
                            size_t w_hs, int ldw, size_t b_off, size_t b_hs, bool has_bias, void* out, size_t o_ss,
                            size_t o_hs, int ldo, int mrows, int N, int Kd, int k, hipStream_t s)
{
    const sp_config& c = M->cfg;
    if (!bf16_path(c) || mrows % 32 || N % 32 || Kd % 16 || lda % 8 || ldw % 8 || ldo % 8 || a_hs % 8 ||
        w_hs % 8 || o_hs % 8)
        return hipErrorInvalidValue;
    const int mtiles = mrows / 32;
    if (N % 128 != 0 && N % 64 == 0 && Kd >= 256 && Kd % 64 == 0) {
        const int nstrips = N / 64;
        const int total = k * c.heads * mtiles * nstrips;
        dim3 grid((unsigned)((total + 7) / 8 * 8));
        hipLaunchKernelGGL(head_gemm_ksplit_kernel, grid, dim3(256), 0, s, (const bf16*)A, a_ss, a_hs, lda, M->arena,
                           M->L.student_stride, w_off, w_hs, ldw, b_off, b_hs, has_bias ? 1 : 0, (bf16*)out, o_ss, o_hs,
                           ldo, mtiles, nstrips, Kd, c.heads, total);
        return hipGetLastError();
    }
#define SP_HEAD_GEMM(NT)                                                                                            \
    do {                                                                                                            \
        const int nstrips = N / (32 * NT);                                                                          \
        const int total = k * c.heads * ((mtiles * nstrips + 3) / 4);                                               \
        dim3 grid((unsigned)((total + 7) / 8 * 8));                                                                 \
        hipLaunchKernelGGL(head_gemm_kernel<NT>, grid, dim3(256), 0, s, (const bf16*)A, a_ss, a_hs, lda, M->arena,  \
                           M->L.student_stride, w_off, w_hs, ldw, b_off, b_hs, has_bias ? 1 : 0, (bf16*)out, o_ss,  \
                           o_hs, ldo, mtiles, nstrips, Kd, c.heads, total);                                         \
    } while (0)
    if (N % 128 == 0) SP_HEAD_GEMM(4);
    else if (N % 64 == 0) SP_HEAD_GEMM(2);
    else SP_HEAD_GEMM(1);
#undef SP_HEAD_GEMM
    return hipGetLastError();
}

bool attention_first_fold_supported(const sp_config& c, int max_seqlen)
{
    (void)max_seqlen;                                       // any length: the softmax is a running one
    return bf16_path(c) && c.hidden / c.heads == kD && c.heads % 4 == 0 && c.heads <= 16;
}

hipError_t launch_attention_first_fold(const sp_model* M, const void* x, const void* qt, void* xbar, const int32_t* cu,
                                       int B, int T, int max_seqlen, int rows, int crows, int cmrows, int k,
                                       hipStream_t s)
{
    const sp_config& c = M->cfg;
    if (!attention_first_fold_supported(c, max_seqlen) || cmrows < B || cmrows > crows) return hipErrorInvalidValue;
    dim3 grid((unsigned)cmrows, (unsigned)k);
#define SP_FOLD(HEADS)                                                                                              \
    do {                                                                                                            \
        auto kern = attention_first_fold_kernel<HEADS>;                                                             \
        constexpr size_t smem = FoldLds<HEADS>::bytes;                                                              \
        static std::atomic<bool> raised{false}; /* the attribute is sticky for the process */                      \
        if (smem > 48 * 1024 && !raised) {                                                                          \
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,      \
                                               (int)smem);                                                          \
            if (e != hipSuccess) return e;                                                                          \
            raised = true;                                                                                          \
        }                                                                                                           \
        hipLaunchKernelGGL(kern, grid, dim3(64 * kFoldWaves), smem, s, (const bf16*)x, (const bf16*)qt, (bf16*)xbar,  \
                           cu, B, T, rows, crows, max_seqlen);                                                      \
    } while (0)
    switch (c.heads) {
        case 4: SP_FOLD(4); break;
        case 8: SP_FOLD(8); break;
        case 12: SP_FOLD(12); break;
        default: SP_FOLD(16); break;
    }
#undef SP_FOLD
    return hipGetLastError();
}

}  // namespace sp
