// Multi-head self-attention over a packed batch: every sequence attends to itself only,
// over exactly its own tokens (cu_seqlens gives the boundaries); head width is 64.
#include "sp_internal.h"

namespace sp {

namespace {

constexpr int kD = 64;          // head width
constexpr int kQPerWg = 128;    // queries per workgroup: 4 waves x 32
constexpr int kKeyTile = 64;    // keys staged in LDS per step
constexpr int kKStride = kKeyTile + 1;   // 16-byte units per k-group of the key tile
constexpr int kVStride = 68;    // bf16 elements per row of the transposed value tile (136 B)

// -------------------------------------------------------------------------------------
// bf16 kernel on the matrix cores.  One workgroup = (student, sequence, head, block of 128
// queries); wave w owns queries q0 + 32w .. + 31.  Per 64-key tile:
//   S^T = K Q^T      (A operand: key rows from LDS, B operand: the wave's queries, kept in
//                     registers for the whole kernel)
//   online softmax   per query = per lane column; a query's keys sit in 16 accumulator
//                    registers of two lanes (l and l + 32)
//   O^T += V^T P^T   (A operand: transposed value tile from LDS; B operand: the
//                     probabilities, which already sit in the B-operand register layout
//                     once the reduction slots of V^T are enumerated in the same key order)
// -------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attention_bf16_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ vt,
                                                             bf16* __restrict__ att,
                                                             const int32_t* __restrict__ cu, int B, int Tn, int rows,
                                                             int H, int heads, int max_seqlen, int nqc, int min_len)
{
    __shared__ uint4 sK[8 * kKStride];             // [d-group of 8][key]
    __shared__ __attribute__((aligned(16))) bf16 sVt[kD * kVStride];   // [d][key]

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
    const int q0 = qc * kQPerWg;
    if (q0 >= L || L <= min_len) return;            // whole workgroup leaves together

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, g = lane >> 5;
    const size_t ld = (size_t)3 * H;
    const bf16* base = qkv + ((size_t)m * rows + t0) * ld + h * kD;
    const int q = q0 + wave * 32 + j;               // this lane's query
    const bool wave_active = q0 + wave * 32 < L;

    // queries: B operand of S^T = K Q^T, four k-steps of 16 over d
    bf16x8 qf[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        uint4 t = {0, 0, 0, 0};
        if (q < L) t = *(const uint4*)(base + (size_t)q * ld + 16 * s + 8 * g);
        qf[s] = __builtin_bit_cast(bf16x8, t);
    }

    f32x16 o[2];
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] = 0.f;
    float mrun = -INFINITY, lrun = 0.f;
    const float sl2 = 0.125f * 1.44269504088896341f;   // 1/sqrt(64) * log2(e)

    // Key tiles start at a token index that is a multiple of 8, so that the transposed values (token-contiguous
    // rows) can be fetched 16 bytes at a time; tokens in front of the sequence are masked below.
    const int lead = t0 & 7;
    const bf16* vbase = vt + ((size_t)m * H + h * kD) * rows + (t0 - lead);
    const int lrow = tid >> 3, lc = tid & 7;
    for (int kt0 = -lead; kt0 < L; kt0 += kKeyTile) {
        // stage the key tile (rows = keys) and the value tile (rows = head dimensions); what lies beyond the
        // sequence is zero-filled
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int r = lrow + 32 * p;                      // key of the tile, or head dimension
            uint4 kk = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
            if (kt0 + r >= 0 && kt0 + r < L) kk = *(const uint4*)(base + (ptrdiff_t)(kt0 + r) * (ptrdiff_t)ld + H + lc * 8);
            if (kt0 + lc * 8 < L) vv = *(const uint4*)(vbase + (size_t)r * rows + (kt0 + lead) + lc * 8);
            sK[lc * kKStride + r] = kk;
            uint2* vd = (uint2*)(sVt + r * kVStride + lc * 8);
            vd[0] = uint2{vv.x, vv.y};
            vd[1] = uint2{vv.z, vv.w};
        }
        __syncthreads();

        if (wave_active) {
            // scores of this wave's 32 queries against the 64 keys: two 32x32 blocks
            f32x16 sc[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int e = 0; e < 16; ++e) sc[kb][e] = 0.f;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const uint4 t = sK[(2 * s + g) * kKStride + kb * 32 + j];
                    sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, t), qf[s], sc[kb], 0, 0, 0);
                }
            }
            // accumulator register v of this lane is key 8*(v/4) + 4*g + v%4 of its block
            float mx = mrun;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = kt0 + kb * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                    const float sv = key >= 0 && key < L ? sc[kb][v] * sl2 : -INFINITY;
                    sc[kb][v] = sv;
                    mx = fmaxf(mx, sv);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32));          // the other half of the query's keys
            const float alpha = exp2f(mrun - mx);        // first tile: exp2(-inf) = 0
            mrun = mx;
            float psum = 0.f;
            bf16x8 pf[2][2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = exp2f(sc[kb][v] - mx);
                    psum += p;
                    pf[kb][v >> 3][v & 7] = (bf16)p;
                }
            lrun = lrun * alpha + psum;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
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
                        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb][s2], o[db], 0, 0, 0);
                    }
                }
        }
        __syncthreads();
    }

    if (wave_active) {
        const float lsum = lrun + __shfl_xor(lrun, 32);
        const float inv = 1.0f / lsum;
        if (q < L) {
            bf16* dst = att + ((size_t)m * rows + t0 + q) * H + h * kD;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    bf16x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (bf16)(o[db][4 * v4 + e] * inv);
                    *(bf16x4*)(dst + db * 32 + 8 * v4 + 4 * g) = w;
                }
        }
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

__global__ __launch_bounds__(256, 3) void attention_bf16_short_kernel(const bf16* __restrict__ qkv,
                                                                      const bf16* __restrict__ vt, bf16* __restrict__ att,
                                                                      const int32_t* __restrict__ cu, int B, int Tn,
                                                                   int rows, int H, int heads, int max_seqlen,
                                                                   int ngroups, int max_len)
{
    __shared__ uint4 sK_all[4][8 * kSKStride];
    __shared__ __attribute__((aligned(16))) bf16 sVt_all[4][kD * kSVStride];

    const int m = blockIdx.y;
    const int b = blockIdx.x / ngroups, hg = blockIdx.x % ngroups;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = hg * 4 + wave;
    int t0 = cu[b], t1 = cu[b + 1];
    t0 = t0 < 0 ? 0 : (t0 > Tn - 1 ? Tn - 1 : t0);
    int L = t1 - t0;
    L = L < 1 ? 1 : L;
    L = L > max_seqlen ? max_seqlen : L;
    L = L > Tn - t0 ? Tn - t0 : L;
    if (L > max_len || h >= heads) return;         // long sequences belong to the cooperative kernel
    uint4* sK = sK_all[wave];
    bf16* sVt = sVt_all[wave];

    const int j = lane & 31, g = lane >> 5;
    const size_t ld = (size_t)3 * H;
    const bf16* base = qkv + ((size_t)m * rows + t0) * ld + h * kD;
    const float sl2 = 0.125f * 1.44269504088896341f;
    const int lkey = lane >> 3, lc = lane & 7;      // key loader: 8 keys x 8 sixteen-byte chunks per instruction
    const int vrow = lane >> 2, vc = lane & 3;      // value loader: 16 head dimensions x 4 chunks of 8 keys
    // key tiles start at a token index that is a multiple of 8 (16-byte fetches of the token-contiguous values);
    // tokens in front of the sequence are masked
    const int lead = t0 & 7;
    const bf16* vbase = vt + ((size_t)m * H + h * kD) * rows + (t0 - lead);

    for (int q0 = 0; q0 < L; q0 += 32) {
        const int q = q0 + j;
        bf16x8 qf[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint4 t = {0, 0, 0, 0};
            if (q < L) t = *(const uint4*)(base + (size_t)q * ld + 16 * s + 8 * g);
            qf[s] = __builtin_bit_cast(bf16x8, t);
        }
        f32x16 o[2];
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] = 0.f;
        float mrun = -INFINITY, lrun = 0.f;

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

            f32x16 sc;
#pragma unroll
            for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const uint4 t = sK[(2 * s + g) * kSKStride + j];
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, t), qf[s], sc, 0, 0, 0);
            }
            float mx = mrun;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = kt0 + 8 * (v >> 2) + 4 * g + (v & 3);
                const float sv = key >= 0 && key < L ? sc[v] * sl2 : -INFINITY;
                sc[v] = sv;
                mx = fmaxf(mx, sv);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float alpha = exp2f(mrun - mx);
            mrun = mx;
            float psum = 0.f;
            bf16x8 pf[2];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float p = exp2f(sc[v] - mx);
                psum += p;
                pf[v >> 3][v & 7] = (bf16)p;
            }
            lrun = lrun * alpha + psum;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const int kbase = 16 * s2 + 4 * g;
#pragma unroll
                for (int db = 0; db < 2; ++db) {
                    const bf16* vr = sVt + (db * 32 + j) * kSVStride + kbase;
                    const bf16x4 lo = *(const bf16x4*)vr, hi = *(const bf16x4*)(vr + 8);
                    const bf16x8 vf = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[s2], o[db], 0, 0, 0);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();       // the slice is rewritten at the top of the next iteration
        }
        const float inv = 1.0f / (lrun + __shfl_xor(lrun, 32));
        if (q < L) {
            bf16* dst = att + ((size_t)m * rows + t0 + q) * H + h * kD;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    bf16x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (bf16)(o[db][4 * v4 + e] * inv);
                    *(bf16x4*)(dst + db * 32 + 8 * v4 + 4 * g) = w;
                }
        }
    }
}

// -------------------------------------------------------------------------------------
// Attention of one query per sequence (its first token), used when only the first-token rows of the last layer are
// needed.  One wave per (student, sequence, head): lanes own keys for the scores and softmax, then head dimensions
// for the weighted sum of the values (row-major here: the 64 lanes read one 128-byte row per key).
// -------------------------------------------------------------------------------------
constexpr int kFirstMaxKeysPerLane = 8;   // sequences of up to 512 tokens

__global__ __launch_bounds__(256) void attention_first_kernel(const bf16* __restrict__ qc, const bf16* __restrict__ qkv,
                                                              bf16* __restrict__ attc,
                                                              const int32_t* __restrict__ cu, int B, int Tn, int rows,
                                                              int crows, int H, int heads, int max_seqlen)
{
    __shared__ float sp_all[4][64 * kFirstMaxKeysPerLane];
    const int m = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int item = blockIdx.x * 4 + wave;             // (sequence, head)
    if (item >= B * heads) return;
    const int b = item / heads, h = item % heads;
    float* sp = sp_all[wave];
    int t0 = cu[b], t1 = cu[b + 1];
    t0 = t0 < 0 ? 0 : (t0 > Tn - 1 ? Tn - 1 : t0);
    int L = t1 - t0;
    L = L < 1 ? 1 : L;
    L = L > max_seqlen ? max_seqlen : L;
    L = L > Tn - t0 ? Tn - t0 : L;
    L = L > 64 * kFirstMaxKeysPerLane ? 64 * kFirstMaxKeysPerLane : L;

    float q[kD];
    {
        const bf16* qr = qc + ((size_t)m * crows + b) * H + h * kD;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const bf16x8 t = *(const bf16x8*)(qr + c * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) q[c * 8 + e] = (float)t[e];
        }
    }
    const size_t ld = (size_t)3 * H;
    const bf16* kbase = qkv + ((size_t)m * rows + t0) * ld + H + h * kD;
    float sc[kFirstMaxKeysPerLane];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < kFirstMaxKeysPerLane; ++i) {
        const int key = lane + 64 * i;
        sc[i] = -INFINITY;
        if (key < L) {
            const bf16* kr = kbase + (size_t)key * ld;
            float d = 0.f;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const bf16x8 t = *(const bf16x8*)(kr + c * 8);
#pragma unroll
                for (int e = 0; e < 8; ++e) d = fmaf(q[c * 8 + e], (float)t[e], d);
            }
            sc[i] = d * (0.125f * 1.44269504088896341f);
            mx = fmaxf(mx, sc[i]);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kFirstMaxKeysPerLane; ++i) {
        const int key = lane + 64 * i;
        const float p = key < L ? exp2f(sc[i] - mx) : 0.f;
        sum += p;
        if (key < L) sp[key] = p;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // lane = head dimension; the value rows sit next to the key rows
    const bf16* vr = kbase + H + lane;
    float o4[4] = {0.f, 0.f, 0.f, 0.f};             // four independent chains, sixteen loads in flight
    int key = 0;
    for (; key + 16 <= L; key += 16) {
        float v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = (float)vr[(size_t)(key + e) * ld];
#pragma unroll
        for (int e = 0; e < 16; ++e) o4[e & 3] = fmaf(sp[key + e], v[e], o4[e & 3]);
    }
    for (; key < L; ++key) o4[0] = fmaf(sp[key], (float)vr[(size_t)key * ld], o4[0]);
    const float o = (o4[0] + o4[1]) + (o4[2] + o4[3]);
    attc[((size_t)m * crows + b) * H + h * kD + lane] = (bf16)(o / sum);
}

// -------------------------------------------------------------------------------------
// fp32 kernel: one thread per query, keys streamed from global memory (all threads of a
// workgroup read the same key row), online softmax in registers, exact division.
// -------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void attention_f32_kernel(const float* __restrict__ qkv, float* __restrict__ att,
                                                           const int32_t* __restrict__ cu, int B, int Tn, int rows,
                                                           int H, int heads, int max_seqlen, int nqc)
{
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
    const int q = qc * 64 + threadIdx.x;
    if (q >= L) return;
    const size_t ld = (size_t)3 * H;
    const float* base = qkv + ((size_t)m * rows + t0) * ld + h * kD;
    float qv[kD], o[kD];
#pragma unroll
    for (int e = 0; e < kD; ++e) { qv[e] = base[(size_t)q * ld + e]; o[e] = 0.f; }
    float mrun = -INFINITY, lrun = 0.f;
    for (int key = 0; key < L; ++key) {
        const float* kr = base + (size_t)key * ld + H;
        const float* vr = kr + H;
        float sdot = 0.f;
#pragma unroll
        for (int e = 0; e < kD; ++e) sdot = fmaf(qv[e], kr[e], sdot);
        sdot *= 0.125f;
        const float mx = fmaxf(mrun, sdot);
        const float alpha = expf(mrun - mx), p = expf(sdot - mx);
        lrun = lrun * alpha + p;
#pragma unroll
        for (int e = 0; e < kD; ++e) o[e] = o[e] * alpha + p * vr[e];
        mrun = mx;
    }
    float* dst = att + ((size_t)m * rows + t0 + q) * H + h * kD;
#pragma unroll
    for (int e = 0; e < kD; ++e) dst[e] = o[e] / lrun;
}

}  // namespace

hipError_t launch_attention(const sp_model* M, const void* qkv, const void* vt, void* att, const int32_t* cu, int B,
                            int T, int max_seqlen, int rows, int k, hipStream_t s)
{
    const sp_config& c = M->cfg;
    if (c.hidden / c.heads != kD) return hipErrorInvalidValue;
    if (c.dtype == SP_DTYPE_BF16) {
        // Sequences of up to 128 tokens: one wave per (sequence, head); longer ones: one workgroup per (sequence,
        // head, 128 queries) sharing the key/value tiles.  Each kernel skips the other's sequences.  (Giving the long
        // sequences of a serving batch to the per-wave kernel as well was measured slower: a 256-token sequence is 72
        // tile iterations in one wave, a long tail behind the ~5 of a typical one.)
        const int kShortLen = 128;
        const int ngroups = (c.heads + 3) / 4;
        hipLaunchKernelGGL(attention_bf16_short_kernel, dim3((unsigned)(B * ngroups), k), dim3(256), 0, s,
                           (const bf16*)qkv, (const bf16*)vt, (bf16*)att, cu, B, T, rows, c.hidden, c.heads, max_seqlen,
                           ngroups, kShortLen);
        if (max_seqlen > kShortLen) {
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            const int nqc = (max_seqlen + kQPerWg - 1) / kQPerWg;
            dim3 grid((unsigned)(B * c.heads * nqc), k);
            hipLaunchKernelGGL(attention_bf16_kernel, grid, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)vt,
                               (bf16*)att, cu, B, T, rows, c.hidden, c.heads, max_seqlen, nqc, kShortLen);
        }
    } else {
        const int nqc = (max_seqlen + 63) / 64;
        dim3 grid((unsigned)(B * c.heads * nqc), k);
        hipLaunchKernelGGL(attention_f32_kernel, grid, dim3(64), 0, s, (const float*)qkv, (float*)att, cu, B, T, rows,
                           c.hidden, c.heads, max_seqlen, nqc);
    }
    return hipGetLastError();
}

hipError_t launch_attention_first(const sp_model* M, const void* qc, const void* qkv, void* attc,
                                  const int32_t* cu, int B, int T, int max_seqlen, int rows, int crows, int k,
                                  hipStream_t s)
{
    const sp_config& c = M->cfg;
    if (c.dtype != SP_DTYPE_BF16 || c.hidden / c.heads != kD || max_seqlen > 64 * kFirstMaxKeysPerLane)
        return hipErrorInvalidValue;
    dim3 grid((unsigned)((B * c.heads + 3) / 4), k);
    hipLaunchKernelGGL(attention_first_kernel, grid, dim3(256), 0, s, (const bf16*)qc, (const bf16*)qkv, (bf16*)attc, cu, B, T, rows, crows, c.hidden, c.heads, max_seqlen);
    return hipGetLastError();
}

}  // namespace sp
