// Bandwidth-bound kernels of the student forward: embedding gather + LayerNorm,
// stand-alone LayerNorm, and the pooled head with the cross-student sum.
#include <type_traits>

#include "sp_internal.h"

namespace sp {

namespace {

constexpr int kMaxChunks = 4;  // 8-element chunks per lane: hidden <= 64 * 8 * kMaxChunks

__device__ inline void load8(const float* p, float (&v)[8])
{
    const f32x4 a = *(const f32x4*)p, b = *(const f32x4*)(p + 4);
    v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3]; v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
}
__device__ inline void load8(const bf16* p, float (&v)[8])
{
    const bf16x8 a = *(const bf16x8*)p;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)a[i];
}
__device__ inline void store8(float* p, const float (&v)[8])
{
    *(f32x4*)p = f32x4{v[0], v[1], v[2], v[3]};
    *(f32x4*)(p + 4) = f32x4{v[4], v[5], v[6], v[7]};
}
__device__ inline void store8(bf16* p, const float (&v)[8])
{
    bf16x8 a;
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = (bf16)v[i];
    *(bf16x8*)p = a;
}

// LayerNorm of one row held across a wave as v[chunk][8]; chunk c of lane l covers
// elements 8*(l + 64c) .. +7.  Two passes over registers: mean, then centred variance.
// gamma and beta are held the same way (a wave keeps them for all the rows it normalises).
// eight values -> eight fp8 (e4m3) codes of v * qscale, saturating, packed in 8 bytes
__device__ inline void store8_fp8(unsigned char* p, const float (&v)[8], float qscale)
{
    int lo = 0, hi = 0;
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[0] * qscale, v[1] * qscale, lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(v[2] * qscale, v[3] * qscale, lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[4] * qscale, v[5] * qscale, hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(v[6] * qscale, v[7] * qscale, hi, true);
    *(int2*)p = int2{lo, hi};
}

// qout (may be null): the same row once more as fp8 codes of value * qscale, for the fp8 projections
// (Q8 is a template parameter: the plain bf16 / fp32 instantiations carry no trace of the second output)
template <typename T, int MAXC, bool Q8 = false>
__device__ inline void ln_row_store(float (&v)[MAXC][8], int nch, int lane, int H, const float (&gg)[MAXC][8],
                                    const float (&bb)[MAXC][8], float eps, T* out, unsigned char* qout = nullptr,
                                    float qscale = 1.f)
{
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i)
        if (lane + 64 * i < nch)
#pragma unroll
            for (int e = 0; e < 8; ++e) s += v[i][e];
    // (1 / H once and the hardware reciprocal square root: a correctly rounded division is ten dependent instructions)
    const float inv_h = __builtin_amdgcn_rcpf((float)H);
    const float mean = wave_sum(s) * inv_h;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i)
        if (lane + 64 * i < nch)
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float d = v[i][e] - mean; q += d * d; }
    const float inv = __builtin_amdgcn_rsqf(wave_sum(q) * inv_h + eps);
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) {
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = gg[i][e] * ((v[i][e] - mean) * inv) + bb[i][e];
            store8(out + c * 8, o);
            if (Q8) store8_fp8(qout + c * 8, o, qscale);
        }
    }
}

template <int MAXC>
__device__ inline void load_gamma_beta(const float* g, const float* b, int nch, int lane, float (&gg)[MAXC][8],
                                       float (&bb)[MAXC][8])
{
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) { load8(g + c * 8, gg[i]); load8(b + c * 8, bb[i]); }
    }
}

// Consecutive rows normalised by one wave (gamma / beta are fetched once for them): 8 for calls that fill the chip
// either way, 1 for small calls, where the row-parallelism is worth more than the saved fetches.
inline int rows_per_wave(int mrows, int k) { return (long)mrows * k >= 32768 ? 8 : 1; }

// One wave per rpw consecutive packed token rows, grid.y = student.
template <typename T, int MAXC, bool Q8>
__global__ __launch_bounds__(256) void embed_ln_kernel(const char* arena, size_t student_stride, size_t tok_off,
                                                       size_t pos_off, size_t g_off, size_t b_off,
                                                       const int32_t* __restrict__ ids,
                                                       const int32_t* __restrict__ cu, int B, int Tn, int rows,
                                                       int mrows, int H, int V, int P, float eps, T* __restrict__ x,
                                                       T* __restrict__ att, int rpw, unsigned char* __restrict__ xq,
                                                       float qscale, unsigned char* __restrict__ attq)
{
    const int m = blockIdx.y, lane = threadIdx.x & 63;
    const int row0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * rpw;
    if (row0 >= mrows) return;
    const int nch = H >> 3;
    const char* sb = arena + (size_t)m * student_stride;
    float gg[MAXC][8], bb[MAXC][8];
    load_gamma_beta<MAXC>((const float*)(sb + g_off), (const float*)(sb + b_off), nch, lane, gg, bb);
    // Token id and position of the wave's rows, found by one lane per row before any row is fetched (rpw <= 64):
    // the sequence of a row is the largest b with cu[b] <= row.  The row loop then has no dependent index loads.
    int my_id = 0, my_pos = 0;
    if (lane < rpw && row0 + lane < Tn) {
        const int row = row0 + lane;
        my_id = ids[row];
        int lo = 0, hi = B;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (cu[mid] <= row) lo = mid; else hi = mid;
        }
        my_pos = row - cu[lo];
        my_pos = my_pos < 0 ? 0 : (my_pos >= P ? P - 1 : my_pos);
        my_id = my_id < 0 ? 0 : (my_id >= V ? V - 1 : my_id);
    }
#pragma unroll 2
    for (int r = 0; r < rpw; ++r) {
        const int row = row0 + r;
        if (row >= mrows) break;
        T* out = x + ((size_t)m * rows + row) * H;
        if (row >= Tn) {
            // Padding rows of the token tile.  They never reach a result, but the projections compute them and the
            // attention kernels fetch values in chunks of eight tokens, so they must hold finite numbers: zero the
            // hidden state here and, once per call, the attention output rows that no kernel writes.
            const float zero8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            T* arow = att + ((size_t)m * rows + row) * H;
            for (int c = lane; c < nch; c += 64) { store8(out + c * 8, zero8); store8(arow + c * 8, zero8); }
            if (Q8)
                for (int c = lane; c < nch; c += 64) {
                    *(int2*)(xq + ((size_t)m * rows + row) * H + c * 8) = int2{0, 0};
                    if (attq) *(int2*)(attq + ((size_t)m * rows + row) * H + c * 8) = int2{0, 0};
                }
            continue;
        }
        const int id = __builtin_amdgcn_readlane(my_id, r), pos = __builtin_amdgcn_readlane(my_pos, r);
        const T* te = (const T*)(sb + tok_off) + (size_t)id * H;
        const T* pe = (const T*)(sb + pos_off) + (size_t)pos * H;
        float v[MAXC][8];
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int c = lane + 64 * i;
            if (c < nch) {
                float a[8], p8[8];
                load8(te + c * 8, a);
                load8(pe + c * 8, p8);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[i][e] = a[e] + p8[e];
            }
        }
        ln_row_store<T, MAXC, Q8>(v, nch, lane, H, gg, bb, eps, out, Q8 ? xq + ((size_t)m * rows + row) * H : nullptr, qscale);
    }
}

template <typename T, int MAXC, bool Q8>
__global__ __launch_bounds__(256) void layernorm_kernel(const char* arena, size_t student_stride, size_t g_off,
                                                        size_t b_off, const T* __restrict__ u, T* __restrict__ out,
                                                        int rows, int mrows, int H, float eps, int rpw,
                                                        unsigned char* __restrict__ outq, float qscale)
{
    const int m = blockIdx.y, lane = threadIdx.x & 63;
    const int row0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * rpw;
    if (row0 >= mrows) return;
    const int nch = H >> 3;
    const char* sb = arena + (size_t)m * student_stride;
    float gg[MAXC][8], bb[MAXC][8];
    load_gamma_beta<MAXC>((const float*)(sb + g_off), (const float*)(sb + b_off), nch, lane, gg, bb);
#pragma unroll 2
    for (int r = 0; r < rpw; ++r) {
        const int row = row0 + r;
        if (row >= mrows) break;
        const T* in = u + ((size_t)m * rows + row) * H;
        float v[MAXC][8];
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int c = lane + 64 * i;
            if (c < nch) load8(in + c * 8, v[i]);
        }
        ln_row_store<T, MAXC, Q8>(v, nch, lane, H, gg, bb, eps, out + ((size_t)m * rows + row) * H,
                                  Q8 ? outq + ((size_t)m * rows + row) * H : nullptr, qscale);
    }
}

// Sum of the slices of a split reduction + bias + residual, then LayerNorm: one wave per row.
template <typename T, int MAXC>
__global__ __launch_bounds__(256) void ln_reduce_kernel(const char* arena, size_t student_stride, size_t g_off,
                                                        size_t b_off, size_t bias_off, const float* __restrict__ part,
                                                        int splits, size_t slice_elems, const T* __restrict__ res,
                                                        T* __restrict__ out, int rows, int mrows, int H, float eps)
{
    const int m = blockIdx.y, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= mrows) return;
    const int nch = H >> 3;
    const char* sb = arena + (size_t)m * student_stride;
    float gg[MAXC][8], bb[MAXC][8];
    load_gamma_beta<MAXC>((const float*)(sb + g_off), (const float*)(sb + b_off), nch, lane, gg, bb);
    const float* bias = (const float*)(sb + bias_off);
    const T* rrow = res + ((size_t)m * rows + row) * H;
    const float* prow = part + (size_t)m * splits * slice_elems + (size_t)row * H;
    float v[MAXC][8];
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) {
            float r8[8], b8[8];
            load8(rrow + c * 8, r8);
            load8(bias + c * 8, b8);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[i][e] = r8[e] + b8[e];
            float p8[kSplitMax][8];                           // all slices requested at once, added in ascending order
#pragma unroll
            for (int sidx = 0; sidx < kSplitMax; ++sidx)
                if (sidx < splits) load8(prow + (size_t)sidx * slice_elems + c * 8, p8[sidx]);
#pragma unroll
            for (int sidx = 0; sidx < kSplitMax; ++sidx)
                if (sidx < splits) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[i][e] += p8[sidx][e];
                }
        }
    }
    ln_row_store<T, MAXC>(v, nch, lane, H, gg, bb, eps, out + ((size_t)m * rows + row) * H);
}

// First-token rows: one wave per (student, sequence).
template <typename T>
__global__ __launch_bounds__(256) void gather_first_kernel(const T* __restrict__ x, const int32_t* __restrict__ cu, int B,
                                                           int Tn, int rows, int H, T* __restrict__ xc,
                                                           T* __restrict__ attc, int crows, int cmrows)
{
    const int m = blockIdx.y, lane = threadIdx.x & 63;
    const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (b >= cmrows) return;
    const int nch = H >> 3;
    T* dst = xc + ((size_t)m * crows + b) * H;
    if (b >= B) {                                  // padding rows of the compact tile: finite contents
        const float zero8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        T* arow = attc + ((size_t)m * crows + b) * H;
        for (int c = lane; c < nch; c += 64) { store8(dst + c * 8, zero8); store8(arow + c * 8, zero8); }
        return;
    }
    int r = cu[b];
    r = r < 0 ? 0 : (r >= Tn ? Tn - 1 : r);
    const T* src = x + ((size_t)m * rows + r) * H;
    for (int c = lane; c < nch; c += 64) {
        float v[8];
        load8(src + c * 8, v);
        store8(dst + c * 8, v);
    }
}

// ---- head -------------------------------------------------------------------------
// Stage 1: one workgroup = (group of kSeqPerWg sequences, student, slice of 64 pooler outputs).
// pooled[n] = tanh(bp[n] + sum_i cls[i] Wp[i][n]); the slice's share of the classifier,
// sum_{n in slice} pooled[n] Wc[n][c], goes to zpart[m][slice][b][c].
constexpr int kSeqPerWg = 8;

// Pooler pre-activations of one slice of 64 outputs for up to kSeqPerWg rows held in LDS (xs[s][H], fp32):
// red[(wave * kSeqPerWg + s) * 64 + n] = sum over the wave's quarter of the inputs i of xs[s][i] * Wp[i][slice * 64 + n].
// A lane fetches 16 bytes (8 outputs) of a weight row, so a wave instruction covers 8 rows of the slice and the wave's
// H / 4 rows are H / 32 instructions per lane, requested sixteen at a time (2-byte loads, one row per instruction,
// took four times as many round trips: the pooler was the longest kernel of a single-sequence call; requesting all
// rows before the token rows are gathered was measured slower than two batches afterwards).  The 8 lanes that share
// an output chunk are then added with shuffles.
template <typename T>
struct RawRow;
template <>
struct RawRow<bf16> {
    bf16x8 v;
    __device__ void load(const bf16* p) { v = *(const bf16x8*)p; }
    __device__ float get(int e) const { return (float)v[e]; }
};
template <>
struct RawRow<float> {
    f32x4 a, b;
    __device__ void load(const float* p) { a = *(const f32x4*)p; b = *(const f32x4*)(p + 4); }
    __device__ float get(int e) const { return e < 4 ? a[e] : b[e - 4]; }
};

template <typename T>
struct PoolerWeights {
    static constexpr int NB = sizeof(T) == 2 ? 16 : 8;       // weight rows in flight per lane
    RawRow<T> w[NB];
    const T* base;
    int nj, stride;
    __device__ void request(const T* Wp, int H, int slice, int lane, int wv)   // addresses only
    {
        nj = H / 32;                                          // rows per lane: the wave's H / 4 rows, 8 per instruction
        stride = 8 * H;
        base = Wp + (size_t)(wv * (H / 4) + (lane >> 3)) * H + slice * 64 + (lane & 7) * 8;
    }
    __device__ void multiply(const float* xs, float* red, int H, int nseq, int lane, int wv)
    {
        const int c8 = (lane & 7) * 8, rl = lane >> 3, row0 = wv * (H / 4) + rl;
        float acc[kSeqPerWg][8];
#pragma unroll
        for (int s = 0; s < kSeqPerWg; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[s][e] = 0.f;
        for (int j0 = 0; j0 < nj; j0 += NB) {
#pragma unroll
            for (int jj = 0; jj < NB; ++jj)
                if (j0 + jj < nj) w[jj].load(base + (size_t)(j0 + jj) * stride);
#pragma unroll
            for (int jj = 0; jj < NB; ++jj)
                if (j0 + jj < nj) {
                    const int i = row0 + (j0 + jj) * 8;
#pragma unroll
                    for (int s = 0; s < kSeqPerWg; ++s)
                        if (s < nseq) {
                            const float xv = xs[s * H + i];
#pragma unroll
                            for (int e = 0; e < 8; ++e) acc[s][e] += xv * w[jj].get(e);
                        }
                }
        }
#pragma unroll
        for (int s = 0; s < kSeqPerWg; ++s)
            if (s < nseq) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    // sum over the eight lanes that share lane % 8: other half of the row, other row of the pair,
                    // other half of the wave
                    float a = acc[s][e];
                    a += dpp_moved<0x128>(a);               // row_ror:8
                    float lo = a, hi = a;
                    swap_rows(lo, hi);
                    a = lo + hi;
                    lo = a;
                    hi = a;
                    swap_halves(lo, hi);
                    a = lo + hi;
                    if (rl == 0) red[(wv * kSeqPerWg + s) * 64 + c8 + e] = a;
                }
            }
    }
};

template <typename T>
__global__ __launch_bounds__(256) void head_pool_kernel(const char* arena, size_t student_stride, size_t wp_off,
                                                        size_t bp_off, size_t wc_off, const T* __restrict__ x,
                                                        const int32_t* __restrict__ cu, int B, int Tn, int rows, int H,
                                                        int C, float* __restrict__ zpart)
{
    extern __shared__ float smem[];
    float* xs = smem;                      // [kSeqPerWg][H]
    float* red = smem + kSeqPerWg * H;     // [4][kSeqPerWg][64]
    const int b0 = blockIdx.x * kSeqPerWg, m = blockIdx.y, slice = blockIdx.z, nslice = gridDim.z;
    const int tid = threadIdx.x, lane = tid & 63, part = tid >> 6;
    const int nseq = (B - b0) < kSeqPerWg ? (B - b0) : kSeqPerWg;
    const char* sb = arena + (size_t)m * student_stride;
    for (int s = 0; s < nseq; ++s) {
        int r = cu ? cu[b0 + s] : b0 + s;    // packed layout: first token of the sequence; compact layout: row b
        r = r < 0 ? 0 : (r >= Tn ? Tn - 1 : r);
        const T* src = x + ((size_t)m * rows + r) * H;
        for (int i = tid; i < H; i += 256) xs[s * H + i] = (float)src[i];
    }
    __syncthreads();
    const int n = slice * 64 + lane;
    if (nseq <= 2) {
        // one or two sequences: latency of the weight fetch is all there is, wide loads (see PoolerWeights)
        PoolerWeights<T> pw;
        pw.request((const T*)(sb + wp_off), H, slice, lane, part);
        pw.multiply(xs, red, H, nseq, lane, part);
    } else {
        // a full group of sequences: a lane owns one output for all of them (measured faster than the wide loads,
        // whose eight-outputs-per-lane sums need 64 accumulators and a shuffle reduction per sequence)
        const T* Wp = (const T*)(sb + wp_off);
        float acc[kSeqPerWg];
#pragma unroll
        for (int s = 0; s < kSeqPerWg; ++s) acc[s] = 0.f;
        const int per = H / 4, i0 = part * per;   // this wave's share of the reduction index (a multiple of 16)
#pragma unroll 8
        for (int i = i0; i < i0 + per; i += 4) {     // unrolled: 32 weight loads in flight per lane
            float w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (float)Wp[(size_t)(i + e) * H + n];
#pragma unroll
            for (int s = 0; s < kSeqPerWg; ++s) {    // rows beyond nseq hold stale data: their sums are never used
                const f32x4 xv = *(const f32x4*)&xs[s * H + i];
                acc[s] += xv[0] * w[0] + xv[1] * w[1] + xv[2] * w[2] + xv[3] * w[3];
            }
        }
#pragma unroll
        for (int s = 0; s < kSeqPerWg; ++s) red[(part * kSeqPerWg + s) * 64 + lane] = acc[s];
    }
    __syncthreads();
    // wave `part` finishes sequences part, part+4: fixed order over the four shares
    const float bpn = ((const float*)(sb + bp_off))[n];
    const T* Wc = (const T*)(sb + wc_off);
    for (int s = part; s < nseq; s += 4) {
        float p = bpn;
#pragma unroll
        for (int q = 0; q < 4; ++q) p += red[(q * kSeqPerWg + s) * 64 + lane];
        p = tanhf(p);
        for (int c = 0; c < C; ++c) {
            const float t = wave_sum(p * (float)Wc[(size_t)n * C + c]);
            if (lane == 0) zpart[(((size_t)m * nslice + slice) * B + (b0 + s)) * C + c] = t;
        }
    }
}

// Stage 2: z[m][b][c] = bc[m][c] + sum over slices (ascending); logits[b][c] = sum_m z (m ascending).
// 256 threads = 8 student lanes x 32 outputs: the students' slice sums run in parallel, the sum over students is taken
// in order by the first lane of each output.
constexpr int kSumStudents = 64;   // most students (sp_config.K is capped at this)

__global__ __launch_bounds__(256) void head_sum_kernel(const char* arena, size_t student_stride, size_t bc_off,
                                                       const float* __restrict__ zpart, int B, int C, int k, int nslice,
                                                       float* __restrict__ z, float* __restrict__ logits)
{
    __shared__ float zs[kSumStudents][32];
    const int ox = threadIdx.x & 31, my = threadIdx.x >> 5;
    const int idx = blockIdx.x * 32 + ox;
    const bool live = idx < B * C;
    const int c = live ? idx % C : 0;
    for (int m = my; m < k; m += 8) {
        float zm = 0.f;
        if (live) {
#pragma unroll 4
            for (int sl = 0; sl < nslice; ++sl) zm += zpart[((size_t)m * nslice + sl) * B * C + idx];
            zm += ((const float*)(arena + (size_t)m * student_stride + bc_off))[c];
            z[(size_t)m * B * C + idx] = zm;
        }
        zs[m][ox] = zm;
    }
    __syncthreads();
    if (my == 0 && live) {
        float total = 0.f;
        for (int m = 0; m < k; ++m) total += zs[m][ox];
        logits[idx] = total;
    }
}

// Stage 1 of the head for calls of a few dozen tokens (same grid and pooler as head_pool_kernel): the first-token
// rows are rebuilt from the slices of the last split reduction: slices (ascending) + bias + residual, LayerNorm,
// rounded to bf16: exactly what ln_reduce_kernel would have stored for these rows (the other rows of the last layer
// reach no result, so that launch is saved).  Taking the sums of stage 2 in the workgroup that finishes last (a ticket
// counter after a device-scope fence) was measured slower than the launch of head_sum_kernel it saves.
__global__ __launch_bounds__(256) void head_small_kernel(const char* arena, size_t student_stride, size_t wp_off,
                                                         size_t bp_off, size_t wc_off, size_t bc_off, size_t g_off,
                                                         size_t b_off, size_t bias_off, const float* __restrict__ part,
                                                         int splits, size_t slice_elems, const bf16* __restrict__ res,
                                                         const int32_t* __restrict__ cu, int B, int Tn, int rows, int H,
                                                         int C, float eps, float* __restrict__ zpart)
{
    extern __shared__ float smem[];
    float* xs = smem;                      // [kSeqPerWg][H]
    float* red = smem + kSeqPerWg * H;     // [4][kSeqPerWg][64]
    const int b0 = blockIdx.x * kSeqPerWg, m = blockIdx.y, slice = blockIdx.z, nslice = gridDim.z;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int nseq = (B - b0) < kSeqPerWg ? (B - b0) : kSeqPerWg;
    const char* sb = arena + (size_t)m * student_stride;
    const float* bias = (const float*)(sb + bias_off);
    const float* gam = (const float*)(sb + g_off);
    const float* bet = (const float*)(sb + b_off);
    PoolerWeights<bf16> pw;
    pw.request((const bf16*)(sb + wp_off), H, slice, lane, wv);
    // A thread owns elements tid + 256 j of a row (H <= 1024: j < 4).  Everything a row needs is requested before
    // anything is used (a loop that loads and uses per element would pay one memory round trip per iteration).
    constexpr int MAXJ = 4;                // hidden <= 1024 (checked by the launcher)
    __shared__ float wsum[2][4];
    float gj[MAXJ], bj[MAXJ], biasj[MAXJ];
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) {
        const int i = tid + 256 * j;
        gj[j] = i < H ? gam[i] : 0.f;
        bj[j] = i < H ? bet[i] : 0.f;
        biasj[j] = i < H ? bias[i] : 0.f;
    }
    for (int s = 0; s < nseq; ++s) {
        int r = cu[b0 + s];
        r = r < 0 ? 0 : (r >= Tn ? Tn - 1 : r);
        const bf16* rrow = res + ((size_t)m * rows + r) * H;
        const float* prow = part + (size_t)m * splits * slice_elems + (size_t)r * H;
        float v[MAXJ], p8[MAXJ][kSplitMax];
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            const int i = tid + 256 * j;
            v[j] = i < H ? (float)rrow[i] : 0.f;
#pragma unroll
            for (int sidx = 0; sidx < kSplitMax; ++sidx)
                p8[j][sidx] = i < H && sidx < splits ? prow[(size_t)sidx * slice_elems + i] : 0.f;
        }
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            v[j] += biasj[j];
#pragma unroll
            for (int sidx = 0; sidx < kSplitMax; ++sidx)      // slices in ascending order
                if (sidx < splits) v[j] += p8[j][sidx];
            if (tid + 256 * j < H) sum += v[j];
        }
        sum = wave_sum(sum);
        if (lane == 0) wsum[0][wv] = sum;
        __syncthreads();
        const float inv_h = __builtin_amdgcn_rcpf((float)H);
        const float mean = (wsum[0][0] + wsum[0][1] + wsum[0][2] + wsum[0][3]) * inv_h;
        float q = 0.f;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j)
            if (tid + 256 * j < H) { const float d = v[j] - mean; q += d * d; }
        q = wave_sum(q);
        if (lane == 0) wsum[1][wv] = q;
        __syncthreads();
        const float inv = __builtin_amdgcn_rsqf((wsum[1][0] + wsum[1][1] + wsum[1][2] + wsum[1][3]) * inv_h + eps);
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            const int i = tid + 256 * j;
            if (i < H) xs[s * H + i] = (float)(bf16)(gj[j] * ((v[j] - mean) * inv) + bj[j]);
        }
        __syncthreads();                       // wsum is rewritten for the next row; xs is read by everybody below
    }
    const int n = slice * 64 + lane;
    pw.multiply(xs, red, H, nseq, lane, wv);
    __syncthreads();
    const float bpn = ((const float*)(sb + bp_off))[n];
    const bf16* Wc = (const bf16*)(sb + wc_off);
    for (int s = wv; s < nseq; s += 4) {
        float p = bpn;
#pragma unroll
        for (int q = 0; q < 4; ++q) p += red[(q * kSeqPerWg + s) * 64 + lane];
        p = tanhf(p);
        for (int c = 0; c < C; ++c) {
            const float t = wave_sum(p * (float)Wc[(size_t)n * C + c]);
            if (lane == 0) zpart[(((size_t)m * nslice + slice) * B + (b0 + s)) * C + c] = t;
        }
    }
}

// logits[i] = sum over students of z[m][i], m ascending.
__global__ void sum_students_kernel(const float* __restrict__ z, int n, int k, float* __restrict__ logits)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float total = 0.f;
#pragma unroll 4
    for (int m = 0; m < k; ++m) total += z[(size_t)m * n + i];
    logits[i] = total;
}

// Classifier on pooled rows and the cross-student sum: one workgroup per sequence, wave w takes students w, w + 4, ...
// (T: type of the classifier matrix in the arena, P: type of the pooled rows)
template <typename T, typename P = T>
__global__ __launch_bounds__(256) void head_classify_kernel(const char* arena, size_t student_stride, size_t wc_off,
                                                            size_t bc_off, const P* __restrict__ pooled, int B, int crows,
                                                            int H, int C, int k, float* __restrict__ z,
                                                            float* __restrict__ logits)
{
    __shared__ float zs[64][16];                 // [student][class]
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int m = wave; m < k; m += 4) {
        const char* sb = arena + (size_t)m * student_stride;
        const T* Wc = (const T*)(sb + wc_off);
        const float* bc = (const float*)(sb + bc_off);
        const P* p = pooled + ((size_t)m * crows + b) * H;
        for (int c = 0; c < C; ++c) {
            float acc = 0.f;
            for (int n = lane; n < H; n += 64) acc += (float)p[n] * (float)Wc[(size_t)n * C + c];
            acc = wave_sum(acc);
            if (lane == 0) { const float v = acc + bc[c]; zs[m][c] = v; z[((size_t)m * B + b) * C + c] = v; }
        }
    }
    __syncthreads();
    if (threadIdx.x < C) {
        float total = 0.f;
        for (int m = 0; m < k; ++m) total += zs[m][threadIdx.x];   // students in training order
        logits[(size_t)b * C + threadIdx.x] = total;
    }
}

}  // namespace

hipError_t launch_head_classify(const sp_model* M, const void* pooled, int B, int crows, int k, float* z, float* logits,
                                hipStream_t s, bool pooled_f32)
{
    const sp_config& c = M->cfg;
    if (!bf16_path(c) || k > 64) return hipErrorInvalidValue;
    if (pooled_f32) {
        hipLaunchKernelGGL((head_classify_kernel<bf16, float>), dim3(B), dim3(256), 0, s, M->arena, M->L.student_stride, M->L.wc,
                           M->L.bc, (const float*)pooled, B, crows, c.hidden, c.classes, k, z, logits);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(head_classify_kernel<bf16>, dim3(B), dim3(256), 0, s, M->arena, M->L.student_stride, M->L.wc,
                       M->L.bc, (const bf16*)pooled, B, crows, c.hidden, c.classes, k, z, logits);
    return hipGetLastError();
}

hipError_t launch_embed_ln(const sp_model* M, const int32_t* ids, const int32_t* cu, int B, int T, int rows, int mrows,
                           int k, void* x, void* att, hipStream_t s, void* xq, float qscale, void* attq)
{
    const sp_config& c = M->cfg;
    const ArenaLayout& L = M->L;
    const int rpw = rows_per_wave(mrows, k);
    dim3 grid((mrows + 4 * rpw - 1) / (4 * rpw), k);
    const int maxc = (c.hidden / 8 + 63) / 64;              // 8-element chunks per lane
#define SP_EMBED(T, MAXC) do {                                                                                     \
    if (xq && std::is_same<T, bf16>::value)                                                                        \
        hipLaunchKernelGGL((embed_ln_kernel<bf16, MAXC, true>), grid, dim3(256), 0, s, M->arena, L.student_stride, L.tok, \
                           L.pos, L.emb_g, L.emb_b, ids, cu, B, T_, rows, mrows, c.hidden, c.vocab, c.max_pos, c.ln_eps,  \
                           (bf16*)x, (bf16*)att, rpw, (unsigned char*)xq, qscale, (unsigned char*)attq);               \
    else                                                                                                           \
    hipLaunchKernelGGL((embed_ln_kernel<T, MAXC, false>), grid, dim3(256), 0, s, M->arena, L.student_stride, L.tok, L.pos, \
                       L.emb_g, L.emb_b, ids, cu, B, T_, rows, mrows, c.hidden, c.vocab, c.max_pos, c.ln_eps, (T*)x, \
                       (T*)att, rpw, (unsigned char*)xq, qscale, (unsigned char*)attq); } while (0)
    const int T_ = T;
    if (maxc > kMaxChunks) return hipErrorInvalidValue;
    if (bf16_path(c)) {
        if (maxc <= 1) SP_EMBED(bf16, 1); else if (maxc == 2) SP_EMBED(bf16, 2); else SP_EMBED(bf16, 4);
    } else {
        if (maxc <= 1) SP_EMBED(float, 1); else if (maxc == 2) SP_EMBED(float, 2); else SP_EMBED(float, 4);
    }
#undef SP_EMBED
    return hipGetLastError();
}

hipError_t launch_layernorm(const sp_model* M, const void* u, void* out, int rows, int mrows, int k, size_t g_off,
                            size_t b_off, hipStream_t s, void* outq, float qscale)
{
    const sp_config& c = M->cfg;
    const int rpw = rows_per_wave(mrows, k);
    dim3 grid((mrows + 4 * rpw - 1) / (4 * rpw), k);
    const int maxc = (c.hidden / 8 + 63) / 64;              // 8-element chunks per lane
    if (maxc > kMaxChunks) return hipErrorInvalidValue;
#define SP_LN(T, MAXC) do {                                                                                         \
    if (outq && std::is_same<T, bf16>::value)                                                                       \
        hipLaunchKernelGGL((layernorm_kernel<bf16, MAXC, true>), grid, dim3(256), 0, s, M->arena, M->L.student_stride, \
                           g_off, b_off, (const bf16*)u, (bf16*)out, rows, mrows, c.hidden, c.ln_eps, rpw,         \
                           (unsigned char*)outq, qscale);                                                          \
    else                                                                                                            \
    hipLaunchKernelGGL((layernorm_kernel<T, MAXC, false>), grid, dim3(256), 0, s, M->arena, M->L.student_stride, g_off,    \
                       b_off, (const T*)u, (T*)out, rows, mrows, c.hidden, c.ln_eps, rpw, (unsigned char*)outq, qscale); } while (0)
    if (bf16_path(c)) {
        if (maxc <= 1) SP_LN(bf16, 1); else if (maxc == 2) SP_LN(bf16, 2); else SP_LN(bf16, 4);
    } else {
        if (maxc <= 1) SP_LN(float, 1); else if (maxc == 2) SP_LN(float, 2); else SP_LN(float, 4);
    }
#undef SP_LN
    return hipGetLastError();
}

// Contents check of a forward's inputs (sp_check_inputs): every thread looks at a strided share of the ids and of the
// offsets and ORs what it finds into one word.
__global__ void clear_word_kernel(unsigned* w) { *w = 0u; }

__global__ __launch_bounds__(256) void check_inputs_kernel(const int32_t* __restrict__ ids,
                                                           const int32_t* __restrict__ cu, int B, int Tn, int max_seqlen,
                                                           int V, unsigned* flags)
{
    unsigned bad = 0;
    const int stride = gridDim.x * blockDim.x, first = blockIdx.x * blockDim.x + threadIdx.x;
    for (int i = first; i < Tn; i += stride) {
        const int id = ids[i];
        if (id < 0 || id >= V) bad |= SP_BAD_ID;
    }
    for (int b = first; b < B; b += stride) {
        const int a = cu[b], e = cu[b + 1];
        if (e <= a) bad |= SP_BAD_ORDER;
        else if (e - a > max_seqlen) bad |= SP_BAD_LENGTH;
    }
    if (first == 0) {
        if (cu[0] != 0) bad |= SP_BAD_CU0;
        if (cu[B] != Tn) bad |= SP_BAD_TOTAL;
    }
    if (bad) atomicOr(flags, bad);
}

hipError_t launch_check_inputs(const int32_t* ids, const int32_t* cu, int B, int T, int max_seqlen, int vocab,
                               unsigned* flags, hipStream_t s)
{
    hipLaunchKernelGGL(clear_word_kernel, dim3(1), dim3(1), 0, s, flags);
    const int blocks = (T + 255) / 256 < 1024 ? (T + 255) / 256 : 1024;
    hipLaunchKernelGGL(check_inputs_kernel, dim3(blocks < 1 ? 1 : blocks), dim3(256), 0, s, ids, cu, B, T, max_seqlen,
                       vocab, flags);
    return hipGetLastError();
}

hipError_t launch_sum_students(const float* z, int n, int k, float* logits, hipStream_t s)
{
    hipLaunchKernelGGL(sum_students_kernel, dim3((n + 255) / 256), dim3(256), 0, s, z, n, k, logits);
    return hipGetLastError();
}

hipError_t launch_ln_reduce(const sp_model* M, const float* partials, int splits, size_t slice_elems, size_t bias_off,
                            const void* residual, void* out, int rows, int mrows, int k, size_t g_off, size_t b_off,
                            hipStream_t s)
{
    const sp_config& c = M->cfg;
    if (!bf16_path(c) || splits < 1 || splits > kSplitMax) return hipErrorInvalidValue;
    dim3 grid((mrows + 3) / 4, k);
    const int maxc = (c.hidden / 8 + 63) / 64;
    if (maxc > kMaxChunks) return hipErrorInvalidValue;
#define SP_LNR(MAXC)                                                                                               \
    hipLaunchKernelGGL((ln_reduce_kernel<bf16, MAXC>), grid, dim3(256), 0, s, M->arena, M->L.student_stride, g_off, \
                       b_off, bias_off, partials, splits, slice_elems, (const bf16*)residual, (bf16*)out, rows, mrows, \
                       c.hidden, c.ln_eps)
    if (maxc <= 1) SP_LNR(1); else if (maxc == 2) SP_LNR(2); else SP_LNR(4);
#undef SP_LNR
    return hipGetLastError();
}

hipError_t launch_gather_first(const sp_model* M, const void* x, const int32_t* cu, int B, int T, int rows, void* xc,
                               void* attc, int crows, int cmrows, int k, hipStream_t s)
{
    const sp_config& c = M->cfg;
    dim3 grid((cmrows + 3) / 4, k);
    if (bf16_path(c))
        hipLaunchKernelGGL(gather_first_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)x, cu, B, T, rows, c.hidden,
                           (bf16*)xc, (bf16*)attc, crows, cmrows);
    else
        hipLaunchKernelGGL(gather_first_kernel<float>, grid, dim3(256), 0, s, (const float*)x, cu, B, T, rows, c.hidden,
                           (float*)xc, (float*)attc, crows, cmrows);
    return hipGetLastError();
}

hipError_t launch_head_small(const sp_model* M, const float* partials, int splits, size_t slice_elems, size_t bias_off,
                             const void* residual, size_t g_off, size_t b_off, const int32_t* cu, int B, int T, int rows,
                             int k, float* z, float* zpart, float* logits, hipStream_t s)
{
    const sp_config& c = M->cfg;
    const ArenaLayout& L = M->L;
    if (!bf16_path(c) || splits < 1 || splits > kSplitMax || c.hidden > 1024 || k > kSumStudents)
        return hipErrorInvalidValue;
    const int nslice = c.hidden / 64;
    dim3 grid((B + kSeqPerWg - 1) / kSeqPerWg, k, nslice);
    const size_t smem = (size_t)(kSeqPerWg * c.hidden + 4 * kSeqPerWg * 64) * sizeof(float);
    hipLaunchKernelGGL(head_small_kernel, grid, dim3(256), smem, s, M->arena, L.student_stride, L.wp, L.bp, L.wc, L.bc,
                       g_off, b_off, bias_off, partials, splits, slice_elems, (const bf16*)residual, cu, B, T, rows,
                       c.hidden, c.classes, c.ln_eps, zpart);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int n = B * c.classes;
    hipLaunchKernelGGL(head_sum_kernel, dim3((n + 31) / 32), dim3(256), 0, s, M->arena, L.student_stride, L.bc, zpart, B,
                       c.classes, k, nslice, z, logits);
    return hipGetLastError();
}

hipError_t launch_head(const sp_model* M, const void* x, const int32_t* cu, int B, int T, int rows, int k, float* z,
                       float* zpart, float* logits, hipStream_t s)
{
    const sp_config& c = M->cfg;
    const ArenaLayout& L = M->L;
    const int nslice = c.hidden / 64;
    dim3 grid((B + kSeqPerWg - 1) / kSeqPerWg, k, nslice);
    const size_t smem = (size_t)(kSeqPerWg * c.hidden + 4 * kSeqPerWg * 64) * sizeof(float);
    if (bf16_path(c))
        hipLaunchKernelGGL(head_pool_kernel<bf16>, grid, dim3(256), smem, s, M->arena, L.student_stride, L.wp, L.bp,
                           L.wc, (const bf16*)x, cu, B, T, rows, c.hidden, c.classes, zpart);
    else
        hipLaunchKernelGGL(head_pool_kernel<float>, grid, dim3(256), smem, s, M->arena, L.student_stride, L.wp, L.bp,
                           L.wc, (const float*)x, cu, B, T, rows, c.hidden, c.classes, zpart);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int n = B * c.classes;
    if (k > kSumStudents) return hipErrorInvalidValue;
    hipLaunchKernelGGL(head_sum_kernel, dim3((n + 31) / 32), dim3(256), 0, s, M->arena, L.student_stride, L.bc,
                       zpart, B, c.classes, k, nslice, z, logits);
    return hipGetLastError();
}

}  // namespace sp
