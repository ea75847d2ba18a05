// Kernels for blocks of rows that belong to several sequences (batch > 1), and the bf16 GEMM for
// more than 16 rows.  Included after kernels.h; the single-sequence kernels there stay as they are.
//
// A block is a list of segments: segment s holds rows [s*ms, s*ms + m[s]) - the tokens of sequence
// seq[s] at positions pos0[s] .. pos0[s] + m[s] - 1.  All segments are ms rows apart (ms = the longest
// segment of the block, <= 16); rows j >= m[s] of a segment are padding: they are computed like the
// segment's last row, write no K/V and are never read back.  A verification block has m[s] = gamma + 1
// for every sequence (no padding), a draft step m[s] = 1; only catch-up blocks are ragged.
#pragma once

#include <type_traits>

namespace msd {

constexpr int MAX_SEGS = 32;

struct Segs {
    int n, ms;
    int seq[MAX_SEGS], m[MAX_SEGS], pos0[MAX_SEGS];
};

struct SeqTab { int v[MAX_SEGS]; };
static_assert(MAX_SEGS == ROUND_TAB, "one round word per sequence of a batch");

// Blocks whose segments run through different models of one shape (the drafter step of a batched round: every
// sequence advances by one token in the drafter its bandit chose).  Segments are ordered by model, so the rows of a
// model are contiguous: group g holds rows [r0[g], r0[g] + m[g]).  Kernels that touch weights or caches take one
// pointer per segment (SegPtrs) or per group (RowGroups).
constexpr int MAX_GROUPS = 8;
struct SegPtrs { const void* p[MAX_SEGS]; };
struct RowGroups {
    int n;
    int r0[MAX_GROUPS], m[MAX_GROUPS];
    const bf16_t* W[MAX_GROUPS][3];
};

// Workgroup barrier that orders LDS accesses only (global loads stay in flight).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// h[r] = E[token of row r]; tokens come from the per-sequence histories hist[seq][max_ctx].   grid (R), block 256
template <typename T>
__global__ void embed_seg_kernel(const int32_t* __restrict__ hist, int max_ctx, const T* __restrict__ E, int d,
                                 float* __restrict__ h, Segs sg) {
    const int r = blockIdx.x, s = r / sg.ms, j = min(r - s * sg.ms, sg.m[s] - 1);
    const size_t t = (size_t)hist[(size_t)sg.seq[s] * max_ctx + sg.pos0[s] + j];
    for (int i = threadIdx.x; i < d; i += blockDim.x) h[(size_t)r * d + i] = El<T>::ld(E[t * d + i]);
}

// The same with one embedding table per segment.
template <typename T>
__global__ void embed_segp_kernel(const int32_t* __restrict__ hist, int max_ctx, SegPtrs E, int d, float* __restrict__ h, Segs sg) {
    const int r = blockIdx.x, s = r / sg.ms, j = min(r - s * sg.ms, sg.m[s] - 1);
    const size_t t = (size_t)hist[(size_t)sg.seq[s] * max_ctx + sg.pos0[s] + j];
    const T* Es = static_cast<const T*>(E.p[s]);
    for (int i = threadIdx.x; i < d; i += blockDim.x) h[(size_t)r * d + i] = El<T>::ld(Es[t * d + i]);
}

// add + RMSNorm with one gain vector per segment (row r belongs to segment r / ms).   grid (R), block 1024
template <typename T>
__global__ __launch_bounds__(1024) void addnorm_segp_kernel(float* __restrict__ h, const float* __restrict__ part, int nsplit,
                                                            size_t sstride, int d, SegPtrs gain, int ms, float eps,
                                                            float* __restrict__ xn, int split) {
    addnorm_body<T>(h, part, nsplit, sstride, d, static_cast<const T*>(gain.p[blockIdx.x / ms]), eps, xn, split);
}

// Rotation table per block row: tab[r][i] = (cos, sin)(position of row r * theta^(-2i/hd)), in fp64.   grid (R), block hd/2
__global__ void rope_table_seg_kernel(Segs sg, int hd, float theta, double2* __restrict__ tab) {
    const int r = blockIdx.x, i = threadIdx.x, half = hd >> 1;
    if (i >= half) return;
    const int s = r / sg.ms, j = min(r - s * sg.ms, sg.m[s] - 1);
    const double freq = pow((double)theta, -2.0 * (double)i / (double)hd);
    double sn, cs;
    sincos((double)(sg.pos0[s] + j) * freq, &sn, &cs);
    tab[r * half + i] = make_double2(cs, sn);
}

// RoPE + K/V append per block row; kc / vc are the planes of sequence 0, sequence b's are kv_seq_stride
// elements further.   grid (H + 2KH, R), block 64
template <typename T>
__global__ void rope_kv_seg_kernel(const float* __restrict__ part, int nsplit, size_t sstride, int N, Segs sg, int H, int KH,
                                   int hd, const double2* __restrict__ tab, float* __restrict__ q, T* __restrict__ kc,
                                   T* __restrict__ vc, size_t kv_seq_stride, int max_ctx, int interleaved, int q_split) {
    const int r = blockIdx.y, s = r / sg.ms, j = r - s * sg.ms;
    const bool valid = j < sg.m[s];
    const size_t so = (size_t)sg.seq[s] * kv_seq_stride;
    rope_kv_body<T>(part, nsplit, sstride, N, sg.pos0[s] + min(j, sg.m[s] - 1), H, KH, hd, tab, q, kc + so, vc + so, max_ctx,
                    interleaved, q_split, nullptr, valid);
}

// The same with the cache planes of each segment given directly (kc.p[s], vc.p[s]: the planes of the segment's
// sequence in its model, at the layer in hand).
template <typename T>
__global__ void rope_kv_segp_kernel(const float* __restrict__ part, int nsplit, size_t sstride, int N, Segs sg, int H, int KH,
                                    int hd, const double2* __restrict__ tab, float* __restrict__ q, SegPtrs kc, SegPtrs vc,
                                    int max_ctx, int interleaved, int q_split) {
    const int r = blockIdx.y, s = r / sg.ms, j = r - s * sg.ms;
    const bool valid = j < sg.m[s];
    rope_kv_body<T>(part, nsplit, sstride, N, sg.pos0[s] + min(j, sg.m[s] - 1), H, KH, hd, tab, q,
                    static_cast<T*>(const_cast<void*>(kc.p[s])), static_cast<T*>(const_cast<void*>(vc.p[s])), max_ctx, interleaved,
                    q_split, nullptr, valid);
}

// Attention partials per (chunk, head, segment); records of segment s start s * H * nch_max chunk records
// into part.   grid (nch_max, H, segments), block 256
template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_partial_seg_kernel(const float* __restrict__ q, const T* __restrict__ kc,
                                                               const T* __restrict__ vc, size_t kv_seq_stride, Segs sg, int H,
                                                               int KH, int max_ctx, float scale, float* __restrict__ part,
                                                               int nch_max) {
    const int s = blockIdx.z, m = sg.m[s], pos0 = sg.pos0[s], c = blockIdx.x;
    if (c * ATT_CH >= pos0 + m) return;                 // workgroup-uniform
    const size_t so = (size_t)sg.seq[s] * kv_seq_stride;
    attn_partial_body<T, HD>(q + (size_t)s * sg.ms * H * HD, kc + so, vc + so, m, pos0, H, KH, max_ctx, scale,
                             part + (size_t)s * H * nch_max * 16 * (HD + 2), nch_max, c, (int)blockIdx.y);
}

template <int HD, bool MULTI>
__global__ __launch_bounds__(256, 3) void attn_partial_mfma_seg_kernel(const float* __restrict__ q, const bf16_t* __restrict__ kc,
                                                                    const bf16_t* __restrict__ vc, size_t kv_seq_stride, Segs sg,
                                                                    int H, int KH, int max_ctx, float scale,
                                                                    float* __restrict__ part, int nch_max, size_t q_lo_off, int cpw) {
    // workgroup blockIdx.x takes chunks blockIdx.x * cpw .. + cpw - 1 of its (sequence, head) and writes record blockIdx.x
    const int s = blockIdx.z, m = sg.m[s], pos0 = sg.pos0[s], c = blockIdx.x * cpw;
    if (c * ATT_CH >= pos0 + m) return;                 // workgroup-uniform
    const size_t so = (size_t)sg.seq[s] * kv_seq_stride;
    const bf16_t* qs = reinterpret_cast<const bf16_t*>(q) + (size_t)s * sg.ms * H * HD;
    float* ps = part + (size_t)s * H * nch_max * 16 * (HD + 2);
    attn_partial_mfma_body<HD, MULTI>(reinterpret_cast<const float*>(qs), kc + so, vc + so, m, pos0, H, KH, max_ctx, scale, ps, nch_max, c,
                                      (int)blockIdx.y, q_lo_off, cpw, (int)blockIdx.x);
}

// One chunk per workgroup, cache planes per segment (see rope_kv_segp_kernel).   grid (nch_max, H, segments), block 256
template <int HD>
__global__ __launch_bounds__(256, 3) void attn_partial_mfma_segp_kernel(const float* __restrict__ q, SegPtrs kc, SegPtrs vc, Segs sg,
                                                                         int H, int KH, int max_ctx, float scale,
                                                                         float* __restrict__ part, int nch_max, size_t q_lo_off) {
    const int s = blockIdx.z, m = sg.m[s], pos0 = sg.pos0[s], c = blockIdx.x;
    if (c * ATT_CH >= pos0 + m) return;                 // workgroup-uniform
    const bf16_t* qs = reinterpret_cast<const bf16_t*>(q) + (size_t)s * sg.ms * H * HD;
    attn_partial_mfma_body<HD, false>(reinterpret_cast<const float*>(qs), static_cast<const bf16_t*>(kc.p[s]),
                                      static_cast<const bf16_t*>(vc.p[s]), m, pos0, H, KH, max_ctx, scale,
                                      part + (size_t)s * H * nch_max * 16 * (HD + 2), nch_max, c, (int)blockIdx.y, q_lo_off);
}

// grid (H, R), block HD
template <int HD>
__global__ void attn_combine_seg_kernel(const float* __restrict__ part, int nch_max, int H, float* __restrict__ out, int split,
                                        Segs sg, int cpw) {
    const int r = blockIdx.y, s = r / sg.ms, j = min(r - s * sg.ms, sg.m[s] - 1);
    const int nch = ((sg.pos0[s] + sg.m[s] + ATT_CH - 1) / ATT_CH + cpw - 1) / cpw;    // records: one per cpw chunks
    attn_combine_body<HD>(part + (size_t)s * H * nch_max * 16 * (HD + 2), nch, nch_max, H, out, split, (int)blockIdx.x, j, r,
                          (size_t)gridDim.y * H * HD);
}

// out[dst row][n] = sum of split-K partials of block row r, for the rows that carry logits:
//   dst row = seq * out_seq_rows + out_row0 + (last_only ? 0 : j);  last_only: only the last valid row of a segment.
// grid (ceil(N / 256), R), block 256
__global__ void sum_partials_seg_kernel(const float* __restrict__ part, int nsplit, size_t sstride, int N, float* __restrict__ out,
                                        Segs sg, int out_seq_rows, int out_row0, int last_only) {
    const int r = blockIdx.y, s = r / sg.ms, j = r - s * sg.ms;
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (j >= sg.m[s] || (last_only && j != sg.m[s] - 1) || n >= N) return;
    float y = 0.f;
    for (int k = 0; k < nsplit; ++k) y += part[(size_t)k * sstride + (size_t)r * N + n];
    out[((size_t)sg.seq[s] * out_seq_rows + out_row0 + (last_only ? 0 : j)) * N + n] = y;
}

// Draft token of every sequence b from its row of logits (logits + b * row_stride):
//   hist[b * max_ctx + at.v[b]] = token, draft[b * draft_stride] = token.   grid (batch), block 512
__global__ __launch_bounds__(AK_NT) void sample_seq_kernel(const float* __restrict__ logits, size_t row_stride, int V, float T,
                                                           uint64_t seed, RoundTab rt, uint32_t pos,
                                                           int32_t* __restrict__ hist, int max_ctx, SeqTab at,
                                                           int32_t* __restrict__ draft, int draft_stride) {
    __shared__ AkShared sm;
    const int b = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float xp[AK_CH][4];
    ak_load(logits + (size_t)b * row_stride, V, wave, lane, xp);
    int token;
    if (T <= 0.f) {
        token = ak_argmax(xp, sm, wave, lane);
    } else {
        const float u = philox_uniform(seed, (uint32_t)b, rt.v[b], pos, 2u);
        token = T == 1.0f ? sample_rows_body<true>(xp, V, T, u, sm, wave, lane) : sample_rows_body<false>(xp, V, T, u, sm, wave, lane);
    }
    if (threadIdx.x == 0) {
        hist[(size_t)b * max_ctx + at.v[b]] = token;
        draft[(size_t)b * draft_stride] = token;
    }
}

// Commit of the emitted tokens: hist[b][l_b + n_acc[b]] = token[b].   grid (1), block 64
__global__ void commit_tokens_kernel(const int32_t* __restrict__ n_acc, const int32_t* __restrict__ token, int32_t* __restrict__ hist,
                                     int max_ctx, SeqTab l, int batch) {
    const int b = threadIdx.x;
    if (b >= batch) return;
    const int tok = token[b];
    if (tok >= 0) hist[(size_t)b * max_ctx + l.v[b] + n_acc[b]] = tok;
}

// ------------------------------------------------------------------------------------------
// addnorm_kernel's arithmetic (same order of additions, same results) for many rows of d = 1024 COLS columns: one
// 256-thread workgroup per row, every thread COLS float4 columns, the row of h and all partials of a group of eight
// requested at once (up to 36 requests in flight per thread instead of 9: with one workgroup per CU the time goes with the
// number of requests a CU keeps in flight).       grid (rows), block 256
template <typename T, int COLS>
__global__ __launch_bounds__(256) void addnorm_rows_kernel(float* __restrict__ h, const float* __restrict__ part, int nsplit, size_t sstride,
                                                           const T* __restrict__ gain, float eps, float* __restrict__ xn, int split) {
    __shared__ float red[4];
    constexpr int d = 1024 * COLS;
    const int r = blockIdx.x;
    float* hr = h + (size_t)r * d;
    const float* pr = part + (size_t)r * d;
    float4 v[COLS], gn[COLS];
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
        const int i = threadIdx.x * 4 + 1024 * c;
        v[c] = *reinterpret_cast<const float4*>(hr + i);
        gn[c] = make_float4(El<T>::ld(gain[i]), El<T>::ld(gain[i + 1]), El<T>::ld(gain[i + 2]), El<T>::ld(gain[i + 3]));
    }
    if (nsplit > 0) {
        float4 y[COLS];
#pragma unroll
        for (int c = 0; c < COLS; ++c) y[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int s0 = 0; s0 < nsplit; s0 += 8) {
            float4 p[8][COLS];
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int c = 0; c < COLS; ++c)
                    p[u][c] = *reinterpret_cast<const float4*>(pr + (size_t)min(s0 + u, nsplit - 1) * sstride + threadIdx.x * 4 + 1024 * c);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool on = s0 + u < nsplit;
#pragma unroll
                for (int c = 0; c < COLS; ++c) {
                    y[c].x += on ? p[u][c].x : 0.f; y[c].y += on ? p[u][c].y : 0.f; y[c].z += on ? p[u][c].z : 0.f; y[c].w += on ? p[u][c].w : 0.f;
                }
            }
        }
#pragma unroll
        for (int c = 0; c < COLS; ++c) {
            v[c].x += y[c].x; v[c].y += y[c].y; v[c].z += y[c].z; v[c].w += y[c].w;
            *reinterpret_cast<float4*>(hr + threadIdx.x * 4 + 1024 * c) = v[c];
        }
    }
    // sum of squares in addnorm_kernel's order: a thread of its 1024-thread workgroup holds one column per 4096, i.e. the
    // columns c of this thread belong to threads tid + 256 c there - different wavefronts, summed per wavefront first
    float tot = 0.f;
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
        float ss = v[c].x * v[c].x + v[c].y * v[c].y + v[c].z * v[c].z + v[c].w * v[c].w;
        ss = wave_sum(ss);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < 4; ++w) tot += red[w];
    }
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    if (xn) {
#pragma unroll
        for (int c = 0; c < COLS; ++c) {
            const int i = threadIdx.x * 4 + 1024 * c;
            float4 o;
            o.x = v[c].x * inv * gn[c].x;
            o.y = v[c].y * inv * gn[c].y;
            o.z = v[c].z * inv * gn[c].z;
            o.w = v[c].w * inv * gn[c].w;
            if (split) store_split4(xn, (size_t)gridDim.x * d, (size_t)r * d + i, o);
            else *reinterpret_cast<float4*>(xn + (size_t)r * d + i) = o;
        }
    }
}

// ------------------------------------------------------------------------------------------
// bf16 GEMM on MFMA for blocks of more than 16 rows (verification of a batch: R = batch x (gamma + 1)).
//   out[ks][r][n] = sum over the K-slice of x[r][k] W[n][k],  W in streaming-tile order,
//   x as two bf16 arrays (hi at xh, lo x_lo_off elements behind), row stride ldx.
// One workgroup of 8 wavefronts owns (8 / NRG) TPQ feature tiles x one K-slice x all R rows.  NRG = 4 (TPQ = 4: 128
// features): wavefronts 0-3 the first TPQ tiles, 4-7 the other TPQ; within such a group wavefront w takes the
// 16-row blocks w, w+NRG, ..  (RBW of them).  NRG = 2: four groups of two wavefronts (12 tiles with TPQ = 3) - every
// activation byte staged serves twice the multiplies, and a weight tile is requested by two wavefronts instead of four.
// The K-slice advances in stages of CST 32-wide chunks (2; 128 contiguous bytes per row and term, whole cache lines):
// per stage the R x 64 activations, both terms, are staged in LDS, double-buffered, one workgroup barrier per stage; a
// wavefront reads each activation fragment once and feeds it to the TPQ tiles it holds in registers (2 TPQ MFMAs per
// LDS read pair).  Weights: PD stages in flight in registers; the wavefronts that share tiles request the same lines
// (L1 / L2 hits).  DMA = false: activation pieces are requested one stage ahead into registers and written to LDS at
// the start of the next stage.  DMA = true: they go from memory into LDS directly (see there).
// LO = false leaves out the low-order terms of the activations (plain bf16 activations).
//   grid (ceil(ntiles / ((8 / NRG) TPQ)) * ksplit), block 512, dynamic LDS 2 * (LO ? 8 : 4) CST * 16 NRG RBW * 16 bytes;  R <= 16 NRG RBW.
template <int RBW, int PD, bool LO, int TPQ = 4, int NRG = 4, int CST = 2, bool DMA = false>
__device__ __forceinline__ void gemm_bf16_rows_body(const bf16_t* __restrict__ xh, size_t x_lo_off, int ldx, int R, int K,
                                                    const bf16_t* __restrict__ W0, const bf16_t* __restrict__ W1,
                                                    const bf16_t* __restrict__ W2, int t0, int t1, int ntiles,
                                                    float* __restrict__ out, size_t out_sstride, int N, int ksplit, int cps) {
    extern __shared__ uint4 lds[];                 // [2 buffers][hi | lo][R16 rows][HP pieces, swizzled]
    constexpr int R16 = 16 * NRG * RBW;
    constexpr int NTG = 8 / NRG;                   // groups of wavefronts with tiles of their own
    constexpr int HP = 4 * CST;                    // 16-byte pieces per row, stage and term (a stage is CST 32-wide chunks)
    constexpr int NP = LO ? 2 * HP : HP;           // .. per row and stage: hi (+ lo)
    constexpr int APT = R16 * NP / 512;            // pieces per thread and stage
    const int kchunks = K >> 5;
    const int ks = blockIdx.x % ksplit, tg = blockIdx.x / ksplit;
    const int c0 = ks * cps, nc = min(cps, kchunks - c0);
    const int nst = (nc + CST - 1) / CST;          // stages of CST chunks
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, quad = wave / NRG, wr = wave % NRG;
    const int row16 = lane & 15, g = lane >> 4;
    const int tl0 = tg * NTG * TPQ + quad * TPQ;   // this wavefront's TPQ tiles: tl0 .. tl0 + TPQ - 1
    auto tile_ptr = [&](int i) -> const u32x4* {
        const int t = min(tl0 + i, ntiles - 1);
        const bf16_t* W;
        int tt;
        if (t < t0) { W = W0; tt = t; }
        else if (t < t1) { W = W1; tt = t - t0; }
        else { W = W2; tt = t - t1; }
        return reinterpret_cast<const u32x4*>(W) + ((size_t)tt * kchunks + c0) * 64 + lane;
    };
    const u32x4* wp[TPQ];
#pragma unroll
    for (int i = 0; i < TPQ; ++i) wp[i] = tile_ptr(i);
    // every load is unconditional and clamped into range: chunks past the slice's end re-read its last
    // chunk and are multiplied by zero
    auto wload = [&](u32x4 (&dst)[CST * TPQ], int st) {
#pragma unroll
        for (int cc = 0; cc < CST; ++cc) {
            const size_t co = (size_t)min(CST * st + cc, nc - 1) * 64;   // plain loads: the four wavefronts that share these tiles meet in L1
#pragma unroll
            for (int i = 0; i < TPQ; ++i) dst[cc * TPQ + i] = wp[i][co];
        }
    };
    auto aload = [&](u32x4 (&dst)[APT], int st) {
#pragma unroll
        for (int u = 0; u < APT; ++u) {
            const int idx = tid + 512 * u, row = min(idx / NP, R - 1), which = idx % NP;
            const int c = min(CST * st + ((which % HP) >> 2), nc - 1);
            const bf16_t* src = xh + (size_t)row * ldx + (size_t)(c0 + c) * 32 + (which & 3) * 8 + (which >= HP ? x_lo_off : (size_t)0);
            dst[u] = *reinterpret_cast<const u32x4*>(src);
        }
    };
    // LDS layout of a stage: per term, rows of HP 16-byte pieces (128 or 64 bytes), piece q of row r in position q ^ swz(r):
    // the 16 lanes that read one K sub-block of 16 consecutive rows then touch 16 different 16-byte columns of the 256-byte
    // bank space (measured: 220 B/clk per CU against 63 without the swizzle and 120 for piece-major planes padded by one row)
    auto swz = [](int r) { return CST == 2 ? (r >> 1) & 7 : (r >> 2) & 3; };
    auto astore = [&](const u32x4 (&src)[APT], int buf) {
        uint4* base = lds + (size_t)buf * NP * R16;
#pragma unroll
        for (int u = 0; u < APT; ++u) {
            const int idx = tid + 512 * u, row = idx / NP, which = idx % NP, q = which % HP;
            base[(which >= HP ? R16 * HP : 0) + row * HP + (q ^ swz(row))] = __builtin_bit_cast(uint4, src[u]);
        }
    };
    f32x4 acc[RBW][TPQ];
#pragma unroll
    for (int a = 0; a < RBW; ++a)
#pragma unroll
        for (int i = 0; i < TPQ; ++i) acc[a][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    // Chunks past the slice's end are multiplied by zero: the (re-read, clamped) weight tiles of such a chunk
    // are masked in registers - they arrived long ago, so the mask costs no wait; masking the activation
    // fragments instead would make every LDS read wait for its data at once.
    // The activation fragments of step k+1 (a step = one 16-row block of one chunk) are read from LDS
    // before the MFMAs of step k are issued, so the LDS latency hides behind 8 (4) MFMAs.
    auto wmask = [&](u32x4 (&w)[CST * TPQ], int st) {
#pragma unroll
        for (int cc = 0; cc < CST; ++cc) {
            const uint32_t mask = CST * st + cc < nc ? 0xffffffffu : 0u;
#pragma unroll
            for (int i = 0; i < TPQ; ++i) w[cc * TPQ + i] &= mask;
        }
    };
    auto compute = [&](u32x4 (&w)[CST * TPQ], int buf) {
        const u32x4* base = reinterpret_cast<const u32x4*>(lds) + (size_t)buf * NP * R16;
        constexpr int FD = 1;                   // fragments are read FD steps before their multiplies (2: measured no faster)
        u32x4 fh[FD + 1], fl[FD + 1];
        auto fetch = [&](int k) {               // step k: chunk cc = k / RBW, row block a = k % RBW
            const int cc = k / RBW, a = k % RBW;
            const int rowi = (wr + NRG * a) * 16 + row16;
            const int slot = rowi * HP + ((cc * 4 + g) ^ swz(rowi));
            fh[k % (FD + 1)] = base[slot];
            if constexpr (LO) fl[k % (FD + 1)] = base[R16 * HP + slot];
        };
#pragma unroll
        for (int k = 0; k < FD; ++k) fetch(k);
#pragma unroll
        for (int k = 0; k < CST * RBW; ++k) {
            if (k + FD < CST * RBW) fetch(k + FD);
            const int cc = k / RBW, a = k % RBW;
#pragma unroll
            for (int i = 0; i < TPQ; ++i)
                acc[a][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[cc * TPQ + i]), __builtin_bit_cast(bf16x8, fh[k % (FD + 1)]), acc[a][i], 0, 0, 0);
            if constexpr (LO) {
#pragma unroll
                for (int i = 0; i < TPQ; ++i)
                    acc[a][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[cc * TPQ + i]), __builtin_bit_cast(bf16x8, fl[k % (FD + 1)]), acc[a][i], 0, 0, 0);
            }
        }
        // shape of the schedule: the reads of the steps ahead, then the MFMAs of this one
        __builtin_amdgcn_sched_group_barrier(0x100, (LO ? 2 : 1) * FD, 0);
#pragma unroll
        for (int k = 0; k < CST * RBW; ++k) {
            if (k + FD < CST * RBW) __builtin_amdgcn_sched_group_barrier(0x100, LO ? 2 : 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, LO ? 2 * TPQ : TPQ, 0);
        }
    };
    u32x4 w[PD][CST * TPQ];
    if constexpr (DMA) {
        // Activations go from memory straight into LDS (16 bytes per lane, lane i of a request to slot i of a KiB), without
        // passing registers: one request covers 8 rows x 128 bytes of one term, the lane that fills position p of row r
        // fetches piece p ^ swz(r).  The requests of stage st+1 are issued once this stage's weights have arrived (after the
        // masks touched them: the waits the compiler places for the weights count the requests it knows of, and these it
        // does not) and land while this stage is multiplied; every wavefront waits for everything it has in flight before
        // the barrier (a count of zero: right wherever the compiler puts the weight requests), and the weights of stage
        // st+PD are requested after the barrier, a whole stage before their use.  Nothing is outstanding when the kernel ends.
        static_assert(!DMA || (LO && CST == 2), "direct loads: two terms, stages of two chunks");
        constexpr int RG = R16 / 8, NI = 2 * RG / 8;             // row groups of 8; requests per wavefront and stage
        const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) void*)lds;
        const int rl = lane >> 3, pp = lane & 7;
        auto dma = [&](int st, int buf) {
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int id = wave * NI + j, term = id / RG, rg = id % RG;
                const int row = rg * 8 + rl, q = pp ^ swz(row);
                const int c = min(CST * st + (q >> 2), nc - 1);
                const bf16_t* src = xh + (size_t)min(row, R - 1) * ldx + (size_t)(c0 + c) * 32 + (q & 3) * 8 + (term ? x_lo_off : (size_t)0);
                const unsigned dst = __builtin_amdgcn_readfirstlane(lds0 + (unsigned)(((buf * NP + term * HP) * R16 + rg * 64) * 16));
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(dst), "v"(src) : "memory", "m0");
            }
        };
        dma(0, 0);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < PD; ++u) wload(w[u], u);
        for (int sb = 0; sb < nst; sb += PD) {
#pragma unroll
            for (int u = 0; u < PD; ++u) {
                const int st = sb + u;
                wmask(w[u], st);
                __builtin_amdgcn_sched_barrier(0);
                dma(st + 1, (st + 1) & 1);                 // its buffer was last read in stage st-1, before the last barrier
                __builtin_amdgcn_sched_barrier(0);
                compute(w[u], st & 1);
                __builtin_amdgcn_sched_barrier(0);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                lds_barrier();
                __builtin_amdgcn_sched_barrier(0);
                wload(w[u], st + PD);
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
    // Order of the requests (a wavefront's loads return in order): the activations of stage st+1 are
    // requested before the multiplies of stage st-1 and written to LDS before those of stage st; the only
    // loads requested after them and before that write are weights the next multiplies need anyway.
    u32x4 ar[APT];
    aload(ar, 0);
#pragma unroll
    for (int u = 0; u + 1 < PD; ++u) wload(w[u], u);
    astore(ar, 0);
    aload(ar, 1);
    __builtin_amdgcn_sched_barrier(0);
    wload(w[PD - 1], PD - 1);                      // as in the loop: the youngest requests on entry are weights
    lds_barrier();
    for (int sb = 0; sb < nst; sb += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const int st = sb + u;
            astore(ar, (st + 1) & 1);              // stage st+1 (its buffer was last read in stage st-1, before the last barrier)
            aload(ar, st + 2);                     // returns while this stage is multiplied
            // The activation requests stay ahead of this stage's weight requests: loads return in order, so an
            // activation load scheduled behind them would make the next stage's LDS write wait for weights that
            // are only needed two stages later (a full trip to HBM per stage).
            __builtin_amdgcn_sched_barrier(0);
            wmask(w[u], st);
            compute(w[u], st & 1);
            wload(w[u], st + PD);
            lds_barrier();
        }
    }
    }
#pragma unroll
    for (int a = 0; a < RBW; ++a) {
        const int row = (wr + NRG * a) * 16 + row16;
        if (row < R) {
#pragma unroll
            for (int i = 0; i < TPQ; ++i)
                if (tl0 + i < ntiles) {
                    float* o = out + (size_t)ks * out_sstride + (size_t)row * N + (size_t)(tl0 + i) * 16 + g * 4;
                    *reinterpret_cast<float4*>(o) = make_float4(acc[a][i][0], acc[a][i][1], acc[a][i][2], acc[a][i][3]);
                }
        }
    }
}

template <int RBW, int PD, bool LO, int TPQ = 4, int NRG = 4, int CST = 2, bool DMA = false>
__global__ __launch_bounds__(512) void gemm_bf16_rows_kernel(const bf16_t* __restrict__ xh, size_t x_lo_off, int ldx, int R, int K,
                                                             const bf16_t* __restrict__ W0, const bf16_t* __restrict__ W1,
                                                             const bf16_t* __restrict__ W2, int t0, int t1, int ntiles,
                                                             float* __restrict__ out, size_t out_sstride, int N, int ksplit,
                                                             int cps) {
    gemm_bf16_rows_body<RBW, PD, LO, TPQ, NRG, CST, DMA>(xh, x_lo_off, ldx, R, K, W0, W1, W2, t0, t1, ntiles, out, out_sstride, N, ksplit, cps);
}

// One launch for several row groups with weights of their own (same shapes): blockIdx.y is the group; its rows
// [r0, r0 + m) of x are multiplied with its matrices into the same rows of out.  m <= 64 RBW per group.
//   grid (ceil(ntiles / 8) * ksplit, groups), block 512, dynamic LDS as gemm_bf16_rows_kernel<RBW, ..>
template <int RBW, int PD>
__global__ __launch_bounds__(512) void gemm_bf16_rows_grouped_kernel(const bf16_t* __restrict__ xh, size_t x_lo_off, int ldx, int K,
                                                                     int t0, int t1, int ntiles, float* __restrict__ out,
                                                                     size_t out_sstride, int N, int ksplit, int cps, RowGroups gg) {
    const int g = blockIdx.y;
    gemm_bf16_rows_body<RBW, PD, true, 4>(xh + (size_t)gg.r0[g] * ldx, x_lo_off, ldx, gg.m[g], K, gg.W[g][0], gg.W[g][1], gg.W[g][2], t0,
                                        t1, ntiles, out + (size_t)gg.r0[g] * N, out_sstride, N, ksplit, cps);
}

}  // namespace msd
