// Device kernels of the MetaSD hot path for gfx950 (CDNA4): wave64, MFMA, LDS.
//
// Every kernel here is launched by metasd.hip; shapes are validated on the host before launch
// (see check_model / the asserts next to each launcher), kernels themselves only guard ragged tails.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace msd {

typedef uint16_t bf16_t;  // raw bf16 bit pattern
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------------
// element conversion

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even float -> bf16 (inf / nan pass through by truncation)
__device__ __forceinline__ bf16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) != 0x7f800000u) u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> struct El;
template <> struct El<float> {
    static __device__ __forceinline__ float ld(float v) { return v; }
    static __device__ __forceinline__ float st(float v) { return v; }
};
template <> struct El<bf16_t> {
    static __device__ __forceinline__ float ld(bf16_t v) { return bf2f(v); }
    static __device__ __forceinline__ bf16_t st(float v) { return f2bf(v); }
};

// ------------------------------------------------------------------------------------------
// wavefront (64 lanes) reductions

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
// inclusive prefix sum over the lanes of a wavefront
__device__ __forceinline__ double wave_scan_incl(double v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        double t = __shfl_up(v, o, 64);
        if (lane >= o) v += t;
    }
    return v;
}

// ------------------------------------------------------------------------------------------
// Tagged words: how workgroups of one launch hand small results to each other through global memory.
// A word is (launch epoch << 32 | 32-bit payload), written and polled with relaxed agent-scope atomics
// (they go through to memory, past the per-XCD L2).  The reader knows a word belongs to this launch as
// soon as the epoch matches: no flag, no fence, and nothing to clear between launches - the buffer is
// zeroed once and epochs only grow.  Polls are bounded; the caller decides what a timeout means.
__device__ __forceinline__ void tw_put(unsigned long long* slot, uint32_t epoch, uint32_t payload) {
    __hip_atomic_store(slot, ((unsigned long long)epoch << 32) | (unsigned long long)payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool tw_get(const unsigned long long* slot, uint32_t epoch, int spin_limit, uint32_t* payload) {
    for (int it = 0; it < spin_limit; ++it) {
        const unsigned long long w = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(w >> 32) == epoch) { *payload = (uint32_t)w; return true; }
        __builtin_amdgcn_s_sleep(2);
    }
    return false;
}

// dst[0 .. n) = 0 (16-byte pieces).   grid ceil(n / 256), block 256
__global__ void zero_fill_kernel(uint4* __restrict__ dst, unsigned n) {
    const unsigned i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = make_uint4(0u, 0u, 0u, 0u);
}

// ------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11)
// counter (c0..c3), key = 64-bit seed; ten rounds, Weyl-sequence key schedule.

__device__ __forceinline__ void philox4x32_10(uint64_t seed, uint32_t& c0, uint32_t& c1, uint32_t& c2, uint32_t& c3) {
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
}

// Round words of the Philox counters of a launch: one per row (n == number of rows <= ROUND_TAB: independent
// sequences of a batch, each with its own round count) or the same for every row (n == 0: v[0]).
constexpr int ROUND_TAB = 32;
struct RoundTab {
    int n;
    uint32_t v[ROUND_TAB];
};
__device__ __forceinline__ uint32_t round_of(const RoundTab& rt, int row) { return rt.n ? rt.v[row] : rt.v[0]; }

// uniform in [0,1): top 24 bits of word 0 at counter (seq, round, pos, stream)
__device__ __forceinline__ float philox_uniform(uint64_t seed, uint32_t seq, uint32_t round, uint32_t pos, uint32_t stream) {
    uint32_t c0 = seq, c1 = round, c2 = pos, c3 = stream;
    philox4x32_10(seed, c0, c1, c2, c3);
    return (float)(c0 >> 8) * (1.0f / 16777216.0f);
}

__global__ void philox_words_kernel(uint64_t seed, uint32_t c0_start, int n, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t* out) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t a = c0_start + (uint32_t)i, b = c1, c = c2, d = c3;
    philox4x32_10(seed, a, b, c, d);
    out[4 * i + 0] = a; out[4 * i + 1] = b; out[4 * i + 2] = c; out[4 * i + 3] = d;
}

// ------------------------------------------------------------------------------------------
// Activations handed to the bf16 GEMM are stored as two bf16 terms, x = hi + lo with hi = bf16(x),
// lo = bf16(x - hi): array hi[n] at `base`, array lo[n] right behind it (n = elements of the whole
// block).  The producer pays the conversion once; every GEMM workgroup then copies 16-byte pieces.
__device__ __forceinline__ void store_split4(float* base, size_t n, size_t at, const float4& v) {
    bf16_t* hi = reinterpret_cast<bf16_t*>(base) + at;
    bf16_t* lo = hi + n;
    const bf16_t h0 = f2bf(v.x), h1 = f2bf(v.y), h2 = f2bf(v.z), h3 = f2bf(v.w);
    *reinterpret_cast<uint2*>(hi) = make_uint2((uint32_t)h0 | ((uint32_t)h1 << 16), (uint32_t)h2 | ((uint32_t)h3 << 16));
    const bf16_t l0 = f2bf(v.x - bf2f(h0)), l1 = f2bf(v.y - bf2f(h1)), l2 = f2bf(v.z - bf2f(h2)), l3 = f2bf(v.w - bf2f(h3));
    *reinterpret_cast<uint2*>(lo) = make_uint2((uint32_t)l0 | ((uint32_t)l1 << 16), (uint32_t)l2 | ((uint32_t)l3 << 16));
}
__device__ __forceinline__ void store_split1(float* base, size_t n, size_t at, float v) {
    bf16_t* hi = reinterpret_cast<bf16_t*>(base) + at;
    const bf16_t h = f2bf(v);
    hi[0] = h;
    hi[n] = f2bf(v - bf2f(h));
}

// ------------------------------------------------------------------------------------------
// Drafter heads on the target's hidden states (the white-box drafters of the paper's Sec. 4): the input of the head's first
// projection, x[r] = [embedding row h[r] ; feature of the position before row r], 2 d values per row.  The feature comes
// from the table of the target's features (feat[p] = residual stream after the target's last layer at position p; row r at
// position pos0 + r takes feat[pos0 + r - 1], zeros for position 0) or, est != nullptr, from the head's own estimate of
// it (est[src.idx[r]]: one row for the draft steps of a chain after the first, the rows of a tree level take their parents').  split != 0: written as two bf16 arrays.     grid (m), block 256
struct FeatSrc { uint8_t idx[16]; };   // estimates: the row of `est` that row r takes (chain steps: 0; tree levels: the parent node)
__global__ void feat_cat_kernel(const float* __restrict__ h, const float* __restrict__ feat, const float* __restrict__ est, FeatSrc src,
                                int pos0, int d, float* __restrict__ out, int split) {
    const int r = blockIdx.x;
    const int p = pos0 + r - 1;
    const float* f = est ? est + (size_t)src.idx[r & 15] * d : feat + (size_t)(p < 0 ? 0 : p) * d;
    for (int i = threadIdx.x * 4; i < 2 * d; i += blockDim.x * 4) {
        float4 v;
        if (i < d) v = *reinterpret_cast<const float4*>(h + (size_t)r * d + i);
        else if (!est && p < 0) v = make_float4(0.f, 0.f, 0.f, 0.f);
        else v = *reinterpret_cast<const float4*>(f + (i - d));
        if (split) store_split4(out, (size_t)gridDim.x * 2 * d, (size_t)r * 2 * d + i, v);
        else *reinterpret_cast<float4*>(out + (size_t)r * 2 * d + i) = v;
    }
}

// dst[0 .. n4) = src[0 .. n4) (16-byte pieces): rows of the residual stream into the feature table / the estimate
__global__ void copy_f4_kernel(const float4* __restrict__ src, float4* __restrict__ dst, unsigned n4) {
    const unsigned i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) dst[i] = src[i];
}

// ------------------------------------------------------------------------------------------
// residual add of split-K partial sums + RMSNorm:      grid (m), block 1024, d % 4 == 0
//   h[r] += sum_s part[s][r]   (skipped when nsplit == 0)
//   xn[r] = h[r] / sqrt(mean(h[r]^2) + eps) * gain          (fp32; T is the type of the gain)
// split != 0: xn is written as two bf16 arrays (see store_split4), the form the bf16 GEMM stages.

template <typename T>
__device__ __forceinline__ void addnorm_body(float* __restrict__ h, const float* __restrict__ part, int nsplit, size_t sstride, int d,
                                             const T* __restrict__ gain, float eps, float* __restrict__ xn, int split) {
    __shared__ float red[16];
    constexpr int KEEP = 2;                 // float4 columns per thread kept in registers (d <= 8192); beyond that via memory
    const int r = blockIdx.x;
    float* hr = h + (size_t)r * d;
    const float* pr = part + (size_t)r * d;
    float4 keep[KEEP], gk[KEEP];
    float ss = 0.f;
    int k = 0;
    for (int i = threadIdx.x * 4; i < d; i += 4096, ++k) {
        float4 v = *reinterpret_cast<const float4*>(hr + i);
        if (nsplit > 0) {
            float4 y = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int s0 = 0; s0 < nsplit; s0 += 8) {      // eight partials in flight; added in the fixed order s = 0, 1, ..
                // every request unconditional (past the last partial: that one again, then dropped by a select): a branch
                // around a request would make the compiler wait for all of them one by one
                float4 p[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    p[u] = *reinterpret_cast<const float4*>(pr + (size_t)min(s0 + u, nsplit - 1) * sstride + i);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const bool on = s0 + u < nsplit;
                    y.x += on ? p[u].x : 0.f; y.y += on ? p[u].y : 0.f; y.z += on ? p[u].z : 0.f; y.w += on ? p[u].w : 0.f;
                }
            }
            v.x += y.x; v.y += y.y; v.z += y.z; v.w += y.w;
            *reinterpret_cast<float4*>(hr + i) = v;
        }
        if (k < KEEP) {
            keep[k] = v;
            if (xn) gk[k] = make_float4(El<T>::ld(gain[i]), El<T>::ld(gain[i + 1]), El<T>::ld(gain[i + 2]), El<T>::ld(gain[i + 3]));   // requested with the row, not after the reduction
        }
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += red[w];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    if (xn) {
        k = 0;
        for (int i = threadIdx.x * 4; i < d; i += 4096, ++k) {
            const float4 v = k < KEEP ? keep[k < KEEP ? k : 0] : *reinterpret_cast<const float4*>(hr + i);
            const float4 gn = k < KEEP ? gk[k < KEEP ? k : 0]
                                       : make_float4(El<T>::ld(gain[i]), El<T>::ld(gain[i + 1]), El<T>::ld(gain[i + 2]), El<T>::ld(gain[i + 3]));
            float4 o;
            o.x = v.x * inv * gn.x;
            o.y = v.y * inv * gn.y;
            o.z = v.z * inv * gn.z;
            o.w = v.w * inv * gn.w;
            if (split) store_split4(xn, (size_t)gridDim.x * d, (size_t)r * d + i, o);
            else *reinterpret_cast<float4*>(xn + (size_t)r * d + i) = o;
        }
    }
}

template <typename T>
__global__ __launch_bounds__(1024) void addnorm_kernel(float* __restrict__ h, const float* __restrict__ part, int nsplit,
                                                       size_t sstride, int d, const T* __restrict__ gain, float eps,
                                                       float* __restrict__ xn, int split) {
    addnorm_body<T>(h, part, nsplit, sstride, d, gain, eps, xn, split);
}

// out[i] = sum_s part[s][i]                         (only for logits when the head GEMM is split)
// inv (optional): 1/rms per row, N columns per row (the GEMM ran on an input that was not yet normalised)
__global__ void sum_partials_kernel(const float* __restrict__ part, int nsplit, size_t sstride, size_t n, float* __restrict__ out,
                                    const float* __restrict__ inv, int N) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float y = 0.f;
    for (int s = 0; s < nsplit; ++s) y += part[(size_t)s * sstride + i];
    if (inv) y *= inv[i / (size_t)N];
    out[i] = y;
}

// ------------------------------------------------------------------------------------------
// fp32 skinny GEMM (fp32 models): one wavefront per output feature, lanes stride over K.
//   out[r][n] = sum_k x[r][k] * W[n][k],  r < m <= 16,  W row-major [n][K], K % 4 == 0.
// Up to three matrices are concatenated along n (boundaries n0 <= n1 <= N).     grid ceil(N/4), block 256

__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ x, int ldx, int m, int K,
                                                       const float* __restrict__ W0, const float* __restrict__ W1,
                                                       const float* __restrict__ W2, int n0, int n1, int N,
                                                       float* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const float* w = n < n0 ? W0 + (size_t)n * K : (n < n1 ? W1 + (size_t)(n - n0) * K : W2 + (size_t)(n - n1) * K);
    float acc[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    for (int k = lane * 4; k < K; k += 256) {
        const float4 wv = *reinterpret_cast<const float4*>(w + k);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (r < m) {
                const float4 xv = *reinterpret_cast<const float4*>(x + (size_t)r * ldx + k);
                acc[r] += wv.x * xv.x + wv.y * xv.y + wv.z * xv.z + wv.w * xv.w;
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        if (r < m) {
            const float s = wave_sum(acc[r]);
            if (lane == 0) out[(size_t)r * N + n] = s;
        }
    }
}

// ------------------------------------------------------------------------------------------
// bf16 skinny GEMM on MFMA with weights streamed from HBM in tile order.
//
// Weights are in streaming-tile order (see pack_weight_kernel): tile (t, c) is 1 KiB holding
// output features 16t..16t+15 and inputs 32c..32c+31; lane l owns 16 bytes = 8 consecutive inputs
// 32c + 8(l/16).. of feature 16t + l%16 - exactly the A operand of v_mfma_f32_16x16x32_bf16, so
// one wavefront load instruction reads one contiguous KiB.  The activations (m <= 16 rows, fp32
// values) are the B operand, staged once per workgroup in LDS as two bf16 terms x = hi + lo
// (hi = bf16(x), lo = bf16(x - hi), written in that form by the producing kernel): each weight tile
// feeds two MFMAs, which keeps ~16 mantissa bits of the activations at no HBM cost (the matrix
// cores idle >95 % of the time here anyway).
// D[i][j] = sum_k A[i][k] B[k][j]: lane l gets D[4(l/16)+v][l%16], v = 0..3, i.e. 4 consecutive
// output features of activation row l%16.
//
// Work split: workgroup = (tile group tg, k-split ks); its 4 wavefronts take tiles
// tg*tpb + wave, +4, ...; the k-split covers chunks [ks*cps, ks*cps + cps).  Partial sums go to
// out[ks][r][n] (row stride N, split stride m*N) and are added by the consumer kernel.
// Up to three matrices are concatenated along n at tile boundaries t0 <= t1 <= ntiles.
//   grid (ceil(ntiles/tpb) * ksplit), block 256, dynamic LDS 2 * m * (cps*4 + 1) * 16 bytes.

constexpr int GEMM_U = 8;  // tiles in flight per wavefront (8 KiB)

__device__ __forceinline__ uint32_t pack_bf16x2(bf16_t lo, bf16_t hi) { return (uint32_t)lo | ((uint32_t)hi << 16); }

// Optional prologues for short, narrow blocks (drafter steps: m <= 4 rows, d_model <= 1024), where the
// split-K partials of the previous GEMM are few enough that every workgroup can afford to consume them
// itself; each one removes a kernel from the dependent chain of a layer:
//   PRO_NORM     x = RMSNorm(h_in + sum of the previous GEMM's partials) * gain.  Every workgroup forms
//                the full rows (it needs their sum of squares), keeps them in LDS, and stages its
//                slice; workgroup 0 also writes the rows to h_out (a second buffer: the others still
//                read h_in).  Replaces addnorm_kernel.
//   PRO_ACT      x = SiLU(gate) * up or GELU(up) from the partials of the gate | up GEMM.  Replaces ffn_act_kernel.
//   PRO_COMBINE  x = attention output merged from the per-chunk partials.  Replaces attn_combine_kernel.
enum { PRO_PLAIN = 0, PRO_NORM = 1, PRO_ACT = 2, PRO_COMBINE = 3 };

// Plain streaming read (measurement aid: the read rate of the machine the benchmark runs on, next to the 8 TB/s
// nominal peak).  The access pattern of the weight-streaming GEMMs without their arithmetic: every wavefront owns a
// contiguous run of 1-KiB chunks (16 bytes per lane and load) and keeps 16 loads in flight; the workgroup leaves
// one word per wavefront in sink so that the reads cannot be dropped.   grid (any), block 256
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, size_t nchunks, uint32_t* __restrict__ sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t nwaves = (size_t)gridDim.x * 4, gw = (size_t)blockIdx.x * 4 + wave;
    const size_t per = (nchunks + nwaves - 1) / nwaves;
    const size_t c0 = min(gw * per, nchunks), c1 = min(c0 + per, nchunks);
    u32x4 acc = {0u, 0u, 0u, 0u};
    if (c1 > c0) {
        const u32x4* wp = src + c0 * 64 + lane;
        const size_t nc = c1 - c0;                 // every load is clamped into the run: the tail re-reads its last chunk
        u32x4 a[8], b[8];
        auto valid = [&](size_t c) -> uint32_t { return c < nc ? 0xffffffffu : 0u; };   // clamped re-reads do not count
#pragma unroll
        for (int u = 0; u < 8; ++u) a[u] = __builtin_nontemporal_load(wp + min((size_t)u, nc - 1) * 64);
#pragma unroll
        for (int u = 0; u < 8; ++u) b[u] = __builtin_nontemporal_load(wp + min((size_t)(8 + u), nc - 1) * 64);
        for (size_t c = 16; c < nc + 16; c += 16) {
#pragma unroll
            for (int u = 0; u < 8; ++u) acc ^= a[u] & valid(c - 16 + u);
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] = __builtin_nontemporal_load(wp + min(c + u, nc - 1) * 64);
#pragma unroll
            for (int u = 0; u < 8; ++u) acc ^= b[u] & valid(c - 8 + u);
#pragma unroll
            for (int u = 0; u < 8; ++u) b[u] = __builtin_nontemporal_load(wp + min(c + 8 + u, nc - 1) * 64);
        }
        // the loads of the last turn lie past the run (c >= nc): nothing more to add
    }
    uint32_t w = (acc[0] ^ acc[1]) ^ (acc[2] ^ acc[3]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) w ^= __shfl_xor(w, o, 64);
    if (lane == 0) sink[blockIdx.x * 4 + wave] = w;
}

struct GemmPro {
    const float* src;      // NORM: h_in [m][K];  ACT: partials [s][m][(1|2) K];  COMBINE: attention partials
                           // (PLAIN: sstride = offset in elements from the hi array x to the lo array; optional:
                           //  src = sums of squares [ns tile groups][16], h_out = 1/rms per row [m], eps)
    const float* part;     // NORM: partials [s][m][K] of the previous GEMM (ns may be 0)
    float* h_out;          // NORM: updated residual stream [m][K]
    const bf16_t* gain;    // NORM
    size_t sstride;        // NORM / ACT: split stride of the partials (floats)
    int ns;                // NORM / ACT: number of partials
    float eps;             // NORM
    int act;               // ACT: 1 SwiGLU, 0 GELU
    int nchunks, hd;       // COMBINE: attention chunks, head dim
    int row0;              // PLAIN with src: first row of the sums-of-squares table that belongs to this block
};

// Epilogue variant for the two projections that feed the residual stream (attention output, FFN down):
// EPI_RESIDUAL.  The split-K siblings of a tile group (consecutive workgroup ids ks = 0 .. ksplit-1) do not
// leave their partial sums to a later kernel: siblings 0 .. ksplit-2 publish them as tagged words, and the
// last sibling adds them in the order s = 0, 1, .. (its own last), then
//     h += sum;   xg = h * gain -> the two-bf16 form the next GEMM stages (not yet normalised);
//     ssq[tile group][row] = sum of h^2 over the group's 64 columns.
// RMSNorm's 1/rms commutes with the next GEMM, so that GEMM runs on h * gain and the kernels that
// consume its output scale by 1/sqrt(sum_groups ssq / D + eps): the add+norm kernel disappears from
// the chain.  The last sibling only waits for workgroups with lower ids; a timeout sets *abort.
enum { EPI_PARTIALS = 0, EPI_RESIDUAL = 1 };

struct GemmEpi {
    unsigned long long* xw;   // tagged words [ksplit - 1][m][N]
    float* h;                 // residual stream [m][N], updated in place
    const bf16_t* gain;       // gain of the norm that follows [N]
    float* xsplit;            // h * gain as two bf16 arrays (hi [m][N], then lo [m][N])
    float* ssq;               // [ceil(ntiles / tpb)][16]
    int* abort;
    uint32_t epoch;
    int spin_limit;
};

template <int PRO, int EPI = EPI_PARTIALS>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const float* __restrict__ x, int ldx, int m, int K,
                                                        const bf16_t* __restrict__ W0, const bf16_t* __restrict__ W1,
                                                        const bf16_t* __restrict__ W2, int t0, int t1, int ntiles,
                                                        float* __restrict__ out, int N, int ksplit, int cps, int tpb,
                                                        GemmPro pro, GemmEpi epi) {
    extern __shared__ uint4 xs[];   // [2 (hi, lo)][m][rs]  (+ [m][K] floats for PRO_NORM)
    const int kchunks = K >> 5;
    const int ks = blockIdx.x % ksplit, tg = blockIdx.x / ksplit;
    const int c0 = ks * cps;
    const int nc = min(cps, kchunks - c0);
    const int rs = cps * 4 + 1;  // LDS row stride in 16-byte units (+1 pads away bank conflicts)
    uint4* xlo = xs + m * rs;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ngroups = (nc + GEMM_U - 1) / GEMM_U;
    // weight tiles of chunk group gi of tile t (tiles past the slice's end read as zero)
    auto tile_base = [&](int t) -> const u32x4* {
        const bf16_t* W;
        int tl;
        if (t < t0) { W = W0; tl = t; }
        else if (t < t1) { W = W1; tl = t - t0; }
        else { W = W2; tl = t - t1; }
        return reinterpret_cast<const u32x4*>(W) + ((size_t)tl * kchunks + c0) * 64 + lane;
    };
    // every load is unconditional (chunks past the slice's end re-read its last tile and are
    // multiplied by zero activations): a branch around a load would make the compiler drain the
    // whole load queue before the first multiply and undo the two-buffer pipeline below
    auto issue = [&](u32x4 (&w)[GEMM_U], const u32x4* wp, int gi) {
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u) w[u] = __builtin_nontemporal_load(wp + (size_t)min(gi * GEMM_U + u, nc - 1) * 64);
    };
    u32x4 wa[GEMM_U], wb[GEMM_U];
    const int tfirst = tg * tpb + wave;
    const u32x4* wp = tile_base(min(tfirst, ntiles - 1));   // a wavefront without a tile still loads (unconditional requests keep the counters exact)
    const int total = m * nc * 4, per = nc * 4;
    auto convert_store = [&](const float (&v)[8], int idx) {
        const int r = idx / per, c = idx - r * per;
        bf16_t hi[8], lo[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            hi[e] = f2bf(v[e]);
            lo[e] = f2bf(v[e] - bf2f(hi[e]));
        }
        xs[r * rs + c] = make_uint4(pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3]), pack_bf16x2(hi[4], hi[5]), pack_bf16x2(hi[6], hi[7]));
        xlo[r * rs + c] = make_uint4(pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3]), pack_bf16x2(lo[4], lo[5]), pack_bf16x2(lo[6], lo[7]));
    };
    if constexpr (PRO == PRO_PLAIN) {
        // When the input is h * gain of a residual epilogue (not yet normalised), workgroup 0 also turns the
        // per-tile-group sums of squares into 1/rms per row for the kernels that consume this GEMM's output.
        // (all rows of an entry come with four 16-byte loads, every load independent of the others: one memory
        // round trip for the whole table instead of one per row - this wavefront is on the kernel's critical path)
        if (pro.src && blockIdx.x == 0 && wave == 0) {
            float4 t[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) t[q] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
            for (int i0 = 0; i0 < pro.ns; i0 += 64) {
                const int i = i0 + lane;
                const float sc = i < pro.ns ? 1.f : 0.f;
                const float4* e = reinterpret_cast<const float4*>(pro.src + (size_t)min(i, pro.ns - 1) * 16);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 v = e[q];
                    t[q].x += sc * v.x; t[q].y += sc * v.y; t[q].z += sc * v.z; t[q].w += sc * v.w;
                }
            }
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) {                  // table row rr is this block's row rr - pro.row0
                const float4 tq = t[rr >> 2];
                float tr = (rr & 3) == 0 ? tq.x : (rr & 3) == 1 ? tq.y : (rr & 3) == 2 ? tq.z : tq.w;
                if (rr >= pro.row0 && rr - pro.row0 < m) {     // wavefront-uniform
                    tr = wave_sum(tr);
                    if (lane == 0) pro.h_out[rr - pro.row0] = 1.0f / sqrtf(tr / (float)K + pro.eps);
                }
            }
        }
        // Order of the requests (a wavefront's loads return in order): first the activations of this
        // workgroup's slice (L2 hits, needed first), then the first KiBs of the weight stream, which
        // stay in flight while the activations are converted and written to LDS.
        // x is given as two bf16 arrays (hi at x, lo at x + pro.sstride elements), row stride ldx.
        constexpr int XB = 6;                         // 8-element pieces per thread and batch
        const bf16_t* xh = reinterpret_cast<const bf16_t*>(x);
        auto piece = [&](int idx) -> const bf16_t* {  // clamped: every load is unconditional and in range
            const int ic = min(idx, total - 1);
            const int r = ic / per, c = ic - r * per;
            return xh + (size_t)r * ldx + (size_t)c0 * 32 + (size_t)c * 8;
        };
        u32x4 a[XB], b[XB];   // (ext vectors: arrays of the HIP struct type end up in scratch memory)
#pragma unroll
        for (int u = 0; u < XB; ++u) {
            const bf16_t* src = piece((int)threadIdx.x + u * 256);
            a[u] = *reinterpret_cast<const u32x4*>(src);
            b[u] = *reinterpret_cast<const u32x4*>(src + pro.sstride);
        }
        issue(wa, wp, 0);
#pragma unroll
        for (int u = 0; u < XB; ++u) {
            const int idx = (int)threadIdx.x + u * 256;
            if (idx < total) { const int r = idx / per, c = idx - r * per; xs[r * rs + c] = __builtin_bit_cast(uint4, a[u]); xlo[r * rs + c] = __builtin_bit_cast(uint4, b[u]); }
        }
        for (int base = XB * 256; base < total; base += XB * 256) {   // taller / wider blocks: further batches
#pragma unroll
            for (int u = 0; u < XB; ++u) {
                const bf16_t* src = piece(base + (int)threadIdx.x + u * 256);
                a[u] = *reinterpret_cast<const u32x4*>(src);
                b[u] = *reinterpret_cast<const u32x4*>(src + pro.sstride);
            }
#pragma unroll
            for (int u = 0; u < XB; ++u) {
                const int idx = base + (int)threadIdx.x + u * 256;
                if (idx < total) { const int r = idx / per, c = idx - r * per; xs[r * rs + c] = __builtin_bit_cast(uint4, a[u]); xlo[r * rs + c] = __builtin_bit_cast(uint4, b[u]); }
            }
        }
    } else if constexpr (PRO == PRO_NORM) {
        float* vrow = reinterpret_cast<float*>(xs + 2 * m * rs);     // [m][K] updated residual rows
        float* red = vrow + (size_t)m * K;                           // [m][4] per-wavefront sums of squares
        for (int r = 0; r < m; ++r) {
            float ss = 0.f;
            for (int i = (int)threadIdx.x * 4; i < K; i += 1024) {
                float4 v = *reinterpret_cast<const float4*>(pro.src + (size_t)r * K + i);
                if (pro.ns > 0) {
                    float4 y = make_float4(0.f, 0.f, 0.f, 0.f);
                    for (int s0 = 0; s0 < pro.ns; s0 += 8) {      // eight partials in flight, added in the order s = 0, 1, ..
                        float4 pp[8];
#pragma unroll
                        for (int u = 0; u < 8; ++u)
                            pp[u] = (s0 + u < pro.ns) ? *reinterpret_cast<const float4*>(pro.part + (size_t)(s0 + u) * pro.sstride + (size_t)r * K + i)
                                                      : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                        for (int u = 0; u < 8; ++u)
                            if (s0 + u < pro.ns) { y.x += pp[u].x; y.y += pp[u].y; y.z += pp[u].z; y.w += pp[u].w; }
                    }
                    v.x += y.x; v.y += y.y; v.z += y.z; v.w += y.w;
                }
                *reinterpret_cast<float4*>(vrow + (size_t)r * K + i) = v;
                ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
            }
            ss = wave_sum(ss);
            if (lane == 0) red[r * 4 + wave] = ss;
        }
        issue(wa, wp, 0);
        __syncthreads();
        if (blockIdx.x == 0)
            for (int i = (int)threadIdx.x * 4; i < m * K; i += 1024)
                *reinterpret_cast<float4*>(pro.h_out + i) = *reinterpret_cast<const float4*>(vrow + i);
        for (int idx = (int)threadIdx.x; idx < total; idx += 256) {
            const int r = idx / per, c = idx - r * per, k0 = c0 * 32 + c * 8;
            const float tot = (red[r * 4] + red[r * 4 + 1]) + (red[r * 4 + 2] + red[r * 4 + 3]);
            const float inv = 1.0f / sqrtf(tot / (float)K + pro.eps);
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = vrow[(size_t)r * K + k0 + e] * inv * bf2f(pro.gain[k0 + e]);
            convert_store(v, idx);
        }
    } else if constexpr (PRO == PRO_ACT) {
        issue(wa, wp, 0);
        const int ldp = (pro.act == 1 ? 2 : 1) * K;
        for (int idx = (int)threadIdx.x; idx < total; idx += 256) {
            const int r = idx / per, c = idx - r * per, k0 = c0 * 32 + c * 8;
            const float* pg = pro.src + (size_t)r * ldp + k0;
            float gsum[8], usum[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) gsum[e] = usum[e] = 0.f;
            for (int s0 = 0; s0 < pro.ns; s0 += 2) {              // two partials in flight, added in order
                float4 ga[2], gb[2], ua[2], ub[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const bool ok = s0 + u < pro.ns;
                    const float* q = pg + (size_t)(ok ? s0 + u : 0) * pro.sstride;
                    ga[u] = *reinterpret_cast<const float4*>(q);
                    gb[u] = *reinterpret_cast<const float4*>(q + 4);
                    if (pro.act == 1) { ua[u] = *reinterpret_cast<const float4*>(q + K); ub[u] = *reinterpret_cast<const float4*>(q + K + 4); }
                    else { ua[u] = make_float4(0.f, 0.f, 0.f, 0.f); ub[u] = ua[u]; }
                }
#pragma unroll
                for (int u = 0; u < 2; ++u)
                    if (s0 + u < pro.ns) {
                        gsum[0] += ga[u].x; gsum[1] += ga[u].y; gsum[2] += ga[u].z; gsum[3] += ga[u].w;
                        gsum[4] += gb[u].x; gsum[5] += gb[u].y; gsum[6] += gb[u].z; gsum[7] += gb[u].w;
                        usum[0] += ua[u].x; usum[1] += ua[u].y; usum[2] += ua[u].z; usum[3] += ua[u].w;
                        usum[4] += ub[u].x; usum[5] += ub[u].y; usum[6] += ub[u].z; usum[7] += ub[u].w;
                    }
            }
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                v[e] = pro.act == 1 ? gsum[e] / (1.0f + expf(-gsum[e])) * usum[e] : 0.5f * gsum[e] * (1.0f + erff(gsum[e] * 0.70710678118654752f));
            convert_store(v, idx);
        }
    } else {   // PRO_COMBINE: eight threads per 8-element piece, each merging every eighth chunk
        issue(wa, wp, 0);
        const size_t cs = (size_t)16 * (pro.hd + 2);
        const int sub = (int)threadIdx.x & 7;
        for (int ib = 0; ib < total; ib += 32) {
            const int idx = ib + ((int)threadIdx.x >> 3), ic = min(idx, total - 1);
            const int r = ic / per, c = ic - r * per, k0 = c0 * 32 + c * 8;
            const int head = k0 / pro.hd, col = k0 - head * pro.hd;
            const float* base = pro.src + ((size_t)head * pro.nchunks * 16 + r) * (pro.hd + 2);
            float mc[4], lc[4];
            float2 oc[4][4];
            float M = -INFINITY;
#pragma unroll
            for (int u = 0; u < 4; ++u) {                          // chunks sub, sub + 8, .. (up to 32 chunks per pass)
                const int ch = sub + 8 * u;
                const bool ok = ch < pro.nchunks;
                const float* rec = base + (size_t)(ok ? ch : 0) * cs;
                mc[u] = ok ? rec[pro.hd] : -INFINITY;
                lc[u] = ok ? rec[pro.hd + 1] : 0.f;
                const float2* op = reinterpret_cast<const float2*>(rec + col);
                oc[u][0] = op[0]; oc[u][1] = op[1]; oc[u][2] = op[2]; oc[u][3] = op[3];
                M = fmaxf(M, mc[u]);
            }
            for (int ch0 = 32; ch0 < pro.nchunks; ch0 += 8)        // longer contexts: the maximum needs every chunk
                if (ch0 + sub < pro.nchunks) M = fmaxf(M, base[(size_t)(ch0 + sub) * cs + pro.hd]);
            M = fmaxf(M, __shfl_xor(M, 1, 64));
            M = fmaxf(M, __shfl_xor(M, 2, 64));
            M = fmaxf(M, __shfl_xor(M, 4, 64));
            float Lsum = 0.f, o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = 0.f;
            auto merge = [&](float mcv, float lcv, const float2 (&ov)[4]) {
                const float w = (mcv == -INFINITY) ? 0.f : expf(mcv - M);
                Lsum += lcv * w;
                o[0] += ov[0].x * w; o[1] += ov[0].y * w; o[2] += ov[1].x * w; o[3] += ov[1].y * w;
                o[4] += ov[2].x * w; o[5] += ov[2].y * w; o[6] += ov[3].x * w; o[7] += ov[3].y * w;
            };
#pragma unroll
            for (int u = 0; u < 4; ++u) merge(mc[u], lc[u], oc[u]);
            for (int ch = 32 + sub; ch < pro.nchunks; ch += 8) {
                const float* rec = base + (size_t)ch * cs;
                const float2* op = reinterpret_cast<const float2*>(rec + col);
                const float2 ov[4] = {op[0], op[1], op[2], op[3]};
                merge(rec[pro.hd], rec[pro.hd + 1], ov);
            }
#pragma unroll
            for (int sh = 1; sh < 8; sh <<= 1) {
                Lsum += __shfl_xor(Lsum, sh, 64);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] += __shfl_xor(o[e], sh, 64);
            }
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = o[e] / Lsum;
            if (sub == 0 && idx < total) convert_store(v, idx);
        }
    }
    __syncthreads();
    const int row = lane & 15, g = lane >> 4;
    const bool rowok = row < m;
    const uint4* xa = xs + (rowok ? row : 0) * rs + g;
    const uint4* xb = xlo + (rowok ? row : 0) * rs + g;
    const uint4 zero = make_uint4(0, 0, 0, 0);
    f32x4 acc, acl;
    auto multiply = [&](const u32x4 (&w)[GEMM_U], int gi) {
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u) {
            const int c = gi * GEMM_U + u;
            const bool live = rowok && c < nc;
            uint4 ah = xa[min(c, nc - 1) * 4], al = xb[min(c, nc - 1) * 4];
            if (!live) { ah = zero; al = zero; }
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[u]), __builtin_bit_cast(bf16x8, ah), acc, 0, 0, 0);
            acl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[u]), __builtin_bit_cast(bf16x8, al), acl, 0, 0, 0);
        }
    };
    __shared__ float epi_red[4][16];
    for (int tt = wave; tt < tpb; tt += 4) {
        const int t = tg * tpb + tt;
        const bool live_tile = t < ntiles;
        if (!live_tile && EPI == EPI_PARTIALS) break;
        if (tt != wave && live_tile) {
            wp = tile_base(t);
            issue(wa, wp, 0);
        }
        acc = f32x4{0.f, 0.f, 0.f, 0.f};
        acl = f32x4{0.f, 0.f, 0.f, 0.f};
        if (live_tile) {
            // two register buffers: the next group of tiles is in flight while this one is multiplied
            int gi = 0;
            for (; gi + 2 < ngroups; gi += 2) {
                issue(wb, wp, gi + 1);
                multiply(wa, gi);
                issue(wa, wp, gi + 2);
                multiply(wb, gi + 1);
            }
            if (gi + 2 == ngroups) {
                issue(wb, wp, gi + 1);
                multiply(wa, gi);
                multiply(wb, gi + 1);
            } else {
                multiply(wa, gi);
            }
        }
        const float4 mine = make_float4(acc[0] + acl[0], acc[1] + acl[1], acc[2] + acl[2], acc[3] + acl[3]);
        if constexpr (EPI == EPI_PARTIALS) {
            if (rowok) {
                float* o = out + (size_t)ks * m * N + (size_t)row * N + (size_t)t * 16 + g * 4;
                *reinterpret_cast<float4*>(o) = mine;
            }
        } else {
            const size_t col = (size_t)t * 16 + g * 4;
            const bool own = rowok && live_tile;
            if (ks < ksplit - 1) {                     // publish this sibling's partial tile
                if (own) {
                    unsigned long long* dst = epi.xw + ((size_t)ks * m + row) * N + col;
                    tw_put(dst + 0, epi.epoch, __float_as_uint(mine.x));
                    tw_put(dst + 1, epi.epoch, __float_as_uint(mine.y));
                    tw_put(dst + 2, epi.epoch, __float_as_uint(mine.z));
                    tw_put(dst + 3, epi.epoch, __float_as_uint(mine.w));
                }
            } else {                                   // last sibling: reduce, residual, gain, sum of squares
                float ss = 0.f;
                if (own) {
                    float4 hv = *reinterpret_cast<const float4*>(epi.h + (size_t)row * N + col);
                    float4 y = make_float4(0.f, 0.f, 0.f, 0.f);
                    bool ok = true;
                    for (int sb0 = 0; sb0 < ksplit - 1 && ok; sb0 += 8) {      // up to eight siblings (32 words) in flight
                        const int nb = min(8, ksplit - 1 - sb0);
                        unsigned long long w[8][4];
                        ok = false;
                        for (int it = 0; it < epi.spin_limit && !ok; ++it) {
                            ok = true;
#pragma unroll
                            for (int u = 0; u < 8; ++u) {
                                const unsigned long long* src = epi.xw + ((size_t)(sb0 + min(u, nb - 1)) * m + row) * N + col;
#pragma unroll
                                for (int v = 0; v < 4; ++v) w[u][v] = __hip_atomic_load(src + v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            }
#pragma unroll
                            for (int u = 0; u < 8; ++u)
#pragma unroll
                                for (int v = 0; v < 4; ++v) ok = ok && (uint32_t)(w[u][v] >> 32) == epi.epoch;
                            if (!ok) __builtin_amdgcn_s_sleep(2);
                        }
#pragma unroll
                        for (int u = 0; u < 8; ++u)
                            if (u < nb) {
                                y.x += __uint_as_float((uint32_t)w[u][0]); y.y += __uint_as_float((uint32_t)w[u][1]);
                                y.z += __uint_as_float((uint32_t)w[u][2]); y.w += __uint_as_float((uint32_t)w[u][3]);
                            }
                    }
                    if (!ok) {
                        // a sibling never showed up: report it and leave the residual stream as it was (the host
                        // fails the round at the next accept; nothing is added from words of another launch)
                        __hip_atomic_store(epi.abort, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    } else {
                        y.x += mine.x; y.y += mine.y; y.z += mine.z; y.w += mine.w;
                        hv.x += y.x; hv.y += y.y; hv.z += y.z; hv.w += y.w;
                        *reinterpret_cast<float4*>(epi.h + (size_t)row * N + col) = hv;
                        const uint2 gn = *reinterpret_cast<const uint2*>(epi.gain + col);
                        const float4 xg = make_float4(hv.x * bf2f((bf16_t)(gn.x & 0xffffu)), hv.y * bf2f((bf16_t)(gn.x >> 16)),
                                                      hv.z * bf2f((bf16_t)(gn.y & 0xffffu)), hv.w * bf2f((bf16_t)(gn.y >> 16)));
                        store_split4(epi.xsplit, (size_t)m * N, (size_t)row * N + col, xg);
                        ss = hv.x * hv.x + hv.y * hv.y + hv.z * hv.z + hv.w * hv.w;
                    }
                }
                ss += __shfl_xor(ss, 16, 64);
                ss += __shfl_xor(ss, 32, 64);
                if (g == 0) epi_red[wave][row] = ss;   // 16 columns of this wavefront's tile
            }
        }
    }
    if constexpr (EPI == EPI_RESIDUAL) {
        if (ks == ksplit - 1) {                        // workgroup-uniform
            __syncthreads();
            if (threadIdx.x < 16) {
                const int r = (int)threadIdx.x;
                epi.ssq[(size_t)tg * 16 + r] = (epi_red[0][r] + epi_red[1][r]) + (epi_red[2][r] + epi_red[3][r]);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Residual-stream GEMM without split-K partials, for a projection whose whole input block fits in LDS
// (the attention output projection: K = d_model).  One workgroup of 8 wavefronts per 16-feature tile;
// wavefront w streams the w-th eighth of the tile's K range against its own slice of the activations
// (staged privately: no workgroup barrier before the multiplies), the eight partial tiles are added
// through LDS, and wavefront 0 applies the residual epilogue of EPI_RESIDUAL directly: h += out,
// h * gain in the two-bf16 form, sums of squares per tile.  No sibling workgroups, nothing to wait for.
//   grid (ntiles), block 512, dynamic LDS 2 * 8 * m * (cpw*4 + 1) * 16 + 8 * 64 * 16 bytes, cpw = ceil(K/32/8).
// ssq is [ntiles][16] here (one entry per tile).

__global__ __launch_bounds__(512) void gemm_fullk_residual_kernel(const bf16_t* __restrict__ xh, size_t x_lo_off, int ldx, int m, int K,
                                                                  const bf16_t* __restrict__ W, int ntiles, int N,
                                                                  float* __restrict__ h, const bf16_t* __restrict__ gain,
                                                                  float* __restrict__ xsplit, float* __restrict__ ssq) {
    extern __shared__ uint4 lds[];
    const int kchunks = K >> 5;
    const int cpw = (kchunks + 7) >> 3;            // chunks per wavefront
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blockIdx.x;
    const int c0 = wave * cpw, nc = max(0, min(cpw, kchunks - c0));
    const int rs = cpw * 4 + 1;
    uint4* xs = lds + (size_t)wave * 2 * m * rs;   // this wavefront's [2 (hi, lo)][m][rs]
    uint4* xlo = xs + m * rs;
    f32x4* red = reinterpret_cast<f32x4*>(lds + (size_t)8 * 2 * m * rs);   // [8][64]
    const u32x4* wp = reinterpret_cast<const u32x4*>(W) + ((size_t)t * kchunks + c0) * 64 + lane;
    const int ngroups = (nc + GEMM_U - 1) / GEMM_U;
    auto issue = [&](u32x4 (&w)[GEMM_U], int gi) {
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u) w[u] = __builtin_nontemporal_load(wp + (size_t)min(gi * GEMM_U + u, max(nc, 1) - 1) * 64);
    };
    u32x4 wa[GEMM_U], wb[GEMM_U];
    // The epilogue's inputs (this tile's block of the residual stream and of the gain) are requested first of all, by every
    // wavefront alike (only wavefront 0 uses them): their trip to memory overlaps the stream instead of following it.
    const int erow = (lane & 15) < m ? (lane & 15) : 0;
    const size_t ecol = (size_t)t * 16 + (lane >> 4) * 4;
    const float4 h_pre = *reinterpret_cast<const float4*>(h + (size_t)erow * N + ecol);
    const uint2 gn_pre = *reinterpret_cast<const uint2*>(gain + ecol);
    // activations of this wavefront's slice next (they come back first), then the weight stream
    {
        const int total = m * nc * 4, per = nc * 4;
        constexpr int XB = 6;
        for (int base = 0; base < total; base += XB * 64) {
            u32x4 a[XB], b[XB];
#pragma unroll
            for (int u = 0; u < XB; ++u) {
                const int ic = min(base + lane + u * 64, total - 1);
                const int r = ic / per, c = ic - r * per;
                const bf16_t* src = xh + (size_t)r * ldx + (size_t)c0 * 32 + (size_t)c * 8;
                a[u] = *reinterpret_cast<const u32x4*>(src);
                b[u] = *reinterpret_cast<const u32x4*>(src + x_lo_off);
            }
            if (base == 0 && nc > 0) issue(wa, 0);
#pragma unroll
            for (int u = 0; u < XB; ++u) {
                const int idx = base + lane + u * 64;
                if (idx < total) { const int r = idx / per, c = idx - r * per; xs[r * rs + c] = __builtin_bit_cast(uint4, a[u]); xlo[r * rs + c] = __builtin_bit_cast(uint4, b[u]); }
            }
        }
    }
    const int row = lane & 15, g = lane >> 4;
    const bool rowok = row < m;
    const uint4* xa = xs + (rowok ? row : 0) * rs + g;
    const uint4* xb = xlo + (rowok ? row : 0) * rs + g;
    const uint4 zero = make_uint4(0, 0, 0, 0);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acl = {0.f, 0.f, 0.f, 0.f};
    auto multiply = [&](const u32x4 (&w)[GEMM_U], int gi) {
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u) {
            const int c = gi * GEMM_U + u;
            const bool live = rowok && c < nc;
            uint4 ah = xa[min(c, nc - 1) * 4], al = xb[min(c, nc - 1) * 4];
            if (!live) { ah = zero; al = zero; }
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[u]), __builtin_bit_cast(bf16x8, ah), acc, 0, 0, 0);
            acl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[u]), __builtin_bit_cast(bf16x8, al), acl, 0, 0, 0);
        }
    };
    if (nc > 0) {
        // the LDS writes above are this wavefront's own; its reads below follow them in program order
        int gi = 0;
        for (; gi + 2 < ngroups; gi += 2) {
            issue(wb, gi + 1);
            multiply(wa, gi);
            issue(wa, gi + 2);
            multiply(wb, gi + 1);
        }
        if (gi + 2 == ngroups) {
            issue(wb, gi + 1);
            multiply(wa, gi);
            multiply(wb, gi + 1);
        } else {
            multiply(wa, gi);
        }
    }
    red[wave * 64 + lane] = acc + acl;
    __syncthreads();
    if (wave != 0) return;
    f32x4 y = red[lane];
#pragma unroll
    for (int w = 1; w < 8; ++w) y += red[w * 64 + lane];      // fixed order: deterministic
    float ss = 0.f;
    if (rowok) {
        const size_t col = (size_t)t * 16 + g * 4;
        float4 hv = h_pre;
        hv.x += y[0]; hv.y += y[1]; hv.z += y[2]; hv.w += y[3];
        *reinterpret_cast<float4*>(h + (size_t)row * N + col) = hv;
        const uint2 gn = gn_pre;
        const float4 xg = make_float4(hv.x * bf2f((bf16_t)(gn.x & 0xffffu)), hv.y * bf2f((bf16_t)(gn.x >> 16)),
                                      hv.z * bf2f((bf16_t)(gn.y & 0xffffu)), hv.w * bf2f((bf16_t)(gn.y >> 16)));
        store_split4(xsplit, (size_t)m * N, (size_t)row * N + col, xg);
        ss = hv.x * hv.x + hv.y * hv.y + hv.z * hv.z + hv.w * hv.w;
    }
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if (g == 0) ssq[(size_t)t * 16 + row] = ss;
}

// The same projection for an input block too large for LDS (the FFN down projection: K = d_ffn): each wavefront
// still owns an eighth of the tile's K range, but stages its activations group by group (8 chunks = 256
// inputs at a time, the granularity of its weight register buffers) into two small private LDS buffers:
// while group g is multiplied, the activations of group g+1 are requested (L2 hits) and written to the other
// buffer.  Wavefront-private, so no workgroup barrier inside the stream; LDS reduction over the eight
// wavefronts and the residual epilogue as in gemm_fullk_residual_kernel.  No sibling workgroups.
//   XB = ceil(m / 2): 16-byte pieces per lane, term and group.
//   DBUF = false (9 .. 16 rows, where two buffers per wavefront no longer fit): one buffer - the next group's activations
//   wait in registers while the current group is multiplied and are written when its LDS reads have been issued (a
//   wavefront's LDS operations are served in order); a group is 8 KiB of weights per wavefront, so that costs nothing
//   the stream would notice.
//   grid (ntiles), block 512, dynamic LDS 8 * (DBUF ? 2 : 1) * 2 * m * 33 * 16 + 8 * 64 * 16 bytes.
template <int XB, bool DBUF = true>
__global__ __launch_bounds__(512) void gemm_fullk_roll_residual_kernel(const bf16_t* __restrict__ xh, size_t x_lo_off, int ldx, int m, int K,
                                                                       const bf16_t* __restrict__ W, int ntiles, int N,
                                                                       float* __restrict__ h, const bf16_t* __restrict__ gain,
                                                                       float* __restrict__ xsplit, float* __restrict__ ssq) {
    extern __shared__ uint4 lds[];
    constexpr int RS = GEMM_U * 4 + 1;             // LDS row stride (16-byte pieces), +1 against bank conflicts
    const int kchunks = K >> 5;
    const int cpw = (kchunks + 7) >> 3;            // chunks per wavefront
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blockIdx.x;
    const int c0 = min(wave * cpw, kchunks - 1), nc = max(0, min(cpw, kchunks - wave * cpw));
    constexpr int NB = DBUF ? 2 : 1, B1 = DBUF ? 1 : 0;                    // buffers per wavefront; the "other" buffer
    uint4* xbuf = lds + (size_t)wave * NB * 2 * m * RS;                    // [NB buffers][2 (hi, lo)][m][RS]
    f32x4* red = reinterpret_cast<f32x4*>(lds + (size_t)8 * NB * 2 * m * RS);   // [8][64]
    const u32x4* wp = reinterpret_cast<const u32x4*>(W) + ((size_t)t * kchunks + c0) * 64 + lane;
    const int ngroups = (nc + GEMM_U - 1) / GEMM_U;
    const int last = max(nc, 1) - 1;
    // every load is unconditional and clamped into valid memory; chunks past the slice's end meet masked weights
    auto issue = [&](u32x4 (&w)[GEMM_U], int gi) {
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u) w[u] = __builtin_nontemporal_load(wp + (size_t)min(gi * GEMM_U + u, last) * 64);
    };
    const int npieces = m * GEMM_U * 4;            // pieces per term and group
    auto sload = [&](u32x4 (&a)[XB], u32x4 (&b)[XB], int gi) {
#pragma unroll
        for (int u = 0; u < XB; ++u) {
            const int idx = min(lane + 64 * u, npieces - 1), r = idx / (GEMM_U * 4), c = idx - r * (GEMM_U * 4);
            const int col = min((c0 + gi * GEMM_U) * 32 + c * 8, K - 8);
            const bf16_t* src = xh + (size_t)r * ldx + col;
            a[u] = *reinterpret_cast<const u32x4*>(src);
            b[u] = *reinterpret_cast<const u32x4*>(src + x_lo_off);
        }
    };
    auto sstore = [&](const u32x4 (&a)[XB], const u32x4 (&b)[XB], int buf) {
        uint4* xs = xbuf + (size_t)buf * 2 * m * RS;
#pragma unroll
        for (int u = 0; u < XB; ++u) {
            const int idx = lane + 64 * u;
            if (idx < npieces) {
                const int r = idx / (GEMM_U * 4), c = idx - r * (GEMM_U * 4);
                xs[r * RS + c] = __builtin_bit_cast(uint4, a[u]);
                xs[(m + r) * RS + c] = __builtin_bit_cast(uint4, b[u]);
            }
        }
    };
    const int row = lane & 15, g = lane >> 4;
    const bool rowok = row < m;
    const int rowc = rowok ? row : 0;              // rows beyond m read row 0: their output columns are never stored
    f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acl = {0.f, 0.f, 0.f, 0.f};
    auto multiply = [&](const u32x4 (&w)[GEMM_U], int buf, int gi) {
        const u32x4* xs = reinterpret_cast<const u32x4*>(xbuf + (size_t)buf * 2 * m * RS);
#pragma unroll
        for (int u = 0; u < GEMM_U; ++u) {
            const uint32_t mask = gi * GEMM_U + u < nc ? 0xffffffffu : 0u;
            const u32x4 wm = w[u] & mask;
            const u32x4 ah = xs[rowc * RS + u * 4 + g], al = xs[(m + rowc) * RS + u * 4 + g];
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wm), __builtin_bit_cast(bf16x8, ah), acc, 0, 0, 0);
            acl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wm), __builtin_bit_cast(bf16x8, al), acl, 0, 0, 0);
        }
    };
    u32x4 wa[GEMM_U], wb[GEMM_U], xa[XB], xb[XB];
    // the epilogue's inputs are requested first of all (see gemm_fullk_residual_kernel)
    const size_t ecol = (size_t)t * 16 + g * 4;
    const float4 h_pre = *reinterpret_cast<const float4*>(h + (size_t)rowc * N + ecol);
    const uint2 gn_pre = *reinterpret_cast<const uint2*>(gain + ecol);
    if (nc > 0) {
        sload(xa, xb, 0);                          // activations first: they come back first
        issue(wa, 0);
        sstore(xa, xb, 0);
        int gi = 0;
        for (; gi + 2 < ngroups; gi += 2) {
            sload(xa, xb, gi + 1);
            issue(wb, gi + 1);
            multiply(wa, 0, gi);
            sstore(xa, xb, B1);
            sload(xa, xb, gi + 2);
            issue(wa, gi + 2);
            multiply(wb, B1, gi + 1);
            sstore(xa, xb, 0);
        }
        if (gi + 2 == ngroups) {
            sload(xa, xb, gi + 1);
            issue(wb, gi + 1);
            multiply(wa, 0, gi);
            sstore(xa, xb, B1);
            multiply(wb, B1, gi + 1);
        } else {
            multiply(wa, 0, gi);
        }
    }
    red[wave * 64 + lane] = acc + acl;
    __syncthreads();
    if (wave != 0) return;
    f32x4 y = red[lane];
#pragma unroll
    for (int w = 1; w < 8; ++w) y += red[w * 64 + lane];      // fixed order: deterministic
    float ss = 0.f;
    if (rowok) {
        const size_t col = (size_t)t * 16 + g * 4;
        float4 hv = h_pre;
        hv.x += y[0]; hv.y += y[1]; hv.z += y[2]; hv.w += y[3];
        *reinterpret_cast<float4*>(h + (size_t)row * N + col) = hv;
        const uint2 gn = gn_pre;
        const float4 xg = make_float4(hv.x * bf2f((bf16_t)(gn.x & 0xffffu)), hv.y * bf2f((bf16_t)(gn.x >> 16)),
                                      hv.z * bf2f((bf16_t)(gn.y & 0xffffu)), hv.w * bf2f((bf16_t)(gn.y >> 16)));
        store_split4(xsplit, (size_t)m * N, (size_t)row * N + col, xg);
        ss = hv.x * hv.x + hv.y * hv.y + hv.z * hv.z + hv.w * hv.w;
    }
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if (g == 0) ssq[(size_t)t * 16 + row] = ss;
}

// Row-major bf16 W[n_out][n_in] -> streaming-tile order.  One thread per 16-byte piece.
// rope_hd > 0 (q and k projections): inside every head of rope_hd output features the rows are
// re-ordered so that tile j holds the rotary pairs (i, i + rope_hd/2), i = 8j .. 8j+7, side by side:
// packed row 16j + c  <-  source row (c even ? 8j + c/2 : 8j + c/2 + rope_hd/2).  The GEMM epilogue
// then finds both members of a pair in one lane and writes them back to their natural positions.
__global__ void pack_weight_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int n_out, int n_in, int rope_hd) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // index of a 16-byte piece in dst
    const size_t total = (size_t)n_out * n_in / 8;
    if (i >= total) return;
    const int kchunks = n_in >> 5;
    const int lane = (int)(i & 63);
    const size_t tile = i >> 6;
    const int c = (int)(tile % kchunks);
    const size_t t = tile / kchunks;
    size_t rowi = t * 16 + (lane & 15);
    if (rope_hd > 0) {
        const size_t head = rowi / rope_hd;
        const int rr = (int)(rowi - head * rope_hd), j = rr >> 4, cc = rr & 15;
        rowi = head * rope_hd + (size_t)(8 * j + (cc >> 1) + ((cc & 1) ? (rope_hd >> 1) : 0));
    }
    const size_t col = (size_t)c * 32 + (size_t)(lane >> 4) * 8;
    dst[i] = src[(rowi * n_in + col) / 8];
}

// ------------------------------------------------------------------------------------------
// Token trees (multi-candidate verification with tree attention, the white-box setting of the paper's Sec. 4).
// A tree block holds nodes of a draft tree in breadth-first order: node 0 is the root (the last committed token, cache slot
// and position `base`), node i > 0 hangs under a node with a lower index.  Node i lives in cache slot base + i, is rotated
// for position base + depth(i), and attends to every committed position (< base) and to its ancestors and itself.
// Block row r is node i0 + r.  on == 0: an ordinary causal block (row r at slot = position pos0 + r).
// on == 2: not a tree but the streaming cache of a drafter (the StreamingLLM strategy of the paper's appendix on KV cache
// strategies): an ordinary block whose row at position p attends to the first `sink` positions and to the last `i0`
// positions up to p that are not below `base`, the start of the contiguous tail of the cache (what lies between the
// sinks and the tail was skipped when the drafter was switched in and holds nothing).
constexpr int TREE_MAX = 16;
struct TreeBlk {
    int on, base, i0, sink;
    uint16_t anc[TREE_MAX];    // bit j: node j is this node or one of its ancestors
    uint8_t depth[TREE_MAX];
};
__device__ __forceinline__ bool tree_allowed(const TreeBlk& tb, int p, int row, int pos0) {
    if (tb.on == 2) {
        const int pr = pos0 + row;
        return p <= pr && (p < tb.sink || p >= max(tb.base, pr - tb.i0 + 1));
    }
    const int j = p - tb.base;
    return j < 0 || (j < TREE_MAX && ((tb.anc[tb.i0 + row] >> j) & 1));
}
// streaming cache: no row of the block (positions pos0 ..) attends to anything in positions [p0, p0 + n)
__device__ __forceinline__ bool stream_skips(const TreeBlk& tb, int p0, int n, int pos0) {
    return tb.on == 2 && p0 >= tb.sink && p0 + n <= max(tb.base, pos0 - tb.i0 + 1);
}

// ------------------------------------------------------------------------------------------
// RoPE (rotate-half pairing, angle = pos * theta^(-2i/hd)) on q and k, K/V cache append.
//   part: split-K partials of the fused q|k|v projection, [s][r][N], N = (H + 2 KH) * hd.
//   q out fp32 [m][H*hd] (q_split: as two bf16 arrays, see below); cache planes (type T) [kv_head][max_ctx][hd].
//   grid (ceil((H + 2KH) / k), m), block 64 k

// The rotation table of a forward block, tab[r][i] = (cos, sin)((pos0 + r) * theta^(-2i/hd)) in fp64 (the rotation is
// applied in fp64 and rounded once), is built once per forward by embed_rope_kernel and used by every layer.

// Body for block row r = blockIdx.y at position pos; write_kv = false for padding rows (q is still written).
template <typename T>
__device__ __forceinline__ void rope_kv_body(const float* __restrict__ part, int nsplit, size_t sstride, int N, int pos, int H,
                                             int KH, int hd, const double2* __restrict__ tab, float* __restrict__ q,
                                             T* __restrict__ kc, T* __restrict__ vc, int max_ctx, int interleaved, int q_split,
                                             const float* __restrict__ inv, bool write_kv) {
    // 64 threads per head; a workgroup of 64 k threads takes k consecutive heads
    const int head = (int)blockIdx.x * ((int)blockDim.x >> 6) + ((int)threadIdx.x >> 6), r = blockIdx.y, i = threadIdx.x & 63, half = hd >> 1;
    if (i >= half || head >= H + 2 * KH) return;
    // interleaved (rope-ordered packed weights): q / k columns hold the pair (i, i + half) at 16(i/8) + 2(i%8), +1
    const bool il = interleaved && head < H + KH;
    const size_t base = (size_t)r * N + (size_t)head * hd;
    const size_t ca = base + (il ? 16 * (i >> 3) + 2 * (i & 7) : i), cb = il ? ca + 1 : ca + half;
    const double2 cssn = tab[r * half + i];
    const float sc = inv ? inv[r] : 1.f;               // requested with the partials, not after them
    float a = 0.f, b = 0.f;
    for (int s0 = 0; s0 < nsplit; s0 += 8) {          // eight partials in flight, added in order
        float pa[8], pb[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool ok = s0 + u < nsplit;
            pa[u] = ok ? part[(size_t)(s0 + u) * sstride + ca] : 0.f;
            pb[u] = ok ? part[(size_t)(s0 + u) * sstride + cb] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (s0 + u < nsplit) { a += pa[u]; b += pb[u]; }
    }
    if (inv) { a *= sc; b *= sc; }                      // 1/rms of the input row (the projection ran on h * gain)
    if (head < H + KH) {
        const double cs = cssn.x, sn = cssn.y;
        const float ra = (float)((double)a * cs - (double)b * sn);
        const float rb = (float)((double)a * sn + (double)b * cs);
        a = ra; b = rb;
    }
    if (head < H) {
        if (q_split) {   // q as two bf16 terms (hi = bf16(q), lo = bf16(q - hi)): [m][H hd] hi, then [m][H hd] lo
            bf16_t* qh = reinterpret_cast<bf16_t*>(q) + (size_t)r * H * hd + (size_t)head * hd;
            bf16_t* ql = qh + (size_t)gridDim.y * H * hd;
            const bf16_t ah = f2bf(a), bh = f2bf(b);
            qh[i] = ah; qh[i + half] = bh;
            ql[i] = f2bf(a - bf2f(ah)); ql[i + half] = f2bf(b - bf2f(bh));
            return;
        }
        float* qd = q + (size_t)r * H * hd + (size_t)head * hd;
        qd[i] = a;
        qd[i + half] = b;
        return;
    }
    if (!write_kv) return;
    T* dst;
    if (head < H + KH) dst = kc + ((size_t)(head - H) * max_ctx + pos) * hd;
    else dst = vc + ((size_t)(head - H - KH) * max_ctx + pos) * hd;
    dst[i] = El<T>::st(a);
    dst[i + half] = El<T>::st(b);
}

// Token embedding and rotation table of a block in one launch: h[r][:] = E[tok[r]][:], and (first hd/2
// threads of row r's workgroup) tab[r][i] = (cos, sin)((pos0 + r) * theta^(-2i/hd)).   grid (m), block 256
template <typename T>
__global__ void embed_rope_kernel(const int32_t* __restrict__ tok, const T* __restrict__ E, int d, float* __restrict__ h, int pos0,
                                  int hd, float theta, double2* __restrict__ tab, TreeBlk tb) {
    const int r = blockIdx.x, i = threadIdx.x, half = hd >> 1;
    const size_t t = (size_t)tok[r];
    for (int k = i; k < d; k += blockDim.x) h[(size_t)r * d + k] = El<T>::ld(E[t * d + k]);
    if (i < half) {
        const double freq = pow((double)theta, -2.0 * (double)i / (double)hd);
        const int pos = tb.on == 1 ? tb.base + (int)tb.depth[tb.i0 + r] : pos0 + r;     // a tree node is rotated for its depth, not its slot
        double sn, cs;
        sincos((double)pos * freq, &sn, &cs);
        tab[r * half + i] = make_double2(cs, sn);
    }
}

template <typename T>
__global__ void rope_kv_kernel(const float* __restrict__ part, int nsplit, size_t sstride, int N, int pos0, int H, int KH,
                               int hd, const double2* __restrict__ tab, float* __restrict__ q, T* __restrict__ kc,
                               T* __restrict__ vc, int max_ctx, int interleaved, int q_split, const float* __restrict__ inv) {
    rope_kv_body<T>(part, nsplit, sstride, N, pos0 + (int)blockIdx.y, H, KH, hd, tab, q, kc, vc, max_ctx, interleaved, q_split, inv,
                    true);
}

// ------------------------------------------------------------------------------------------
// Decode attention over the KV cache for a block of m <= 16 query rows at positions pos0..pos0+m-1
// (row r sees positions 0..pos0+r), split along the KV length in chunks of 128 positions.
// K and V chunks are staged in LDS with coalesced 16-byte loads; scores, softmax and PV in fp32.
//   partial kernel: grid (nchunks, H), block 256 -> part[h][c][16][HD+2] = (o[HD], max, sum)
//   combine kernel: grid (H, m), block HD        -> out[r][h*HD + :] = sum_c o_c e^{m_c-M} / sum_c l_c e^{m_c-M}

constexpr int ATT_CH = 128;

template <typename T, int HD>
__device__ __forceinline__ void attn_partial_body(const float* __restrict__ q, const T* __restrict__ kc,
                                                  const T* __restrict__ vc, int m, int pos0, int H, int KH, int max_ctx,
                                                  float scale, float* __restrict__ part, int nchunks, int c, int h,
                                                  const TreeBlk* tb = nullptr) {
    constexpr int EPV = 16 / (int)sizeof(T);     // elements per 16-byte piece
    constexpr int RS = HD + EPV;                 // padded LDS row stride (elements)
    constexpr int VPR = HD / EPV;                // 16-byte pieces per row
    constexpr int KVB = ATT_CH * RS * (int)sizeof(T);
    constexpr int REDB = 256 * 16 * 4;
    __shared__ __align__(16) unsigned char kvraw[KVB > REDB ? KVB : REDB];
    __shared__ float qs[16 * HD];
    __shared__ float ss[16 * ATT_CH];
    __shared__ float mrow[16], lrow[16];
    T* kv = reinterpret_cast<T*>(kvraw);

    const int kh = h / (H / KH);
    const int L = pos0 + m;
    const int p0 = c * ATT_CH;
    const int np = min(ATT_CH, L - p0);
    const int tid = threadIdx.x;

    for (int idx = tid; idx < m * HD; idx += 256) {
        const int r = idx / HD, i = idx - r * HD;
        qs[idx] = q[(size_t)r * H * HD + (size_t)h * HD + i];
    }
    const T* kbase = kc + ((size_t)kh * max_ctx + p0) * HD;
    for (int idx = tid; idx < np * VPR; idx += 256) {
        const int p = idx / VPR, v = idx - p * VPR;
        *reinterpret_cast<uint4*>(kv + p * RS + v * EPV) = *reinterpret_cast<const uint4*>(kbase + (size_t)p * HD + v * EPV);
    }
    __syncthreads();

    {   // scores: thread = (position p, row half rh); 8 rows per thread
        const int p = tid & (ATT_CH - 1), rh = tid >> 7;
        const int rbeg = rh * 8;
        if (rbeg < m) {
            float acc[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = 0.f;
            if (p < np) {
                for (int i = 0; i < HD; i += 8) {
                    float kf[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) kf[e] = El<T>::ld(kv[p * RS + i + e]);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        if (rbeg + j < m) {
                            const float* qq = qs + (rbeg + j) * HD + i;
#pragma unroll
                            for (int e = 0; e < 8; ++e) acc[j] += kf[e] * qq[e];
                        }
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = rbeg + j;
                if (r < m) {
                    const bool see = tb ? tree_allowed(*tb, p0 + p, r, pos0) : (p0 + p <= pos0 + r);
                    ss[r * ATT_CH + p] = (p < np && see) ? acc[j] * scale : -INFINITY;
                }
            }
        }
    }
    __syncthreads();

    {   // chunk-local softmax numerators and statistics; wave w takes rows w, w+4, ...
        const int wave = tid >> 6, lane = tid & 63;
        for (int r = wave; r < m; r += 4) {
            const float a = ss[r * ATT_CH + lane], b = ss[r * ATT_CH + lane + 64];
            const float mx = wave_max(fmaxf(a, b));
            const float ea = (mx == -INFINITY) ? 0.f : expf(a - mx);
            const float eb = (mx == -INFINITY) ? 0.f : expf(b - mx);
            const float sum = wave_sum(ea + eb);
            ss[r * ATT_CH + lane] = ea;
            ss[r * ATT_CH + lane + 64] = eb;
            if (lane == 0) { mrow[r] = mx; lrow[r] = sum; }
        }
    }
    __syncthreads();   // all reads of the K tile are done

    const T* vbase = vc + ((size_t)kh * max_ctx + p0) * HD;
    for (int idx = tid; idx < np * VPR; idx += 256) {
        const int p = idx / VPR, v = idx - p * VPR;
        *reinterpret_cast<uint4*>(kv + p * RS + v * EPV) = *reinterpret_cast<const uint4*>(vbase + (size_t)p * HD + v * EPV);
    }
    __syncthreads();

    constexpr int G = 256 / HD;   // position groups
    const int col = tid % HD, g = tid / HD;
    float o[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) o[r] = 0.f;
    for (int p = g; p < np; p += G) {
        const float v = El<T>::ld(kv[p * RS + col]);
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (r < m) o[r] += ss[r * ATT_CH + p] * v;
    }
    __syncthreads();   // all reads of the V tile are done: reuse it for the cross-group reduction
    float* red = reinterpret_cast<float*>(kvraw);
#pragma unroll
    for (int r = 0; r < 16; ++r)
        if (r < m) red[(g * 16 + r) * HD + col] = o[r];
    __syncthreads();
    float* dst = part + ((size_t)h * nchunks + c) * 16 * (HD + 2);
    for (int idx = tid; idx < m * HD; idx += 256) {
        const int r = idx / HD, cc = idx - r * HD;
        float s = 0.f;
#pragma unroll
        for (int gg = 0; gg < G; ++gg) s += red[(gg * 16 + r) * HD + cc];
        dst[r * (HD + 2) + cc] = s;
    }
    if (tid < m) {
        dst[tid * (HD + 2) + HD] = mrow[tid];
        dst[tid * (HD + 2) + HD + 1] = lrow[tid];
    }
}

template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_partial_kernel(const float* __restrict__ q, const T* __restrict__ kc,
                                                           const T* __restrict__ vc, int m, int pos0, int H, int KH,
                                                           int max_ctx, float scale, float* __restrict__ part, int nchunks) {
    attn_partial_body<T, HD>(q, kc, vc, m, pos0, H, KH, max_ctx, scale, part, nchunks, (int)blockIdx.x, (int)blockIdx.y);
}
// the same for a tree block (row r = node tb.i0 + r in slot pos0 + r)
template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_partial_tree_kernel(const float* __restrict__ q, const T* __restrict__ kc,
                                                                const T* __restrict__ vc, int m, int pos0, int H, int KH,
                                                                int max_ctx, float scale, float* __restrict__ part, int nchunks, TreeBlk tb) {
    attn_partial_body<T, HD>(q, kc, vc, m, pos0, H, KH, max_ctx, scale, part, nchunks, (int)blockIdx.x, (int)blockIdx.y, &tb);
}

// Source of a block's fresh q / k / v when the attention kernel forms them itself (no rope_kv_kernel launch): the split-K
// partial sums of the QKV projection (rope-ordered q and k columns: pair (i, i + hd/2) of a head at columns 16(i/8) + 2(i%8), +1),
// the rotation table of the block, the optional 1/rms per row, and where the new K / V rows go.  The arithmetic per element is
// rope_kv_body's: partials added in order from zero, scaled, rotated in fp64, rounded once.
struct QkvIn {
    const float* part;     // [nsplit][m][N]
    int nsplit;
    size_t sstride;        // m * N
    int N;                 // (H + 2 KH) * hd
    const double2* tab;    // [m][hd/2] (cos, sin)
    const float* inv;      // [m] or nullptr
    bf16_t* kc;            // cache planes of this layer, written for positions pos0 .. pos0+m-1
    bf16_t* vc;
};

// bf16-cache variant on MFMA.  One workgroup (4 wavefronts) per (chunk of 128 positions, query head):
//   S^T[pos][row] = K[pos][:] . q[row][:]   A = K rows straight from global (16 B per lane, no LDS),
//                                           B = q as two bf16 terms (hi + lo); wavefront w owns
//                                           positions 32w .. 32w+31 of the chunk;
//   softmax numerators p = exp(s - max) per row over the chunk (shuffles across the 4 lane groups,
//   LDS across the 4 wavefronts), written to LDS as P[row][pos] in two bf16 terms;
//   O^T[hd][row] = V^T[hd][pos] . P^T[pos][row]   A = V gathered from the LDS-staged V chunk,
//                                           wavefront w owns head-dim tiles {w, w+4, ..}.
// Output layout and the combine kernel are shared with the generic kernel above.

// q_lo_off: distance (elements) from the hi array of q to its lo array (rows of the whole block x H x HD).
// MULTI: the workgroup walks cpw consecutive chunks starting at chunk c and keeps a running (max, sum, O) per row
// (each new chunk rescales what is there by exp(old max - new max)); it writes one record, number rec of head h,
// so the records written and merged later shrink by the factor cpw.  Without MULTI: one chunk, record c.
// QKV (one chunk per workgroup only): q, and the K / V rows of the block's own positions, are formed here from the QKV
// projection's partial sums instead of being read (see QkvIn).  The pieces (four consecutive columns of one row: all of q of
// this head, and the new K and V rows that fall into this chunk) are dealt out over the 256 threads and requested before the
// cache loads, so they arrive in the same trip to memory; q and the new K rows pass through LDS into the MFMA fragment layout,
// the new V rows go straight into the staged V chunk.  The first query head of each KV head also writes the new rows to the
// cache.  Every workgroup forms the new rows it needs itself: nothing in this launch reads what another workgroup writes.
template <int HD, bool MULTI = false, bool QKV = false>
__device__ __forceinline__ void attn_partial_mfma_body(const float* __restrict__ q, const bf16_t* __restrict__ kc,
                                                       const bf16_t* __restrict__ vc, int m, int pos0, int H, int KH,
                                                       int max_ctx, float scale, float* __restrict__ part, int nchunks, int c,
                                                       int h, size_t q_lo_off, int cpw = 1, int rec = 0, const TreeBlk* tb = nullptr,
                                                       const QkvIn* qi = nullptr) {
    static_assert(!(MULTI && QKV), "fresh q/k/v are formed for a single chunk per workgroup");
    constexpr int RS = HD + 8;                 // padded LDS row stride of the V chunk (elements)
    constexpr int VPR = HD / 8;                // 16-byte pieces per row
    constexpr int PS = ATT_CH + 8;             // padded row stride of P (elements)
    constexpr int KC = HD / 32;                // 32-wide head-dim chunks
    constexpr int NT = HD / 16;                // 16-wide head-dim tiles
    __shared__ __align__(16) bf16_t vs[ATT_CH * RS];
    __shared__ __align__(16) bf16_t phi[16 * PS];
    __shared__ __align__(16) bf16_t plo[16 * PS];
    __shared__ float wmax[4][16], wsum[4][16];

    const int kh = h / (H / KH);
    const int L = pos0 + m;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = lane & 15, g = lane >> 4;
    const bool rowok = row < m;
    constexpr int VIT = ATT_CH * VPR / 256;    // 16-byte pieces of a V chunk per thread
    constexpr int NTW = (NT + 3) / 4;          // head-dim tiles per wavefront

    // ---- q fragments (B operand): q[row][32 kc + 8 g .. +8], already split into two bf16 terms by rope_kv_kernel
    uint4 qh[KC], ql[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        qh[k] = make_uint4(0, 0, 0, 0);
        ql[k] = make_uint4(0, 0, 0, 0);
        if (!QKV && rowok) {
            const bf16_t* src = reinterpret_cast<const bf16_t*>(q) + (size_t)row * H * HD + (size_t)h * HD + k * 32 + g * 8;
            qh[k] = *reinterpret_cast<const uint4*>(src);
            ql[k] = *reinterpret_cast<const uint4*>(src + q_lo_off);
        }
    }
    const bf16_t* kbase = kc + (size_t)kh * max_ctx * HD;
    constexpr int QS = HD + 8;                 // padded row stride (elements) of q and of the new K rows in LDS
    constexpr int C4 = HD / 4;                 // four-column pieces per row
    constexpr int half = HD / 2;
    // running state of this lane's query row (MULTI): maximum, sum, and this wavefront's O^T tiles
    float run_max = -INFINITY, run_sum = 0.f;
    f32x4 orun[NTW];
#pragma unroll
    for (int i = 0; i < NTW; ++i) orun[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nloop = MULTI ? cpw : 1;
    for (int ci = 0; ci < nloop; ++ci) {
        const int p0 = (c + ci) * ATT_CH;
        if (MULTI && p0 >= L) break;               // workgroup-uniform
        const int np = min(ATT_CH, L - p0);
        if (!MULTI && tb && stream_skips(*tb, p0, ATT_CH, pos0)) {
            // a streaming cache holds nothing any row attends to in this chunk: an empty record (weight zero in the merge)
            float* dst = part + ((size_t)h * nchunks + c) * 16 * (HD + 2);
            for (int i = tid; i < m * (HD + 2); i += 256) dst[i] = (i % (HD + 2)) == HD ? -INFINITY : 0.f;
            return;
        }
        // the block's own rows that fall into this chunk: rows r_lo .. r_lo + nnew - 1
        const int r_lo = max(0, p0 - pos0), nnew = QKV ? max(0, min(m, p0 + ATT_CH - pos0) - r_lo) : 0;
        // ---- fresh q / k / v: the pieces of this thread (piece number tid + 256 j), two per trip.  Requests are unconditional
        // (clamped to valid addresses, unused values dropped later) so that the code up to the first use is one straight line
        // and the wait for the pieces does not have to wait for the cache rows requested after them.
        constexpr int GRP = 2;
        const int n_q = m * C4, n_kv = nnew * C4, n_items = QKV ? n_q + 2 * n_kv : 0;
        float4 raw[GRP][4];
        double2 rot[GRP][2];
        float rsc[GRP];
        auto item_at = [&](int idx, int& kind, int& r, int& cc) {      // idx < n_items; kinds: 0 q, 1 K, 2 V
            const int k1 = idx - n_q, k2 = k1 - n_kv;
            kind = idx < n_q ? 0 : (k2 < 0 ? 1 : 2);
            const int loc = kind == 0 ? idx : (kind == 1 ? k1 : k2);
            const int rr = loc / C4;
            cc = loc - rr * C4;
            r = kind == 0 ? rr : r_lo + rr;
        };
        auto item_src = [&](int kind, int r, int cc) {
            const size_t col = kind == 0 ? (size_t)h * HD : kind == 1 ? (size_t)(H + kh) * HD : (size_t)(H + KH + kh) * HD;
            return qi->part + (size_t)r * qi->N + col + 4 * cc;
        };
        auto item_request = [&](int j0) {
            const int ns1 = qi->nsplit - 1;
#pragma unroll
            for (int j = 0; j < GRP; ++j) {
                const int idx = min(tid + 256 * (j0 + j), n_items - 1);
                int kind, r, cc;
                item_at(idx, kind, r, cc);
                const float* src = item_src(kind, r, cc);
#pragma unroll
                for (int s = 0; s < 4; ++s) raw[j][s] = *reinterpret_cast<const float4*>(src + (size_t)min(s, ns1) * qi->sstride);
                const double2* t = qi->tab + (size_t)r * half + 8 * (cc >> 2) + 2 * (cc & 3);   // pairs i, i + 1 of columns 4 cc ..
                rot[j][0] = t[0]; rot[j][1] = t[1];
                rsc[j] = *(qi->inv ? qi->inv + r : reinterpret_cast<const float*>(qi->tab));
            }
        };
        if constexpr (QKV) {
            item_request(0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- issue the V chunk loads (consumed last); rows beyond the ragged end re-read the last row and are zeroed when staged
        const bf16_t* vbase = vc + ((size_t)kh * max_ctx + p0) * HD;
        uint4 vreg[VIT];
#pragma unroll
        for (int it = 0; it < VIT; ++it) {
            const int idx = tid + it * 256;
            const int p = idx / VPR, v = idx - p * VPR;
            vreg[it] = *reinterpret_cast<const uint4*>(vbase + (size_t)min(p, np - 1) * HD + v * 8);
        }
        // ---- K rows of this wavefront's 32 positions: two 16-position tiles (A operand straight from the cache)
        u32x4 kf[2][KC];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int pl = wave * 32 + t * 16 + row;                       // this lane's K row within the chunk
            const int pg = min(p0 + pl, L - 1);                            // clamp: stays inside the cache
            const u32x4* kp = reinterpret_cast<const u32x4*>(kbase + (size_t)pg * HD + g * 8);
#pragma unroll
            for (int k = 0; k < KC; ++k) kf[t][k] = kp[k * 4];             // +32 elements = 4 x 16 bytes
        }
        if constexpr (QKV) {
            __builtin_amdgcn_sched_barrier(0);
            __shared__ __align__(16) bf16_t kn[16 * QS];                   // the new K rows of this chunk, rotated
            bf16_t* qs_hi = phi;                                            // q as two bf16 terms: phi / plo are free until the scores exist
            bf16_t* qs_lo = plo;
            const bool kv_writer = h % (H / KH) == 0;
            auto item_finish = [&](int j0) {
#pragma unroll
                for (int j = 0; j < GRP; ++j) {
                    const int idx = tid + 256 * (j0 + j);
                    float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        const float w = s < qi->nsplit ? 1.f : 0.f;      // a repeated request counts as + 0 (the sums stay the ordered ones)
                        f.x += w * raw[j][s].x; f.y += w * raw[j][s].y; f.z += w * raw[j][s].z; f.w += w * raw[j][s].w;
                    }
                    if (idx < n_items) {
                        int kind, r, cc;
                        item_at(idx, kind, r, cc);
                        if (qi->nsplit > 4) {                               // more than four partials: the rest one by one
                            const float* src = item_src(kind, r, cc);
                            for (int s = 4; s < qi->nsplit; ++s) {
                                const float4 x = *reinterpret_cast<const float4*>(src + (size_t)s * qi->sstride);
                                f.x += x.x; f.y += x.y; f.z += x.z; f.w += x.w;
                            }
                        }
                        if (qi->inv) { const float sc = rsc[j]; f.x *= sc; f.y *= sc; f.z *= sc; f.w *= sc; }
                        if (kind == 2) {
                            const uint2 pk = make_uint2(pack_bf16x2(f2bf(f.x), f2bf(f.y)), pack_bf16x2(f2bf(f.z), f2bf(f.w)));
                            *reinterpret_cast<uint2*>(vs + (pos0 + r - p0) * RS + 4 * cc) = pk;
                            if (kv_writer) *reinterpret_cast<uint2*>(qi->vc + ((size_t)kh * max_ctx + pos0 + r) * HD + 4 * cc) = pk;
                        } else {
                            // columns 4 cc .. + 3 hold (a_i, b_i, a_{i+1}, b_{i+1}): elements i, i + 1 and their partners hd/2 further on
                            const int i = 8 * (cc >> 2) + 2 * (cc & 3);
                            const float a0 = (float)((double)f.x * rot[j][0].x - (double)f.y * rot[j][0].y);
                            const float b0 = (float)((double)f.x * rot[j][0].y + (double)f.y * rot[j][0].x);
                            const float a1 = (float)((double)f.z * rot[j][1].x - (double)f.w * rot[j][1].y);
                            const float b1 = (float)((double)f.z * rot[j][1].y + (double)f.w * rot[j][1].x);
                            const bf16_t a0h = f2bf(a0), a1h = f2bf(a1), b0h = f2bf(b0), b1h = f2bf(b1);
                            if (kind == 0) {
                                *reinterpret_cast<uint32_t*>(qs_hi + r * QS + i) = pack_bf16x2(a0h, a1h);
                                *reinterpret_cast<uint32_t*>(qs_hi + r * QS + i + half) = pack_bf16x2(b0h, b1h);
                                *reinterpret_cast<uint32_t*>(qs_lo + r * QS + i) = pack_bf16x2(f2bf(a0 - bf2f(a0h)), f2bf(a1 - bf2f(a1h)));
                                *reinterpret_cast<uint32_t*>(qs_lo + r * QS + i + half) = pack_bf16x2(f2bf(b0 - bf2f(b0h)), f2bf(b1 - bf2f(b1h)));
                            } else {
                                *reinterpret_cast<uint32_t*>(kn + (r - r_lo) * QS + i) = pack_bf16x2(a0h, a1h);
                                *reinterpret_cast<uint32_t*>(kn + (r - r_lo) * QS + i + half) = pack_bf16x2(b0h, b1h);
                            }
                        }
                    }
                }
            };
            item_finish(0);
            for (int j0 = GRP; j0 * 256 < n_items; j0 += GRP) {           // more than two pieces per thread: further trips
                item_request(j0);
                item_finish(j0);
            }
            __syncthreads();
            if (rowok) {
#pragma unroll
                for (int k = 0; k < KC; ++k) {
                    qh[k] = *reinterpret_cast<const uint4*>(qs_hi + row * QS + k * 32 + g * 8);
                    ql[k] = *reinterpret_cast<const uint4*>(qs_lo + row * QS + k * 32 + g * 8);
                }
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int pg = min(p0 + wave * 32 + t * 16 + row, L - 1);
                if (pg >= pos0) {                                          // what was read from the cache there is not written yet
#pragma unroll
                    for (int k = 0; k < KC; ++k)
                        kf[t][k] = __builtin_bit_cast(u32x4, *reinterpret_cast<const uint4*>(kn + (pg - pos0 - r_lo) * QS + k * 32 + g * 8));
                }
            }
            if (kv_writer && tid < nnew * VPR) {                           // the new K rows to the cache, 16 bytes per thread
                const int rr = tid / VPR, v = tid - rr * VPR;
                *reinterpret_cast<uint4*>(qi->kc + ((size_t)kh * max_ctx + pos0 + r_lo + rr) * HD + v * 8) =
                    *reinterpret_cast<const uint4*>(kn + rr * QS + v * 8);
            }
        }
        // ---- scores
        f32x4 sacc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acl = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[t][k]), __builtin_bit_cast(bf16x8, qh[k]), acc, 0, 0, 0);
                acl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[t][k]), __builtin_bit_cast(bf16x8, ql[k]), acl, 0, 0, 0);
            }
            sacc[t] = acc + acl;
        }
        // lane (g, row) holds positions wave*32 + t*16 + 4g + v of query row `row`
        float sv[8];
        float lmax = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int pl = wave * 32 + t * 16 + g * 4 + v;
                const bool see = tb ? tree_allowed(*tb, p0 + pl, rowok ? row : 0, pos0) : (p0 + pl) <= pos0 + row;
                const bool ok = rowok && pl < np && see;
                const float x = ok ? sacc[t][v] * scale : -INFINITY;
                sv[t * 4 + v] = x;
                lmax = fmaxf(lmax, x);
            }
        lmax = fmaxf(lmax, __shfl_xor(lmax, 16, 64));
        lmax = fmaxf(lmax, __shfl_xor(lmax, 32, 64));
        if (g == 0) wmax[wave][row] = lmax;
        // ---- stage V into LDS while the maxima settle
#pragma unroll
        for (int it = 0; it < VIT; ++it) {
            const int idx = tid + it * 256;
            const int p = idx / VPR, v = idx - p * VPR;
            if (!(QKV && p < np && p0 + p >= pos0))                       // the block's own rows are in place already
                *reinterpret_cast<uint4*>(vs + p * RS + v * 8) = p < np ? vreg[it] : make_uint4(0, 0, 0, 0);
        }
        __syncthreads();
        const float cmx = fmaxf(fmaxf(wmax[0][row], wmax[1][row]), fmaxf(wmax[2][row], wmax[3][row]));
        const float mx = MULTI ? fmaxf(run_max, cmx) : cmx;
        float lsum = 0.f;
        bf16_t ph[8], pl8[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float e = (mx == -INFINITY) ? 0.f : expf(sv[i] - mx);   // expf(-inf) = 0 for masked positions
            lsum += e;
            ph[i] = f2bf(e);
            pl8[i] = f2bf(e - bf2f(ph[i]));
        }
        lsum += __shfl_xor(lsum, 16, 64);
        lsum += __shfl_xor(lsum, 32, 64);
        if (g == 0) wsum[wave][row] = lsum;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int pl = wave * 32 + t * 16 + g * 4;
            *reinterpret_cast<uint2*>(phi + row * PS + pl) = make_uint2(pack_bf16x2(ph[t * 4], ph[t * 4 + 1]), pack_bf16x2(ph[t * 4 + 2], ph[t * 4 + 3]));
            *reinterpret_cast<uint2*>(plo + row * PS + pl) = make_uint2(pack_bf16x2(pl8[t * 4], pl8[t * 4 + 1]), pack_bf16x2(pl8[t * 4 + 2], pl8[t * 4 + 3]));
        }
        __syncthreads();
        // what the earlier chunks left is rescaled to the new maximum
        const float alpha = (MULTI && run_max != -INFINITY) ? expf(run_max - mx) : 0.f;
        // ---- O^T tiles: wavefront w takes head-dim tiles w, w+4, ..
        float* dst = part + ((size_t)h * nchunks + (MULTI ? rec : c)) * 16 * (HD + 2);
#pragma unroll
        for (int ti = 0; ti < NTW; ++ti) {
            const int nt = wave + 4 * ti;
            if (nt < NT) {                                                  // wavefront-uniform
                f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acl = {0.f, 0.f, 0.f, 0.f};
                const int col = nt * 16 + row;                              // A operand row index i = lane % 16 -> head-dim column
#pragma unroll
                for (int k = 0; k < ATT_CH / 32; ++k) {
                    const bf16_t* vp = vs + (k * 32 + g * 8) * RS + col;
                    const uint4 a = make_uint4(pack_bf16x2(vp[0], vp[RS]), pack_bf16x2(vp[2 * RS], vp[3 * RS]),
                                               pack_bf16x2(vp[4 * RS], vp[5 * RS]), pack_bf16x2(vp[6 * RS], vp[7 * RS]));
                    const uint4 bh = *reinterpret_cast<const uint4*>(phi + row * PS + k * 32 + g * 8);
                    const uint4 bl = *reinterpret_cast<const uint4*>(plo + row * PS + k * 32 + g * 8);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, bh), acc, 0, 0, 0);
                    acl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, bl), acl, 0, 0, 0);
                }
                if constexpr (MULTI) {
                    orun[ti] = orun[ti] * alpha + (acc + acl);
                } else if (rowok) {
                    float* o = dst + row * (HD + 2) + nt * 16 + g * 4;       // D[i = 4g + v][j = row]
                    o[0] = acc[0] + acl[0]; o[1] = acc[1] + acl[1]; o[2] = acc[2] + acl[2]; o[3] = acc[3] + acl[3];
                }
            }
        }
        if constexpr (MULTI) {
            run_sum = run_sum * alpha + ((wsum[0][row] + wsum[1][row]) + (wsum[2][row] + wsum[3][row]));
            run_max = mx;
            const bool last = ci + 1 == nloop || p0 + ATT_CH >= L;
            if (!last) {
                __syncthreads();                   // the next chunk overwrites vs, phi, plo, wmax and wsum
            } else {
#pragma unroll
                for (int ti = 0; ti < NTW; ++ti) {
                    const int nt = wave + 4 * ti;
                    if (nt < NT && rowok) {
                        float* o = dst + row * (HD + 2) + nt * 16 + g * 4;
                        o[0] = orun[ti][0]; o[1] = orun[ti][1]; o[2] = orun[ti][2]; o[3] = orun[ti][3];
                    }
                }
                if (tid < m) {                     // wavefront 0, g = 0: this lane's row is tid
                    dst[tid * (HD + 2) + HD] = run_max;
                    dst[tid * (HD + 2) + HD + 1] = run_sum;
                }
            }
        } else if (tid < m) {
            dst[tid * (HD + 2) + HD] = fmaxf(fmaxf(wmax[0][tid], wmax[1][tid]), fmaxf(wmax[2][tid], wmax[3][tid]));
            dst[tid * (HD + 2) + HD + 1] = (wsum[0][tid] + wsum[1][tid]) + (wsum[2][tid] + wsum[3][tid]);
        }
    }
}

template <int HD>
__global__ __launch_bounds__(256) void attn_partial_mfma_kernel(const float* __restrict__ q, const bf16_t* __restrict__ kc,
                                                                const bf16_t* __restrict__ vc, int m, int pos0, int H, int KH,
                                                                int max_ctx, float scale, float* __restrict__ part, int nchunks) {
    attn_partial_mfma_body<HD>(q, kc, vc, m, pos0, H, KH, max_ctx, scale, part, nchunks, (int)blockIdx.x, (int)blockIdx.y,
                               (size_t)m * H * HD);
}
// The same with q and the block's own K / V rows formed from the QKV projection's partial sums (tb.on selects the tree mask).
template <int HD>
__global__ __launch_bounds__(256, 3) void attn_partial_mfma_qkv_kernel(QkvIn qi, const bf16_t* __restrict__ kc, const bf16_t* __restrict__ vc,
                                                                    int m, int pos0, int H, int KH, int max_ctx, float scale,
                                                                    float* __restrict__ part, int nchunks, TreeBlk tb) {
    attn_partial_mfma_body<HD, false, true>(nullptr, kc, vc, m, pos0, H, KH, max_ctx, scale, part, nchunks, (int)blockIdx.x,
                                            (int)blockIdx.y, 0, 1, 0, tb.on ? &tb : nullptr, &qi);
}
template <int HD>
__global__ __launch_bounds__(256) void attn_partial_mfma_tree_kernel(const float* __restrict__ q, const bf16_t* __restrict__ kc,
                                                                     const bf16_t* __restrict__ vc, int m, int pos0, int H, int KH,
                                                                     int max_ctx, float scale, float* __restrict__ part, int nchunks,
                                                                     TreeBlk tb) {
    attn_partial_mfma_body<HD>(q, kc, vc, m, pos0, H, KH, max_ctx, scale, part, nchunks, (int)blockIdx.x, (int)blockIdx.y,
                               (size_t)m * H * HD, 1, 0, &tb);
}

// Merge of the chunk records of (head h, block row r): nchunks records are merged, records of one head are
// nch_stride chunks apart; the result goes to row r_out of out (split: as two bf16 arrays lo_off elements apart).
template <int HD>
__device__ __forceinline__ void attn_combine_body(const float* __restrict__ part, int nchunks, int nch_stride, int H,
                                                  float* __restrict__ out, int split, int h, int r, int r_out, size_t lo_off) {
    const int col = threadIdx.x;
    const float* base = part + ((size_t)h * nch_stride * 16 + r) * (HD + 2);
    const size_t cs = (size_t)16 * (HD + 2);
    // up to 24 records (3072 positions): everything is requested at once - one trip to memory instead of one per group of
    // eight and pass (slots past the end re-read the last record and get weight zero; 8 slots when that is enough)
    auto merge_all = [&](auto slots) {
        constexpr int NS = decltype(slots)::value;
        float mc[NS], lc[NS], oc[NS];
#pragma unroll
        for (int u = 0; u < NS; ++u) {
            const float* rec = base + (size_t)min(u, nchunks - 1) * cs;
            mc[u] = rec[HD]; lc[u] = rec[HD + 1]; oc[u] = rec[col];
        }
        float M = -INFINITY;
#pragma unroll
        for (int u = 0; u < NS; ++u) M = fmaxf(M, u < nchunks ? mc[u] : -INFINITY);
        float Lsum = 0.f, o = 0.f;
#pragma unroll
        for (int u = 0; u < NS; ++u) {                   // same order and arithmetic as the general loop below
            const float w = (u >= nchunks || mc[u] == -INFINITY) ? 0.f : expf(mc[u] - M);
            Lsum += lc[u] * w;
            o += oc[u] * w;
        }
        if (split) store_split1(out, lo_off, (size_t)r_out * H * HD + (size_t)h * HD + col, o / Lsum);
        else out[(size_t)r_out * H * HD + (size_t)h * HD + col] = o / Lsum;
    };
    if (nchunks <= 8) { merge_all(std::integral_constant<int, 8>{}); return; }
    if (nchunks <= 24) { merge_all(std::integral_constant<int, 24>{}); return; }
    float M = -INFINITY;
    for (int c0 = 0; c0 < nchunks; c0 += 8) {           // eight chunk records in flight
        float mc[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) mc[u] = (c0 + u < nchunks) ? base[(c0 + u) * cs + HD] : -INFINITY;
#pragma unroll
        for (int u = 0; u < 8; ++u) M = fmaxf(M, mc[u]);
    }
    float Lsum = 0.f, o = 0.f;
    for (int c0 = 0; c0 < nchunks; c0 += 8) {
        float mc[8], lc[8], oc[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool ok = c0 + u < nchunks;
            mc[u] = ok ? base[(c0 + u) * cs + HD] : -INFINITY;
            lc[u] = ok ? base[(c0 + u) * cs + HD + 1] : 0.f;
            oc[u] = ok ? base[(c0 + u) * cs + col] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float w = (mc[u] == -INFINITY) ? 0.f : expf(mc[u] - M);
            Lsum += lc[u] * w;
            o += oc[u] * w;
        }
    }
    if (split) store_split1(out, lo_off, (size_t)r_out * H * HD + (size_t)h * HD + col, o / Lsum);
    else out[(size_t)r_out * H * HD + (size_t)h * HD + col] = o / Lsum;
}

template <typename T, int HD>
__global__ void attn_combine_kernel(const float* __restrict__ part, int nchunks, int H, float* __restrict__ out, int split) {
    attn_combine_body<HD>(part, nchunks, nchunks, H, out, split, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.y,
                          (size_t)gridDim.y * H * HD);
}

// ------------------------------------------------------------------------------------------
// FFN activation on split-K partials:  SwiGLU  out = silu(gate) * up  (part columns: gate | up),
//                                      GELU    out = 0.5 u (1 + erf(u / sqrt 2)).

// Four consecutive columns per thread (f % 4 == 0), the same arithmetic per element as ffn_act_kernel.   grid ceil(m f / 1024), block 256
__global__ void ffn_act4_kernel(const float* __restrict__ part, int nsplit, size_t sstride, int m, int f, int act,
                                float* __restrict__ out, int split, const float* __restrict__ inv) {
    const size_t idx = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (idx >= (size_t)m * f) return;
    const int r = (int)(idx / f), i = (int)(idx - (size_t)r * f);
    const size_t cg = (size_t)r * (act == 1 ? 2 : 1) * f + i, cu = cg + f;
    float4 g = make_float4(0.f, 0.f, 0.f, 0.f), u = g;
    const float sc = inv ? inv[r] : 1.f;               // requested with the partials, not after them
    for (int s0 = 0; s0 < nsplit; s0 += 4) {            // four partials in flight, added in order
        float4 pg[4], pu[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool ok = s0 + k < nsplit;
            pg[k] = ok ? *reinterpret_cast<const float4*>(part + (size_t)(s0 + k) * sstride + cg) : make_float4(0.f, 0.f, 0.f, 0.f);
            pu[k] = (ok && act == 1) ? *reinterpret_cast<const float4*>(part + (size_t)(s0 + k) * sstride + cu) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (s0 + k < nsplit) {
                g.x += pg[k].x; g.y += pg[k].y; g.z += pg[k].z; g.w += pg[k].w;
                u.x += pu[k].x; u.y += pu[k].y; u.z += pu[k].z; u.w += pu[k].w;
            }
    }
    if (inv) { g.x *= sc; g.y *= sc; g.z *= sc; g.w *= sc; u.x *= sc; u.y *= sc; u.z *= sc; u.w *= sc; }
    auto f1 = [&](float gg, float uu) { return act == 1 ? gg / (1.0f + expf(-gg)) * uu : 0.5f * gg * (1.0f + erff(gg * 0.70710678118654752f)); };
    const float4 y = make_float4(f1(g.x, u.x), f1(g.y, u.y), f1(g.z, u.z), f1(g.w, u.w));
    if (split) store_split4(out, (size_t)m * f, idx, y);
    else *reinterpret_cast<float4*>(out + idx) = y;
}

__global__ void ffn_act_kernel(const float* __restrict__ part, int nsplit, size_t sstride, int m, int f, int act,
                               float* __restrict__ out, int split, const float* __restrict__ inv) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)m * f) return;
    const int r = (int)(idx / f), i = (int)(idx - (size_t)r * f);
    const size_t cg = (size_t)r * (act == 1 ? 2 : 1) * f + i, cu = cg + f;
    float g = 0.f, u = 0.f;
    for (int s0 = 0; s0 < nsplit; s0 += 4) {            // four partials in flight, added in order
        float pg[4], pu[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool ok = s0 + k < nsplit;
            pg[k] = ok ? part[(size_t)(s0 + k) * sstride + cg] : 0.f;
            pu[k] = (ok && act == 1) ? part[(size_t)(s0 + k) * sstride + cu] : 0.f;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (s0 + k < nsplit) { g += pg[k]; u += pu[k]; }
    }
    if (inv) { const float sc = inv[r]; g *= sc; u *= sc; }
    const float y = act == 1 ? g / (1.0f + expf(-g)) * u : 0.5f * g * (1.0f + erff(g * 0.70710678118654752f));
    if (split) store_split1(out, (size_t)m * f, idx, y);
    else out[idx] = y;
}

// ------------------------------------------------------------------------------------------
// Vocab-wide softmax + accept test + residual / bonus inverse-CDF draw, one workgroup of 512
// threads per (sequence row, block position).  The logits of the position (target row and, for
// j < gamma, drafter row) are read from HBM exactly once into registers: wavefront w owns the
// contiguous vocabulary segment [4096 w, 4096 w + 4096), lane l the float4 at 256 c + 4 l of
// chunk c = 0..15 (128 data registers per lane; 512 threads leave the compiler 256 registers, with
// 1024 threads and 128 registers the same code spills).
//
// Arithmetic: exp(x - max) per element in fp32 (hardware exp2); p = e_p / Z_p and q = e_q / Z_q per
// element in fp32 with 1/Z carried as two floats (so the element error is one random rounding, not a
// common factor); sums - Z_p, Z_q, the residual mass, sum min(p, q), the CDF - in fp32 inside a
// thread (64 values) and in fp64 across threads.  The accept ratio p(d)/q(d) is formed in fp64.
// The search for the drawn token is hierarchical (wavefront totals, then chunk totals inside the
// one wavefront that holds the target, then a lane scan, then the four elements of that lane).

constexpr int AK_NT = 512, AK_WAVES = 8, AK_CH = 16, AK_SEG = AK_CH * 256;  // V <= 32768

struct AkShared {
    float fmx[2][AK_WAVES];
    double dz[2][AK_WAVES];
    double dw[2][AK_WAVES];
    int ival[AK_WAVES];
    int token;
};

// exp(a) for a <= 0 (or -inf): hardware 2^(a log2 e).  The fp32 product rounds the argument, so the
// relative error grows with |a| (about 4e-7 at a = -10); it is random per element, which leaves
// sums over the vocabulary and the accept ratio far inside their near-tie windows.  Results below
// the normal range flush to zero.
__device__ __forceinline__ float ak_exp(float a) {
    return __builtin_amdgcn_exp2f(a * 1.44269502162933349609375f);   // a = -inf gives 0
}

// exp((x - mx) / T): for T = 1 the fp32 difference is the correctly rounded argument; otherwise
// the argument is scaled in fp64 before it is rounded.
template <bool UNIT_T>
__device__ __forceinline__ float ak_expx(float x, float mx, double invT) {
    if constexpr (UNIT_T) return ak_exp(x - mx);
    else return ak_exp((float)(((double)x - (double)mx) * invT));
}

__device__ __forceinline__ void ak_load(const float* __restrict__ row, int V, int wave, int lane, float (&x)[AK_CH][4]) {
#pragma unroll
    for (int c = 0; c < AK_CH; ++c) {
        const int idx = wave * AK_SEG + c * 256 + lane * 4;
        if (idx < V) {
            const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row + idx));
            x[c][0] = v[0]; x[c][1] = v[1]; x[c][2] = v[2]; x[c][3] = v[3];
        } else {
            x[c][0] = x[c][1] = x[c][2] = x[c][3] = -INFINITY;
        }
    }
}

__device__ __forceinline__ float ak_thread_max(const float (&x)[AK_CH][4]) {
    float lm = -INFINITY;
#pragma unroll
    for (int c = 0; c < AK_CH; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) lm = fmaxf(lm, x[c][e]);
    return lm;
}

// x <- exp((x - mx)/T) in place; returns this thread's sum.  Inside a thread the 64 values are
// added in fp32 (rounding errors are random and average out over the 512 threads: about 1e-8 of
// the total); across threads every sum is fp64.
template <bool UNIT_T>
__device__ __forceinline__ double ak_exp_inplace(float (&x)[AK_CH][4], float mx, double invT) {
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < AK_CH; ++c) {
        float s4 = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float v = ak_expx<UNIT_T>(x[c][e], mx, invT);
            x[c][e] = v;
            s4 += v;
        }
        s += s4;
    }
    return (double)s;
}

__device__ __forceinline__ float ak_chunk_sum(const float (&w)[AK_CH][4], int c) {
    return (w[c][0] + w[c][1]) + (w[c][2] + w[c][3]);
}

// Inverse CDF in ascending vocabulary order over the non-negative weights w (registers):
// smallest v with sum_{i<=v} w_i > u * Z, where wtot[0..16) in LDS are the wavefront totals
// (already visible to every thread) and Z their sum.  If rounding leaves no such v, the last
// index with weight.  The winner is written to sm.token; the caller synchronises before reading.
__device__ __forceinline__ void ak_search(const float (&w)[AK_CH][4], const double* wtot, double Z, float u, int V, AkShared& sm,
                                          int wave, int lane) {
    const double target = (double)u * Z;
    int wstar = -1, wlast = 0;
    double base = 0.0, run = 0.0;
#pragma unroll
    for (int k = 0; k < AK_WAVES; ++k) {
        const double ww = wtot[k];
        if (ww > 0.0) wlast = k;
        if (wstar < 0) {
            if (run + ww > target) { wstar = k; base = run; }
            else run += ww;
        }
    }
    bool take_last = false;
    if (wstar < 0) { wstar = wlast; take_last = true; }
    if (wave != wstar) return;   // wave-uniform
    int cstar = -1, clast = -1;
    double cb = base;
#pragma unroll
    for (int c = 0; c < AK_CH; ++c) {
        const double ct = wave_sum((double)ak_chunk_sum(w, c));
        if (ct > 0.0) clast = c;
        if (cstar < 0 && !take_last) {
            if (cb + ct > target) cstar = c;
            else cb += ct;
        }
    }
    if (cstar < 0) { cstar = clast < 0 ? 0 : clast; take_last = true; }
    float w4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < AK_CH; ++c)
        if (c == cstar) { w4[0] = w[c][0]; w4[1] = w[c][1]; w4[2] = w[c][2]; w4[3] = w[c][3]; }
    const double sc = (double)((w4[0] + w4[1]) + (w4[2] + w4[3]));
    const double incl = wave_scan_incl(sc, lane);
    unsigned long long bal = __ballot(take_last ? (sc > 0.0) : (cb + incl > target));
    if (bal == 0ull) { take_last = true; bal = __ballot(sc > 0.0); }
    int lstar;
    if (bal == 0ull) lstar = 0;
    else lstar = take_last ? (63 - __clzll((long long)bal)) : (__ffsll((long long)bal) - 1);
    if (lane == lstar) {
        double acc = cb + incl - sc;
        int tok = -1, lastpos = -1;
        const int idx0 = wave * AK_SEG + cstar * 256 + lane * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc += (double)w4[e];
            if (w4[e] > 0.f) lastpos = idx0 + e;
            if (tok < 0 && !take_last && acc > target) tok = idx0 + e;
        }
        if (tok < 0) tok = lastpos >= 0 ? lastpos : min(idx0, V - 1);
        sm.token = tok;
    }
}

// argmax with lowest index on ties; returns the index in every thread
__device__ int ak_argmax(const float (&x)[AK_CH][4], AkShared& sm, int wave, int lane) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int c = 0; c < AK_CH; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = wave * AK_SEG + c * 256 + lane * 4 + e;
            if (x[c][e] > bv) { bv = x[c][e]; bi = idx; }   // ascending c, e within a lane
        }
    // lanes of one chunk interleave, so order by (value desc, index asc)
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { sm.fmx[0][wave] = bv; sm.ival[wave] = bi; }
    __syncthreads();
    float rv = sm.fmx[0][0];
    int ri = sm.ival[0];
#pragma unroll
    for (int w = 1; w < AK_WAVES; ++w) {
        const float ov = sm.fmx[0][w];
        const int oi = sm.ival[w];
        if (ov > rv || (ov == rv && oi < ri)) { rv = ov; ri = oi; }
    }
    return ri;
}

// One (row b, position j) of the accept step.  cand[(b*(gamma+1)+j)] = (candidate token, test result).
//   j < gamma : test u_acc < min(1, p(d)/q(d)); candidate = draw from norm(max(0, p - q)) (from p if p == q)
//   j == gamma: candidate = draw from p (bonus token); test result unused (1)
//   T == 0    : test = [d == argmax P_j], candidate = argmax P_j
template <bool UNIT_T>
__device__ __forceinline__ void accept_rows_body(const float* __restrict__ P, const float* __restrict__ Q,
                                                 const int32_t* __restrict__ d, int gamma, int V, float T, uint64_t seed,
                                                 const RoundTab& rt, uint32_t seq0, int2* __restrict__ cand,
                                                 double* __restrict__ bd, AkShared& sm) {
    const int j = blockIdx.x, b = blockIdx.y;
    const uint32_t round = round_of(rt, b);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float* Prow = P + ((size_t)b * (gamma + 1) + j) * V;
    const bool has_q = j < gamma;
    const float* Qrow = has_q ? Q + ((size_t)b * gamma + j) * V : nullptr;
    const int dtok = has_q ? min(max(d[(size_t)b * gamma + j], 0), V - 1) : -1;   // clamped: stays in bounds for any input
    float xp[AK_CH][4], xq[AK_CH][4];
    ak_load(Prow, V, wave, lane, xp);
    if (T <= 0.f) {
        const int am = ak_argmax(xp, sm, wave, lane);
        if (threadIdx.x == 0) {
            cand[(size_t)b * (gamma + 1) + j] = make_int2(am, has_q ? (dtok == am) : 1);
            if (has_q && bd) bd[(size_t)b * gamma + j] = (dtok == am) ? 1.0 : 0.0;
        }
        return;
    }
    const double invT = 1.0 / (double)T;
    if (has_q) ak_load(Qrow, V, wave, lane, xq);
    // the two logits of the draft token (tiny second read, issued with the stream)
    float pdl = 0.f, qdl = 0.f;
    if (has_q) { pdl = Prow[dtok]; qdl = Qrow[dtok]; }
    if (threadIdx.x == 0) sm.token = -1;
    // ---- maxima
    {
        const float a = wave_max(ak_thread_max(xp));
        const float c = has_q ? wave_max(ak_thread_max(xq)) : -INFINITY;
        if (lane == 0) { sm.fmx[0][wave] = a; sm.fmx[1][wave] = c; }
    }
    __syncthreads();
    float mp = sm.fmx[0][0], mq = sm.fmx[1][0];
#pragma unroll
    for (int k = 1; k < AK_WAVES; ++k) { mp = fmaxf(mp, sm.fmx[0][k]); mq = fmaxf(mq, sm.fmx[1][k]); }
    // ---- exp and the two normalisers
    {
        const double a = wave_sum(ak_exp_inplace<UNIT_T>(xp, mp, invT));
        const double c = has_q ? wave_sum(ak_exp_inplace<UNIT_T>(xq, mq, invT)) : 0.0;
        if (lane == 0) { sm.dz[0][wave] = a; sm.dz[1][wave] = c; }
    }
    __syncthreads();
    double Zp = 0.0, Zq = 0.0;
#pragma unroll
    for (int k = 0; k < AK_WAVES; ++k) { Zp += sm.dz[0][k]; Zq += sm.dz[1][k]; }
    const float u_res = philox_uniform(seed, seq0 + (uint32_t)b, round, 0u, 1u);
    int accept = 1;
    if (!has_q) {   // bonus position: draw from p
        ak_search(xp, sm.dz[0], Zp, u_res, V, sm, wave, lane);
        __syncthreads();
        if (threadIdx.x == 0) cand[(size_t)b * (gamma + 1) + j] = make_int2(sm.token, 1);
        return;
    }
    const double ipz = 1.0 / Zp, iqz = 1.0 / Zq;
    const float ip_hi = (float)ipz, ip_lo = (float)(ipz - (double)ip_hi);
    const float iq_hi = (float)iqz, iq_lo = (float)(iqz - (double)iq_hi);
    // ---- accept test on the draft token
    {
        const double pd = (double)ak_expx<UNIT_T>(pdl, mp, invT) * ipz, qd = (double)ak_expx<UNIT_T>(qdl, mq, invT) * iqz;
        if (qd > 0.0) {
            const double ratio = pd / qd;
            const float u_acc = philox_uniform(seed, seq0 + (uint32_t)b, round, (uint32_t)j, 0u);
            accept = (double)u_acc < (ratio < 1.0 ? ratio : 1.0);
        }
    }
    // ---- residual weights max(0, p - q) (kept in xq) and sum min(p, q)
    {
        float fw = 0.f, fm = 0.f;
#pragma unroll
        for (int c = 0; c < AK_CH; ++c) {
            float mn4 = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float pv = fmaf(xp[c][e], ip_lo, xp[c][e] * ip_hi), qv = fmaf(xq[c][e], iq_lo, xq[c][e] * iq_hi);
                mn4 += fminf(pv, qv);
                xq[c][e] = fmaxf(pv - qv, 0.f);
            }
            fw += ak_chunk_sum(xq, c);
            fm += mn4;
        }
        double tw = (double)fw, tm = (double)fm;
        tw = wave_sum(tw);
        tm = wave_sum(tm);
        if (lane == 0) { sm.dw[0][wave] = tw; sm.dw[1][wave] = tm; }
    }
    __syncthreads();
    double Zr = 0.0, bdj = 0.0;
#pragma unroll
    for (int k = 0; k < AK_WAVES; ++k) { Zr += sm.dw[0][k]; bdj += sm.dw[1][k]; }
    if (Zr > 0.0) ak_search(xq, sm.dw[0], Zr, u_res, V, sm, wave, lane);
    else ak_search(xp, sm.dz[0], Zp, u_res, V, sm, wave, lane);   // p == q: a rejection has probability 0; draw from p
    __syncthreads();
    if (threadIdx.x == 0) {
        cand[(size_t)b * (gamma + 1) + j] = make_int2(sm.token, accept);
        if (bd) bd[(size_t)b * gamma + j] = bdj;
    }
}

__global__ __launch_bounds__(AK_NT) void accept_rows_kernel(const float* __restrict__ P, const float* __restrict__ Q,
                                                            const int32_t* __restrict__ d, int gamma, int V, float T,
                                                            uint64_t seed, RoundTab rt, uint32_t seq0,
                                                            int2* __restrict__ cand, double* __restrict__ bd) {
    __shared__ AkShared sm;
    if (T == 1.0f) accept_rows_body<true>(P, Q, d, gamma, V, T, seed, rt, seq0, cand, bd, sm);
    else accept_rows_body<false>(P, Q, d, gamma, V, T, seed, rt, seq0, cand, bd, sm);
}

// ------------------------------------------------------------------------------------------
// The same accept step with every (row, position) split over four workgroups of 256 threads, one
// per quarter of the vocabulary (8192 entries: wavefront w of quarter q owns [8192 q + 2048 w, +2048),
// 64 data registers per lane).  Four such workgroups fit on a CU, so the loads of one overlap the
// arithmetic of another, and 64 rows x 6 positions give 1536 equal pieces for 1024 resident slots
// instead of 384 items for 256.  The quarters of an item meet twice through 64-bit words in global
// memory, each word = (launch epoch << 32 | payload), written and polled with relaxed agent-scope
// atomics: a reader knows a word is this launch's as soon as the epoch matches, so there are no
// flags, no fences and nothing to clear between launches (the buffer starts zeroed and epochs only
// grow).  Sums travel as two floats (hi + lo, 48 bits) so that all four workgroups use identical values.
//   meeting A: each quarter's maxima m_k and sums z_k = sum exp(x - m_k) of P_j and Q_j.  With
//              M = max m_k the normaliser is Z = sum_k z_k exp(m_k - M), and an element's probability
//              is exp(x - m_k) * (exp(m_k - M) / Z): the per-quarter factor is folded into 1/Z, so no
//              element is touched twice.
//   meeting B: each quarter's residual mass and sum min(p, q) -> Z_res, the BD term, and the quarter
//              that holds u Z_res; only that quarter searches (wavefront, chunk, lane, element).
// The candidate of the position is published as one more tagged word, and the workgroup (quarter 0,
// bonus position) of every row waits for the row's gamma + 1 candidates and writes N_acc, the
// emitted token and the mask - no second kernel.
// Liveness: workgroups are dispatched in id order on every XCD, and a workgroup only waits for
// workgroups with ids below its own or in its own group of four, so the oldest unfinished item
// always has everything it waits for resident or done.  The polls are bounded all the same: after
// spin_limit polls the item is marked failed (token -2) and every wave exits.

constexpr int AS_NT = 256, AS_WAVES = 4, AS_CH = 8, AS_WSEG = AS_CH * 256, AS_Q = 4, AS_QSEG = AS_WAVES * AS_WSEG;
constexpr int AS_WORDS = 10;                                   // exchange words per quarter
constexpr int AS_XCHG_BYTES = AS_Q * AS_WORDS * 8;             // per (row, position)
constexpr uint32_t AS_CAND_ACCEPT = 1u << 30, AS_CAND_FAIL = 1u << 29;

struct AsShared {
    float fmx[2][AS_WAVES];
    double dz[2][AS_WAVES];
    double dw[2][AS_WAVES];
    int ival[AS_WAVES];
    float xw[AS_Q][AS_WORDS];
    int token, fail;
};

__device__ __forceinline__ void as_put(unsigned long long* slot, uint32_t epoch, uint32_t payload) { tw_put(slot, epoch, payload); }
__device__ __forceinline__ bool as_get(const unsigned long long* slot, uint32_t epoch, int spin_limit, uint32_t* payload) {
    return tw_get(slot, epoch, spin_limit, payload);
}

// Publish NW floats of this quarter (words first .. first + NW) and collect the same words of all four.
// `mine` must hold the same values in every thread.  Returns false after a timeout (sm.fail is set).
template <int NW>
__device__ __forceinline__ bool as_exchange(unsigned long long* slots, int q, uint32_t epoch, const float (&mine)[NW], int first,
                                            AsShared& sm, int spin_limit) {
    const int t = (int)threadIdx.x;
    if (t < NW) as_put(slots + q * AS_WORDS + first + t, epoch, __float_as_uint(mine[t]));
    if (t < AS_Q * NW) {
        const int qq = t / NW, ww = t - qq * NW;
        uint32_t bits = 0;
        if (as_get(slots + qq * AS_WORDS + first + ww, epoch, spin_limit, &bits)) sm.xw[qq][first + ww] = __uint_as_float(bits);
        else sm.fail = 1;
    }
    __syncthreads();
    return sm.fail == 0;
}

__device__ __forceinline__ void as_load(const float* __restrict__ row, int V, int seg0, int lane, float (&x)[AS_CH][4]) {
#pragma unroll
    for (int c = 0; c < AS_CH; ++c) {
        const int idx = seg0 + c * 256 + lane * 4;
        if (idx < V) {
            const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row + idx));
            x[c][0] = v[0]; x[c][1] = v[1]; x[c][2] = v[2]; x[c][3] = v[3];
        } else {
            x[c][0] = x[c][1] = x[c][2] = x[c][3] = -INFINITY;
        }
    }
}

__device__ __forceinline__ float as_thread_max(const float (&x)[AS_CH][4]) {
    float lm = -INFINITY;
#pragma unroll
    for (int c = 0; c < AS_CH; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) lm = fmaxf(lm, x[c][e]);
    return lm;
}

// x <- exp((x - mx)/T) in place (mx finite); returns this thread's sum (fp32 inside the thread).
template <bool UNIT_T>
__device__ __forceinline__ double as_exp_inplace(float (&x)[AS_CH][4], float mx, double invT) {
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < AS_CH; ++c) {
        float s4 = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float v = ak_expx<UNIT_T>(x[c][e], mx, invT);
            x[c][e] = v;
            s4 += v;
        }
        s += s4;
    }
    return (double)s;
}

// Quarter, wavefront, chunk, lane, element holding the target u * Z of the inverse CDF over scale * w.
// tq[0..4): the quarters' totals in the common scale (identical in all four workgroups); wtot: this quarter's
// wavefront totals of w (LDS); scale: this quarter's factor.  Only the quarter that holds the target continues;
// it leaves the token in sm.token.  Returns (workgroup-uniform) whether this workgroup is that quarter.
// Rounding gaps fall back to the last index with weight, level by level.
__device__ __forceinline__ bool as_search(const float (&w)[AS_CH][4], const double* wtot, double scale, const double (&tq)[AS_Q],
                                          double Z, float u, int V, int q, AsShared& sm, int wave, int lane) {
    const double target = (double)u * Z;
    int qstar = -1, qlast = 0;
    double base = 0.0, run = 0.0;
#pragma unroll
    for (int k = 0; k < AS_Q; ++k) {
        if (tq[k] > 0.0) qlast = k;
        if (qstar < 0) {
            if (run + tq[k] > target) { qstar = k; base = run; }
            else run += tq[k];
        }
    }
    bool take_last = false;
    if (qstar < 0) { qstar = qlast; take_last = true; }
    if (q != qstar) return false;
    int wstar = -1, wlast = 0;
    double wbase = base;
#pragma unroll
    for (int k = 0; k < AS_WAVES; ++k) {
        const double ww = wtot[k] * scale;
        if (ww > 0.0) wlast = k;
        if (wstar < 0 && !take_last) {
            if (wbase + ww > target) wstar = k;
            else wbase += ww;
        }
    }
    if (wstar < 0) { wstar = wlast; take_last = true; }
    if (wave == wstar) {   // wave-uniform
        int cstar = -1, clast = -1;
        double cb = wbase;
#pragma unroll
        for (int c = 0; c < AS_CH; ++c) {
            const double ct = wave_sum((double)((w[c][0] + w[c][1]) + (w[c][2] + w[c][3]))) * scale;
            if (ct > 0.0) clast = c;
            if (cstar < 0 && !take_last) {
                if (cb + ct > target) cstar = c;
                else cb += ct;
            }
        }
        if (cstar < 0) { cstar = clast < 0 ? 0 : clast; take_last = true; }
        float w4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < AS_CH; ++c)
            if (c == cstar) { w4[0] = w[c][0]; w4[1] = w[c][1]; w4[2] = w[c][2]; w4[3] = w[c][3]; }
        const double sc = (double)((w4[0] + w4[1]) + (w4[2] + w4[3])) * scale;
        const double incl = wave_scan_incl(sc, lane);
        unsigned long long bal = __ballot(take_last ? (sc > 0.0) : (cb + incl > target));
        if (bal == 0ull) { take_last = true; bal = __ballot(sc > 0.0); }
        int lstar;
        if (bal == 0ull) lstar = 0;
        else lstar = take_last ? (63 - __clzll((long long)bal)) : (__ffsll((long long)bal) - 1);
        if (lane == lstar) {
            double acc = cb + incl - sc;
            int tok = -1, lastpos = -1;
            const int idx0 = q * AS_QSEG + wave * AS_WSEG + cstar * 256 + lane * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc += (double)w4[e] * scale;
                if (w4[e] > 0.f) lastpos = idx0 + e;
                if (tok < 0 && !take_last && acc > target) tok = idx0 + e;
            }
            if (tok < 0) tok = lastpos >= 0 ? lastpos : min(idx0, V - 1);
            sm.token = tok;
        }
    }
    __syncthreads();
    return true;
}

template <bool UNIT_T>
__device__ __forceinline__ void accept_split_item(const float* __restrict__ P, const float* __restrict__ Q,
                                                  const int32_t* __restrict__ d, int gamma, int V, float T, uint64_t seed,
                                                  const RoundTab& rt, uint32_t seq0, unsigned long long* __restrict__ cand,
                                                  double* __restrict__ bd, unsigned long long* __restrict__ xchg, uint32_t epoch,
                                                  int spin_limit, AsShared& sm) {
    const int q = blockIdx.x, j = blockIdx.y, b = blockIdx.z;
    const uint32_t round = round_of(rt, b);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t item = (size_t)b * (gamma + 1) + j;
    unsigned long long* slots = xchg + item * (AS_Q * AS_WORDS);
    const float* Prow = P + item * V;
    const bool has_q = j < gamma;
    const float* Qrow = has_q ? Q + ((size_t)b * gamma + j) * V : nullptr;
    const int dtok = has_q ? min(max(d[(size_t)b * gamma + j], 0), V - 1) : -1;   // clamped: stays in bounds for any input
    const int seg0 = q * AS_QSEG + wave * AS_WSEG;
    float xp[AS_CH][4], xq[AS_CH][4];
    as_load(Prow, V, seg0, lane, xp);
    auto fail_out = [&]() { if (threadIdx.x == 0) as_put(cand + item, epoch, AS_CAND_FAIL); };
    if (T <= 0.f) {   // greedy: argmax with the lowest index on ties
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int c = 0; c < AS_CH; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int idx = seg0 + c * 256 + lane * 4 + e;
                if (xp[c][e] > bv) { bv = xp[c][e]; bi = idx; }
            }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(bv, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        if (lane == 0) { sm.fmx[0][wave] = bv; sm.ival[wave] = bi; }
        __syncthreads();
        float rv = sm.fmx[0][0];
        int ri = sm.ival[0];
#pragma unroll
        for (int k = 1; k < AS_WAVES; ++k)
            if (sm.fmx[0][k] > rv || (sm.fmx[0][k] == rv && sm.ival[k] < ri)) { rv = sm.fmx[0][k]; ri = sm.ival[k]; }
        const float mine[2] = {rv, __int_as_float(ri)};
        if (!as_exchange<2>(slots, q, epoch, mine, 0, sm, spin_limit)) { fail_out(); return; }
        if (q == 0 && threadIdx.x == 0) {
            float gv = sm.xw[0][0];
            int gi = __float_as_int(sm.xw[0][1]);
            for (int k = 1; k < AS_Q; ++k) {
                const float ov = sm.xw[k][0];
                const int oi = __float_as_int(sm.xw[k][1]);
                if (ov > gv || (ov == gv && oi < gi)) { gv = ov; gi = oi; }
            }
            const bool acc = has_q ? (dtok == gi) : true;
            as_put(cand + item, epoch, (acc ? AS_CAND_ACCEPT : 0u) | (uint32_t)gi);
            if (has_q && bd) bd[(size_t)b * gamma + j] = acc ? 1.0 : 0.0;
        }
        return;
    }
    const double invT = 1.0 / (double)T;
    if (has_q) as_load(Qrow, V, seg0, lane, xq);
    float pdl = 0.f, qdl = 0.f;
    if (has_q) { pdl = Prow[dtok]; qdl = Qrow[dtok]; }
    // ---- local maxima
    {
        const float a = wave_max(as_thread_max(xp));
        const float c = has_q ? wave_max(as_thread_max(xq)) : -INFINITY;
        if (lane == 0) { sm.fmx[0][wave] = a; sm.fmx[1][wave] = c; }
    }
    __syncthreads();
    float lmp = sm.fmx[0][0], lmq = sm.fmx[1][0];
#pragma unroll
    for (int k = 1; k < AS_WAVES; ++k) { lmp = fmaxf(lmp, sm.fmx[0][k]); lmq = fmaxf(lmq, sm.fmx[1][k]); }
    // a quarter beyond the vocabulary (or fully masked) has no maximum: it exponentiates against 0 and contributes nothing
    const float emp = lmp > -INFINITY ? lmp : 0.f, emq = lmq > -INFINITY ? lmq : 0.f;
    // ---- local exp and sums
    {
        const double a = wave_sum(as_exp_inplace<UNIT_T>(xp, emp, invT));
        const double c = has_q ? wave_sum(as_exp_inplace<UNIT_T>(xq, emq, invT)) : 0.0;
        if (lane == 0) { sm.dz[0][wave] = a; sm.dz[1][wave] = c; }
    }
    __syncthreads();
    // ---- meeting A
    double zpq[AS_Q], Zp = 0.0, Zq = 0.0, sp_mine, sq_mine;
    float mp, mq;
    {
        double lp = 0.0, lq = 0.0;
#pragma unroll
        for (int k = 0; k < AS_WAVES; ++k) { lp += sm.dz[0][k]; lq += sm.dz[1][k]; }
        const float ph = (float)lp, qh = (float)lq;
        const float mine[6] = {lmp, lmq, ph, (float)(lp - (double)ph), qh, (float)(lq - (double)qh)};
        if (!as_exchange<6>(slots, q, epoch, mine, 0, sm, spin_limit)) { fail_out(); return; }
        mp = fmaxf(fmaxf(sm.xw[0][0], sm.xw[1][0]), fmaxf(sm.xw[2][0], sm.xw[3][0]));
        mq = fmaxf(fmaxf(sm.xw[0][1], sm.xw[1][1]), fmaxf(sm.xw[2][1], sm.xw[3][1]));
        sp_mine = 0.0; sq_mine = 0.0;
#pragma unroll
        for (int k = 0; k < AS_Q; ++k) {
            // factor of quarter k: exp((m_k - M)/T); 0 for a quarter without a maximum
            const double sp = sm.xw[k][0] > -INFINITY ? (double)ak_expx<UNIT_T>(sm.xw[k][0], mp, invT) : 0.0;
            const double sq = sm.xw[k][1] > -INFINITY ? (double)ak_expx<UNIT_T>(sm.xw[k][1], mq, invT) : 0.0;
            zpq[k] = ((double)sm.xw[k][2] + (double)sm.xw[k][3]) * sp;
            Zp += zpq[k];
            Zq += ((double)sm.xw[k][4] + (double)sm.xw[k][5]) * sq;
            if (k == q) { sp_mine = sp; sq_mine = sq; }
        }
    }
    const float u_res = philox_uniform(seed, seq0 + (uint32_t)b, round, 0u, 1u);
    if (!has_q) {   // bonus position: draw from p
        if (as_search(xp, sm.dz[0], sp_mine, zpq, Zp, u_res, V, q, sm, wave, lane) && threadIdx.x == 0)
            as_put(cand + item, epoch, AS_CAND_ACCEPT | (uint32_t)sm.token);
        return;
    }
    const double ipz = sp_mine / Zp, iqz = sq_mine / Zq;      // this quarter's exp(m_k - M) / Z
    const float ip_hi = (float)ipz, ip_lo = (float)(ipz - (double)ip_hi);
    const float iq_hi = (float)iqz, iq_lo = (float)(iqz - (double)iq_hi);
    bool accept = true;
    {
        const double pd = (double)ak_expx<UNIT_T>(pdl, mp, invT) / Zp, qd = (double)ak_expx<UNIT_T>(qdl, mq, invT) / Zq;
        if (qd > 0.0) {
            const double ratio = pd / qd;
            const float u_acc = philox_uniform(seed, seq0 + (uint32_t)b, round, (uint32_t)j, 0u);
            accept = (double)u_acc < (ratio < 1.0 ? ratio : 1.0);
        }
    }
    // ---- residual weights max(0, p - q) (kept in xq) and sum min(p, q)
    {
        float fw = 0.f, fm = 0.f;
#pragma unroll
        for (int c = 0; c < AS_CH; ++c) {
            float mn4 = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float pv = fmaf(xp[c][e], ip_lo, xp[c][e] * ip_hi), qv = fmaf(xq[c][e], iq_lo, xq[c][e] * iq_hi);
                mn4 += fminf(pv, qv);
                xq[c][e] = fmaxf(pv - qv, 0.f);
            }
            fw += (xq[c][0] + xq[c][1]) + (xq[c][2] + xq[c][3]);
            fm += mn4;
        }
        const double tw = wave_sum((double)fw), tm = wave_sum((double)fm);
        if (lane == 0) { sm.dw[0][wave] = tw; sm.dw[1][wave] = tm; }
    }
    __syncthreads();
    // ---- meeting B
    double zrq[AS_Q], Zr = 0.0, bdj = 0.0;
    {
        double lr = 0.0, lm = 0.0;
#pragma unroll
        for (int k = 0; k < AS_WAVES; ++k) { lr += sm.dw[0][k]; lm += sm.dw[1][k]; }
        const float rh = (float)lr, mh = (float)lm;
        const float mine[4] = {rh, (float)(lr - (double)rh), mh, (float)(lm - (double)mh)};
        if (!as_exchange<4>(slots, q, epoch, mine, 6, sm, spin_limit)) { fail_out(); return; }
#pragma unroll
        for (int k = 0; k < AS_Q; ++k) {
            zrq[k] = (double)sm.xw[k][6] + (double)sm.xw[k][7];
            Zr += zrq[k];
            bdj += (double)sm.xw[k][8] + (double)sm.xw[k][9];
        }
    }
    bool mine_wins;
    if (Zr > 0.0) mine_wins = as_search(xq, sm.dw[0], 1.0, zrq, Zr, u_res, V, q, sm, wave, lane);
    else mine_wins = as_search(xp, sm.dz[0], sp_mine, zpq, Zp, u_res, V, q, sm, wave, lane);   // p == q: draw from p
    if (mine_wins && threadIdx.x == 0) {
        if (bd) bd[(size_t)b * gamma + j] = bdj;
        as_put(cand + item, epoch, (accept ? AS_CAND_ACCEPT : 0u) | (uint32_t)sm.token);
    }
}

// grid (4 quarters, gamma + 1 positions, rows), block 256.  cand: one tagged word per (row, position);
// xchg: AS_XCHG_BYTES per (row, position); both zero-filled before their first use.
__global__ __launch_bounds__(AS_NT) void accept_split_kernel(const float* __restrict__ P, const float* __restrict__ Q,
                                                             const int32_t* __restrict__ d, int gamma, int V, float T,
                                                             uint64_t seed, RoundTab rt, uint32_t seq0,
                                                             unsigned long long* __restrict__ cand, double* __restrict__ bd,
                                                             unsigned long long* __restrict__ xchg, uint32_t epoch, int spin_limit,
                                                             int32_t* __restrict__ n_acc, int32_t* __restrict__ token,
                                                             uint32_t* __restrict__ mask, int32_t* __restrict__ hist, int l) {
    __shared__ AsShared sm;
    if (threadIdx.x == 0) { sm.token = -1; sm.fail = 0; }
    if (T == 1.0f) accept_split_item<true>(P, Q, d, gamma, V, T, seed, rt, seq0, cand, bd, xchg, epoch, spin_limit, sm);
    else accept_split_item<false>(P, Q, d, gamma, V, T, seed, rt, seq0, cand, bd, xchg, epoch, spin_limit, sm);
    // ---- per row: first failed test, emitted token, mask (one thread of the bonus position's first quarter)
    if (blockIdx.x == 0 && (int)blockIdx.y == gamma && threadIdx.x == 0) {
        const int b = blockIdx.z;
        int n = gamma, tok = -2;
        uint32_t mk = 0, cn = 0;
        bool ok = true;
        for (int j = gamma; j >= 0 && ok; --j) {
            uint32_t w = 0;
            ok = as_get(cand + (size_t)b * (gamma + 1) + j, epoch, spin_limit, &w) && !(w & AS_CAND_FAIL);
            if (!ok) break;
            if (j == gamma) { cn = w; continue; }
            if (w & AS_CAND_ACCEPT) mk |= 1u << j;
            else { n = j; cn = w; }
        }
        if (ok) tok = (int)(cn & 0x1fffffffu);
        else { n = 0; mk = 0; }
        n_acc[b] = n;
        token[b] = tok;
        if (mask) mask[b] = mk;
        if (hist && tok >= 0) hist[l + n] = tok;
    }
}

// Per row: N_acc = first failed test, emitted token = candidate of that position, mask bits.
// hist (optional): hist[b*hist_stride + l + n] = token  (commit of the emitted token).
__global__ void accept_finalize_kernel(const int2* __restrict__ cand, int rows, int gamma, int32_t* __restrict__ n_acc,
                                       int32_t* __restrict__ token, uint32_t* __restrict__ mask, int32_t* __restrict__ hist,
                                       int l) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= rows) return;
    int n = gamma;
    uint32_t mk = 0;
    for (int j = gamma - 1; j >= 0; --j) {
        const int a = cand[(size_t)b * (gamma + 1) + j].y;
        if (a) mk |= 1u << j;
        else n = j;
    }
    const int tok = cand[(size_t)b * (gamma + 1) + n].x;
    n_acc[b] = n;
    token[b] = tok;
    if (mask) mask[b] = mk;
    if (hist && tok >= 0) hist[l + n] = tok;
}

// Token draw from one row of logits: argmax (T = 0) or inverse CDF of softmax(logits / T) with the
// stream-2 uniform at (seq0 + row, round, pos).  grid (rows), block 512.  tok[row * tok_stride]
// (and tok_copy[row] when given).
template <bool UNIT_T>
__device__ __forceinline__ int sample_rows_body(float (&xp)[AK_CH][4], int V, float T, float u, AkShared& sm, int wave, int lane) {
    if (threadIdx.x == 0) sm.token = -1;
    const float a = wave_max(ak_thread_max(xp));
    if (lane == 0) sm.fmx[0][wave] = a;
    __syncthreads();
    float mp = sm.fmx[0][0];
#pragma unroll
    for (int k = 1; k < AK_WAVES; ++k) mp = fmaxf(mp, sm.fmx[0][k]);
    const double s = wave_sum(ak_exp_inplace<UNIT_T>(xp, mp, 1.0 / (double)T));
    if (lane == 0) sm.dz[0][wave] = s;
    __syncthreads();
    double Zp = 0.0;
#pragma unroll
    for (int k = 0; k < AK_WAVES; ++k) Zp += sm.dz[0][k];
    ak_search(xp, sm.dz[0], Zp, u, V, sm, wave, lane);
    __syncthreads();
    return sm.token;
}

__global__ __launch_bounds__(AK_NT) void sample_rows_kernel(const float* __restrict__ logits, int V, float T, uint64_t seed,
                                                            uint32_t round, uint32_t pos, uint32_t seq0,
                                                            int32_t* __restrict__ tok, int tok_stride,
                                                            int32_t* __restrict__ tok_copy) {
    __shared__ AkShared sm;
    const int b = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float xp[AK_CH][4];
    ak_load(logits + (size_t)b * V, V, wave, lane, xp);
    int token;
    if (T <= 0.f) {
        token = ak_argmax(xp, sm, wave, lane);
    } else {
        const float u = philox_uniform(seed, seq0 + (uint32_t)b, round, pos, 2u);
        token = T == 1.0f ? sample_rows_body<true>(xp, V, T, u, sm, wave, lane) : sample_rows_body<false>(xp, V, T, u, sm, wave, lane);
    }
    if (threadIdx.x == 0) {
        tok[(size_t)b * tok_stride] = token;
        if (tok_copy) tok_copy[b] = token;
    }
}

// ------------------------------------------------------------------------------------------
// Greedy draft trees: the children of a node are its drafter's most likely next tokens.

struct TreeShape {
    int n;                          // nodes including the root
    int8_t parent[TREE_MAX];        // parent[0] = -1; parent[i] < i
    int8_t rank[TREE_MAX];          // node i is the rank[i]-th most likely next token after its parent (0 = most likely)
};
constexpr int TREE_RANKS = 8;

// Row r holds the drafter's logits at node node0 + r.  The TREE_RANKS largest logits of the row are found in order (ties: the
// lower token first) and every child of the node gets its token: hist[base + i] = tok[i] = winner[rank[i]].
//   grid (rows), block 512
__global__ __launch_bounds__(AK_NT) void tree_children_kernel(const float* __restrict__ logits, int V, TreeShape ts, int node0,
                                                              int32_t* __restrict__ hist_base, int32_t* __restrict__ tok) {
    __shared__ AkShared sm;
    __shared__ int win[TREE_RANKS];
    const int node = node0 + (int)blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float x[AK_CH][4];
    ak_load(logits + (size_t)blockIdx.x * V, V, wave, lane, x);
    int need = 0;                                   // ranks 0 .. need-1 are used by some child
    for (int i = node + 1; i < ts.n; ++i)
        if (ts.parent[i] == node) need = max(need, (int)ts.rank[i] + 1);
    for (int k = 0; k < need; ++k) {
        __syncthreads();                            // the previous turn's readers of sm are done
        const int w = ak_argmax(x, sm, wave, lane);
        if (threadIdx.x == 0) win[k] = w;
#pragma unroll
        for (int c = 0; c < AK_CH; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (wave * AK_SEG + c * 256 + lane * 4 + e == w) x[c][e] = -INFINITY;
    }
    __syncthreads();
    if (threadIdx.x == 0)
        for (int i = node + 1; i < ts.n; ++i)
            if (ts.parent[i] == node) {
                const int t = win[ts.rank[i]];
                hist_base[i] = t;
                tok[i] = t;
            }
}

// Greedy acceptance over a verified tree: amax[i] = the target's most likely token after node i.  Walk from the root:
// while the current node has a child whose token is the target's choice, step to it.  n_acc = nodes stepped to,
// token = the target's choice at the last node reached.  res: [0] n_acc, [1] token, [2 ..] the nodes of the path.
// Commits the tokens: hist_base[1 + j] = tok[path[j]], hist_base[1 + n_acc] = token.     grid (1), block 64
__global__ void accept_tree_kernel(const int32_t* __restrict__ amax, const int32_t* __restrict__ tok, TreeShape ts,
                                   int32_t* __restrict__ res, int32_t* __restrict__ hist_base) {
    if (threadIdx.x != 0) return;
    int cur = 0, n = 0;
    int path[TREE_MAX];
    for (;;) {
        const int want = amax[cur];
        int next = -1;
        for (int i = cur + 1; i < ts.n && next < 0; ++i)
            if (ts.parent[i] == cur && tok[i] == want) next = i;
        if (next < 0) break;
        path[n++] = next;
        cur = next;
    }
    const int token = amax[cur];
    res[0] = n;
    res[1] = token;
    for (int j = 0; j < n; ++j) res[2 + j] = path[j];
    for (int j = 0; j < n; ++j) hist_base[1 + j] = tok[path[j]];     // path[j] >= j + 1: reads from tok, a separate array
    hist_base[1 + n] = token;
}

// ------------------------------------------------------------------------------------------
// Sampled draft trees (T > 0): the children of a node, in ascending rank, are successive draws without replacement from
// q = softmax(logits / T); the walk over the verified tree is recursive rejection sampling (Jeon et al., "Recursive
// speculative decoding", 2024 - for one child per node it is the accept step of the chain).  Uniforms: child node v uses
// position v - 1 (draft stream for its draw, accept stream for its test), the emitted token position 0 of the residual
// stream, so a chain-shaped tree uses exactly the counters of a chain round.

// the children of `node` in ascending rank; returns how many
__device__ __forceinline__ int tree_children_of(const TreeShape& ts, int node, int (&ch)[TREE_RANKS]) {
    int n = 0;
    for (int r = 0; r < TREE_RANKS; ++r)
        for (int i = node + 1; i < ts.n; ++i)
            if (ts.parent[i] == node && ts.rank[i] == r && n < TREE_RANKS) ch[n++] = i;
    return n;
}

// this thread's sum of its 64 values, in the order of ak_exp_inplace
__device__ __forceinline__ float ak_thread_sum(const float (&x)[AK_CH][4]) {
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < AK_CH; ++c) s += (x[c][0] + x[c][1]) + (x[c][2] + x[c][3]);
    return s;
}

// sm.dz[which][wave] <- the wavefront totals of x; returns their sum (every thread).  Two barriers.
__device__ __forceinline__ double ak_totals(const float (&x)[AK_CH][4], AkShared& sm, int which, int wave, int lane) {
    const double a = wave_sum((double)ak_thread_sum(x));
    __syncthreads();                                   // earlier readers of sm.dz are done
    if (lane == 0) sm.dz[which][wave] = a;
    __syncthreads();
    double Z = 0.0;
#pragma unroll
    for (int k = 0; k < AK_WAVES; ++k) Z += sm.dz[which][k];
    return Z;
}

// element `idx` of the vocabulary as held in x: the value (0 elsewhere); with zero = true the owner also clears it
__device__ __forceinline__ float ak_take(float (&x)[AK_CH][4], int idx, int wave, int lane, bool zero) {
    float v = 0.f;
    const int off = idx - wave * AK_SEG - lane * 4;     // = 256 c + e for the owner
    if (off >= 0 && off < AK_SEG && (off & 255) < 4) {
        const int cd = off >> 8, ed = off & 3;
#pragma unroll
        for (int c = 0; c < AK_CH; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (c == cd && e == ed) { v = x[c][e]; if (zero) x[c][e] = 0.f; }
    }
    return v;
}

// Row r holds the drafter's logits at node node0 + r; every child of the node gets its token:
// hist[base + i] = tok[i] = the draw.   grid (rows), block 512
template <bool UNIT_T>
__device__ __forceinline__ void tree_children_sample_body(const float* __restrict__ logits, int V, float T, uint64_t seed, uint32_t seq,
                                                          uint32_t round, const TreeShape& ts, int node0,
                                                          int32_t* __restrict__ hist_base, int32_t* __restrict__ tok, AkShared& sm) {
    const int node = node0 + (int)blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int ch[TREE_RANKS];
    const int nch = tree_children_of(ts, node, ch);
    if (nch == 0) return;                              // workgroup-uniform
    float x[AK_CH][4];
    ak_load(logits + (size_t)blockIdx.x * V, V, wave, lane, x);
    const float a = wave_max(ak_thread_max(x));
    if (lane == 0) sm.fmx[0][wave] = a;
    __syncthreads();
    float mx = sm.fmx[0][0];
#pragma unroll
    for (int k = 1; k < AK_WAVES; ++k) mx = fmaxf(mx, sm.fmx[0][k]);
    ak_exp_inplace<UNIT_T>(x, mx, 1.0 / (double)T);
    for (int c = 0; c < nch; ++c) {
        const double Z = ak_totals(x, sm, 0, wave, lane);
        const float u = philox_uniform(seed, seq, round, (uint32_t)(ch[c] - 1), 2u);
        ak_search(x, sm.dz[0], Z, u, V, sm, wave, lane);
        __syncthreads();
        const int t = sm.token;
        if (threadIdx.x == 0) { hist_base[ch[c]] = t; tok[ch[c]] = t; }
        ak_take(x, t, wave, lane, true);               // drawn: out of the urn
    }
}

__global__ __launch_bounds__(AK_NT) void tree_children_sample_kernel(const float* __restrict__ logits, int V, float T, uint64_t seed,
                                                                     uint32_t seq, uint32_t round, TreeShape ts, int node0,
                                                                     int32_t* __restrict__ hist_base, int32_t* __restrict__ tok) {
    __shared__ AkShared sm;
    if (T == 1.0f) tree_children_sample_body<true>(logits, V, T, seed, seq, round, ts, node0, hist_base, tok, sm);
    else tree_children_sample_body<false>(logits, V, T, seed, seq, round, ts, node0, hist_base, tok, sm);
}

// x *= 1 / Z (1/Z applied as two floats)
__device__ __forceinline__ void ak_scale(float (&x)[AK_CH][4], double Z) {
    const double iz = 1.0 / Z;
    const float hi = (float)iz, lo = (float)(iz - (double)hi);
#pragma unroll
    for (int c = 0; c < AK_CH; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) x[c][e] = fmaf(x[c][e], lo, x[c][e] * hi);
}

// x <- softmax(row / T) as fp32 probabilities
template <bool UNIT_T>
__device__ __forceinline__ void ak_normalised(const float* __restrict__ row, int V, double invT, float (&x)[AK_CH][4], AkShared& sm, int wave,
                                              int lane) {
    ak_load(row, V, wave, lane, x);
    const float a = wave_max(ak_thread_max(x));
    __syncthreads();
    if (lane == 0) sm.fmx[0][wave] = a;
    __syncthreads();
    float mx = sm.fmx[0][0];
#pragma unroll
    for (int k = 1; k < AK_WAVES; ++k) mx = fmaxf(mx, sm.fmx[0][k]);
    ak_exp_inplace<UNIT_T>(x, mx, invT);
    ak_scale(x, ak_totals(x, sm, 0, wave, lane));
}

// The walk, node by node in parallel.  What happens at a node - which child is accepted, or which token is emitted when none
// is - depends on that node's two distributions, its children's tokens and their uniforms only, not on how the walk got
// there; so one workgroup per node decides it (P[i], Q[i]: target / drafter logits at node i, Q only for nodes with
// children; tok[i]: the node's token; the two distributions are held in registers as probabilities and updated in place
// after every rejection), and accept_tree_walk_kernel then follows the decisions from the root.
//   step[i] = (accepted child or -1, token emitted if the walk ends at node i).     grid (nodes), block 512
template <bool UNIT_T>
__device__ __forceinline__ void accept_tree_node_body(const float* __restrict__ P, const float* __restrict__ Q,
                                                      const int32_t* __restrict__ tok, int V, float T, uint64_t seed, uint32_t seq,
                                                      uint32_t round, const TreeShape& ts, int2* __restrict__ step, AkShared& sm,
                                                      float* pick) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const double invT = 1.0 / (double)T;
    const int cur = blockIdx.x;
    float xp[AK_CH][4], xq[AK_CH][4];
    int ch[TREE_RANKS];
    const int nch = tree_children_of(ts, cur, ch);
    ak_normalised<UNIT_T>(P + (size_t)cur * V, V, invT, xp, sm, wave, lane);
    if (nch > 0) ak_normalised<UNIT_T>(Q + (size_t)cur * V, V, invT, xq, sm, wave, lane);
    int next = -1;
#pragma unroll 1
    for (int c = 0; c < nch; ++c) {
        int child = ch[0];
#pragma unroll
        for (int i = 1; i < TREE_RANKS; ++i) child = c == i ? ch[i] : child;
        const int x = min(max(tok[child], 0), V - 1);          // clamped: stays in bounds for any input
        const int off = x - wave * AK_SEG - lane * 4;
        const bool owner = off >= 0 && off < AK_SEG && (off & 255) < 4;
        const float pv = ak_take(xp, x, wave, lane, false), qv = ak_take(xq, x, wave, lane, true);   // q(x) leaves the urn either way
        __syncthreads();
        if (owner) { pick[0] = pv; pick[1] = qv; }
        __syncthreads();
        const double pd = (double)pick[0], qd = (double)pick[1];
        bool acc = true;
        if (qd > 0.0) {
            const double ratio = pd / qd;
            const float u = philox_uniform(seed, seq, round, (uint32_t)(child - 1), 0u);
            acc = (double)u < (ratio < 1.0 ? ratio : 1.0);
        }
        if (acc) { next = child; break; }
        // rejected: p <- norm(max(0, p - q)) with q still counting q(x); q <- q without x, renormalised
#pragma unroll
        for (int cc = 0; cc < AK_CH; ++cc)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float qe = (owner && cc == (off >> 8) && e == (off & 3)) ? qv : xq[cc][e];
                xp[cc][e] = fmaxf(xp[cc][e] - qe, 0.f);
            }
        const double Zr = ak_totals(xp, sm, 0, wave, lane);
        if (Zr > 0.0) ak_scale(xp, Zr);
        else ak_normalised<UNIT_T>(P + (size_t)cur * V, V, invT, xp, sm, wave, lane);   // p == q to rounding: a rejection has probability 0; keep p
        const double Sq = ak_totals(xq, sm, 1, wave, lane);
        if (Sq > 0.0) ak_scale(xq, Sq);
    }
    int token = -1;
    if (next < 0) {
        const double Z = ak_totals(xp, sm, 0, wave, lane);
        const float u = philox_uniform(seed, seq, round, 0u, 1u);
        ak_search(xp, sm.dz[0], Z, u, V, sm, wave, lane);
        __syncthreads();
        token = sm.token;
    }
    if (threadIdx.x == 0) step[cur] = make_int2(next, token);
}

__global__ __launch_bounds__(AK_NT) void accept_tree_node_kernel(const float* __restrict__ P, const float* __restrict__ Q,
                                                                 const int32_t* __restrict__ tok, int V, float T, uint64_t seed,
                                                                 uint32_t seq, uint32_t round, TreeShape ts, int2* __restrict__ step) {
    __shared__ AkShared sm;
    __shared__ float pick[2];
    if (T == 1.0f) accept_tree_node_body<true>(P, Q, tok, V, T, seed, seq, round, ts, step, sm, pick);
    else accept_tree_node_body<false>(P, Q, tok, V, T, seed, seq, round, ts, step, sm, pick);
}

// Follows the nodes' decisions from the root; res and hist as accept_tree_kernel.     grid (1), block 64
__global__ void accept_tree_walk_kernel(const int2* __restrict__ step, const int32_t* __restrict__ tok, TreeShape ts,
                                        int32_t* __restrict__ res, int32_t* __restrict__ hist_base) {
    if (threadIdx.x != 0) return;
    int cur = 0, n = 0;
    int path[TREE_MAX];
    while (n < TREE_MAX - 1) {
        const int next = step[cur].x;
        if (next <= cur || next >= ts.n) break;          // -1, or anything that is not a later node
        path[n++] = next;
        cur = next;
    }
    const int token = step[cur].y;
    res[0] = n;
    res[1] = token;
    for (int j = 0; j < n; ++j) res[2 + j] = path[j];
    for (int j = 0; j < n; ++j) hist_base[1 + j] = tok[path[j]];     // path[j] >= j + 1: reads from tok, a separate array
    hist_base[1 + n] = token;
}

// After acceptance the K/V of the accepted nodes move from their tree slots to the positions they were rotated for:
// slot base + path[j] -> base + 1 + j for j < n (path[j] >= j + 1 and ascending, so a thread that owns one element
// offset and walks j upwards never overwrites a source it still needs).   grid (ceil(planes * hd / 256)), block 256
// res: the result words of accept_tree_kernel (n_acc, token, path); limit: at most this many leading path nodes are moved
// (a drafter has only processed the nodes above the deepest level).
template <typename T>
__global__ void kv_compact_kernel(T* __restrict__ kv, int planes, int max_ctx, int hd, int base, const int32_t* __restrict__ res, int limit,
                                  int nodes) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;      // (plane, element of a row)
    if (i >= (size_t)planes * hd) return;
    const size_t plane = i / hd, e = i - plane * hd;
    T* row0 = kv + (plane * max_ctx + base) * hd + e;
    const int n = min(min(res[0], limit), nodes - 1);
    for (int j = 0; j < n; ++j) {
        const int src = min(max(res[2 + j], 1), nodes - 1), dst = 1 + j;        // clamped: stays inside the tree's slots whatever res holds
        if (src != dst) row0[(size_t)dst * hd] = row0[(size_t)src * hd];
    }
}

}  // namespace msd
