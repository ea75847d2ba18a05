// Persistent forward kernel for bf16 models on gfx950: one launch runs a whole block forward
// (m <= 16 rows through every layer and, optionally, the LM head) on one workgroup per compute
// unit, with device-wide barriers between dependent phases.
//
// Why: at m = 6 rows the pass is a pure weight stream (13.2 GB at the 7B shape).  Launching each
// GEMM / attention / element-wise step on its own costs a pipeline drain and refill per step
// (about 320 of them), and a step is only 4-35 us long.  Here every wavefront knows the weight
// tiles it will need in the next phase, so it issues those loads BEFORE it waits at the barrier:
// HBM keeps streaming while activations are exchanged.
//
// Phases per layer (a device-wide barrier after each):
//   QKV      x = h * gain (RMSNorm scale applied to the output), q|k|v projection, rotary
//            embedding, q -> fp32 buffer, k/v -> bf16 cache rows
//   ATTN     (head, 128-position chunk) units on half-workgroups: partial (o, max, sum)
//   COMBINE  merge the chunks of every (row, head)
//   O        h += attn W_o^T
//   GATE/UP  gu = norm(h) [W_gate | W_up]^T
//   DOWN     h += (silu(g) * u) W_down^T
// GEMM phases: the workgroup owns output tiles t = bid, bid + nb, ..; its 8 wavefronts split K,
// reduce through LDS and one of them runs the epilogue - no partial sums in global memory, no
// float atomics, fixed summation order.  Activations are staged in LDS as two bf16 terms; when a
// whole K does not fit (m * K * 4 bytes > PK_XBYTES) K is processed in parts.
//
// Cross-workgroup data (h, q, new K/V rows, attention partials, gu) is written with agent-scope
// write-through stores; a barrier drains them, counts arrivals, and the waiters invalidate their
// caches once (acquire) before reading - no L2 write-back, no per-unit fences.
#pragma once

#include "kernels.h"

namespace msd {

constexpr int PK_NW = 8;                 // wavefronts per workgroup
constexpr int PK_NT = PK_NW * 64;        // threads per workgroup
constexpr int PK_U = 8;                // weight tiles (KiB) a wavefront keeps in flight
constexpr int PK_MAXT = 8;               // output tiles a workgroup accumulates per pass over K
constexpr int PK_XBYTES = 136 * 1024;    // LDS for staged activations (also the attention tiles)
constexpr int PK_RED_FLOATS = 2 * PK_NW * 256;                       // double-buffered cross-wave reduction
constexpr int PK_MISC_FLOATS = PK_NW * 16 + 2 * 2 * 4 * 16 + 16;     // row sums of squares, attention row stats
constexpr int PK_LDS_BYTES = PK_XBYTES + (PK_RED_FLOATS + PK_MISC_FLOATS) * 4;

struct GridBar { int count; int gen; int abort; int pad; };

// Device-wide (all XCDs) visibility without flushing caches: data another workgroup of the same
// launch will read is written with agent-scope relaxed atomic stores (write-through); the writer
// drains its stores before it is counted at the barrier.  A __threadfence() would write back and
// invalidate the whole L2 instead.
__device__ __forceinline__ void st_agent(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void drain_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ int arrive(int* cnt) { return __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

enum { PKPRO_PLAIN = 0, PKPRO_NORM = 1, PKPRO_SWIGLU = 2, PKPRO_GELU = 3 };

// 8 activations -> two bf16 terms (hi = bf16(x), lo = bf16(x - hi)), one 16-byte LDS unit each
__device__ __forceinline__ void store_hilo(uint4* xs, uint4* xlo, int at, const float (&v)[8]) {
    bf16_t hi[8], lo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        hi[e] = f2bf(v[e]);
        lo[e] = f2bf(v[e] - bf2f(hi[e]));
    }
    xs[at] = make_uint4(pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3]), pack_bf16x2(hi[4], hi[5]), pack_bf16x2(hi[6], hi[7]));
    xlo[at] = make_uint4(pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3]), pack_bf16x2(lo[4], lo[5]), pack_bf16x2(lo[6], lo[7]));
}

struct FwdP {
    int n_layers, D, H, KH, hd, F, V, act;
    float eps, theta;
    const void* const* w;      // device copy of the model's weight table
    bf16_t* kv;                // [layer][2][KH][max_ctx][hd]
    int max_ctx;
    const int32_t* tok;        // m tokens
    int m, pos0;
    float* h;                  // [m][D] residual stream
    float* q;                  // [m][H*hd]
    float* ao;                 // [m][H*hd] attention output
    float* gu;                 // [m][2F] fused gate | up (or [m][F] for GELU)
    float* apart;              // [H][nchunks][16][hd+2]
    float* logits;             // nullptr, or rows first_row..m-1 -> [m-first_row][V]
    int first_row;
    GridBar* bar;
    int spin_limit;
    long long* tlog;           // nullptr, or 2 timestamps per barrier written by workgroup 0 (measurement aid)
};

enum { PEPI_QKV = 0, PEPI_RESID = 1, PEPI_GU = 2, PEPI_LOGITS = 3 };

struct GPh {                   // one GEMM phase
    const float* x; int ldx; int K; int pro; const bf16_t* gain;
    const bf16_t* W0; const bf16_t* W1; const bf16_t* W2; int t0, t1, ntiles; int N;
    int epi; int row0;         // row0: first activation row (LM head on the last rows only)
    int layer;
};

struct GIdx {                  // how a phase maps onto this workgroup / wavefront
    int m, kchunks, nparts, pc, ntl;
};

__device__ __forceinline__ GIdx gemm_index(const GPh& G, int m, int bid, int nb) {
    GIdx I;
    I.m = m;
    I.kchunks = G.K >> 5;
    const int pc_max = max(PK_NW, (PK_XBYTES / (32 * m) - 1) / 4); // chunks per part: 2 planes x m rows x (4 pc + 1) x 16 B
    I.nparts = (I.kchunks + pc_max - 1) / pc_max;
    I.pc = (I.kchunks + I.nparts - 1) / I.nparts;
    I.ntl = G.ntiles > bid ? (G.ntiles - bid + nb - 1) / nb : 0;
    return I;
}

__device__ __forceinline__ const u32x4* tile_ptr(const GPh& G, int t, int kchunks) {
    const bf16_t* W;
    int tl;
    if (t < G.t0) { W = G.W0; tl = t; }
    else if (t < G.t1) { W = G.W1; tl = t - G.t0; }
    else { W = G.W2; tl = t - G.t1; }
    return reinterpret_cast<const u32x4*>(W) + (size_t)tl * kchunks * 64;
}

// GEMM phase descriptors: kind 0 QKV, 3 O, 4 gate|up, 5 down of layer L; kind 6 LM head.
// Written with selects on purpose (no branch ladder): every field is a function of (L, kind).
__device__ __forceinline__ void make_gemm(const FwdP& P, int L, int kind, GPh& G) {
    const int D = P.D, F = P.F, DQ = P.H * P.hd, DKV = P.KH * P.hd, nl = P.n_layers;
    const bool qkv = kind == 0, op = kind == 3, gu = kind == 4, dn = kind == 5, head = kind == 6;
    const bool swiglu = P.act == 1;
    const int base = 1 + 9 * L;                                   // attn_norm of layer L in the weight table
    G.layer = L;
    G.row0 = head ? P.first_row : 0;
    G.x = op ? P.ao : (dn ? P.gu : P.h);
    G.ldx = op ? DQ : (dn ? (swiglu ? 2 * F : F) : D);
    G.K = op ? DQ : (dn ? F : D);
    G.pro = op ? PKPRO_PLAIN : (dn ? (swiglu ? PKPRO_SWIGLU : PKPRO_GELU) : PKPRO_NORM);
    const int gi = qkv ? base : (gu ? base + 5 : 1 + 9 * nl);      // norm gain (unused for O and down)
    G.gain = (const bf16_t*)P.w[gi];
    const int w0 = qkv ? base + 1 : op ? base + 4 : gu ? (swiglu ? base + 6 : base + 7) : dn ? base + 8 : 2 + 9 * nl;
    const int w1 = qkv ? base + 2 : (gu && swiglu) ? base + 7 : w0;
    const int w2 = qkv ? base + 3 : w1;
    G.W0 = (const bf16_t*)P.w[w0];
    G.W1 = (const bf16_t*)P.w[w1];
    G.W2 = (const bf16_t*)P.w[w2];
    G.N = qkv ? DQ + 2 * DKV : gu ? (swiglu ? 2 * F : F) : head ? P.V : D;
    G.ntiles = G.N / 16;
    G.t0 = qkv ? DQ / 16 : (gu && swiglu) ? F / 16 : G.ntiles;
    G.t1 = qkv ? (DQ + DKV) / 16 : G.ntiles;
    G.epi = qkv ? PEPI_QKV : gu ? PEPI_GU : head ? PEPI_LOGITS : PEPI_RESID;
}

// Issue the loads of the first group of weight tiles of a phase (part 0, first tile).
// The phase is named by (layer, kind) and its descriptor is rebuilt here and in gemm_run: only two
// integers stay live across the barriers.
__device__ __forceinline__ void gemm_prefetch(const FwdP& P, int L, int kind, int bid, int nb, int wave, int lane, u32x4 (&w)[PK_U]) {
    GPh G;
    make_gemm(P, L, kind, G);
    const GIdx I = gemm_index(G, kind == 6 ? P.m - P.first_row : P.m, bid, nb);
    if (I.ntl == 0) return;
    const int npc = min(I.pc, I.kchunks);
    const int cpw = (npc + PK_NW - 1) / PK_NW;
    const int wc0 = wave * cpw;
    const int nwc = max(0, min(cpw, npc - wc0));
    const int cnt = min(PK_U, nwc);
    const u32x4* wp = tile_ptr(G, bid, I.kchunks) + (size_t)wc0 * 64 + lane;
#pragma unroll
    for (int u = 0; u < PK_U; ++u)
        if (u < cnt) w[u] = __builtin_nontemporal_load(wp + (size_t)u * 64);
}

// Workgroup barrier that orders LDS accesses only: unlike __syncthreads() it does not wait for
// outstanding global loads, so weight tiles prefetched for the next phase stay in flight.
__device__ __forceinline__ void wg_barrier_lds() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Device-wide barrier, in two halves so that the prefetch of the next phase's weights can be
// issued in between (after this wavefront's stores have drained, before the wait):
//     grid_barrier_begin();  [wavefronts 1..7: prefetch]  if (!grid_barrier_end(..)) return;
// Wavefront 0 polls the generation counter, so it must not have loads in flight (memory
// operations of a wavefront return in order); it fetches its first weight group afterwards.
// my_gen is the workgroup's private copy of the generation.  grid_barrier_end returns false when
// the run was aborted (a wait exceeded spin_limit): every wavefront then leaves the kernel.
__device__ __forceinline__ void grid_barrier_begin() { drain_stores(); }

__device__ __forceinline__ bool grid_barrier_end(GridBar* b, int nb, int spin_limit, int& my_gen, int* flag_s, long long* tlog = nullptr) {
    wg_barrier_lds();                                    // every wavefront of the workgroup has drained its stores
    if (threadIdx.x < 64) {
        if (threadIdx.x == 0) {
            int ok = 1;
            if (tlog) tlog[0] = wall_clock64();
            if (arrive(&b->count) == nb - 1) {
                __hip_atomic_store(&b->count, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                drain_stores();                              // the reset lands before the release
                __hip_atomic_fetch_add(&b->gen, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
                int spins = 0;
                while (__hip_atomic_load(&b->gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == my_gen) {
                    if (++spins > spin_limit || __hip_atomic_load(&b->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                        __hip_atomic_store(&b->abort, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        ok = 0;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
            if (__hip_atomic_load(&b->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) ok = 0;
            *flag_s = ok;
            if (tlog) tlog[1] = wall_clock64();
        }
        // one wavefront per compute unit drops stale cache lines: later plain loads of this
        // workgroup see what the other workgroups stored before the barrier
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    wg_barrier_lds();
    my_gen += 1;
    return *flag_s != 0;
}

__device__ __forceinline__ void st_agent4(float* p, float a, float b, float c, float d) {
    st_agent(p, a); st_agent(p + 1, b); st_agent(p + 2, c); st_agent(p + 3, d);
}
__device__ __forceinline__ void st_agent_u32(void* p, uint32_t v) {
    __hip_atomic_store(reinterpret_cast<uint32_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Stage chunks [pc0, pc0 + npc) of the phase's activations into LDS as hi / lo bf16 planes.
// Rows go in batches of 4 so that the global loads of a batch are in flight together (one memory
// round trip per batch instead of one per row).
__device__ __forceinline__ void stage_x(const GPh& G, int m, int pc0, int npc, uint4* xs, float* ssq_s, int tid, int wave, int lane) {
    const int rs = npc * 4 + 1;
    uint4* xlo = xs + m * rs;
    constexpr int RB = 4;
    for (int r0 = 0; r0 < m; r0 += RB) {
        float ss[RB] = {0.f, 0.f, 0.f, 0.f};
        for (int c = tid; c < npc * 4; c += PK_NT) {
            const int k = pc0 * 32 + c * 8;
            float4 a[RB], b[RB], ua[RB], ub[RB];
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                const int r = min(r0 + j, m - 1);                        // clamped rows are loaded twice and not stored
                const float* xr = G.x + (size_t)(G.row0 + r) * G.ldx + k;
                a[j] = *reinterpret_cast<const float4*>(xr);
                b[j] = *reinterpret_cast<const float4*>(xr + 4);
                if (G.pro == PKPRO_SWIGLU) {
                    ua[j] = *reinterpret_cast<const float4*>(xr + G.K);
                    ub[j] = *reinterpret_cast<const float4*>(xr + G.K + 4);
                }
            }
            uint4 gq = make_uint4(0, 0, 0, 0);
            if (G.pro == PKPRO_NORM) gq = *reinterpret_cast<const uint4*>(G.gain + k);
            const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w};
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                if (r0 + j < m) {
                    float v[8] = {a[j].x, a[j].y, a[j].z, a[j].w, b[j].x, b[j].y, b[j].z, b[j].w};
                    if (G.pro == PKPRO_NORM) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            ss[j] += v[e] * v[e];
                            v[e] *= bf2f((bf16_t)(gw[e >> 1] >> ((e & 1) * 16)));
                        }
                    } else if (G.pro == PKPRO_SWIGLU) {
                        const float u[8] = {ua[j].x, ua[j].y, ua[j].z, ua[j].w, ub[j].x, ub[j].y, ub[j].z, ub[j].w};
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = v[e] / (1.0f + expf(-v[e])) * u[e];
                    } else if (G.pro == PKPRO_GELU) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = 0.5f * v[e] * (1.0f + erff(v[e] * 0.70710678118654752f));
                    }
                    store_hilo(xs, xlo, (r0 + j) * rs + c, v);
                }
            }
        }
        if (G.pro == PKPRO_NORM) {
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                const float t = wave_sum(ss[j]);
                if (lane == 0 && r0 + j < m) ssq_s[wave * 16 + r0 + j] += t;   // each wavefront owns its slot: no race
            }
        }
    }
}

// One GEMM phase.  w holds the first group of weight tiles when `prefetched`.
// Tile by tile: stage the activations (once per phase when the whole K fits the LDS, else once
// per tile and K part), stream this wavefront's K slice of the tile, reduce the 8 wavefronts
// through LDS, run the epilogue on one of them.
__device__ __forceinline__ void gemm_run(const FwdP& P, int L, int kind, u32x4 (&w)[PK_U], bool prefetched,
                                         uint4* xs, float* red, float* ssq_s, int bid, int nb, int tid, int wave, int lane) {
    GPh G;
    make_gemm(P, L, kind, G);
    const GIdx I = gemm_index(G, kind == 6 ? P.m - P.first_row : P.m, bid, nb);
    const int m = I.m, N = G.N;
    const int row = lane & 15, g = lane >> 4;
    const bool rowok = row < m;
    const uint4 zero = make_uint4(0, 0, 0, 0);
    bool staged = false;
    // This wavefront's weight stream is a sequence of groups of <= PK_U tiles, ordered by (output
    // tile, K part, offset).  Two register buffers: while group i is multiplied, group i+1 is
    // already being loaded - also across output tiles and K parts.
    u32x4 wb[PK_U];
    struct Grp { int ti, p, c, cnt; const u32x4* ptr; };
    auto locate = [&](int ti, int p, int c) {          // first non-empty group at or after (ti, p, c)
        Grp q;
        q.cnt = 0; q.ptr = nullptr; q.ti = ti; q.p = p; q.c = c;
        while (q.ti < I.ntl) {
            const int pc0 = q.p * I.pc, npc = min(I.pc, I.kchunks - pc0);
            const int cpw = (npc + PK_NW - 1) / PK_NW;
            const int wc0 = wave * cpw;
            const int nwc = max(0, min(cpw, npc - wc0));
            if (q.c < nwc) {
                q.cnt = min(PK_U, nwc - q.c);
                q.ptr = tile_ptr(G, bid + q.ti * nb, I.kchunks) + (size_t)(pc0 + wc0 + q.c) * 64 + lane;
                return q;
            }
            q.c = 0;
            if (++q.p == I.nparts) { q.p = 0; ++q.ti; }
        }
        return q;
    };
    auto issue = [&](u32x4 (&buf)[PK_U], const Grp& q) {
#pragma unroll
        for (int u = 0; u < PK_U; ++u)
            if (u < q.cnt) buf[u] = __builtin_nontemporal_load(q.ptr + (size_t)u * 64);
    };
    Grp cur = locate(0, 0, 0);
    if (cur.cnt > 0 && !prefetched) issue(w, cur);
    int par = 0;                                           // buffer holding the current group: 0 = w, 1 = wb
    for (int ti = 0; ti < I.ntl; ++ti) {
        const int t = bid + ti * nb;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acl = {0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < I.nparts; ++p) {
            const int pc0 = p * I.pc, npc = min(I.pc, I.kchunks - pc0);
            const int rs = npc * 4 + 1;
            if (!staged || I.nparts > 1) {
                wg_barrier_lds();                                    // earlier readers of xs / ssq_s are done (LDS only:
                if (p == 0 && tid < PK_NW * 16) ssq_s[tid] = 0.f;    //  weight loads stay in flight)
                wg_barrier_lds();
                stage_x(G, m, pc0, npc, xs, ssq_s, tid, wave, lane);
                wg_barrier_lds();
                staged = true;
            }
            const int cpw = (npc + PK_NW - 1) / PK_NW;
            const int wc0 = wave * cpw;
            const int nwc = max(0, min(cpw, npc - wc0));
            const uint4* xa = xs + (rowok ? row : 0) * rs + wc0 * 4 + g;
            const uint4* xb = xa + m * rs;
            for (int c = 0; c < nwc; c += PK_U) {                    // here (ti, p, c) is exactly `cur`
                const Grp nx = locate(ti, p, c + PK_U);
                if (par == 0) {
                    if (nx.cnt > 0) issue(wb, nx);
#pragma unroll
                    for (int u = 0; u < PK_U; ++u) {
                        if (u < cur.cnt) {
                            uint4 ah = xa[(c + u) * 4], al = xb[(c + u) * 4];
                            if (!rowok) { ah = zero; al = zero; }
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[u]), __builtin_bit_cast(bf16x8, ah), acc, 0, 0, 0);
                            acl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[u]), __builtin_bit_cast(bf16x8, al), acl, 0, 0, 0);
                        }
                    }
                } else {
                    if (nx.cnt > 0) issue(w, nx);
#pragma unroll
                    for (int u = 0; u < PK_U; ++u) {
                        if (u < cur.cnt) {
                            uint4 ah = xa[(c + u) * 4], al = xb[(c + u) * 4];
                            if (!rowok) { ah = zero; al = zero; }
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wb[u]), __builtin_bit_cast(bf16x8, ah), acc, 0, 0, 0);
                            acl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wb[u]), __builtin_bit_cast(bf16x8, al), acl, 0, 0, 0);
                        }
                    }
                }
                par ^= 1;
                cur = nx;
            }
        }
        // ---- cross-wavefront reduction (double-buffered) and epilogue
        float* rb = red + (ti & 1) * PK_NW * 256;
        if (rowok) *reinterpret_cast<float4*>(rb + wave * 256 + row * 16 + g * 4) =
            make_float4(acc[0] + acl[0], acc[1] + acl[1], acc[2] + acl[2], acc[3] + acl[3]);
        wg_barrier_lds();
        if (wave == (ti & (PK_NW - 1)) && rowok) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int ww = 0; ww < PK_NW; ++ww) {                     // fixed order
                const float4 pv = *reinterpret_cast<const float4*>(rb + ww * 256 + row * 16 + g * 4);
                v.x += pv.x; v.y += pv.y; v.z += pv.z; v.w += pv.w;
            }
            if (G.pro == PKPRO_NORM) {
                float ssq = 0.f;
#pragma unroll
                for (int ww = 0; ww < PK_NW; ++ww) ssq += ssq_s[ww * 16 + row];
                const float ir = 1.0f / sqrtf(ssq / (float)G.K + P.eps);
                v.x *= ir; v.y *= ir; v.z *= ir; v.w *= ir;
            }
            const size_t col = (size_t)t * 16 + g * 4;
            if (G.epi == PEPI_LOGITS) {
                *reinterpret_cast<float4*>(P.logits + (size_t)row * N + col) = v;
            } else if (G.epi == PEPI_GU) {
                st_agent4(P.gu + (size_t)row * N + col, v.x, v.y, v.z, v.w);
            } else if (G.epi == PEPI_RESID) {
                const float4 hv = *reinterpret_cast<const float4*>(P.h + (size_t)row * N + col);
                st_agent4(P.h + (size_t)row * N + col, hv.x + v.x, hv.y + v.y, hv.z + v.z, hv.w + v.w);
            } else {   // PEPI_QKV
                const int hd = P.hd, half = hd >> 1, tph = hd >> 4;
                const int head = t / tph, j = t - head * tph;
                const int pos = P.pos0 + row;
                const size_t plane = (size_t)P.KH * P.max_ctx * hd;
                bf16_t* kc = P.kv + (size_t)G.layer * 2 * plane;
                if (head < P.H + P.KH) {
                    // rope-ordered weight rows: the tile's columns are (a_i, b_i) pairs, i = 8j + c/2
                    const int i0 = j * 8 + g * 2;
                    float a[2] = {v.x, v.z}, b[2] = {v.y, v.w};
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const double freq = pow((double)P.theta, -2.0 * (double)(i0 + e) / (double)hd);
                        double sn, cs;
                        sincos((double)pos * freq, &sn, &cs);
                        const float ra = (float)((double)a[e] * cs - (double)b[e] * sn);
                        const float rb2 = (float)((double)a[e] * sn + (double)b[e] * cs);
                        a[e] = ra; b[e] = rb2;
                    }
                    if (head < P.H) {
                        float* qd = P.q + (size_t)row * P.H * hd + (size_t)head * hd + i0;
                        st_agent(qd, a[0]); st_agent(qd + 1, a[1]);
                        st_agent(qd + half, b[0]); st_agent(qd + half + 1, b[1]);
                    } else {
                        bf16_t* dst = kc + ((size_t)(head - P.H) * P.max_ctx + pos) * hd + i0;
                        st_agent_u32(dst, pack_bf16x2(f2bf(a[0]), f2bf(a[1])));
                        st_agent_u32(dst + half, pack_bf16x2(f2bf(b[0]), f2bf(b[1])));
                    }
                } else {
                    bf16_t* dst = kc + plane + ((size_t)(head - P.H - P.KH) * P.max_ctx + pos) * hd + j * 16 + g * 4;
                    st_agent_u32(dst, pack_bf16x2(f2bf(v.x), f2bf(v.y)));
                    st_agent_u32(dst + 2, pack_bf16x2(f2bf(v.z), f2bf(v.w)));
                }
            }
        }
    }
}

// Attention partials on half-workgroups (4 wavefronts each): same algorithm as
// attn_partial_mfma_kernel; both halves run in lockstep on different (head, chunk) units.
template <int HD>
__device__ __forceinline__ void attn_phase(const FwdP& P, int layer, unsigned char* lds, float* stat_s, int bid, int nb, int tid) {
    constexpr int RS = HD + 8, VPR = HD / 8, PS = ATT_CH + 8, KC = HD / 32, NT = HD / 16;
    constexpr int HALF_BYTES = (ATT_CH * RS + 2 * 16 * PS) * 2;
    const int half_id = tid >> 8, ht = tid & 255, lane = tid & 63, wave = (tid >> 6) & 3;
    const int row = lane & 15, g = lane >> 4;
    const int m = P.m, H = P.H, KH = P.KH, pos0 = P.pos0;
    const bool rowok = row < m;
    bf16_t* vs = reinterpret_cast<bf16_t*>(lds + (size_t)half_id * HALF_BYTES);
    bf16_t* phi = vs + ATT_CH * RS;
    bf16_t* plo = phi + 16 * PS;
    float* wmax = stat_s + half_id * 128;      // [4][16]
    float* wsum = wmax + 64;                   // [4][16]
    const int L = pos0 + m;
    const int nchunks = (L + ATT_CH - 1) / ATT_CH;
    const int nunits = H * nchunks;
    const float scale = 1.0f / sqrtf((float)HD);
    const size_t plane = (size_t)KH * P.max_ctx * HD;
    const bf16_t* kcl = P.kv + (size_t)layer * 2 * plane;
    const bf16_t* vcl = kcl + plane;
    for (int u0 = bid * 2; u0 < nunits; u0 += nb * 2) {
        const int u = u0 + half_id;
        const bool live = u < nunits;
        const int uu = live ? u : nunits - 1;              // a dead half recomputes the last unit and stores nothing
        const int h = uu / nchunks, c = uu - h * nchunks, kh = h / (H / KH);
        const int p0 = c * ATT_CH;
        const int np = min(ATT_CH, L - p0);
        const bf16_t* vbase = vcl + ((size_t)kh * P.max_ctx + p0) * HD;
        constexpr int VIT = ATT_CH * VPR / 256;
        uint4 vreg[VIT];
#pragma unroll
        for (int it = 0; it < VIT; ++it) {
            const int idx = ht + it * 256;
            const int p = idx / VPR, v = idx - p * VPR;
            vreg[it] = (p < np) ? *reinterpret_cast<const uint4*>(vbase + (size_t)p * HD + v * 8) : make_uint4(0, 0, 0, 0);
        }
        uint4 qh[KC], ql[KC];
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            qh[k] = make_uint4(0, 0, 0, 0);
            ql[k] = make_uint4(0, 0, 0, 0);
            if (rowok) {
                const float* src = P.q + (size_t)row * H * HD + (size_t)h * HD + k * 32 + g * 8;
                const float4 a = *reinterpret_cast<const float4*>(src), b = *reinterpret_cast<const float4*>(src + 4);
                const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                bf16_t hi[8], lo[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) { hi[e] = f2bf(v[e]); lo[e] = f2bf(v[e] - bf2f(hi[e])); }
                qh[k] = make_uint4(pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3]), pack_bf16x2(hi[4], hi[5]), pack_bf16x2(hi[6], hi[7]));
                ql[k] = make_uint4(pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3]), pack_bf16x2(lo[4], lo[5]), pack_bf16x2(lo[6], lo[7]));
            }
        }
        const bf16_t* kbase = kcl + (size_t)kh * P.max_ctx * HD;
        f32x4 sacc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int pl = wave * 32 + t * 16 + row;
            const int pg = min(p0 + pl, L - 1);
            const u32x4* kp = reinterpret_cast<const u32x4*>(kbase + (size_t)pg * HD + g * 8);
            u32x4 kf[KC];
#pragma unroll
            for (int k = 0; k < KC; ++k) kf[k] = kp[k * 4];
            f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acl = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[k]), __builtin_bit_cast(bf16x8, qh[k]), acc, 0, 0, 0);
                acl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[k]), __builtin_bit_cast(bf16x8, ql[k]), acl, 0, 0, 0);
            }
            sacc[t] = acc + acl;
        }
        float sv[8];
        float lmax = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int pl = wave * 32 + t * 16 + g * 4 + v;
                const bool ok = rowok && pl < np && (p0 + pl) <= pos0 + row;
                const float x = ok ? sacc[t][v] * scale : -INFINITY;
                sv[t * 4 + v] = x;
                lmax = fmaxf(lmax, x);
            }
        lmax = fmaxf(lmax, __shfl_xor(lmax, 16, 64));
        lmax = fmaxf(lmax, __shfl_xor(lmax, 32, 64));
        __syncthreads();                                   // the previous unit's readers of vs / phi / stats are done
        if (g == 0) wmax[wave * 16 + row] = lmax;
#pragma unroll
        for (int it = 0; it < VIT; ++it) {
            const int idx = ht + it * 256;
            const int p = idx / VPR, v = idx - p * VPR;
            *reinterpret_cast<uint4*>(vs + p * RS + v * 8) = vreg[it];
        }
        __syncthreads();
        const float mx = fmaxf(fmaxf(wmax[row], wmax[16 + row]), fmaxf(wmax[32 + row], wmax[48 + row]));
        float lsum = 0.f;
        bf16_t ph[8], pl8[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float e = (mx == -INFINITY) ? 0.f : expf(sv[i] - mx);
            lsum += e;
            ph[i] = f2bf(e);
            pl8[i] = f2bf(e - bf2f(ph[i]));
        }
        lsum += __shfl_xor(lsum, 16, 64);
        lsum += __shfl_xor(lsum, 32, 64);
        if (g == 0) wsum[wave * 16 + row] = lsum;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int pl = wave * 32 + t * 16 + g * 4;
            *reinterpret_cast<uint2*>(phi + row * PS + pl) = make_uint2(pack_bf16x2(ph[t * 4], ph[t * 4 + 1]), pack_bf16x2(ph[t * 4 + 2], ph[t * 4 + 3]));
            *reinterpret_cast<uint2*>(plo + row * PS + pl) = make_uint2(pack_bf16x2(pl8[t * 4], pl8[t * 4 + 1]), pack_bf16x2(pl8[t * 4 + 2], pl8[t * 4 + 3]));
        }
        __syncthreads();
        float* dst = P.apart + ((size_t)h * nchunks + c) * 16 * (HD + 2);
#pragma unroll
        for (int nt = wave; nt < NT; nt += 4) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acl = {0.f, 0.f, 0.f, 0.f};
            const int col = nt * 16 + row;
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
            if (rowok && live) {
                float* o = dst + row * (HD + 2) + nt * 16 + g * 4;
                st_agent4(o, acc[0] + acl[0], acc[1] + acl[1], acc[2] + acl[2], acc[3] + acl[3]);
            }
        }
        if (ht < m && live) {
            st_agent(dst + ht * (HD + 2) + HD, fmaxf(fmaxf(wmax[ht], wmax[16 + ht]), fmaxf(wmax[32 + ht], wmax[48 + ht])));
            st_agent(dst + ht * (HD + 2) + HD + 1, (wsum[ht] + wsum[16 + ht]) + (wsum[32 + ht] + wsum[48 + ht]));
        }
    }
}

// Merge the chunks: ao[r][h*HD + col] = sum_c o_c e^{m_c - M} / sum_c l_c e^{m_c - M}
template <int HD>
__device__ __forceinline__ void combine_phase(const FwdP& P, int bid, int nb, int tid) {
    const int m = P.m, H = P.H;
    const int nchunks = (P.pos0 + m + ATT_CH - 1) / ATT_CH;
    const size_t cs = (size_t)16 * (HD + 2);
    const int total = m * H * HD;
    for (int idx = bid * PK_NT + tid; idx < total; idx += nb * PK_NT) {
        const int r = idx / (H * HD), rem = idx - r * (H * HD), h = rem / HD, col = rem - h * HD;
        const float* br = P.apart + ((size_t)h * nchunks * 16 + r) * (HD + 2);
        float M = -INFINITY;
        for (int c0 = 0; c0 < nchunks; c0 += 8) {
            float mv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) mv[j] = br[(size_t)min(c0 + j, nchunks - 1) * cs + HD];
#pragma unroll
            for (int j = 0; j < 8; ++j) M = fmaxf(M, mv[j]);
        }
        float Lsum = 0.f, o = 0.f;
        for (int c0 = 0; c0 < nchunks; c0 += 8) {
            float mv[8], lv[8], ov[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float* pc = br + (size_t)min(c0 + j, nchunks - 1) * cs;
                mv[j] = pc[HD]; lv[j] = pc[HD + 1]; ov[j] = pc[col];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (c0 + j < nchunks) {
                    const float w = (mv[j] == -INFINITY) ? 0.f : expf(mv[j] - M);
                    Lsum += lv[j] * w;
                    o += ov[j] * w;
                }
            }
        }
        st_agent(P.ao + (size_t)r * H * HD + (size_t)h * HD + col, o / Lsum);
    }
}

template <int HD>
__global__ __launch_bounds__(PK_NT) void forward_persistent_kernel(const FwdP P) {
    extern __shared__ uint4 lds_raw[];
    __shared__ int bar_flag;
    unsigned char* lds = reinterpret_cast<unsigned char*>(lds_raw);
    uint4* xs = lds_raw;
    float* red = reinterpret_cast<float*>(lds + PK_XBYTES);
    float* ssq_s = red + PK_RED_FLOATS;              // [PK_NW][16]
    float* stat_s = ssq_s + PK_NW * 16;              // attention row statistics, 2 halves x 2 x [4][16]
    const int bid = blockIdx.x, nb = gridDim.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = P.m, D = P.D;
    int my_gen = __hip_atomic_load(&P.bar->gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    drain_stores();                                    // the generation is read before anybody can arrive

    // ---- embedding
    {
        const bf16_t* E = (const bf16_t*)P.w[0];
        for (int idx = bid * PK_NT + tid; idx < m * (D / 4); idx += nb * PK_NT) {
            const int r = idx / (D / 4), i = (idx - r * (D / 4)) * 4;
            const uint2 e = *reinterpret_cast<const uint2*>(E + (size_t)P.tok[r] * D + i);
            st_agent4(P.h + (size_t)r * D + i, bf2f((bf16_t)e.x), bf2f((bf16_t)(e.x >> 16)), bf2f((bf16_t)e.y), bf2f((bf16_t)(e.y >> 16)));
        }
    }
    // Order of phases: QKV_0 | for each layer: ATTN, COMBINE, then the GEMM chain O, GATE|UP, DOWN and
    // QKV of the next layer (or the LM head).  The loop is rotated so that the chain is one inner
    // loop (a single copy of gemm_run) and the attention code sits where no prefetched weights
    // are held: w is cleared right after it, so the registers are free during ATTN.
    const bool pf = wave != 0;                           // wavefront 0 runs the barriers and prefetches nothing
    int tcount = 0;
    auto tl = [&]() -> long long* { if (!P.tlog || bid != 0) return nullptr; long long* p = P.tlog + 2 * tcount; ++tcount; return p; };
    u32x4 w[PK_U];
    for (int L = -1; L < P.n_layers; ++L) {
        if (L >= 0) {
            grid_barrier_begin();                            // q, k, v of this layer are complete
            if (!grid_barrier_end(P.bar, nb, P.spin_limit, my_gen, &bar_flag, tl())) return;
            attn_phase<HD>(P, L, lds, stat_s, bid, nb, tid);
        }
#pragma unroll
        for (int u = 0; u < PK_U; ++u) w[u] = (u32x4){0u, 0u, 0u, 0u};
        int gl = L >= 0 ? L : 0, kind = L >= 0 ? 3 : 0;      // the chain starts with O (or with QKV of layer 0)
        grid_barrier_begin();                                // embedding (L = -1) or attention partials are out
        if (pf) gemm_prefetch(P, gl, kind, bid, nb, wave, lane, w);
        if (!grid_barrier_end(P.bar, nb, P.spin_limit, my_gen, &bar_flag, tl())) return;
        if (L >= 0) {
            combine_phase<HD>(P, bid, nb, tid);
            grid_barrier_begin();
            if (!grid_barrier_end(P.bar, nb, P.spin_limit, my_gen, &bar_flag, tl())) return;
        }
        while (true) {
            gemm_run(P, gl, kind, w, pf, xs, red, ssq_s, bid, nb, tid, wave, lane);
            if (kind == 0 || kind == 6) break;               // QKV hands over to ATTN; the head is the end
            if (kind < 5) kind += 1;
            else if (L + 1 < P.n_layers) { kind = 0; gl = L + 1; }
            else if (P.logits) kind = 6;
            else break;
            grid_barrier_begin();
            if (pf) gemm_prefetch(P, gl, kind, bid, nb, wave, lane, w);
            if (!grid_barrier_end(P.bar, nb, P.spin_limit, my_gen, &bar_flag, tl())) return;
        }
    }
}

}  // namespace msd
