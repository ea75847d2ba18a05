// Host side of the MetaSD hot-path library: C ABI (include/metasd.h), launch plans, bandit.
// Device memory is never allocated here; every buffer comes from the caller.
#include "../../include/metasd.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "kernels.h"
#include "batch.h"

using namespace msd;

// Scratch of metasd_accept_logits_noalloc: candidates and exchange words of up to METASD_ACCEPT_NOALLOC_MAX_ITEMS
// (row, position) items.  Every GPU the library runs on holds its own copy at its own address; host code reaches it
// only through the per-device pointer that noalloc_scratch() asks the runtime for.
static __device__ __align__(256) unsigned char scratch[(size_t)METASD_ACCEPT_NOALLOC_MAX_ITEMS * 336];

namespace {

thread_local std::string g_err = "";

int fail_global(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

constexpr int PER_LAYER = 9;
constexpr int MAX_ROWS = 16;
constexpr size_t ALIGN = 256;
constexpr int LDS_BUDGET = 60 * 1024;
constexpr int ROWS_PD = 2;                    // gemm_bf16_rows_kernel: stages (of two chunks) in flight
constexpr size_t FULLK_LDS_MAX = 150 * 1024;   // gemm_fullk_residual_kernel: the whole activation block in LDS

size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }
size_t elem_size(const metasd_model_desc& d) { return d.dtype == METASD_BF16 ? 2 : 4; }

struct Model {
    metasd_model_desc d{};
    std::vector<const void*> w;
    void* kv = nullptr;
    bool shared_kv = false;  // an early-exit drafter whose layers are the target's first n_layers and whose cache IS the target's
    int kv_layers = 0;       // layers of the cache buffer behind kv (the target's count for a shared cache): sequence stride
    int hd = 0;
    std::vector<int> kvl;   // positions valid in the KV cache, per sequence
    bool head = false;      // a drafter head on the target's hidden states (metasd_set_drafter_head): see forward_rows
    const void* fc = nullptr;   // its input projection W_fc [d][2 d]
    bool stream = false;    // a drafter with a streaming cache (cfg.stream_sink, cfg.stream_window): see forward()
    int tail = 0;           // streaming cache: first position of the contiguous tail (what lies between the sinks and it was skipped)
    const void** d_table = nullptr;   // device copy of w
    const void* layer_w(int L, int i) const { return w[1 + PER_LAYER * L + i]; }
    const void* final_norm() const { return w[1 + PER_LAYER * d.n_layers]; }
    const void* lm_head() const { return w[2 + PER_LAYER * d.n_layers]; }
};

// split of one GEMM launch
struct Split {
    int ksplit, cps, tpb;
    size_t lds;
};

int env_int(const char* name, int dflt) { const char* e = getenv(name); return e ? atoi(e) : dflt; }
// Launch epoch of tagged exchange words (see tw_put in kernels.h): unique per launch in this process, never 0.
// Epochs 0 (a zero-filled buffer) and 1 (the accept flag the one-workgroup accept path leaves in the upper half of a
// candidate word) are never handed out.
uint32_t next_epoch() {
    static std::atomic<uint32_t> e{1};
    uint32_t v = ++e;
    while (v < 2) v = ++e;
    return v;
}
constexpr int KS_CAP = 8;            // split-K siblings wanted for parallelism (LDS capacity can ask for more)
constexpr int ks_cap() { return KS_CAP; }

Split choose_split(int m, int ntiles, int kchunks) {
    constexpr int target_units = 3072, align = 8;   // wavefront work units aimed for; slices are multiples of 8 chunks (whole load groups)
    const int cps_max = std::max(1, ((LDS_BUDGET / 32 / m) - 1) / 4);   // two bf16 terms per activation
    int want = target_units / ntiles;                             // aim for about 3072 wavefront work units, never fewer tiles' worth
    want = std::max(1, std::min(want, ks_cap()));
    want = std::min(want, std::max(1, kchunks / 8));              // at least 8 chunks per slice
    int ks = std::max(want, (kchunks + cps_max - 1) / cps_max);   // LDS capacity wins
    int cps = (kchunks + ks - 1) / ks;
    if (align > 1 && (cps + align - 1) / align * align <= cps_max) cps = (cps + align - 1) / align * align;
    ks = (kchunks + cps - 1) / cps;
    Split s;
    s.ksplit = ks;
    s.cps = cps;
    s.tpb = 4;
    s.lds = (size_t)2 * m * (cps * 4 + 1) * 16;
    return s;
}

// Many-row GEMM (more than 16 rows): tiles per workgroup (8; for more than 128 rows also 6, 4, or 12 - the form that
// loads its activations straight into LDS) and K split.
// A workgroup holds a CU (its LDS), so the launch runs in ceil(workgroups / 256) rounds; measured on the 7B
// shapes at 256 rows a round costs about 0.9 / 0.75 / 0.6 / 1.28 us per 32-wide K chunk with 8 / 6 / 4 / 12 tiles (a
// fixed part for staging the activations plus the multiplies), and the split-K partials are written and read once.
Split choose_split_rows(int ntiles, int kchunks, int R, int forced_tpb) {
    int best = 1, best_tpb = 8;
    double best_cost = 1e30;
    for (int tpb : {8, 6, 4, 12}) {
        if (tpb != 8 && (R <= 128 || (forced_tpb && tpb != forced_tpb))) continue;
        if (tpb == 8 && forced_tpb && forced_tpb != 8 && R > 128) continue;
        const int groups = (ntiles + tpb - 1) / tpb;
        for (int ks = 1; ks <= 8 && kchunks / ks >= 8; ++ks) {
            const int cps = ((kchunks + ks - 1) / ks + 3) / 4 * 4;
            const int rounds = (groups * ks + 255) / 256;
            const double per_chunk = tpb == 12 ? 1.28 : 0.3 + 0.075 * tpb;
            const double cost = (double)rounds * cps * per_chunk + (ks > 1 ? (double)ks * R * ntiles * 16 * 8 / 8e6 : 0.0);   // us
            if (cost < best_cost) { best_cost = cost; best = ks; best_tpb = tpb; }
        }
    }
    int ks = best;
    int cps = ((kchunks + ks - 1) / ks + 3) / 4 * 4;
    ks = (kchunks + cps - 1) / cps;
    Split s;
    s.ksplit = ks; s.cps = cps; s.tpb = best_tpb; s.lds = 0;
    return s;
}

const char* check_model(const metasd_model_desc& d, const char* who, char* buf, size_t n) {
    auto bad = [&](const char* what) { snprintf(buf, n, "%s: %s", who, what); return buf; };
    if (d.n_layers < 1 || d.d_model < 1 || d.n_heads < 1 || d.n_kv_heads < 1 || d.d_ffn < 1 || d.vocab < 1) return bad("non-positive dimension");
    if (d.d_model % d.n_heads) return bad("d_model not divisible by n_heads");
    if (d.n_heads % d.n_kv_heads) return bad("n_heads not divisible by n_kv_heads");
    const int hd = d.d_model / d.n_heads;
    if (hd != 32 && hd != 64 && hd != 128) return bad("head_dim must be 32, 64 or 128");
    if (d.act != METASD_GELU && d.act != METASD_SWIGLU) return bad("act");
    if (d.dtype != METASD_F32 && d.dtype != METASD_BF16) return bad("dtype");
    if (d.dtype == METASD_F32 && hd > 64) return bad("fp32 models support head_dim <= 64");
    if (d.vocab % 4 || d.vocab > AK_WAVES * AK_SEG) return bad("vocab must be a multiple of 4 and <= 32768");
    if (d.dtype == METASD_BF16) {
        if (d.d_model % 32 || d.d_ffn % 32) return bad("bf16: d_model and d_ffn must be multiples of 32");
        if (d.vocab % 16) return bad("bf16: vocab must be a multiple of 16");
    } else if (d.d_model % 4 || d.d_ffn % 4) return bad("fp32: d_model and d_ffn must be multiples of 4");
    if (!(d.rms_eps > 0.f) || !(d.rope_theta > 0.f)) return bad("rms_eps / rope_theta must be positive");
    return nullptr;
}

// Word the split-K siblings of a residual GEMM set when their bounded wait for each other runs out (read back with
// the results of every accept).
struct GridBar { int abort; int pad[3]; };

// Workspace layout shared by metasd_workspace_bytes and metasd_create.
struct Layout {
    size_t hist, h, h2, xn, part, part2, gx, ssq, inv, q, ao, act, apart, rope, P, Q, cand, bd, res, draft, tstep, feat, fest, bar, xchg, tables, table_stride, total;
};

Layout make_layout(const metasd_config& c, const metasd_model_desc& t, const metasd_model_desc* dr) {
    int dmax = t.d_model, fmax = t.d_ffn, vmax = t.vocab, hmax = t.n_heads, hdmax = t.d_model / t.n_heads;
    size_t partmax = 0, gxmax = ALIGN;
    auto acc = [&](const metasd_model_desc& d) {
        // sibling exchange of the residual GEMMs (N = d_model; K = attention width or d_ffn): ksplit - 1 published
        // partial tiles of m rows, for the split choose_split really takes at every block height (LDS capacity
        // can push it past ks_cap())
        if (d.dtype == METASD_BF16)
            for (int m = 1; m <= MAX_ROWS; ++m)
                for (int K : {d.d_model, d.d_ffn})
                    gxmax = std::max(gxmax, (size_t)(choose_split(m, d.d_model / 16, K / 32).ksplit - 1) * m * d.d_model * 8);
        dmax = std::max(dmax, d.d_model); fmax = std::max(fmax, d.d_ffn); vmax = std::max(vmax, d.vocab);
        hmax = std::max(hmax, d.n_heads); hdmax = std::max(hdmax, d.d_model / d.n_heads);
        const int hd = d.d_model / d.n_heads;
        const int ns[5] = {(d.n_heads + 2 * d.n_kv_heads) * hd, d.d_model, (d.act == METASD_SWIGLU ? 2 : 1) * d.d_ffn, d.d_model, d.vocab};
        const int ks[5] = {d.d_model, d.d_model, d.d_model, d.d_ffn, d.d_model};
        if (c.feature_heads && d.dtype == METASD_BF16)   // a drafter head's input projection: N = d, K = 2 d
            partmax = std::max(partmax, (size_t)std::max(choose_split(MAX_ROWS, d.d_model / 16, 2 * d.d_model / 32).ksplit, ks_cap()) *
                                            MAX_ROWS * d.d_model * sizeof(float));
        for (int i = 0; i < 5; ++i) {
            int ksplit = 1;
            if (d.dtype == METASD_BF16) ksplit = choose_split(MAX_ROWS, ns[i] / 16, ks[i] / 32).ksplit;
            // a smaller m never needs more splits for LDS, but may use up to 8 for parallelism
            ksplit = std::max(ksplit, ks_cap());
            partmax = std::max(partmax, (size_t)ksplit * MAX_ROWS * ns[i] * sizeof(float));
            if (c.batch > 1) {
                const int kr = d.dtype == METASD_BF16 ? std::min(8, std::max(1, ks[i] / 32 / 8)) : 1;   // any split choose_split_rows may take
                partmax = std::max(partmax, (size_t)std::max(kr, ksplit) * MAX_ROWS * c.batch * ns[i] * sizeof(float));
            }
        }
    };
    acc(t);
    for (int k = 0; k < c.K; ++k) acc(dr[k]);
    const int nchunks = (c.max_ctx + ATT_CH - 1) / ATT_CH;
    Layout L{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes); return at; };
    const size_t B = (size_t)c.batch, RM = (size_t)MAX_ROWS * B;   // sequences, rows of the largest block
    L.hist = take(B * c.max_ctx * 4);
    L.h = take(RM * dmax * 4);
    L.h2 = take((size_t)MAX_ROWS * dmax * 4);
    L.xn = take(RM * dmax * 4);
    L.part = take(partmax);
    L.part2 = take(partmax);
    L.gx = take(gxmax);                                            // tagged partial sums of the residual GEMMs
    L.ssq = take((size_t)(dmax / 16 + 1) * 16 * 4);              // per tile group (or per tile) and row
    L.inv = take(64);
    L.q = take(RM * dmax * 4);
    L.ao = take(RM * dmax * 4);
    L.act = take(RM * fmax * 4 * 2);          // also the fused gate | up result
    L.apart = take(B * hmax * nchunks * 16 * (hdmax + 2) * 4);
    L.rope = take(RM * (hdmax / 2) * sizeof(double2));
    L.P = take(B * (c.gamma_max + 1) * vmax * 4);
    L.Q = take(B * c.gamma_max * vmax * 4);
    L.cand = take(B * (c.gamma_max + 1) * sizeof(int2));
    L.bd = take(B * c.gamma_max * sizeof(double));
    L.res = take(std::max<size_t>(128, B * 12));                   // batch 1: also the path of a tree round (2 + 15 words)
    L.draft = take(std::max<size_t>(64, B * (c.gamma_max + 1) * 4)); // chain: gamma tokens per sequence; tree: one per node
    L.tstep = take(TREE_MAX * sizeof(int2));                       // sampled tree rounds: the decision of every node
    L.bar = take(sizeof(GridBar));                                 // bd .. bar: the span read back after every round, kept small
    L.xchg = take(B * (c.gamma_max + 1) * AS_XCHG_BYTES);
    // drafter heads: the target's feature of every processed position, and the head's estimate of the latest one
    L.feat = take(c.feature_heads ? (size_t)c.max_ctx * t.d_model * 4 : 0);
    L.fest = take(c.feature_heads ? (size_t)TREE_MAX * t.d_model * 4 : 0);   // one row per tree node (a chain uses row 0)
    int lmax = t.n_layers;
    for (int k = 0; k < c.K; ++k) lmax = std::max(lmax, dr[k].n_layers);
    L.table_stride = align_up((size_t)(1 + PER_LAYER * lmax + 2) * sizeof(void*));
    L.tables = take(L.table_stride * (size_t)(c.K + 1));
    L.total = o;
    return L;
}

// uniform in [0,1) at Philox counter (seq, round, pos, stream): the host twin of philox_uniform
float host_philox_uniform(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3) {
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c0 = n0; c1 = (uint32_t)p1; c2 = n2; c3 = (uint32_t)p0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return (float)(c0 >> 8) * (1.0f / 16777216.0f);
}

// Drafter-selection state of one sequence.  UCB is Alg. 2; the others are the algorithms of the
// paper's appendix on switching costs and non-stationary rewards, and its EXP3 / random baselines.
struct Bandit {
    int K = 0, t = 0, policy = METASD_POLICY_UCB, window = 0;
    double beta = 1.0, param = 1.0;
    uint64_t seed = 0;
    uint32_t seq = 0;           // sequence id: first Philox counter word of this bandit's draws
    std::vector<double> mu;     // reported estimate per arm
    std::vector<int> n;         // reported count per arm
    std::vector<double> aux;    // D-UCB: discounted reward sums; EXP3: weights; SH: reward sums of the phase
    std::vector<int> last;      // D-UCB: round of the arm's latest pull
    std::vector<double> prob;   // EXP3: probabilities of the latest select
    std::vector<std::pair<int, double>> recent;   // SW-UCB: (arm, reward) of the rounds in the window, oldest first
    std::vector<int> alive;     // SH: surviving arms, ascending
    int sh_phases = 0, sh_pos = 0;

    void init(const metasd_config& c) {
        K = c.K; beta = c.ucb_beta; policy = c.policy; param = c.policy_param; window = c.policy_window; seed = c.seed;
        reset();
    }
    void reset() {
        t = 0;
        mu.assign(K, 0.0); n.assign(K, 0);
        aux.assign(K, policy == METASD_POLICY_EXP3 ? 1.0 : 0.0);
        last.assign(K, 0);
        prob.assign(K, 1.0 / std::max(K, 1));
        recent.clear();
        alive.resize(K);
        for (int i = 0; i < K; ++i) alive[i] = i;
        sh_phases = 0;
        for (int v = 1; v < K; v <<= 1) ++sh_phases;   // ceil(log2 K)
        sh_pos = 0;
    }
    int ucb_argmax() const {
        int best = 0;
        double bs = -INFINITY;
        for (int i = 0; i < K; ++i) {
            const double s = mu[i] + beta * std::sqrt(2.0 * std::log((double)t) / (double)n[i]);
            if (s > bs) { bs = s; best = i; }
        }
        return best;
    }
    static int draw(const std::vector<double>& p, double u) {   // first arm whose cumulative probability exceeds u
        double c = 0.0;
        for (size_t i = 0; i < p.size(); ++i) {
            c += p[i];
            if (c > u) return (int)i;
        }
        return (int)p.size() - 1;
    }
    int sh_pulls() const { return std::max(1, window / ((int)alive.size() * std::max(sh_phases, 1))); }

    int select() {
        switch (policy) {
            case METASD_POLICY_UCB:
            case METASD_POLICY_DUCB:
                return t < K ? t : ucb_argmax();
            case METASD_POLICY_SWUCB:
                if (t < K) return t;
                for (int i = 0; i < K; ++i)
                    if (n[i] == 0) return i;            // no pull left in the window: no estimate, try it
                return ucb_argmax();
            case METASD_POLICY_EXP3: {
                double tot = 0.0;
                for (double w : aux) tot += w;
                for (int i = 0; i < K; ++i) prob[i] = (1.0 - param) * (aux[i] / tot) + param / (double)K;
                return draw(prob, (double)host_philox_uniform(seed, seq, (uint32_t)t, 0u, 3u));
            }
            case METASD_POLICY_SH:
                return alive.size() == 1 ? alive[0] : alive[sh_pos / sh_pulls()];
            default: {                                   // METASD_POLICY_RANDOM
                std::vector<double> p(K, 1.0 / (double)K);
                return draw(p, (double)host_philox_uniform(seed, seq, (uint32_t)t, 0u, 3u));
            }
        }
    }

    void plain_mean(int k, double r) { mu[k] = (mu[k] * (double)n[k] + r) / (double)(n[k] + 1); n[k] += 1; }

    void update(int k, double r) {
        switch (policy) {
            case METASD_POLICY_DUCB:
                // discounted sum carried from the arm's latest pull: S <- S gamma^(t - t_last) + r
                aux[k] = (n[k] > 0 ? aux[k] * std::pow(param, (double)(t - last[k])) : 0.0) + r;
                last[k] = t;
                n[k] += 1;
                mu[k] = aux[k] / (double)n[k];
                break;
            case METASD_POLICY_SWUCB: {
                recent.emplace_back(k, r);
                if ((int)recent.size() > window) recent.erase(recent.begin());
                std::vector<double> s(K, 0.0);
                std::fill(n.begin(), n.end(), 0);
                for (const auto& e : recent) { s[e.first] += e.second; n[e.first] += 1; }
                for (int i = 0; i < K; ++i) mu[i] = n[i] ? s[i] / (double)n[i] : 0.0;
                break;
            }
            case METASD_POLICY_EXP3: {
                aux[k] *= std::exp(param * (r / prob[k]) / (double)K);
                const double big = *std::max_element(aux.begin(), aux.end());
                if (big > 1e100) {                       // exact power-of-two rescale, probabilities unchanged
                    int e;
                    std::frexp(big, &e);
                    for (double& w : aux) w = std::ldexp(w, -e);
                }
                plain_mean(k, r);
                break;
            }
            case METASD_POLICY_SH:
                plain_mean(k, r);
                if (alive.size() > 1) {
                    aux[k] += r;
                    if (++sh_pos == (int)alive.size() * sh_pulls()) {   // phase over: keep the better half
                        std::vector<int> order = alive;
                        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return aux[a] > aux[b]; });
                        order.resize((alive.size() + 1) / 2);
                        std::sort(order.begin(), order.end());
                        alive = order;
                        std::fill(aux.begin(), aux.end(), 0.0);
                        sh_pos = 0;
                    }
                }
                break;
            default:                                     // UCB (Alg. 2 mean update), RANDOM
                plain_mean(k, r);
                break;
        }
        t += 1;
    }
};


enum Phase { PH_NONE = 0, PH_READY, PH_DRAFTED, PH_VERIFIED, PH_TREE_DRAFTED, PH_TREE_VERIFIED };

}  // namespace

struct metasd_ctx {
    metasd_config cfg{};
    Model target;
    std::vector<Model> drafters;
    hipStream_t stream = nullptr;
    char* ws = nullptr;
    Layout lay{};
    struct SeqState {
        std::vector<int32_t> hist;   // host mirror of committed tokens
        int l = 0;                   // committed tokens
        int cur_k = -1;              // drafter of the running round
        int round = 0;               // rounds completed since this sequence's context was set: the round word of its Philox counters
        bool ready = false;          // a context has been set
        Bandit bandit;
    };
    std::vector<SeqState> sq;        // one per sequence (cfg.batch)
    int cur_gamma = 0;
    Phase phase = PH_NONE;
    // Pinned host mirror of the workspace span [lay.bd, lay.bar + sizeof(GridBar)): the BD terms, the result words
    // (n_acc, token, mask per sequence), the draft tokens and the abort flag come back in one copy per accept.
    char* hspan = nullptr;
    size_t span_bytes() const { return lay.bar + sizeof(GridBar) - lay.bd; }
    template <typename U> const U* mirror(size_t ws_offset) const { return reinterpret_cast<const U*>(hspan + (ws_offset - lay.bd)); }
    int fetch_results() {          // copy the span and wait for it (the only synchronisation of a round)
        hipError_t e = hipMemcpyAsync(hspan, ws + lay.bd, span_bytes(), hipMemcpyDeviceToHost, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) return fail(METASD_E_HIP, "reading back the accept results: %s", hipGetErrorString(e));
        return 0;
    }
    std::string err;
    // optional per-launch timing of the three bandwidth-bound kernels (metasd_profile)
    struct ProfRec { hipEvent_t a, b; int kind; double bytes; int n, k, m, model; };   // GEMM launches: N, K, rows, model (-1 target, else drafter)
    bool prof_on = false;
    bool fullk = true;               // residual GEMMs whose input fits in LDS run without split-K (METASD_GEMM_FULLK=0: off)
    bool grouped_on = true;          // batched drafting: one forward per step for all arms (METASD_DRAFT_GROUPED=0: one per arm)
    int att_cpw = 0;                 // batched attention: chunks per workgroup, 0 = by the rule in attention_seg_hd (METASD_ATT_CPW=1..64 forces one)
    int rows_tpb = 0;                // many-row GEMM: tiles per workgroup, 0 = by the cost model (METASD_ROWS_TPB=4|6|8|12 forces one)
    bool fullk_roll = true;          // .. and larger inputs with rolling private staging (METASD_GEMM_ROLL=0: sibling reduction instead)
    bool gemm_reduce = true;         // bf16 models: residual GEMMs reduce their split-K partials themselves (METASD_GEMM_REDUCE=0: off)
    float cur_eps = 1e-5f;           // rms_eps of the model whose forward is being launched
    bool fuse_small = true;          // short blocks of narrow bf16 models use the GEMMs with fused prologues (METASD_FUSE_SMALL=0: off)
    int n_cu = 0;
    const TreeBlk* tree = nullptr;   // set while a block of draft-tree nodes is being launched (positions and mask of its rows)
    bool head_est = false;           // a drafter head's forward takes its own estimates (d_fest) as the feature input (draft steps after the first)
    FeatSrc fsrc{};                  // .. row r the estimate fsrc.idx[r] (chain steps: 0; tree levels: the parent node's)
    TreeShape tshape{};              // the tree of the running round (metasd_draft_tree)
    int tdepth[TREE_MAX] = {};       // depth of every node, tlevel[d] = first node of depth d (tlevel[max depth + 1] = n)
    int tlevel[TREE_MAX + 2] = {};
    int tmaxdepth = 0;
    uint16_t tanc[TREE_MAX] = {};
    int accept_fallbacks = 0;        // accept steps taken again with one workgroup per position after an exchange timeout
    std::vector<ProfRec> prof;       // event pool
    size_t prof_used = 0;
    // Next free record, or nullptr when profiling is off / the pool is used up.  The launcher hands
    // the record's two events to the dispatch itself (hipExtLaunchKernelGGL), so they carry the
    // kernel's own begin and end times rather than those of marker packets around it.
    int cur_model = -1;              // model whose forward is being launched (-1 target, k drafter k): label of the timing records
    ProfRec* prof_take(int kind, double bytes, int n = 0, int k = 0, int m = 0) {
        if (!prof_on || prof_used >= prof.size()) return nullptr;
        ProfRec* r = &prof[prof_used++];
        r->kind = kind;
        r->bytes = bytes;
        r->n = n; r->k = k; r->m = m; r->model = cur_model;
        return r;
    }
    // for launches that cannot carry events (cooperative): marker events on the stream around them
    bool prof_begin(int kind, double bytes) {
        if (!prof_on || prof_used >= prof.size()) return false;
        prof[prof_used].kind = kind;
        prof[prof_used].bytes = bytes;
        return hipEventRecord(prof[prof_used].a, stream) == hipSuccess;
    }
    void prof_end() { (void)hipEventRecord(prof[prof_used].b, stream); ++prof_used; }

    int32_t* d_hist() const { return reinterpret_cast<int32_t*>(ws + lay.hist); }
    float* d_h() const { return reinterpret_cast<float*>(ws + lay.h); }
    void* d_xn() const { return ws + lay.xn; }
    float* d_part() const { return reinterpret_cast<float*>(ws + lay.part); }
    unsigned long long* d_gx() const { return reinterpret_cast<unsigned long long*>(ws + lay.gx); }
    float* d_ssq() const { return reinterpret_cast<float*>(ws + lay.ssq); }
    float* d_inv() const { return reinterpret_cast<float*>(ws + lay.inv); }
    unsigned long long* d_xchg() const { return reinterpret_cast<unsigned long long*>(ws + lay.xchg); }
    float* d_part_pp(int i) const { return reinterpret_cast<float*>(ws + (i ? lay.part2 : lay.part)); }
    float* d_h_pp(int i) const { return reinterpret_cast<float*>(ws + (i ? lay.h2 : lay.h)); }
    void* d_q() const { return ws + lay.q; }
    void* d_ao() const { return ws + lay.ao; }
    void* d_act() const { return ws + lay.act; }
    float* d_apart() const { return reinterpret_cast<float*>(ws + lay.apart); }
    double2* d_rope() const { return reinterpret_cast<double2*>(ws + lay.rope); }
    float* d_P() const { return reinterpret_cast<float*>(ws + lay.P); }
    float* d_Q() const { return reinterpret_cast<float*>(ws + lay.Q); }
    int2* d_cand() const { return reinterpret_cast<int2*>(ws + lay.cand); }
    int2* d_tstep() const { return reinterpret_cast<int2*>(ws + lay.tstep); }
    float* d_feat() const { return reinterpret_cast<float*>(ws + lay.feat); }
    float* d_fest() const { return reinterpret_cast<float*>(ws + lay.fest); }
    double* d_bd() const { return reinterpret_cast<double*>(ws + lay.bd); }
    int32_t* d_res() const { return reinterpret_cast<int32_t*>(ws + lay.res); }
    int32_t* d_draft() const { return reinterpret_cast<int32_t*>(ws + lay.draft); }
    GridBar* d_bar() const { return reinterpret_cast<GridBar*>(ws + lay.bar); }

    int fail(int code, const char* fmt, ...) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        err = buf;
        return code;
    }
};

namespace {

#define HIP_TRY(ctx, expr)                                                                              \
    do {                                                                                                \
        hipError_t e_ = (expr);                                                                         \
        if (e_ != hipSuccess) return (ctx)->fail(METASD_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

#define LAUNCH_CHECK(ctx, name)                                                                              \
    do {                                                                                                     \
        hipError_t e_ = hipGetLastError();                                                                   \
        if (e_ != hipSuccess) return (ctx)->fail(METASD_E_HIP, "launch %s: %s", name, hipGetErrorString(e_)); \
    } while (0)

// ---- GEMM launcher: out[.][r][n] over up to three matrices concatenated along n.
// Returns the number of split-K partials written to `part` (their split stride is m*N);
// when direct_out != nullptr the summed result is written there instead and 0 is returned.
template <typename T>
int gemm(metasd_ctx* c, const void* x, int ldx, int m, int K, const void* W0, int n0, const void* W1, int n1,
         const void* W2, int n2, float* direct_out, int* nsplit_out, size_t x_lo_off = 0, const float* ssq = nullptr,
         int ntg = 0, float* inv_out = nullptr, int inv_row0 = 0);

template <>
int gemm<float>(metasd_ctx* c, const void* x, int ldx, int m, int K, const void* W0, int n0, const void* W1, int n1,
                const void* W2, int n2, float* direct_out, int* nsplit_out, size_t, const float*, int, float*, int) {
    const int N = n0 + n1 + n2;
    float* out = direct_out ? direct_out : c->d_part();
    hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 3) / 4), dim3(256), 0, c->stream, (const float*)x, ldx, m, K,
                       (const float*)W0, (const float*)W1, (const float*)W2, n0, n0 + n1, N, out);
    LAUNCH_CHECK(c, "gemm_f32");
    *nsplit_out = direct_out ? 0 : 1;
    return 0;
}

template <>
// x: the activations as two bf16 arrays, hi at x and lo x_lo_off elements behind it (see store_split4).
// ssq != nullptr: x is h * gain of a residual epilogue, not yet normalised; workgroup 0 writes 1/rms per row
// to inv_out (rows inv_row0 ..) for the consumers of this GEMM's output, and a direct result is scaled by it.
int gemm<bf16_t>(metasd_ctx* c, const void* x, int ldx, int m, int K, const void* W0, int n0, const void* W1, int n1,
                 const void* W2, int n2, float* direct_out, int* nsplit_out, size_t x_lo_off, const float* ssq, int ntg,
                 float* inv_out, int inv_row0) {
    const int N = n0 + n1 + n2;
    const int ntiles = N / 16, kchunks = K / 32;
    const Split s = choose_split(m, ntiles, kchunks);
    const bool direct = direct_out && s.ksplit == 1 && !ssq;     // a scaled result always goes through sum_partials
    float* out = direct ? direct_out : c->d_part();
    const int groups = (ntiles + s.tpb - 1) / s.tpb;
    // algorithmic bytes: every weight once, the activations once, the result once
    metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_GEMM, (double)N * K * 2 + (double)m * K * 4 + (double)m * N * 4, N, K, m);
    GemmPro plain{};
    plain.sstride = x_lo_off;
    if (ssq) { plain.src = ssq; plain.row0 = inv_row0; plain.ns = ntg; plain.h_out = inv_out + inv_row0; plain.eps = c->cur_eps; }
    hipExtLaunchKernelGGL(gemm_bf16_kernel<PRO_PLAIN>, dim3(groups * s.ksplit), dim3(256), (uint32_t)s.lds, c->stream,
                          pr ? pr->a : nullptr, pr ? pr->b : nullptr, 0u, (const float*)x, ldx, m, K, (const bf16_t*)W0,
                          (const bf16_t*)W1, (const bf16_t*)W2, n0 / 16, (n0 + n1) / 16, ntiles, out, N, s.ksplit, s.cps, s.tpb,
                          plain, GemmEpi{});
    LAUNCH_CHECK(c, "gemm_bf16");
    if (direct_out && !direct) {
        const size_t n = (size_t)m * N;
        hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, c->d_part(),
                           s.ksplit, n, n, direct_out, ssq ? (const float*)(inv_out + inv_row0) : nullptr, N);
        LAUNCH_CHECK(c, "sum_partials");
    }
    *nsplit_out = direct_out ? 0 : s.ksplit;
    return 0;
}

// The same projection without split-K (gemm_fullk_residual_kernel): used when the input block fits in LDS
// and there are enough tiles to occupy the CUs.
bool fullk_ok(const metasd_ctx* c, int m, int K, int ntiles, size_t* lds_out) {
    const int cpw = (K / 32 + 7) / 8;
    const size_t lds = (size_t)2 * 8 * m * (cpw * 4 + 1) * 16 + (size_t)8 * 64 * 16;
    *lds_out = lds;
    return c->fullk && lds <= FULLK_LDS_MAX && ntiles * 4 >= c->n_cu * 3;
}

// bf16 GEMM into the residual stream (attention output / FFN down projection): the split-K siblings reduce
// among themselves and the last one updates h, writes h * gain in the two-bf16 form for the next GEMM and the
// per-tile-group sums of squares (EPI_RESIDUAL in kernels.h).  N = d_model.
int gemm_residual(metasd_ctx* c, const void* x, int ldx, int m, int K, const void* W, int N, size_t x_lo_off, float* h,
                  const void* gain_next, float* xsplit, float* ssq, int* ntg_out) {
    const int ntiles = N / 16, kchunks = K / 32;
    size_t lds_full = 0;
    if (fullk_ok(c, m, K, ntiles, &lds_full)) {
        metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_GEMM, (double)N * K * 2 + (double)m * K * 4 + (double)m * N * 4, N, K, m);
        hipExtLaunchKernelGGL(gemm_fullk_residual_kernel, dim3(ntiles), dim3(512), (uint32_t)lds_full, c->stream, pr ? pr->a : nullptr,
                              pr ? pr->b : nullptr, 0u, (const bf16_t*)x, x_lo_off, ldx, m, K, (const bf16_t*)W, ntiles, N, h,
                              (const bf16_t*)gain_next, xsplit, ssq);
        LAUNCH_CHECK(c, "gemm_bf16 (full-K residual)");
        *ntg_out = ntiles;
        return 0;
    }
    // up to 8 rows: two private staging buffers per wavefront; 9 .. 16 rows: one (see the kernel)
    const size_t lds_roll = (size_t)8 * (m <= 8 ? 4 : 2) * m * (GEMM_U * 4 + 1) * 16 + (size_t)8 * 64 * 16;
    if (c->fullk && c->fullk_roll && m <= 16 && ntiles * 4 >= c->n_cu * 3 && kchunks >= 8 * GEMM_U && lds_roll <= FULLK_LDS_MAX) {
        metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_GEMM, (double)N * K * 2 + (double)m * K * 4 + (double)m * N * 4, N, K, m);
        hipEvent_t ea = pr ? pr->a : nullptr, eb = pr ? pr->b : nullptr;
#define ROLL_GO(XB, DB) hipExtLaunchKernelGGL((gemm_fullk_roll_residual_kernel<XB, DB>), dim3(ntiles), dim3(512), (uint32_t)lds_roll, c->stream, ea, eb, 0u, \
                                              (const bf16_t*)x, x_lo_off, ldx, m, K, (const bf16_t*)W, ntiles, N, h, (const bf16_t*)gain_next, xsplit, ssq)
        if (m <= 6) ROLL_GO(3, true);
        else if (m <= 8) ROLL_GO(4, true);
        else if (m <= 10) ROLL_GO(5, false);
        else if (m <= 12) ROLL_GO(6, false);
        else if (m <= 14) ROLL_GO(7, false);
        else ROLL_GO(8, false);
#undef ROLL_GO
        LAUNCH_CHECK(c, "gemm_bf16 (full-K residual, rolling staging)");
        *ntg_out = ntiles;
        return 0;
    }
    const Split s = choose_split(m, ntiles, kchunks);
    const int groups = (ntiles + s.tpb - 1) / s.tpb;
    if ((size_t)(s.ksplit - 1) * m * N * 8 > c->lay.ssq - c->lay.gx)
        return c->fail(METASD_E_WORKSPACE, "residual GEMM (m %d, K %d, N %d): %d split-K siblings exceed the exchange area of the workspace", m, K, N, s.ksplit);
    metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_GEMM, (double)N * K * 2 + (double)m * K * 4 + (double)m * N * 4, N, K, m);
    GemmPro plain{};
    plain.sstride = x_lo_off;
    GemmEpi epi{};
    epi.xw = c->d_gx(); epi.h = h; epi.gain = (const bf16_t*)gain_next; epi.xsplit = xsplit; epi.ssq = ssq;
    epi.abort = &reinterpret_cast<GridBar*>(c->d_bar())->abort;
    epi.epoch = next_epoch();
    epi.spin_limit = std::max(0, env_int("METASD_GEMM_SPIN_LIMIT", 1 << 18));
    hipExtLaunchKernelGGL((gemm_bf16_kernel<PRO_PLAIN, EPI_RESIDUAL>), dim3(groups * s.ksplit), dim3(256), (uint32_t)s.lds, c->stream,
                          pr ? pr->a : nullptr, pr ? pr->b : nullptr, 0u, (const float*)x, ldx, m, K, (const bf16_t*)W,
                          (const bf16_t*)W, (const bf16_t*)W, ntiles, ntiles, ntiles, (float*)nullptr, N, s.ksplit, s.cps, s.tpb,
                          plain, epi);
    LAUNCH_CHECK(c, "gemm_bf16 (residual epilogue)");
    *ntg_out = groups;
    return 0;
}

// bf16 GEMM whose prologue forms the activations itself (PRO_NORM / PRO_ACT / PRO_COMBINE, see kernels.h).
// Partials go to part_out (split stride m*N), or, when direct_out is given and no split is needed, there.
template <int PRO>
int gemm_pro(metasd_ctx* c, const GemmPro& pro, int m, int K, const void* W0, int n0, const void* W1, int n1, const void* W2,
             int n2, float* part_out, float* direct_out, int* nsplit_out) {
    const int N = n0 + n1 + n2;
    const int ntiles = N / 16, kchunks = K / 32;
    const Split s = choose_split(m, ntiles, kchunks);
    float* out = (direct_out && s.ksplit == 1) ? direct_out : part_out;
    const int groups = (ntiles + s.tpb - 1) / s.tpb;
    const size_t lds = s.lds + (PRO == PRO_NORM ? (size_t)m * K * 4 + (size_t)m * 16 : 0);
    metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_GEMM, (double)N * K * 2 + (double)m * K * 4 + (double)m * N * 4, N, K, m);
    hipExtLaunchKernelGGL(gemm_bf16_kernel<PRO>, dim3(groups * s.ksplit), dim3(256), (uint32_t)lds, c->stream, pr ? pr->a : nullptr,
                          pr ? pr->b : nullptr, 0u, (const float*)nullptr, K, m, K, (const bf16_t*)W0, (const bf16_t*)W1,
                          (const bf16_t*)W2, n0 / 16, (n0 + n1) / 16, ntiles, out, N, s.ksplit, s.cps, s.tpb, pro, GemmEpi{});
    LAUNCH_CHECK(c, "gemm_bf16 (fused prologue)");
    if (direct_out && s.ksplit > 1) {
        const size_t n = (size_t)m * N;
        hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, part_out, s.ksplit, n, n,
                           direct_out, (const float*)nullptr, N);
        LAUNCH_CHECK(c, "sum_partials");
    }
    *nsplit_out = direct_out ? 0 : s.ksplit;
    return 0;
}

// combine == false: only the per-chunk records (the consumer merges them itself)
// qi (bf16 caches, head_dim >= 64 only): q and the block's own K / V rows come from the QKV projection's partial sums inside
// the attention kernel (no separate rope launch)
template <typename T, int HD>
int attention_hd(metasd_ctx* c, const Model& M, int L, int pos0, int m, bool combine, const QkvIn* qi) {
    const metasd_model_desc& d = M.d;
    const size_t plane = (size_t)d.n_kv_heads * c->cfg.max_ctx * HD;
    const T* kc = (const T*)M.kv + (size_t)L * 2 * plane;
    const T* vc = kc + plane;
    const int nchunks = (pos0 + m + ATT_CH - 1) / ATT_CH;
    const float scale = 1.0f / sqrtf((float)HD);
    // algorithmic bytes: K and V of every cached position once per KV head, q in, partials out
    metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_ATTN, 2.0 * d.n_kv_heads * (double)(pos0 + m) * HD * sizeof(T) +
                                                                 (double)m * d.n_heads * HD * 4);
    hipEvent_t ea = pr ? pr->a : nullptr, eb = pr ? pr->b : nullptr;
    if constexpr (sizeof(T) == 2 && HD >= 64) {
        if (qi)
            hipExtLaunchKernelGGL((attn_partial_mfma_qkv_kernel<HD>), dim3(nchunks, d.n_heads), dim3(256), 0u, c->stream, ea, eb, 0u, *qi,
                                  kc, vc, m, pos0, d.n_heads, d.n_kv_heads, c->cfg.max_ctx, scale, c->d_apart(), nchunks,
                                  c->tree ? *c->tree : TreeBlk{});
        else if (c->tree)
            hipExtLaunchKernelGGL((attn_partial_mfma_tree_kernel<HD>), dim3(nchunks, d.n_heads), dim3(256), 0u, c->stream, ea, eb, 0u,
                                  (const float*)c->d_q(), kc, vc, m, pos0, d.n_heads, d.n_kv_heads, c->cfg.max_ctx, scale,
                                  c->d_apart(), nchunks, *c->tree);
        else
            hipExtLaunchKernelGGL((attn_partial_mfma_kernel<HD>), dim3(nchunks, d.n_heads), dim3(256), 0u, c->stream, ea, eb, 0u,
                                  (const float*)c->d_q(), kc, vc, m, pos0, d.n_heads, d.n_kv_heads, c->cfg.max_ctx, scale,
                                  c->d_apart(), nchunks);
    } else {
        if (c->tree)
            hipExtLaunchKernelGGL((attn_partial_tree_kernel<T, HD>), dim3(nchunks, d.n_heads), dim3(256), 0u, c->stream, ea, eb, 0u,
                                  (const float*)c->d_q(), kc, vc, m, pos0, d.n_heads, d.n_kv_heads, c->cfg.max_ctx, scale,
                                  c->d_apart(), nchunks, *c->tree);
        else
            hipExtLaunchKernelGGL((attn_partial_kernel<T, HD>), dim3(nchunks, d.n_heads), dim3(256), 0u, c->stream, ea, eb, 0u,
                                  (const float*)c->d_q(), kc, vc, m, pos0, d.n_heads, d.n_kv_heads, c->cfg.max_ctx, scale,
                                  c->d_apart(), nchunks);
    }
    LAUNCH_CHECK(c, "attn_partial");
    if (!combine) return 0;
    hipLaunchKernelGGL((attn_combine_kernel<T, HD>), dim3(d.n_heads, m), dim3(HD), 0, c->stream, c->d_apart(), nchunks,
                       d.n_heads, (float*)c->d_ao(), sizeof(T) == 2 ? 1 : 0);
    LAUNCH_CHECK(c, "attn_combine");
    return 0;
}

template <typename T>
int attention(metasd_ctx* c, const Model& M, int L, int pos0, int m, bool combine = true, const QkvIn* qi = nullptr) {
    if (qi && (sizeof(T) != 2 || M.hd < 64)) return c->fail(METASD_E_INVALID, "attention: fused q/k/v needs a bf16 cache and head_dim >= 64");
    switch (M.hd) {
        case 32: return attention_hd<T, 32>(c, M, L, pos0, m, combine, nullptr);
        case 64: return attention_hd<T, 64>(c, M, L, pos0, m, combine, qi);
        default:
            if constexpr (sizeof(T) == 2) return attention_hd<T, 128>(c, M, L, pos0, m, combine, qi);
            return c->fail(METASD_E_INVALID, "fp32 head_dim 128 unsupported");
    }
}

// Forward of m <= 16 rows whose tokens are hist[pos0 .. pos0+m) at positions pos0..; appends K/V.
// logits: nullptr = none; otherwise rows [first_row, m) of the block get logits, written
// consecutively to `logits` (row stride V).
template <typename T>
int forward_rows(metasd_ctx* c, Model& M, int pos0, int m, float* logits, int first_row) {
    const metasd_model_desc& d = M.d;
    const int D = d.d_model, H = d.n_heads, KH = d.n_kv_heads, hd = M.hd, F = d.d_ffn, V = d.vocab;
    const int DQ = H * hd, DKV = KH * hd;
    hipStream_t st = c->stream;
    float* h = c->d_h();
    float* xn = (float*)c->d_xn();
    float* part = c->d_part();
    int ns = 0, rc;
    constexpr int split = sizeof(T) == 2 ? 1 : 0;   // bf16 models: activations for the GEMM are stored as two bf16 arrays
    hipLaunchKernelGGL(embed_rope_kernel<T>, dim3(m), dim3(256), 0, st, c->d_hist() + pos0, (const T*)M.w[0], D, h, pos0, hd, d.rope_theta,
                       c->d_rope(), c->tree ? *c->tree : TreeBlk{});
    LAUNCH_CHECK(c, "embed + rope table");
    if (M.head) {
        // a drafter head starts from W_fc . [embedding ; feature of the position before] instead of the embedding
        float* cat = (float*)c->d_act();
        hipLaunchKernelGGL(feat_cat_kernel, dim3(m), dim3(256), 0, st, (const float*)h, (const float*)c->d_feat(),
                           c->head_est ? (const float*)c->d_fest() : (const float*)nullptr, c->fsrc, pos0, D, cat, split);
        LAUNCH_CHECK(c, "feat_cat");
        int dummy;
        if ((rc = gemm<T>(c, cat, 2 * D, m, 2 * D, M.fc, D, nullptr, 0, nullptr, 0, h, &dummy, (size_t)m * 2 * D))) return rc;
    }
    for (int L = 0; L < d.n_layers; ++L) {
        // h += previous FFN output (split partials); xn = norm(h)
        hipLaunchKernelGGL(addnorm_kernel<T>, dim3(m), dim3(1024), 0, st, h, part, ns, (size_t)m * D, D, (const T*)M.layer_w(L, 0),
                           d.rms_eps, xn, split);
        LAUNCH_CHECK(c, "addnorm");
        if ((rc = gemm<T>(c, xn, D, m, D, M.layer_w(L, 1), DQ, M.layer_w(L, 2), DKV, M.layer_w(L, 3), DKV, nullptr, &ns, (size_t)m * D))) return rc;
        const int NQKV = DQ + 2 * DKV;
        const size_t plane = (size_t)KH * c->cfg.max_ctx * hd;
        T* kc = (T*)M.kv + (size_t)L * 2 * plane;
        hipLaunchKernelGGL(rope_kv_kernel<T>, dim3((H + 2 * KH + 3) / 4, m), dim3(256), 0, st, part, ns, (size_t)m * NQKV, NQKV, pos0, H, KH,
                           hd, (const double2*)c->d_rope(), (float*)c->d_q(), kc, kc + plane, c->cfg.max_ctx, sizeof(T) == 2 ? 1 : 0,
                           (sizeof(T) == 2 && hd >= 64) ? 1 : 0, (const float*)nullptr);
        LAUNCH_CHECK(c, "rope_kv");
        if ((rc = attention<T>(c, M, L, pos0, m))) return rc;
        if ((rc = gemm<T>(c, c->d_ao(), DQ, m, DQ, M.layer_w(L, 4), D, nullptr, 0, nullptr, 0, nullptr, &ns, (size_t)m * DQ))) return rc;
        hipLaunchKernelGGL(addnorm_kernel<T>, dim3(m), dim3(1024), 0, st, h, part, ns, (size_t)m * D, D, (const T*)M.layer_w(L, 5),
                           d.rms_eps, xn, split);
        LAUNCH_CHECK(c, "addnorm");
        if (d.act == METASD_SWIGLU) {
            if ((rc = gemm<T>(c, xn, D, m, D, M.layer_w(L, 6), F, M.layer_w(L, 7), F, nullptr, 0, nullptr, &ns, (size_t)m * D))) return rc;
        } else {
            if ((rc = gemm<T>(c, xn, D, m, D, M.layer_w(L, 7), F, nullptr, 0, nullptr, 0, nullptr, &ns, (size_t)m * D))) return rc;
        }
        const size_t nact = (size_t)m * F;
        const int NF = (d.act == METASD_SWIGLU ? 2 : 1) * F;
        hipLaunchKernelGGL(ffn_act4_kernel, dim3((unsigned)((nact / 4 + 255) / 256)), dim3(256), 0, st, part, ns, (size_t)m * NF, m, F,
                           d.act, (float*)c->d_act(), split, (const float*)nullptr);
        LAUNCH_CHECK(c, "ffn_act");
        if ((rc = gemm<T>(c, c->d_act(), F, m, F, M.layer_w(L, 8), D, nullptr, 0, nullptr, 0, nullptr, &ns, (size_t)m * F))) return rc;
    }
    if (logits || c->cfg.feature_heads) {          // with drafter heads the finished residual rows are wanted in any case
        hipLaunchKernelGGL(addnorm_kernel<T>, dim3(m), dim3(1024), 0, st, h, part, ns, (size_t)m * D, D, (const T*)M.final_norm(),
                           d.rms_eps, xn, split);
        LAUNCH_CHECK(c, "addnorm");
    }
    if (logits) {
        int dummy;
        const void* xrow = split ? (const void*)((const bf16_t*)xn + (size_t)first_row * D) : (const void*)(xn + (size_t)first_row * D);
        if ((rc = gemm<T>(c, xrow, D, m - first_row, D, M.lm_head(), V, nullptr, 0, nullptr, 0, logits, &dummy, (size_t)m * D)))
            return rc;
    }
    return 0;
}

// bf16 models, general case: the two projections into the residual stream reduce their split-K partials
// inside the GEMM and hand the next GEMM h * gain directly (EPI_RESIDUAL); the kernels that consume a
// projection of such an input scale by 1/rms.  8 launches per layer instead of 10 (no add+norm kernels).
int forward_rows_residual(metasd_ctx* c, Model& M, int pos0, int m, float* logits, int first_row) {
    typedef bf16_t T;
    const metasd_model_desc& d = M.d;
    const int D = d.d_model, H = d.n_heads, KH = d.n_kv_heads, hd = M.hd, F = d.d_ffn, V = d.vocab;
    const int DQ = H * hd, DKV = KH * hd, NQKV = DQ + 2 * DKV;
    hipStream_t st = c->stream;
    float* h = c->d_h();
    float* xn = (float*)c->d_xn();
    float* part = c->d_part();
    float* ssq = c->d_ssq();
    float* inv = c->d_inv();
    int ns = 0, rc, ntg = 0;
    c->cur_eps = d.rms_eps;
    hipLaunchKernelGGL(embed_rope_kernel<T>, dim3(m), dim3(256), 0, st, c->d_hist() + pos0, (const T*)M.w[0], D, h, pos0, hd, d.rope_theta,
                       c->d_rope(), c->tree ? *c->tree : TreeBlk{});
    LAUNCH_CHECK(c, "embed + rope table");
    if (M.head) {
        // a drafter head starts from W_fc . [embedding ; feature of the position before] instead of the embedding (as in forward_rows)
        float* cat = (float*)c->d_act();
        hipLaunchKernelGGL(feat_cat_kernel, dim3(m), dim3(256), 0, st, (const float*)h, (const float*)c->d_feat(),
                           c->head_est ? (const float*)c->d_fest() : (const float*)nullptr, c->fsrc, pos0, D, cat, 1);
        LAUNCH_CHECK(c, "feat_cat");
        int dummy;
        if ((rc = gemm<T>(c, cat, 2 * D, m, 2 * D, M.fc, D, nullptr, 0, nullptr, 0, h, &dummy, (size_t)m * 2 * D))) return rc;
    }
    // first norm: a plain RMSNorm of the embedding rows (normalised x, no scaling downstream)
    hipLaunchKernelGGL(addnorm_kernel<T>, dim3(m), dim3(1024), 0, st, h, part, 0, (size_t)m * D, D, (const T*)M.layer_w(0, 0), d.rms_eps,
                       xn, 1);
    LAUNCH_CHECK(c, "addnorm");
    bool scaled = false;            // does xn hold h * gain (true) or the normalised rows (false)?
    for (int L = 0; L < d.n_layers; ++L) {
        if ((rc = gemm<T>(c, xn, D, m, D, M.layer_w(L, 1), DQ, M.layer_w(L, 2), DKV, M.layer_w(L, 3), DKV, nullptr, &ns, (size_t)m * D,
                          scaled ? ssq : nullptr, ntg, inv, 0))) return rc;
        const size_t plane = (size_t)KH * c->cfg.max_ctx * hd;
        T* kc = (T*)M.kv + (size_t)L * 2 * plane;
        // (forming q / k / v inside the attention kernel, as the short-block path below does, was measured here and is slower
        // at the 7B shape: 3.32 against 3.29 ms per pass - the wider kernel loses what the launch saves)
        hipLaunchKernelGGL(rope_kv_kernel<T>, dim3((H + 2 * KH + 3) / 4, m), dim3(256), 0, st, part, ns, (size_t)m * NQKV, NQKV, pos0, H, KH, hd,
                           (const double2*)c->d_rope(), (float*)c->d_q(), kc, kc + plane, c->cfg.max_ctx, 1, hd >= 64 ? 1 : 0,
                           scaled ? (const float*)inv : nullptr);
        LAUNCH_CHECK(c, "rope_kv");
        if ((rc = attention<T>(c, M, L, pos0, m))) return rc;
        if ((rc = gemm_residual(c, c->d_ao(), DQ, m, DQ, M.layer_w(L, 4), D, (size_t)m * DQ, h, M.layer_w(L, 5), xn, ssq, &ntg))) return rc;
        if (d.act == METASD_SWIGLU) {
            if ((rc = gemm<T>(c, xn, D, m, D, M.layer_w(L, 6), F, M.layer_w(L, 7), F, nullptr, 0, nullptr, &ns, (size_t)m * D, ssq, ntg, inv, 0))) return rc;
        } else {
            if ((rc = gemm<T>(c, xn, D, m, D, M.layer_w(L, 7), F, nullptr, 0, nullptr, 0, nullptr, &ns, (size_t)m * D, ssq, ntg, inv, 0))) return rc;
        }
        const size_t nact = (size_t)m * F;
        const int NF = (d.act == METASD_SWIGLU ? 2 : 1) * F;
        hipLaunchKernelGGL(ffn_act4_kernel, dim3((unsigned)((nact / 4 + 255) / 256)), dim3(256), 0, st, part, ns, (size_t)m * NF, m, F, d.act,
                           (float*)c->d_act(), 1, (const float*)inv);
        LAUNCH_CHECK(c, "ffn_act");
        const void* gain_next = L + 1 < d.n_layers ? M.layer_w(L + 1, 0) : M.final_norm();
        if ((rc = gemm_residual(c, c->d_act(), F, m, F, M.layer_w(L, 8), D, (size_t)m * F, h, gain_next, xn, ssq, &ntg))) return rc;
        scaled = true;
    }
    if (logits) {
        int dummy;
        const void* xrow = (const void*)((const bf16_t*)xn + (size_t)first_row * D);
        if ((rc = gemm<T>(c, xrow, D, m - first_row, D, M.lm_head(), V, nullptr, 0, nullptr, 0, logits, &dummy, (size_t)m * D, ssq, ntg, inv,
                          first_row))) return rc;
    }
    return 0;
}

// Short blocks of narrow bf16 models (drafter steps; d_model <= 2048, METASD_FUSE_DMAX): the same forward with the add+norm, the FFN
// activation and the attention combine folded into the prologue of the GEMM that consumes them -
// 5 launches per layer instead of 10 (q / k / v are formed inside the attention kernel).  The residual stream and the partials ping-pong between two
// buffers, because a GEMM's workgroups read the old ones while others already write the new ones.
constexpr int fused_max_rows() { return 4; }
bool fused_small_ok(const Model& M, int m) {
    const metasd_model_desc& d = M.d;
    constexpr int dmax = 2048;
    // the add+norm prologue keeps the block's residual rows in LDS (m * d_model floats) beside the staged activations:
    // within the 64 KiB a kernel gets without asking for more
    return d.dtype == METASD_BF16 && m <= fused_max_rows() && d.d_model <= dmax && d.d_ffn <= 4 * dmax && M.hd >= 64 &&
           (size_t)m * d.d_model * 4 <= 40 * 1024;
}

int forward_rows_fused(metasd_ctx* c, Model& M, int pos0, int m, float* logits, int first_row) {
    typedef bf16_t T;
    const metasd_model_desc& d = M.d;
    const int D = d.d_model, H = d.n_heads, KH = d.n_kv_heads, hd = M.hd, F = d.d_ffn, V = d.vocab;
    const int DQ = H * hd, DKV = KH * hd, NQKV = DQ + 2 * DKV;
    hipStream_t st = c->stream;
    int hp = 0, pp = 0, ns = 0, rc;     // current residual buffer, current partials buffer, partials in it
    hipLaunchKernelGGL(embed_rope_kernel<T>, dim3(m), dim3(256), 0, st, c->d_hist() + pos0, (const T*)M.w[0], D, c->d_h_pp(0), pos0, hd,
                       d.rope_theta, c->d_rope(), c->tree ? *c->tree : TreeBlk{});
    LAUNCH_CHECK(c, "embed + rope table");
    auto norm_pro = [&](const void* gain, int row0) {
        GemmPro p{};
        p.src = c->d_h_pp(hp) + (size_t)row0 * D;
        p.part = c->d_part_pp(pp) + (size_t)row0 * D;
        p.h_out = c->d_h_pp(hp ^ 1) + (size_t)row0 * D;
        p.gain = (const bf16_t*)gain;
        p.sstride = (size_t)m * D;
        p.ns = ns;
        p.eps = d.rms_eps;
        return p;
    };
    const int nchunks = (pos0 + m + ATT_CH - 1) / ATT_CH;
    for (int L = 0; L < d.n_layers; ++L) {
        // QKV projection of norm(h + previous FFN output)
        if ((rc = gemm_pro<PRO_NORM>(c, norm_pro(M.layer_w(L, 0), 0), m, D, M.layer_w(L, 1), DQ, M.layer_w(L, 2), DKV, M.layer_w(L, 3), DKV,
                                     c->d_part_pp(pp ^ 1), nullptr, &ns))) return rc;
        hp ^= 1; pp ^= 1;
        const size_t plane = (size_t)KH * c->cfg.max_ctx * hd;
        T* kc = (T*)M.kv + (size_t)L * 2 * plane;
        // q, and the new K / V rows, are summed and rotated inside the attention kernel (no rope launch)
        {
            const QkvIn qi{c->d_part_pp(pp), ns, (size_t)m * NQKV, NQKV, (const double2*)c->d_rope(), nullptr, kc, kc + plane};
            if ((rc = attention<T>(c, M, L, pos0, m, false, &qi))) return rc;
        }
        // output projection of the merged attention output
        {
            GemmPro p{};
            p.src = c->d_apart(); p.nchunks = nchunks; p.hd = hd;
            if ((rc = gemm_pro<PRO_COMBINE>(c, p, m, DQ, M.layer_w(L, 4), D, nullptr, 0, nullptr, 0, c->d_part_pp(pp ^ 1), nullptr, &ns))) return rc;
            pp ^= 1;
        }
        // gate | up projection of norm(h + attention output)
        if (d.act == METASD_SWIGLU)
            rc = gemm_pro<PRO_NORM>(c, norm_pro(M.layer_w(L, 5), 0), m, D, M.layer_w(L, 6), F, M.layer_w(L, 7), F, nullptr, 0,
                                    c->d_part_pp(pp ^ 1), nullptr, &ns);
        else
            rc = gemm_pro<PRO_NORM>(c, norm_pro(M.layer_w(L, 5), 0), m, D, M.layer_w(L, 7), F, nullptr, 0, nullptr, 0, c->d_part_pp(pp ^ 1),
                                    nullptr, &ns);
        if (rc) return rc;
        hp ^= 1; pp ^= 1;
        // down projection of the activation
        {
            GemmPro p{};
            p.src = c->d_part_pp(pp); p.ns = ns; p.sstride = (size_t)m * (d.act == METASD_SWIGLU ? 2 : 1) * F; p.act = d.act == METASD_SWIGLU ? 1 : 0;
            if ((rc = gemm_pro<PRO_ACT>(c, p, m, F, M.layer_w(L, 8), D, nullptr, 0, nullptr, 0, c->d_part_pp(pp ^ 1), nullptr, &ns))) return rc;
            pp ^= 1;
        }
    }
    if (logits) {
        int dummy;
        if ((rc = gemm_pro<PRO_NORM>(c, norm_pro(M.final_norm(), first_row), m - first_row, D, M.lm_head(), V, nullptr, 0, nullptr, 0,
                                     c->d_part_pp(pp ^ 1), logits, &dummy))) return rc;
    }
    return 0;
}

int upload_table(metasd_ctx* c, Model& M) {
    HIP_TRY(c, hipMemcpyAsync((void*)M.d_table, M.w.data(), M.w.size() * sizeof(void*), hipMemcpyHostToDevice, c->stream));
    return 0;
}

// Forward over tokens hist[pos0 .. pos0+n) in blocks of <= 16 rows (later blocks see the KV of
// earlier ones).  logits (optional): want_all ? all n rows (n <= 16) : the last row only.
int model_index(const metasd_ctx* c, const Model& M) { return &M == &c->target ? -1 : (int)(&M - c->drafters.data()); }

int forward_blocks(metasd_ctx* c, Model& M, int pos0, int n, float* logits, bool want_all);

// A drafter with a streaming cache attends to the sinks and to the last stream_window positions of its cache's tail: the
// block mask of the attention kernels (TreeBlk, on == 2) carries that for the duration of its forward passes.
int forward(metasd_ctx* c, Model& M, int pos0, int n, float* logits, bool want_all) {
    if (!M.stream || c->tree) return forward_blocks(c, M, pos0, n, logits, want_all);
    TreeBlk wb{};
    wb.on = 2; wb.base = M.tail; wb.i0 = c->cfg.stream_window; wb.sink = c->cfg.stream_sink;
    c->tree = &wb;
    const int rc = forward_blocks(c, M, pos0, n, logits, want_all);
    c->tree = nullptr;
    return rc;
}

int forward_blocks(metasd_ctx* c, Model& M, int pos0, int n, float* logits, bool want_all) {
    c->cur_model = model_index(c, M);
    if (pos0 + n > c->cfg.max_ctx) return c->fail(METASD_E_OVERFLOW, "positions %d..%d exceed max_ctx %d", pos0, pos0 + n, c->cfg.max_ctx);
    int done = 0;
    while (done < n) {
        const int m = std::min(MAX_ROWS, n - done);
        const bool last = done + m == n;
        float* lg = (last && logits) ? logits : nullptr;
        const int first_row = want_all ? 0 : m - 1;
        int rc;
        const bool is_target = &M == &c->target;
        // the short-block path never writes the finished residual rows: not for the target when its features are wanted
        const bool fused = c->fuse_small && fused_small_ok(M, m) && !(is_target && c->cfg.feature_heads);
        if (M.d.dtype != METASD_BF16) rc = forward_rows<float>(c, M, pos0 + done, m, lg, first_row);
        else if (M.head) rc = c->gemm_reduce ? forward_rows_residual(c, M, pos0 + done, m, lg, first_row)     // these two paths carry the head's
                                             : forward_rows<bf16_t>(c, M, pos0 + done, m, lg, first_row);      // input projection
        else if (fused) rc = forward_rows_fused(c, M, pos0 + done, m, lg, first_row);
        else if (c->gemm_reduce) rc = forward_rows_residual(c, M, pos0 + done, m, lg, first_row);
        else rc = forward_rows<bf16_t>(c, M, pos0 + done, m, lg, first_row);
        if (rc) return rc;
        const int D = M.d.d_model;
        if (is_target && c->cfg.feature_heads) {        // the target's features of the block's positions
            const unsigned n4 = (unsigned)((size_t)m * D / 4);
            hipLaunchKernelGGL(copy_f4_kernel, dim3((n4 + 255) / 256), dim3(256), 0, c->stream, (const float4*)c->d_h(),
                               (float4*)(c->d_feat() + (size_t)(pos0 + done) * D), n4);
            LAUNCH_CHECK(c, "feature rows");
        }
        if (M.head && c->tree && c->tree->on == 1) {     // a tree level (one block): the estimates at its nodes, for their children
            const unsigned n4 = (unsigned)((size_t)m * D / 4);
            hipLaunchKernelGGL(copy_f4_kernel, dim3((n4 + 255) / 256), dim3(256), 0, c->stream, (const float4*)c->d_h(),
                               (float4*)(c->d_fest() + (size_t)c->tree->i0 * D), n4);
            LAUNCH_CHECK(c, "feature estimates");
        } else if (M.head && last) {                     // the head's estimate of the last row's feature: input of its next step
            hipLaunchKernelGGL(copy_f4_kernel, dim3((D / 4 + 255) / 256), dim3(256), 0, c->stream,
                               (const float4*)(c->d_h() + (size_t)(m - 1) * D), (float4*)c->d_fest(), (unsigned)(D / 4));
            LAUNCH_CHECK(c, "feature estimate");
        }
        done += m;
    }
    M.kvl[0] = pos0 + n;
    return 0;
}


// ================================================================================================
// Blocks of rows from several sequences (cfg.batch > 1): the plain step-by-step forward on the
// segment-aware kernels of batch.h.  Rows R = sg.n * sg.ms; row-wise kernels (add+norm, activation)
// are the single-sequence ones launched over R rows.

// GEMM over R rows into split-K partials part[s][R][N] (split stride R*N).
template <typename T>
int gemm_rows(metasd_ctx* c, const void* x, int ldx, int R, int K, const void* W0, int n0, const void* W1, int n1, const void* W2,
              int n2, int* nsplit_out);

template <>
int gemm_rows<float>(metasd_ctx* c, const void* x, int ldx, int R, int K, const void* W0, int n0, const void* W1, int n1,
                     const void* W2, int n2, int* nsplit_out) {
    const int N = n0 + n1 + n2;
    for (int r0 = 0; r0 < R; r0 += MAX_ROWS) {
        hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 3) / 4), dim3(256), 0, c->stream, (const float*)x + (size_t)r0 * ldx, ldx,
                           std::min(MAX_ROWS, R - r0), K, (const float*)W0, (const float*)W1, (const float*)W2, n0, n0 + n1, N,
                           c->d_part() + (size_t)r0 * N);
        LAUNCH_CHECK(c, "gemm_f32");
    }
    *nsplit_out = 1;
    return 0;
}

// more than 64 KiB of dynamic LDS needs the function attribute (set once per variant; harmless below the limit)
template <int RBW, bool LO, int TPQ = 4, int PD = ROWS_PD, int NRG = 4, int CST = 2, bool DMA = false>
int launch_gemm_rows(metasd_ctx* c, const bf16_t* xh, size_t x_lo_off, int ldx, int R, int r0, int nr, int K, const void* W0,
                     const void* W1, const void* W2, int t0, int t1, int ntiles, int N, const Split& s, metasd_ctx::ProfRec* pr) {
    const size_t lds = (size_t)2 * (LO ? 8 : 4) * CST * (16 * NRG * RBW) * 16;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)gemm_bf16_rows_kernel<RBW, PD, LO, TPQ, NRG, CST, DMA>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return c->fail(METASD_E_HIP, "gemm_bf16_rows_kernel: cannot reserve %zu bytes of LDS", lds);
        attr_set = true;
    }
    constexpr int TPW = (8 / NRG) * TPQ;           // tiles per workgroup
    const int groups = (ntiles + TPW - 1) / TPW;
    hipExtLaunchKernelGGL((gemm_bf16_rows_kernel<RBW, PD, LO, TPQ, NRG, CST, DMA>), dim3(groups * s.ksplit), dim3(512), (uint32_t)lds, c->stream,
                          pr ? pr->a : nullptr, pr ? pr->b : nullptr, 0u, xh + (size_t)r0 * ldx, x_lo_off, ldx, nr, K, (const bf16_t*)W0,
                          (const bf16_t*)W1, (const bf16_t*)W2, t0, t1, ntiles, c->d_part() + (size_t)r0 * N, (size_t)R * N, N, s.ksplit, s.cps);
    LAUNCH_CHECK(c, "gemm_bf16_rows");
    return 0;
}

template <>
int gemm_rows<bf16_t>(metasd_ctx* c, const void* x, int ldx, int R, int K, const void* W0, int n0, const void* W1, int n1,
                      const void* W2, int n2, int* nsplit_out) {
    const size_t x_lo_off = (size_t)R * ldx;      // producers write hi [R][ldx], then lo [R][ldx]
    if (R <= MAX_ROWS) return gemm<bf16_t>(c, x, ldx, R, K, W0, n0, W1, n1, W2, n2, nullptr, nsplit_out, x_lo_off);
    const int N = n0 + n1 + n2, ntiles = N / 16, kchunks = K / 32;
    const Split s = choose_split_rows(ntiles, kchunks, R, c->rows_tpb);
    metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_GEMM, (double)N * K * 2 + (double)R * K * 4 + (double)R * N * 4 * s.ksplit, N, K, R);
    const bf16_t* xh = (const bf16_t*)x;
    const int t0 = n0 / 16, t1 = (n0 + n1) / 16;
    int rc = 0;
    // more than 256 rows: two passes over the weights, 256 rows each (a 512-row variant would spill registers)
    for (int r0 = 0; r0 < R && !rc; r0 += 256) {
        const int nr = std::min(256, R - r0);
        metasd_ctx::ProfRec* p = r0 ? nullptr : pr;
#define ROWS_ARGS (c, xh, x_lo_off, ldx, R, r0, nr, K, W0, W1, W2, t0, t1, ntiles, N, s, p)
#define ROWS_GO(RBW, TPQ) launch_gemm_rows<RBW, true, TPQ> ROWS_ARGS
        if (nr <= 64) rc = ROWS_GO(1, 4);
        else if (nr <= 128) rc = ROWS_GO(2, 4);
        else if (s.tpb == 12) rc = launch_gemm_rows<8, true, 3, ROWS_PD, 2, 2, true> ROWS_ARGS;     // activations straight into LDS
        else if (s.tpb == 4) rc = ROWS_GO(4, 2);
        else if (s.tpb == 6) rc = ROWS_GO(4, 3);
        else rc = ROWS_GO(4, 4);
#undef ROWS_GO
#undef ROWS_ARGS
    }
    *nsplit_out = s.ksplit;
    return rc;
}

template <typename T, int HD>
int attention_seg_hd(metasd_ctx* c, const Model& M, int L, const Segs& sg) {
    const metasd_model_desc& d = M.d;
    const int R = sg.n * sg.ms;
    const size_t plane = (size_t)d.n_kv_heads * c->cfg.max_ctx * HD;
    const size_t seq_stride = (size_t)M.kv_layers * 2 * plane;
    const T* kc = (const T*)M.kv + (size_t)L * 2 * plane;
    const T* vc = kc + plane;
    int nch_max = 1;
    double kvpos = 0.0;
    for (int s = 0; s < sg.n; ++s) {
        nch_max = std::max(nch_max, (sg.pos0[s] + sg.m[s] + ATT_CH - 1) / ATT_CH);
        kvpos += (double)(sg.pos0[s] + sg.m[s]);
    }
    const float scale = 1.0f / sqrtf((float)HD);
    metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_ATTN, 2.0 * d.n_kv_heads * kvpos * HD * sizeof(T) + (double)R * d.n_heads * HD * 4);
    hipEvent_t ea = pr ? pr->a : nullptr, eb = pr ? pr->b : nullptr;
    int cpw = 1;                       // chunks per workgroup (bf16 MFMA kernel): fewer, larger records while the grid still fills the chip
    if constexpr (sizeof(T) == 2 && HD >= 64) {
        // Measured at 32 sequences x 4096 positions (7B shape, head_dim 128): 391 + 53 us (partial + merge) with one chunk per
        // workgroup, 380 + 10 us with eight; with head_dim 64 the chunks are too small for the loop to pay (37 -> 51 us).
        if (HD >= 128)
            for (int t = 8; t >= 2 && cpw == 1; t /= 2)
                if ((size_t)d.n_heads * sg.n * ((nch_max + t - 1) / t) >= (size_t)c->n_cu * 4) cpw = t;
        if (c->att_cpw > 0) cpw = c->att_cpw;
        const dim3 grid((nch_max + cpw - 1) / cpw, d.n_heads, sg.n);
        if (cpw > 1)
            hipExtLaunchKernelGGL((attn_partial_mfma_seg_kernel<HD, true>), grid, dim3(256), 0u, c->stream, ea, eb, 0u, (const float*)c->d_q(), kc,
                                  vc, seq_stride, sg, d.n_heads, d.n_kv_heads, c->cfg.max_ctx, scale, c->d_apart(), nch_max,
                                  (size_t)R * d.n_heads * HD, cpw);
        else
            hipExtLaunchKernelGGL((attn_partial_mfma_seg_kernel<HD, false>), grid, dim3(256), 0u, c->stream, ea, eb, 0u, (const float*)c->d_q(), kc,
                                  vc, seq_stride, sg, d.n_heads, d.n_kv_heads, c->cfg.max_ctx, scale, c->d_apart(), nch_max,
                                  (size_t)R * d.n_heads * HD, cpw);
    } else {
        hipExtLaunchKernelGGL((attn_partial_seg_kernel<T, HD>), dim3(nch_max, d.n_heads, sg.n), dim3(256), 0u, c->stream, ea, eb, 0u,
                              (const float*)c->d_q(), kc, vc, seq_stride, sg, d.n_heads, d.n_kv_heads, c->cfg.max_ctx, scale,
                              c->d_apart(), nch_max);
    }
    LAUNCH_CHECK(c, "attn_partial (segments)");
    hipLaunchKernelGGL((attn_combine_seg_kernel<HD>), dim3(d.n_heads, R), dim3(HD), 0, c->stream, c->d_apart(), nch_max, d.n_heads,
                       (float*)c->d_ao(), sizeof(T) == 2 ? 1 : 0, sg, cpw);
    LAUNCH_CHECK(c, "attn_combine (segments)");
    return 0;
}

template <typename T>
int attention_seg(metasd_ctx* c, const Model& M, int L, const Segs& sg) {
    switch (M.hd) {
        case 32: return attention_seg_hd<T, 32>(c, M, L, sg);
        case 64: return attention_seg_hd<T, 64>(c, M, L, sg);
        default:
            if constexpr (sizeof(T) == 2) return attention_seg_hd<T, 128>(c, M, L, sg);
            return c->fail(METASD_E_INVALID, "fp32 head_dim 128 unsupported");
    }
}

// add the split-K partials to the residual rows and normalise: many rows of 2048 or 4096 columns go through the form that
// keeps more requests in flight per CU (same arithmetic in the same order)
template <typename T>
void launch_addnorm_many(metasd_ctx* c, int R, float* h, const float* part, int ns, int D, const T* gain, float eps, float* xn, int split) {
    if (R > MAX_ROWS && D == 4096)
        hipLaunchKernelGGL((addnorm_rows_kernel<T, 4>), dim3(R), dim3(256), 0, c->stream, h, part, ns, (size_t)R * D, gain, eps, xn, split);
    else if (R > MAX_ROWS && D == 2048)
        hipLaunchKernelGGL((addnorm_rows_kernel<T, 2>), dim3(R), dim3(256), 0, c->stream, h, part, ns, (size_t)R * D, gain, eps, xn, split);
    else
        hipLaunchKernelGGL(addnorm_kernel<T>, dim3(R), dim3(1024), 0, c->stream, h, part, ns, (size_t)R * D, D, gain, eps, xn, split);
}

// Forward of the block sg through model M; appends K/V of the valid rows.  logits == nullptr: none.
// Otherwise the rows that carry logits are written to logits[(seq * out_seq_rows + out_row0 + j) * V]
// (last_only: only the last valid row of each segment, at j = 0).
template <typename T>
int forward_segs_t(metasd_ctx* c, Model& M, const Segs& sg, float* logits, int out_seq_rows, int out_row0, int last_only) {
    const metasd_model_desc& d = M.d;
    const int D = d.d_model, H = d.n_heads, KH = d.n_kv_heads, hd = M.hd, F = d.d_ffn, V = d.vocab;
    const int DQ = H * hd, DKV = KH * hd, NQKV = DQ + 2 * DKV;
    const int R = sg.n * sg.ms;
    hipStream_t st = c->stream;
    float* h = c->d_h();
    float* xn = (float*)c->d_xn();
    float* part = c->d_part();
    int ns = 0, rc;
    constexpr int split = sizeof(T) == 2 ? 1 : 0;
    const size_t plane = (size_t)KH * c->cfg.max_ctx * hd;
    const size_t seq_stride = (size_t)M.kv_layers * 2 * plane;
    hipLaunchKernelGGL(embed_seg_kernel<T>, dim3(R), dim3(256), 0, st, (const int32_t*)c->d_hist(), c->cfg.max_ctx, (const T*)M.w[0], D, h, sg);
    LAUNCH_CHECK(c, "embed (segments)");
    hipLaunchKernelGGL(rope_table_seg_kernel, dim3(R), dim3(hd / 2), 0, st, sg, hd, d.rope_theta, c->d_rope());
    LAUNCH_CHECK(c, "rope_table (segments)");
    for (int L = 0; L < d.n_layers; ++L) {
        launch_addnorm_many<T>(c, R, h, part, ns, D, (const T*)M.layer_w(L, 0), d.rms_eps, xn, split);
        LAUNCH_CHECK(c, "addnorm");
        if ((rc = gemm_rows<T>(c, xn, D, R, D, M.layer_w(L, 1), DQ, M.layer_w(L, 2), DKV, M.layer_w(L, 3), DKV, &ns))) return rc;
        T* kc = (T*)M.kv + (size_t)L * 2 * plane;
        hipLaunchKernelGGL(rope_kv_seg_kernel<T>, dim3(H + 2 * KH, R), dim3(64), 0, st, part, ns, (size_t)R * NQKV, NQKV, sg, H, KH, hd,
                           (const double2*)c->d_rope(), (float*)c->d_q(), kc, kc + plane, seq_stride, c->cfg.max_ctx, split,
                           (split && hd >= 64) ? 1 : 0);
        LAUNCH_CHECK(c, "rope_kv (segments)");
        if ((rc = attention_seg<T>(c, M, L, sg))) return rc;
        if ((rc = gemm_rows<T>(c, c->d_ao(), DQ, R, DQ, M.layer_w(L, 4), D, nullptr, 0, nullptr, 0, &ns))) return rc;
        launch_addnorm_many<T>(c, R, h, part, ns, D, (const T*)M.layer_w(L, 5), d.rms_eps, xn, split);
        LAUNCH_CHECK(c, "addnorm");
        if (d.act == METASD_SWIGLU) {
            if ((rc = gemm_rows<T>(c, xn, D, R, D, M.layer_w(L, 6), F, M.layer_w(L, 7), F, nullptr, 0, &ns))) return rc;
        } else {
            if ((rc = gemm_rows<T>(c, xn, D, R, D, M.layer_w(L, 7), F, nullptr, 0, nullptr, 0, &ns))) return rc;
        }
        const size_t nact = (size_t)R * F;
        const int NF = (d.act == METASD_SWIGLU ? 2 : 1) * F;
        hipLaunchKernelGGL(ffn_act4_kernel, dim3((unsigned)((nact / 4 + 255) / 256)), dim3(256), 0, st, part, ns, (size_t)R * NF, R, F, d.act,
                           (float*)c->d_act(), split, (const float*)nullptr);
        LAUNCH_CHECK(c, "ffn_act");
        if ((rc = gemm_rows<T>(c, c->d_act(), F, R, F, M.layer_w(L, 8), D, nullptr, 0, nullptr, 0, &ns))) return rc;
    }
    if (logits) {
        launch_addnorm_many<T>(c, R, h, part, ns, D, (const T*)M.final_norm(), d.rms_eps, xn, split);
        LAUNCH_CHECK(c, "addnorm");
        if ((rc = gemm_rows<T>(c, xn, D, R, D, M.lm_head(), V, nullptr, 0, nullptr, 0, &ns))) return rc;
        hipLaunchKernelGGL(sum_partials_seg_kernel, dim3((V + 255) / 256, R), dim3(256), 0, st, (const float*)part, ns, (size_t)R * V, V,
                           logits, sg, out_seq_rows, out_row0, last_only);
        LAUNCH_CHECK(c, "sum_partials (segments)");
    }
    for (int s = 0; s < sg.n; ++s) M.kvl[sg.seq[s]] = sg.pos0[s] + sg.m[s];
    return 0;
}

int forward_segs(metasd_ctx* c, Model& M, const Segs& sg, float* logits, int out_seq_rows, int out_row0, int last_only) {
    c->cur_model = model_index(c, M);
    for (int s = 0; s < sg.n; ++s)
        if (sg.pos0[s] + sg.m[s] > c->cfg.max_ctx)
            return c->fail(METASD_E_OVERFLOW, "sequence %d: positions %d..%d exceed max_ctx %d", sg.seq[s], sg.pos0[s], sg.pos0[s] + sg.m[s], c->cfg.max_ctx);
    if (M.d.dtype == METASD_BF16) return forward_segs_t<bf16_t>(c, M, sg, logits, out_seq_rows, out_row0, last_only);
    return forward_segs_t<float>(c, M, sg, logits, out_seq_rows, out_row0, last_only);
}

// ---- one drafter step of a batched round as a single forward: every sequence advances by one token in the drafter
// its bandit chose.  All drafters must have the same shape (bf16, head_dim >= 64); segments are ordered by arm, each
// kernel that touches weights or caches takes them per segment / per group (25 launches per step instead of 25 per
// arm in use - the draft phase of a batch is bound by the host's launch rate otherwise).

bool same_shape(const metasd_model_desc& a, const metasd_model_desc& b) {
    return a.n_layers == b.n_layers && a.d_model == b.d_model && a.n_heads == b.n_heads && a.n_kv_heads == b.n_kv_heads &&
           a.d_ffn == b.d_ffn && a.vocab == b.vocab && a.act == b.act && a.dtype == b.dtype && a.rms_eps == b.rms_eps &&
           a.rope_theta == b.rope_theta;
}

bool grouped_step_supported(const metasd_ctx* c) {
    if (!c->grouped_on || c->cfg.K > MAX_GROUPS) return false;
    const metasd_model_desc& d0 = c->drafters[0].d;
    if (d0.dtype != METASD_BF16 || c->drafters[0].hd < 64) return false;
    for (int a = 1; a < c->cfg.K; ++a)
        if (!same_shape(d0, c->drafters[a].d)) return false;
    return true;
}

template <int RBW>
int launch_gemm_rows_grouped(metasd_ctx* c, const void* x, int ldx, int R, int K, const RowGroups& gg, int n0, int n1, int N, const Split& s,
                             metasd_ctx::ProfRec* pr) {
    const size_t lds = (size_t)2 * 16 * (64 * RBW) * 16;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)gemm_bf16_rows_grouped_kernel<RBW, ROWS_PD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return c->fail(METASD_E_HIP, "gemm_bf16_rows_grouped_kernel: cannot reserve %zu bytes of LDS", lds);
        attr_set = true;
    }
    const int ntiles = N / 16, groups = (ntiles + 7) / 8;
    hipExtLaunchKernelGGL((gemm_bf16_rows_grouped_kernel<RBW, ROWS_PD>), dim3(groups * s.ksplit, gg.n), dim3(512), (uint32_t)lds, c->stream,
                          pr ? pr->a : nullptr, pr ? pr->b : nullptr, 0u, (const bf16_t*)x, (size_t)R * ldx, ldx, K, n0 / 16, (n0 + n1) / 16,
                          ntiles, c->d_part(), (size_t)R * N, N, s.ksplit, s.cps, gg);
    LAUNCH_CHECK(c, "gemm_bf16_rows (grouped)");
    return 0;
}

// x: R rows in the two-bf16 form (hi, then lo R * ldx elements further); gg: the row groups and their matrices.
int gemm_rows_grouped(metasd_ctx* c, const void* x, int ldx, int R, int K, const RowGroups& gg, int n0, int n1, int n2, int* nsplit_out) {
    const int N = n0 + n1 + n2, ntiles = N / 16, kchunks = K / 32;
    int mmax = 1;
    for (int g = 0; g < gg.n; ++g) mmax = std::max(mmax, gg.m[g]);
    const Split s = choose_split_rows(ntiles, kchunks, 64, 8);
    metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_GEMM, (double)gg.n * N * K * 2 + (double)R * K * 4 + (double)R * N * 4 * s.ksplit, N, K, R);
    *nsplit_out = s.ksplit;
    if (mmax <= 64) return launch_gemm_rows_grouped<1>(c, x, ldx, R, K, gg, n0, n1, N, s, pr);
    if (mmax <= 128) return launch_gemm_rows_grouped<2>(c, x, ldx, R, K, gg, n0, n1, N, s, pr);
    return launch_gemm_rows_grouped<4>(c, x, ldx, R, K, gg, n0, n1, N, s, pr);
}

// sg: the segments ordered by arm (ms <= 16 rows each, at most 256 rows per arm); arm[s]: the drafter of segment s.
// The logits of each segment's last valid row go to logits[(seq * out_seq_rows + out_row0) * V].
template <int HD>
int forward_step_grouped(metasd_ctx* c, const Segs& sg, const int* arm, float* logits, int out_seq_rows, int out_row0) {
    typedef bf16_t T;
    c->cur_model = arm[0];
    const metasd_model_desc& d = c->drafters[arm[0]].d;
    const int D = d.d_model, H = d.n_heads, KH = d.n_kv_heads, hd = HD, F = d.d_ffn, V = d.vocab;
    const int DQ = H * hd, DKV = KH * hd, NQKV = DQ + 2 * DKV;
    const int R = sg.n * sg.ms;
    hipStream_t st = c->stream;
    float* h = c->d_h();
    float* xn = (float*)c->d_xn();
    float* part = c->d_part();
    int ns = 0, rc;
    const size_t plane = (size_t)KH * c->cfg.max_ctx * hd;
    // groups of consecutive segments with one arm
    RowGroups gg{};
    for (int s0 = 0; s0 < sg.n;) {
        int s1 = s0;
        while (s1 < sg.n && arm[s1] == arm[s0]) ++s1;
        gg.r0[gg.n] = s0 * sg.ms; gg.m[gg.n] = (s1 - s0) * sg.ms; ++gg.n;
        s0 = s1;
    }
    auto seg_ptrs = [&](auto&& of_model) {
        SegPtrs p{};
        for (int s = 0; s < sg.n; ++s) p.p[s] = of_model(c->drafters[arm[s]], s);
        return p;
    };
    auto weights = [&](int L, int i0, int i1, int i2) {
        RowGroups g = gg;
        for (int q = 0; q < g.n; ++q) {
            const Model& M = c->drafters[arm[g.r0[q] / sg.ms]];
            g.W[q][0] = (const bf16_t*)(L < 0 ? M.lm_head() : M.layer_w(L, i0));
            g.W[q][1] = i1 >= 0 ? (const bf16_t*)M.layer_w(L, i1) : nullptr;
            g.W[q][2] = i2 >= 0 ? (const bf16_t*)M.layer_w(L, i2) : nullptr;
        }
        return g;
    };
    hipLaunchKernelGGL(embed_segp_kernel<T>, dim3(R), dim3(256), 0, st, (const int32_t*)c->d_hist(), c->cfg.max_ctx,
                       seg_ptrs([](const Model& M, int) { return (const void*)M.w[0]; }), D, h, sg);
    LAUNCH_CHECK(c, "embed (grouped)");
    hipLaunchKernelGGL(rope_table_seg_kernel, dim3(R), dim3(hd / 2), 0, st, sg, hd, d.rope_theta, c->d_rope());
    LAUNCH_CHECK(c, "rope_table (segments)");
    int nch_max = 1;
    double kvpos = 0.0;
    for (int s = 0; s < sg.n; ++s) {
        nch_max = std::max(nch_max, (sg.pos0[s] + sg.m[s] + ATT_CH - 1) / ATT_CH);
        kvpos += (double)(sg.pos0[s] + sg.m[s]);
    }
    const float scale = 1.0f / sqrtf((float)HD);
    for (int L = 0; L < d.n_layers; ++L) {
        hipLaunchKernelGGL(addnorm_segp_kernel<T>, dim3(R), dim3(1024), 0, st, h, part, ns, (size_t)R * D, D,
                           seg_ptrs([&](const Model& M, int) { return (const void*)M.layer_w(L, 0); }), sg.ms, d.rms_eps, xn, 1);
        LAUNCH_CHECK(c, "addnorm (grouped)");
        if ((rc = gemm_rows_grouped(c, xn, D, R, D, weights(L, 1, 2, 3), DQ, DKV, DKV, &ns))) return rc;
        const SegPtrs kcs = seg_ptrs([&](const Model& M, int s) { return (const void*)((const T*)M.kv + (size_t)L * 2 * plane + (size_t)sg.seq[s] * M.kv_layers * 2 * plane); });
        const SegPtrs vcs = seg_ptrs([&](const Model& M, int s) { return (const void*)((const T*)M.kv + (size_t)L * 2 * plane + plane + (size_t)sg.seq[s] * M.kv_layers * 2 * plane); });
        hipLaunchKernelGGL(rope_kv_segp_kernel<T>, dim3(H + 2 * KH, R), dim3(64), 0, st, part, ns, (size_t)R * NQKV, NQKV, sg, H, KH, hd,
                           (const double2*)c->d_rope(), (float*)c->d_q(), kcs, vcs, c->cfg.max_ctx, 1, 1);
        LAUNCH_CHECK(c, "rope_kv (grouped)");
        {
            metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_ATTN, 2.0 * KH * kvpos * HD * sizeof(T) + (double)R * H * HD * 4);
            hipExtLaunchKernelGGL((attn_partial_mfma_segp_kernel<HD>), dim3(nch_max, H, sg.n), dim3(256), 0u, st, pr ? pr->a : nullptr,
                                  pr ? pr->b : nullptr, 0u, (const float*)c->d_q(), kcs, vcs, sg, H, KH, c->cfg.max_ctx, scale, c->d_apart(),
                                  nch_max, (size_t)R * H * HD);
            LAUNCH_CHECK(c, "attn_partial (grouped)");
            hipLaunchKernelGGL((attn_combine_seg_kernel<HD>), dim3(H, R), dim3(HD), 0, st, c->d_apart(), nch_max, H, (float*)c->d_ao(), 1, sg, 1);
            LAUNCH_CHECK(c, "attn_combine (segments)");
        }
        if ((rc = gemm_rows_grouped(c, c->d_ao(), DQ, R, DQ, weights(L, 4, -1, -1), D, 0, 0, &ns))) return rc;
        hipLaunchKernelGGL(addnorm_segp_kernel<T>, dim3(R), dim3(1024), 0, st, h, part, ns, (size_t)R * D, D,
                           seg_ptrs([&](const Model& M, int) { return (const void*)M.layer_w(L, 5); }), sg.ms, d.rms_eps, xn, 1);
        LAUNCH_CHECK(c, "addnorm (grouped)");
        if (d.act == METASD_SWIGLU) {
            if ((rc = gemm_rows_grouped(c, xn, D, R, D, weights(L, 6, 7, -1), F, F, 0, &ns))) return rc;
        } else {
            if ((rc = gemm_rows_grouped(c, xn, D, R, D, weights(L, 7, -1, -1), F, 0, 0, &ns))) return rc;
        }
        const size_t nact = (size_t)R * F;
        const int NF = (d.act == METASD_SWIGLU ? 2 : 1) * F;
        hipLaunchKernelGGL(ffn_act4_kernel, dim3((unsigned)((nact / 4 + 255) / 256)), dim3(256), 0, st, part, ns, (size_t)R * NF, R, F, d.act,
                           (float*)c->d_act(), 1, (const float*)nullptr);
        LAUNCH_CHECK(c, "ffn_act");
        if ((rc = gemm_rows_grouped(c, c->d_act(), F, R, F, weights(L, 8, -1, -1), D, 0, 0, &ns))) return rc;
    }
    hipLaunchKernelGGL(addnorm_segp_kernel<T>, dim3(R), dim3(1024), 0, st, h, part, ns, (size_t)R * D, D,
                       seg_ptrs([](const Model& M, int) { return (const void*)M.final_norm(); }), sg.ms, d.rms_eps, xn, 1);
    LAUNCH_CHECK(c, "addnorm (grouped)");
    if ((rc = gemm_rows_grouped(c, xn, D, R, D, weights(-1, 0, -1, -1), V, 0, 0, &ns))) return rc;
    hipLaunchKernelGGL(sum_partials_seg_kernel, dim3((V + 255) / 256, R), dim3(256), 0, st, (const float*)part, ns, (size_t)R * V, V,
                       logits, sg, out_seq_rows, out_row0, 1);
    LAUNCH_CHECK(c, "sum_partials (segments)");
    for (int s = 0; s < sg.n; ++s) c->drafters[arm[s]].kvl[sg.seq[s]] = sg.pos0[s] + sg.m[s];
    return 0;
}

// Model M processes, for every listed sequence, the tokens at positions [M.kvl[seq], upto[seq]) in blocks of
// at most 16 rows per sequence.  logits (optional): the logits of each sequence's last token go to
// logits[(seq * out_seq_rows + out_row0) * V].
int catch_up(metasd_ctx* c, Model& M, const std::vector<int>& seqs, const std::vector<int>& upto, float* logits, int out_seq_rows,
             int out_row0) {
    for (;;) {
        Segs sg{};
        int pend_max = 0;
        bool more = false;
        for (size_t i = 0; i < seqs.size(); ++i) {
            const int b = seqs[i], pend = upto[i] - M.kvl[b];
            if (pend <= 0) continue;
            const int s = sg.n++;
            sg.seq[s] = b; sg.pos0[s] = M.kvl[b]; sg.m[s] = std::min(MAX_ROWS, pend);
            pend_max = std::max(pend_max, sg.m[s]);
            more = more || pend > MAX_ROWS;
        }
        if (sg.n == 0) return 0;
        sg.ms = pend_max;
        // logits are only needed from a sequence's last block; every block that ends a sequence computes them
        bool ends = false;
        for (int s = 0; s < sg.n; ++s) {
            size_t i = 0;
            while (seqs[i] != sg.seq[s]) ++i;
            ends = ends || sg.pos0[s] + sg.m[s] == upto[i];
        }
        if (int rc = forward_segs(c, M, sg, (logits && ends) ? logits : nullptr, out_seq_rows, out_row0, 1)) return rc;
        if (!more) return 0;
    }
}

int launch_sample(hipStream_t st, const float* logits, int rows, int V, float T, uint64_t seed, uint32_t round, uint32_t pos,
                  uint32_t seq0, int32_t* tok, int stride, int32_t* tok_copy) {
    hipLaunchKernelGGL(sample_rows_kernel, dim3(rows), dim3(AK_NT), 0, st, logits, V, T, seed, round, pos, seq0, tok, stride,
                       tok_copy);
    return hipGetLastError() == hipSuccess ? 0 : METASD_E_HIP;
}

bool accept_split_enabled() { return env_int("METASD_ACCEPT_SPLIT", 1) != 0; }   // read per launch: tests toggle it

// xchg != nullptr: four workgroups per (row, position) (accept_split_kernel); else one (accept_rows_kernel).
// rounds: the round word of the Philox counters, one per row (rt.n == rows) or the same for every row (rt.n == 0: rt.v[0]).
int launch_accept(hipStream_t st, const float* P, const float* Q, const int32_t* d, int rows, int gamma, int V, float T,
                  uint64_t seed, const RoundTab& rt, uint32_t seq0, int2* cand, double* bd, int32_t* n_acc, int32_t* token,
                  uint32_t* mask, int32_t* hist, int l, unsigned long long* xchg, hipEvent_t ev_begin = nullptr,
                  hipEvent_t ev_end = nullptr) {
    if (xchg && accept_split_enabled()) {   // one launch: the kernel also writes N_acc, the token and the mask
        hipExtLaunchKernelGGL(accept_split_kernel, dim3(AS_Q, gamma + 1, rows), dim3(AS_NT), 0u, st, ev_begin, ev_end, 0u, P, Q, d, gamma,
                              V, T, seed, rt, seq0, (unsigned long long*)cand, bd, xchg, next_epoch(),
                              std::max(0, env_int("METASD_ACCEPT_SPIN_LIMIT", 1 << 18)), n_acc, token, mask,
                              hist, l);
        return hipGetLastError() == hipSuccess ? 0 : METASD_E_HIP;
    }
    hipExtLaunchKernelGGL(accept_rows_kernel, dim3(gamma + 1, rows), dim3(AK_NT), 0u, st, ev_begin, ev_end, 0u, P, Q, d, gamma, V,
                          T, seed, rt, seq0, cand, bd);
    if (hipGetLastError() != hipSuccess) return METASD_E_HIP;
    hipLaunchKernelGGL(accept_finalize_kernel, dim3((rows + 63) / 64), dim3(64), 0, st, cand, rows, gamma, n_acc, token, mask,
                       hist, l);
    return hipGetLastError() == hipSuccess ? 0 : METASD_E_HIP;
}

bool valid_vocab(int V) { return V >= 4 && V % 4 == 0 && V <= AK_WAVES * AK_SEG; }

// ---- one round over a batch of independent sequences (cfg.batch > 1): every sequence drafts with its own
// arm (sequences that share an arm share that drafter's forward), one verification block over all
// batch x (gamma + 1) rows, one accept launch over all rows.

// A drafter that shares the target's cache has, by definition, processed exactly what the target has.
void sync_shared_kv(metasd_ctx* c) {
    for (auto& D : c->drafters)
        if (D.shared_kv) D.kvl = c->target.kvl;
}

RoundTab seq_rounds(const metasd_ctx* c) {
    RoundTab rt{};
    rt.n = c->cfg.batch;
    for (int b = 0; b < rt.n; ++b) rt.v[b] = (uint32_t)c->sq[b].round;
    return rt;
}
RoundTab one_round(uint32_t round) {
    RoundTab rt{};
    rt.v[0] = round;
    return rt;
}

int draft_batch(metasd_ctx* c, const int32_t* k, int gamma) {
    const int B = c->cfg.batch, V = c->target.d.vocab;
    for (int b = 0; b < B; ++b) {
        if (k[b] < 0 || k[b] >= c->cfg.K) return c->fail(METASD_E_INVALID, "draft: drafter index of sequence %d out of range", b);
        if (c->sq[b].l + gamma + 1 > c->cfg.max_ctx)
            return c->fail(METASD_E_OVERFLOW, "draft: sequence %d: l + gamma + 1 = %d exceeds max_ctx %d", b, c->sq[b].l + gamma + 1, c->cfg.max_ctx);
    }
    sync_shared_kv(c);
    SeqTab at{};
    const bool can_group = grouped_step_supported(c);
    for (int j = 0; j < gamma; ++j) {
        // one forward for all arms when more than one arm is in use and every sequence has 1..16 tokens to process in its
        // drafter (always so after the first step; in the first step unless a drafter was idle for many rounds)
        bool grouped = can_group;
        int arms_used = 0, pend_max = 0, rows_max = 0;
        for (int a = 0; a < c->cfg.K && grouped; ++a) {
            int nseq = 0;
            for (int b = 0; b < B; ++b)
                if (k[b] == a) {
                    ++nseq;
                    const int pend = c->sq[b].l + j - c->drafters[a].kvl[b];
                    if (pend < 1 || pend > MAX_ROWS) grouped = false;
                    pend_max = std::max(pend_max, pend);
                }
            arms_used += nseq > 0;
            rows_max = std::max(rows_max, nseq);
        }
        if (grouped && arms_used > 1 && rows_max * pend_max <= 256) {
            Segs sg{};
            int arm[MAX_SEGS];
            sg.ms = pend_max;
            for (int a = 0; a < c->cfg.K; ++a)
                for (int b = 0; b < B; ++b)
                    if (k[b] == a) {
                        const int s = sg.n++;
                        sg.seq[s] = b; sg.pos0[s] = c->drafters[a].kvl[b]; sg.m[s] = c->sq[b].l + j - c->drafters[a].kvl[b];
                        arm[s] = a;
                    }
            for (int s = 0; s < sg.n; ++s)
                if (sg.pos0[s] + sg.m[s] > c->cfg.max_ctx) return c->fail(METASD_E_OVERFLOW, "draft: sequence %d exceeds max_ctx", sg.seq[s]);
            const int rc = c->drafters[0].hd == 64 ? forward_step_grouped<64>(c, sg, arm, c->d_Q(), gamma, j)
                                                    : forward_step_grouped<128>(c, sg, arm, c->d_Q(), gamma, j);
            if (rc) return rc;
        } else
        for (int a = 0; a < c->cfg.K; ++a) {
            std::vector<int> seqs, upto;
            for (int b = 0; b < B; ++b)
                if (k[b] == a) { seqs.push_back(b); upto.push_back(c->sq[b].l + j); }
            if (seqs.empty()) continue;
            // j = 0: every committed token the drafter has not seen (ends with the last committed one);
            // j > 0: the draft token d_j at position l + j - 1
            if (int rc = catch_up(c, c->drafters[a], seqs, upto, c->d_Q(), gamma, j)) return rc;
        }
        for (int b = 0; b < B; ++b) at.v[b] = c->sq[b].l + j;
        hipLaunchKernelGGL(sample_seq_kernel, dim3(B), dim3(AK_NT), 0, c->stream, (const float*)c->d_Q() + (size_t)j * V, (size_t)gamma * V, V,
                           c->cfg.temperature, c->cfg.seed, seq_rounds(c), (uint32_t)j, c->d_hist(), c->cfg.max_ctx, at,
                           c->d_draft() + j, gamma);
        LAUNCH_CHECK(c, "sample (batch)");
    }
    for (int b = 0; b < B; ++b) c->sq[b].cur_k = k[b];
    return 0;
}

int verify_batch(metasd_ctx* c, int gamma) {
    Segs sg{};
    sg.n = c->cfg.batch;
    sg.ms = gamma + 1;
    for (int b = 0; b < sg.n; ++b) { sg.seq[b] = b; sg.m[b] = gamma + 1; sg.pos0[b] = c->sq[b].l - 1; }
    return forward_segs(c, c->target, sg, c->d_P(), gamma + 1, 0, 0);
}

int accept_batch(metasd_ctx* c, int gamma, int32_t* n_acc_out, int32_t* token_out, uint32_t* mask_out, double* bd_out) {
    const int B = c->cfg.batch, V = c->target.d.vocab, gm = c->cfg.gamma_max;
    int32_t* res = c->d_res();
    metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_ACCEPT, (double)B * (2 * gamma + 1) * V * 4);
    if (launch_accept(c->stream, c->d_P(), c->d_Q(), c->d_draft(), B, gamma, V, c->cfg.temperature, c->cfg.seed, seq_rounds(c), 0u,
                      c->d_cand(), c->d_bd(), res, res + B, (uint32_t*)(res + 2 * B), nullptr, 0, c->d_xchg(), pr ? pr->a : nullptr,
                      pr ? pr->b : nullptr))
        return c->fail(METASD_E_HIP, "launch accept kernels failed");
    SeqTab lt{};
    for (int b = 0; b < B; ++b) lt.v[b] = c->sq[b].l;
    hipLaunchKernelGGL(commit_tokens_kernel, dim3(1), dim3(64), 0, c->stream, (const int32_t*)res, (const int32_t*)(res + B), c->d_hist(),
                       c->cfg.max_ctx, lt, B);
    LAUNCH_CHECK(c, "commit_tokens");
    if (int rc = c->fetch_results()) return rc;
    (void)gm;
    const int32_t* hn = c->mirror<int32_t>(c->lay.res);
    bool timed_out = false;
    for (int b = 0; b < B; ++b) timed_out = timed_out || hn[B + b] == -2;
    if (timed_out && !c->mirror<GridBar>(c->lay.bar)->abort) {
        // some position's workgroups did not meet within their bounded wait: nothing of those rows was committed and the
        // logits are untouched - take the whole step again with one workgroup per position
        if (launch_accept(c->stream, c->d_P(), c->d_Q(), c->d_draft(), B, gamma, V, c->cfg.temperature, c->cfg.seed, seq_rounds(c), 0u,
                          c->d_cand(), c->d_bd(), res, res + B, (uint32_t*)(res + 2 * B), nullptr, 0, nullptr))
            return c->fail(METASD_E_HIP, "launch accept kernels failed");
        hipLaunchKernelGGL(commit_tokens_kernel, dim3(1), dim3(64), 0, c->stream, (const int32_t*)res, (const int32_t*)(res + B), c->d_hist(),
                           c->cfg.max_ctx, lt, B);
        LAUNCH_CHECK(c, "commit_tokens");
        if (int rc = c->fetch_results()) return rc;
        c->accept_fallbacks += 1;
    }
    const int32_t* ht = hn + B;
    const uint32_t* hm = (const uint32_t*)(hn + 2 * B);
    const int32_t* hd = c->mirror<int32_t>(c->lay.draft);
    const double* hbd = c->mirror<double>(c->lay.bd);
    if (c->mirror<GridBar>(c->lay.bar)->abort) {
        (void)hipMemsetAsync(c->d_bar(), 0, sizeof(GridBar), c->stream);
        c->phase = PH_NONE;
        for (auto& q : c->sq) q.ready = false;
        return c->fail(METASD_E_HIP, "a bounded device-side wait between workgroups timed out; call metasd_set_context (for every sequence) to start over");
    }
    for (int b = 0; b < B; ++b) {
        if (ht[b] == -2) { c->phase = PH_NONE; for (auto& q : c->sq) q.ready = false; return c->fail(METASD_E_HIP, "accept: the workgroups of a position did not meet (exchange timed out); call metasd_set_context to start over"); }
        if (hn[b] < 0 || hn[b] > gamma || ht[b] < 0 || ht[b] >= V) return c->fail(METASD_E_HIP, "accept: device returned n_acc %d token %d for sequence %d", hn[b], ht[b], b);
    }
    for (int b = 0; b < B; ++b) {
        metasd_ctx::SeqState& S = c->sq[b];
        const int l = S.l, n = hn[b];
        for (int j = 0; j < n; ++j) S.hist[l + j] = hd[(size_t)b * gamma + j];
        S.hist[l + n] = ht[b];
        S.l = l + n + 1;
        S.round += 1;
        c->target.kvl[b] = l + n;
        c->drafters[S.cur_k].kvl[b] = std::min(l + n, l + gamma - 1);
        if (n_acc_out) n_acc_out[b] = n;
        if (token_out) token_out[b] = ht[b];
        if (mask_out) mask_out[b] = hm[b];
        if (bd_out) {
            double sum = 0.0;
            for (int j = 0; j < gamma; ++j) sum += hbd[(size_t)b * gamma + j];
            bd_out[b] = sum / (double)gamma;
        }
    }
    sync_shared_kv(c);
    c->phase = PH_READY;
    return METASD_OK;
}

}  // namespace

namespace {
template <typename T>
int compact_kv(metasd_ctx* c, Model& M, int base, int limit) {
    const int planes = M.d.n_layers * 2 * M.d.n_kv_heads;
    const size_t total = (size_t)planes * M.hd;
    hipLaunchKernelGGL(kv_compact_kernel<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, c->stream, (T*)M.kv, planes, c->cfg.max_ctx, M.hd,
                       base, (const int32_t*)c->d_res(), limit, c->tshape.n);
    LAUNCH_CHECK(c, "kv_compact");
    return 0;
}

}  // namespace

// ================================================================================================ C ABI

extern "C" {

const char* metasd_last_error(const metasd_ctx* c) { return c ? c->err.c_str() : g_err.c_str(); }

int32_t metasd_kv_bytes(const metasd_model_desc* m, int32_t max_ctx, size_t* bytes_out) {
    if (!m || !bytes_out || max_ctx < 1) return fail_global(METASD_E_INVALID, "metasd_kv_bytes: bad argument");
    char buf[256];
    if (const char* e = check_model(*m, "model", buf, sizeof buf)) return fail_global(METASD_E_INVALID, "%s", e);
    *bytes_out = (size_t)m->n_layers * 2 * m->n_kv_heads * (size_t)max_ctx * (m->d_model / m->n_heads) * elem_size(*m);
    return METASD_OK;
}

static int check_config(const metasd_config* cfg, const metasd_model_desc* target, const metasd_model_desc* drafters) {
    if (!cfg || !target || !drafters) return fail_global(METASD_E_INVALID, "NULL config or descriptor");
    if (cfg->K < 1 || cfg->K > METASD_MAX_K) return fail_global(METASD_E_INVALID, "K must be in 1..%d", METASD_MAX_K);
    if (cfg->gamma_max < 1 || cfg->gamma_max > METASD_MAX_GAMMA) return fail_global(METASD_E_INVALID, "gamma_max must be in 1..%d", METASD_MAX_GAMMA);
    if (cfg->batch < 1 || cfg->batch > METASD_MAX_BATCH) return fail_global(METASD_E_INVALID, "batch must be in 1..%d", METASD_MAX_BATCH);
    if (cfg->max_ctx < cfg->gamma_max + 2) return fail_global(METASD_E_INVALID, "max_ctx too small");
    if (!(cfg->temperature >= 0.f)) return fail_global(METASD_E_INVALID, "temperature must be >= 0");
    if (cfg->reward != METASD_REWARD_BE && cfg->reward != METASD_REWARD_BD) return fail_global(METASD_E_INVALID, "reward");
    if (!(cfg->ucb_beta >= 0.0)) return fail_global(METASD_E_INVALID, "ucb_beta must be >= 0");
    switch (cfg->policy) {
        case METASD_POLICY_UCB: case METASD_POLICY_RANDOM: break;
        case METASD_POLICY_DUCB: case METASD_POLICY_EXP3:
            if (!(cfg->policy_param > 0.0 && cfg->policy_param <= 1.0)) return fail_global(METASD_E_INVALID, "policy_param must be in (0, 1] for this policy");
            break;
        case METASD_POLICY_SWUCB: case METASD_POLICY_SH:
            if (cfg->policy_window < 1) return fail_global(METASD_E_INVALID, "policy_window must be >= 1 for this policy");
            break;
        default: return fail_global(METASD_E_INVALID, "unknown policy %d", cfg->policy);
    }
    if (cfg->stream_window < 0 || cfg->stream_sink < 0) return fail_global(METASD_E_INVALID, "stream_sink and stream_window must be >= 0");
    if (cfg->stream_window > 0 && cfg->batch > 1) return fail_global(METASD_E_INVALID, "streaming drafter caches: contexts with one sequence only");
    if (cfg->feature_heads != 0 && cfg->feature_heads != 1) return fail_global(METASD_E_INVALID, "feature_heads must be 0 or 1");
    if (cfg->feature_heads && cfg->batch > 1) return fail_global(METASD_E_INVALID, "drafter heads on the target's hidden states: contexts with one sequence only");
    char buf[256];
    if (const char* e = check_model(*target, "target", buf, sizeof buf)) return fail_global(METASD_E_INVALID, "%s", e);
    for (int k = 0; k < cfg->K; ++k) {
        char who[32];
        snprintf(who, sizeof who, "drafter %d", k);
        if (const char* e = check_model(drafters[k], who, buf, sizeof buf)) return fail_global(METASD_E_INVALID, "%s", e);
        if (drafters[k].vocab != target->vocab) return fail_global(METASD_E_INVALID, "%s: vocab differs from the target's", who);
    }
    return METASD_OK;
}

int32_t metasd_workspace_bytes(const metasd_config* cfg, const metasd_model_desc* target, const metasd_model_desc* drafters,
                               size_t* bytes_out) {
    if (!bytes_out) return fail_global(METASD_E_INVALID, "NULL bytes_out");
    if (int rc = check_config(cfg, target, drafters)) return rc;
    *bytes_out = make_layout(*cfg, *target, drafters).total;
    return METASD_OK;
}

int32_t metasd_pack_weight(void* dst, const void* src, int32_t n_out, int32_t n_in, int32_t rope_head_dim, void* hip_stream) {
    if (!dst || !src || dst == src) return fail_global(METASD_E_INVALID, "metasd_pack_weight: NULL or aliased pointers");
    if (n_out < 16 || n_in < 32 || n_out % 16 || n_in % 32) return fail_global(METASD_E_INVALID, "metasd_pack_weight: n_out %% 16 and n_in %% 32 must be 0");
    if (rope_head_dim != 0 && (rope_head_dim < 32 || rope_head_dim % 32 || n_out % rope_head_dim))
        return fail_global(METASD_E_INVALID, "metasd_pack_weight: rope_head_dim must be 0 or a multiple of 32 dividing n_out");
    const size_t total = (size_t)n_out * n_in / 8;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)hip_stream,
                       (const uint4*)src, (uint4*)dst, n_out, n_in, rope_head_dim);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_global(METASD_E_HIP, "pack_weight: %s", hipGetErrorString(e));
    return METASD_OK;
}

int32_t metasd_create(metasd_ctx** out, const metasd_config* cfg, const metasd_model_desc* target,
                      const metasd_model_desc* drafters, const void* const* target_weights,
                      const void* const* const* drafter_weights, void* target_kv, void* const* drafter_kv, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
    if (!out) return fail_global(METASD_E_INVALID, "NULL out");
    *out = nullptr;
    if (int rc = check_config(cfg, target, drafters)) return rc;
    if (!target_weights || !drafter_weights || !target_kv || !drafter_kv || !workspace) return fail_global(METASD_E_INVALID, "NULL pointer argument");
    if ((uintptr_t)workspace % ALIGN) return fail_global(METASD_E_INVALID, "workspace must be 256-byte aligned");
    const Layout lay = make_layout(*cfg, *target, drafters);
    if (workspace_bytes < lay.total) return fail_global(METASD_E_WORKSPACE, "workspace too small: need %zu bytes, got %zu", lay.total, workspace_bytes);
    auto fill = [&](Model& M, const metasd_model_desc& d, const void* const* w, void* kv, const char* who) -> int {
        M.d = d;
        M.hd = d.d_model / d.n_heads;
        M.kv = kv;
        M.kv_layers = d.n_layers;
        M.kvl.assign(cfg->batch, 0);
        const int nw = 1 + PER_LAYER * d.n_layers + 2;
        M.w.assign(w, w + nw);
        for (int i = 0; i < nw; ++i) {
            const bool gate = i >= 1 && i < nw - 2 && (i - 1) % PER_LAYER == 6;
            if (!M.w[i] && !(gate && d.act == METASD_GELU)) return fail_global(METASD_E_INVALID, "%s: weight %d is NULL", who, i);
            if ((uintptr_t)M.w[i] % 16) return fail_global(METASD_E_INVALID, "%s: weight %d is not 16-byte aligned", who, i);
        }
        if (!kv || (uintptr_t)kv % 16) return fail_global(METASD_E_INVALID, "%s: KV cache NULL or misaligned", who);
        return 0;
    };
    metasd_ctx* c = new (std::nothrow) metasd_ctx();
    if (!c) return fail_global(METASD_E_INVALID, "out of host memory");
    c->cfg = *cfg;
    c->stream = (hipStream_t)hip_stream;
    c->ws = (char*)workspace;
    c->lay = lay;
    int rc = fill(c->target, *target, target_weights, target_kv, "target");
    c->drafters.resize(cfg->K);
    for (int k = 0; k < cfg->K && !rc; ++k) {
        if (!drafter_weights[k]) rc = fail_global(METASD_E_INVALID, "drafter %d: NULL weight table", k);
        else {
            char who[32];
            snprintf(who, sizeof who, "drafter %d", k);
            rc = fill(c->drafters[k], drafters[k], drafter_weights[k], drafter_kv[k], who);
            if (!rc && drafter_kv[k] == target_kv) {
                // shared cache: the drafter must be the target's first layers, tensor for tensor, or its K/V would not be the target's
                Model& D = c->drafters[k];
                const metasd_model_desc &a = D.d, &b = *target;
                bool same = a.n_layers <= b.n_layers && a.d_model == b.d_model && a.n_heads == b.n_heads && a.n_kv_heads == b.n_kv_heads &&
                            a.d_ffn == b.d_ffn && a.act == b.act && a.dtype == b.dtype && a.rms_eps == b.rms_eps && a.rope_theta == b.rope_theta;
                for (int i = 0; same && i < 1 + PER_LAYER * a.n_layers; ++i) same = D.w[i] == c->target.w[i];
                if (!same) rc = fail_global(METASD_E_INVALID, "%s: shares the target's KV cache but its layers are not the target's first %d layers (same shapes and weight pointers required)", who, a.n_layers);
                D.shared_kv = true;
                D.kv_layers = b.n_layers;
            }
            if (!rc) c->drafters[k].stream = cfg->stream_window > 0 && !c->drafters[k].shared_kv;
        }
    }
    if (rc) { delete c; return rc; }
    c->sq.resize(cfg->batch);
    for (int b = 0; b < cfg->batch; ++b) {
        c->sq[b].hist.assign(cfg->max_ctx, 0);
        c->sq[b].bandit.init(*cfg);
        c->sq[b].bandit.seq = (uint32_t)b;
    }
    hipError_t e = hipHostMalloc((void**)&c->hspan, c->span_bytes(), hipHostMallocDefault);
    if (e != hipSuccess) {
        rc = fail_global(METASD_E_HIP, "hipHostMalloc: %s", hipGetErrorString(e));
        delete c;
        return rc;
    }
    {
        int dev = 0, ncu = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ncu < 1) {
            rc = fail_global(METASD_E_HIP, "cannot query the device");
            (void)hipHostFree(c->hspan);
            delete c;
            return rc;
        }
        if (const char* ev = getenv("METASD_FUSE_SMALL")) c->fuse_small = ev[0] != '0';
        if (const char* ev = getenv("METASD_GEMM_REDUCE")) c->gemm_reduce = ev[0] != '0';
        if (const char* ev = getenv("METASD_GEMM_ROLL")) c->fullk_roll = ev[0] != '0';
        if (const char* ev = getenv("METASD_DRAFT_GROUPED")) c->grouped_on = ev[0] != '0';
        if (const char* ev = getenv("METASD_ATT_CPW")) { const int v = atoi(ev); c->att_cpw = (v >= 1 && v <= 64) ? v : 0; }
        if (const char* ev = getenv("METASD_ROWS_TPB")) { const int v = atoi(ev); c->rows_tpb = (v == 4 || v == 6 || v == 8 || v == 12) ? v : 0; }
        {
            const int roll_lds = (int)FULLK_LDS_MAX;
            if (hipFuncSetAttribute((const void*)gemm_fullk_roll_residual_kernel<3, true>, hipFuncAttributeMaxDynamicSharedMemorySize, roll_lds) != hipSuccess ||
                hipFuncSetAttribute((const void*)gemm_fullk_roll_residual_kernel<4, true>, hipFuncAttributeMaxDynamicSharedMemorySize, roll_lds) != hipSuccess ||
                hipFuncSetAttribute((const void*)gemm_fullk_roll_residual_kernel<5, false>, hipFuncAttributeMaxDynamicSharedMemorySize, roll_lds) != hipSuccess ||
                hipFuncSetAttribute((const void*)gemm_fullk_roll_residual_kernel<6, false>, hipFuncAttributeMaxDynamicSharedMemorySize, roll_lds) != hipSuccess ||
                hipFuncSetAttribute((const void*)gemm_fullk_roll_residual_kernel<7, false>, hipFuncAttributeMaxDynamicSharedMemorySize, roll_lds) != hipSuccess ||
                hipFuncSetAttribute((const void*)gemm_fullk_roll_residual_kernel<8, false>, hipFuncAttributeMaxDynamicSharedMemorySize, roll_lds) != hipSuccess) {
                c->fullk_roll = false;
                (void)hipGetLastError();
            }
        }
        if (hipFuncSetAttribute((const void*)gemm_fullk_residual_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)FULLK_LDS_MAX) != hipSuccess) { c->fullk = false; (void)hipGetLastError(); }
        c->n_cu = ncu;
    }
    c->target.d_table = (const void**)(c->ws + lay.tables);
    for (int k = 0; k < cfg->K; ++k) c->drafters[k].d_table = (const void**)(c->ws + lay.tables + lay.table_stride * (size_t)(k + 1));
    e = hipMemsetAsync(c->d_bar(), 0, sizeof(GridBar), c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->d_gx(), 0, c->lay.ssq - c->lay.gx, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->d_xchg(), 0, (size_t)cfg->batch * (cfg->gamma_max + 1) * AS_XCHG_BYTES, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->d_cand(), 0, (size_t)cfg->batch * (cfg->gamma_max + 1) * sizeof(int2), c->stream);
    if (e == hipSuccess) e = hipMemcpyAsync((void*)c->target.d_table, c->target.w.data(), c->target.w.size() * sizeof(void*), hipMemcpyHostToDevice, c->stream);
    for (int k = 0; k < cfg->K && e == hipSuccess; ++k)
        e = hipMemcpyAsync((void*)c->drafters[k].d_table, c->drafters[k].w.data(), c->drafters[k].w.size() * sizeof(void*), hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) {
        rc = fail_global(METASD_E_HIP, "context set-up: %s", hipGetErrorString(e));
        (void)hipHostFree(c->hspan);
        delete c;
        return rc;
    }
    *out = c;
    return METASD_OK;
}

int32_t metasd_destroy(metasd_ctx* c) {
    if (!c) return METASD_OK;
    if (c->hspan) (void)hipHostFree(c->hspan);
    for (auto& r : c->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    delete c;
    return METASD_OK;
}

int32_t metasd_set_context(metasd_ctx* c, int32_t seq, const int32_t* tokens, int32_t n, int32_t kv_prefilled) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (seq < 0 || seq >= c->cfg.batch || !tokens || n < 1) return c->fail(METASD_E_INVALID, "set_context: bad seq / tokens / n");
    if (n + c->cfg.gamma_max + 1 > c->cfg.max_ctx) return c->fail(METASD_E_OVERFLOW, "set_context: n + gamma_max + 1 = %d exceeds max_ctx %d", n + c->cfg.gamma_max + 1, c->cfg.max_ctx);
    for (int i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= c->target.d.vocab) return c->fail(METASD_E_INVALID, "set_context: token %d out of range at %d", tokens[i], i);
    if (c->phase == PH_DRAFTED || c->phase == PH_VERIFIED || c->phase == PH_TREE_DRAFTED || c->phase == PH_TREE_VERIFIED)
        return c->fail(METASD_E_ORDER, "set_context: a round is in flight (finish it with metasd_accept first)");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    metasd_ctx::SeqState& S = c->sq[seq];
    std::copy(tokens, tokens + n, S.hist.begin());
    HIP_TRY(c, hipMemcpyAsync(c->d_hist() + (size_t)seq * c->cfg.max_ctx, S.hist.data(), (size_t)n * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    S.l = n;
    S.bandit.reset();
    S.ready = true;
    S.round = 0;                    // this sequence's Philox round word restarts with its query; the others carry on
    bool all = true;
    for (const auto& q : c->sq) all = all && q.ready;
    c->phase = all ? PH_READY : PH_NONE;
    c->target.kvl[seq] = kv_prefilled ? n - 1 : 0;
    for (auto& d : c->drafters) { d.kvl[seq] = (kv_prefilled || d.shared_kv) ? n - 1 : 0; d.tail = 0; }
    if (!kv_prefilled && n > 1) {
        if (c->cfg.batch == 1) { if (int rc = forward(c, c->target, 0, n - 1, nullptr, false)) return rc; }
        else if (int rc = catch_up(c, c->target, std::vector<int>{seq}, std::vector<int>{n - 1}, nullptr, 0, 0)) return rc;
    }
    return METASD_OK;
}

int32_t metasd_swap_weight(metasd_ctx* c, int32_t model, int32_t index, const void* dev_ptr) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (model < -1 || model >= c->cfg.K) return c->fail(METASD_E_INVALID, "swap_weight: model %d out of range", model);
    Model& M = model < 0 ? c->target : c->drafters[model];
    if (index < 0 || index >= (int)M.w.size() || !dev_ptr || (uintptr_t)dev_ptr % 16) return c->fail(METASD_E_INVALID, "swap_weight: bad index or pointer");
    M.w[index] = dev_ptr;
    HIP_TRY(c, hipStreamSynchronize(c->stream));        // no launch in flight reads the old table
    if (int rc = upload_table(c, M)) return rc;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return METASD_OK;
}

// ---- bandit

int32_t metasd_bandit_select(metasd_ctx* c, int32_t seq, int32_t* k_out) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (seq < 0 || seq >= c->cfg.batch || !k_out) return c->fail(METASD_E_INVALID, "bandit_select: bad argument");
    *k_out = c->sq[seq].bandit.select();
    return METASD_OK;
}

int32_t metasd_bandit_update(metasd_ctx* c, int32_t seq, int32_t k, int32_t n_acc, int32_t gamma, double bd_reward) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (seq < 0 || seq >= c->cfg.batch || k < 0 || k >= c->cfg.K || gamma < 1 || n_acc < 0 || n_acc > gamma) return c->fail(METASD_E_INVALID, "bandit_update: bad argument");
    double r = (double)n_acc / (double)gamma;
    if (c->cfg.reward == METASD_REWARD_BD) {
        if (!(bd_reward >= 0.0 && bd_reward <= 1.0 + 1e-9)) return c->fail(METASD_E_INVALID, "bandit_update: BD reward %g not in [0,1]", bd_reward);
        r = bd_reward;
    }
    c->sq[seq].bandit.update(k, r);
    return METASD_OK;
}

int32_t metasd_bandit_state(const metasd_ctx* c, int32_t seq, double* mu, int32_t* n, int32_t* t) {
    if (!c || seq < 0 || seq >= c->cfg.batch) return fail_global(METASD_E_INVALID, "bandit_state: bad argument");
    const Bandit& B = c->sq[seq].bandit;
    if (mu) std::copy(B.mu.begin(), B.mu.end(), mu);
    if (n) std::copy(B.n.begin(), B.n.end(), n);
    if (t) *t = B.t;
    return METASD_OK;
}

// ---- round

int32_t metasd_set_drafter_head(metasd_ctx* c, int32_t k, const void* w_fc) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (!c->cfg.feature_heads) return c->fail(METASD_E_INVALID, "set_drafter_head: the context was created without metasd_config.feature_heads");
    if (k < 0 || k >= c->cfg.K || !w_fc) return c->fail(METASD_E_INVALID, "set_drafter_head: bad drafter index or NULL weight");
    if (c->phase != PH_NONE) return c->fail(METASD_E_ORDER, "set_drafter_head: call it before the first metasd_set_context");
    Model& D = c->drafters[k];
    const metasd_model_desc& t = c->target.d;
    if (D.d.d_model != t.d_model || D.d.dtype != t.dtype) return c->fail(METASD_E_INVALID, "set_drafter_head: the head must have the target's width and dtype");
    if (D.shared_kv) return c->fail(METASD_E_INVALID, "set_drafter_head: a head keeps a cache of its own");
    if (t.d_ffn < t.d_model) return c->fail(METASD_E_INVALID, "set_drafter_head: needs d_ffn >= d_model (the input block is staged in the FFN buffer)");
    D.head = true;
    D.fc = w_fc;
    D.stream = false;
    return METASD_OK;
}

int32_t metasd_draft(metasd_ctx* c, const int32_t* k, int32_t gamma) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (!k || k[0] < 0 || k[0] >= c->cfg.K) return c->fail(METASD_E_INVALID, "draft: drafter index out of range");
    if (gamma < 1 || gamma > c->cfg.gamma_max) return c->fail(METASD_E_INVALID, "draft: gamma %d not in 1..%d", gamma, c->cfg.gamma_max);
    if (c->phase != PH_READY) return c->fail(METASD_E_ORDER, "draft: call set_context first (for every sequence) / finish the previous round with accept");
    if (c->cfg.batch > 1) {
        if (int rc = draft_batch(c, k, gamma)) return rc;
        c->cur_gamma = gamma;
        c->phase = PH_DRAFTED;
        return METASD_OK;
    }
    if (c->sq[0].l + gamma + 1 > c->cfg.max_ctx) return c->fail(METASD_E_OVERFLOW, "draft: l + gamma + 1 = %d exceeds max_ctx %d", c->sq[0].l + gamma + 1, c->cfg.max_ctx);
    sync_shared_kv(c);
    Model& D = c->drafters[k[0]];
    const int V = D.d.vocab, l = c->sq[0].l;
    const float T = c->cfg.temperature;
    for (int j = 0; j < gamma; ++j) {
        float* Qj = c->d_Q() + (size_t)j * V;
        int rc;
        if (j == 0 && D.stream) {
            // switched in: the sinks it has not seen, then the last stream_window committed tokens; a longer backlog is skipped
            const int S = std::min(c->cfg.stream_sink, l);
            int have = D.kvl[0];
            rc = 0;
            if (have < S) { rc = forward(c, D, have, S - have, S == l ? Qj : nullptr, false); have = S; }
            const int start = std::max(have, l - c->cfg.stream_window);
            if (start > have) D.tail = start;
            if (!rc && start < l) rc = forward(c, D, start, l - start, Qj, false);
        } else if (j == 0) rc = forward(c, D, D.kvl[0], l - D.kvl[0], Qj, false);   // catch-up, ends with the last committed token
        else {
            c->head_est = D.head;                      // a drafter head goes on from its own estimate of the last feature
            rc = forward(c, D, l + j - 1, 1, Qj, false);
            c->head_est = false;
        }
        if (rc) return rc;
        if (launch_sample(c->stream, Qj, 1, V, T, c->cfg.seed, (uint32_t)c->sq[0].round, (uint32_t)j, 0u, c->d_hist() + l + j, 1,
                          c->d_draft() + j))
            return c->fail(METASD_E_HIP, "launch sample_rows failed");
    }
    c->sq[0].cur_k = k[0];
    c->cur_gamma = gamma;
    c->phase = PH_DRAFTED;
    return METASD_OK;
}

int32_t metasd_verify(metasd_ctx* c, int32_t gamma) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (c->phase != PH_DRAFTED) return c->fail(METASD_E_ORDER, "verify: draft has not been run for this round");
    if (gamma != c->cur_gamma) return c->fail(METASD_E_INVALID, "verify: gamma %d differs from the drafted %d", gamma, c->cur_gamma);
    if (c->cfg.batch > 1) { if (int rc = verify_batch(c, gamma)) return rc; }
    else if (int rc = forward(c, c->target, c->sq[0].l - 1, gamma + 1, c->d_P(), true)) return rc;
    c->phase = PH_VERIFIED;
    return METASD_OK;
}

int32_t metasd_accept(metasd_ctx* c, int32_t gamma, int32_t* n_acc_out, int32_t* token_out, uint32_t* mask_out, double* bd_out) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (c->phase != PH_VERIFIED) return c->fail(METASD_E_ORDER, "accept: verify has not been run for this round");
    if (gamma != c->cur_gamma) return c->fail(METASD_E_INVALID, "accept: gamma %d differs from the drafted %d", gamma, c->cur_gamma);
    if (c->cfg.batch > 1) return accept_batch(c, gamma, n_acc_out, token_out, mask_out, bd_out);
    const int V = c->target.d.vocab, l = c->sq[0].l;
    int32_t* res = c->d_res();
    metasd_ctx::ProfRec* pr = c->prof_take(METASD_PROF_ACCEPT, (double)(2 * gamma + 1) * V * 4);
    if (launch_accept(c->stream, c->d_P(), c->d_Q(), c->d_hist() + l, 1, gamma, V, c->cfg.temperature, c->cfg.seed,
                      one_round((uint32_t)c->sq[0].round), 0u, c->d_cand(), c->d_bd(), res, res + 1, (uint32_t*)(res + 2), c->d_hist(), l,
                      c->d_xchg(), pr ? pr->a : nullptr, pr ? pr->b : nullptr))
        return c->fail(METASD_E_HIP, "launch accept kernels failed");
    if (int rc = c->fetch_results()) return rc;
    const int32_t* hres = c->mirror<int32_t>(c->lay.res);     // n_acc, token, mask
    if (hres[1] == -2 && !c->mirror<GridBar>(c->lay.bar)->abort) {
        // the four workgroups of some position did not meet within their bounded wait: nothing was committed, the
        // logits are untouched - take the step again with one workgroup per position (no meeting between workgroups)
        if (launch_accept(c->stream, c->d_P(), c->d_Q(), c->d_hist() + l, 1, gamma, V, c->cfg.temperature, c->cfg.seed,
                          one_round((uint32_t)c->sq[0].round), 0u, c->d_cand(), c->d_bd(), res, res + 1, (uint32_t*)(res + 2), c->d_hist(), l, nullptr))
            return c->fail(METASD_E_HIP, "launch accept kernels failed");
        if (int rc = c->fetch_results()) return rc;
        c->accept_fallbacks += 1;
    }
    const int32_t* hd = c->mirror<int32_t>(c->lay.draft);
    const double* hbd = c->mirror<double>(c->lay.bd);
    if (c->mirror<GridBar>(c->lay.bar)->abort) {
        (void)hipMemsetAsync(c->d_bar(), 0, sizeof(GridBar), c->stream);
        c->phase = PH_NONE;
        return c->fail(METASD_E_HIP, "a bounded device-side wait between workgroups timed out (split-K reduction or device-wide barrier); call metasd_set_context to start over");
    }
    const int n = hres[0], token = hres[1];
    if (token == -2) { c->phase = PH_NONE; return c->fail(METASD_E_HIP, "accept: the workgroups of a position did not meet (exchange timed out); call metasd_set_context to start over"); }
    if (n < 0 || n > gamma || token < 0 || token >= V) return c->fail(METASD_E_HIP, "accept: device returned n_acc %d token %d", n, token);
    for (int j = 0; j < n; ++j) c->sq[0].hist[l + j] = hd[j];
    c->sq[0].hist[l + n] = token;
    // commit: rows 0..n of the verification block stay in the target's cache; the drafter keeps
    // the committed prefix it has processed (it never saw d_gamma)
    c->sq[0].l = l + n + 1;
    c->target.kvl[0] = l + n;
    c->drafters[c->sq[0].cur_k].kvl[0] = std::min(l + n, l + gamma - 1);
    // a drafter head keeps nothing it computed from estimated features: it will re-read the committed tokens of this round with
    // the target's own features (which the verification pass has just left in the feature table)
    if (c->drafters[c->sq[0].cur_k].head) c->drafters[c->sq[0].cur_k].kvl[0] = l;
    c->sq[0].round += 1;
    sync_shared_kv(c);
    c->phase = PH_READY;
    if (n_acc_out) *n_acc_out = n;
    if (token_out) *token_out = token;
    if (mask_out) *mask_out = (uint32_t)hres[2];
    if (bd_out) {
        double s = 0.0;
        for (int j = 0; j < gamma; ++j) s += hbd[j];
        *bd_out = s / (double)gamma;
    }
    return METASD_OK;
}

// ---- token trees (greedy): draft a tree of candidates, verify it in one pass with tree attention, accept the longest
// path that the target's own greedy choices follow

int32_t metasd_draft_tree(metasd_ctx* c, int32_t k, const metasd_tree* tree) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (c->cfg.batch != 1) return c->fail(METASD_E_INVALID, "draft_tree: contexts with one sequence only");
    if (k < 0 || k >= c->cfg.K || !tree) return c->fail(METASD_E_INVALID, "draft_tree: bad drafter index or NULL tree");
    if (c->drafters[k].stream) return c->fail(METASD_E_INVALID, "draft_tree: drafters with a streaming cache draft chains only");
    if (c->phase != PH_READY) return c->fail(METASD_E_ORDER, "draft_tree: call set_context first / finish the previous round");
    const int n = tree->n;
    if (n < 2 || n > TREE_MAX || n > c->cfg.gamma_max + 1) return c->fail(METASD_E_INVALID, "draft_tree: tree of %d nodes; 2 .. min(%d, gamma_max + 1) supported", n, TREE_MAX);
    TreeShape ts{};
    ts.n = n;
    ts.parent[0] = -1;
    c->tdepth[0] = 0;
    c->tanc[0] = 1;
    for (int i = 1; i < n; ++i) {
        const int p = tree->parent[i], r = tree->rank[i];
        if (p < 0 || p >= i || r < 0 || r >= TREE_RANKS) return c->fail(METASD_E_INVALID, "draft_tree: node %d: parent must be an earlier node, rank 0..%d", i, TREE_RANKS - 1);
        c->tdepth[i] = c->tdepth[p] + 1;
        if (c->tdepth[i] < c->tdepth[i - 1]) return c->fail(METASD_E_INVALID, "draft_tree: nodes must come in breadth-first order (depth never decreases)");
        for (int j = 1; j < i; ++j)
            if (tree->parent[j] == p && tree->rank[j] == r) return c->fail(METASD_E_INVALID, "draft_tree: nodes %d and %d are the same child of node %d", j, i, p);
        ts.parent[i] = (int8_t)p;
        ts.rank[i] = (int8_t)r;
        c->tanc[i] = (uint16_t)(c->tanc[p] | (1u << i));
    }
    c->tmaxdepth = c->tdepth[n - 1];
    for (int d = 0, i = 0; d <= c->tmaxdepth + 1; ++d) {
        while (i < n && c->tdepth[i] < d) ++i;
        c->tlevel[d] = i;
    }
    if (c->tlevel[c->tmaxdepth] > c->cfg.gamma_max) return c->fail(METASD_E_INVALID, "draft_tree: %d nodes above the deepest level exceed gamma_max %d", c->tlevel[c->tmaxdepth], c->cfg.gamma_max);
    const int l = c->sq[0].l, base = l - 1;
    if (l + n + 1 > c->cfg.max_ctx) return c->fail(METASD_E_OVERFLOW, "draft_tree: l + nodes + 1 = %d exceeds max_ctx %d", l + n + 1, c->cfg.max_ctx);
    sync_shared_kv(c);
    Model& D = c->drafters[k];
    const int V = D.d.vocab;
    TreeBlk tb{};
    tb.on = 1; tb.base = base;
    for (int i = 0; i < n; ++i) { tb.anc[i] = c->tanc[i]; tb.depth[i] = (uint8_t)c->tdepth[i]; }
    for (int d = 0; d < c->tmaxdepth; ++d) {
        const int i0 = c->tlevel[d], m = c->tlevel[d + 1] - i0;
        float* Qd = c->d_Q() + (size_t)i0 * V;
        int rc;
        if (d == 0) rc = forward(c, D, D.kvl[0], l - D.kvl[0], Qd, false);      // the committed backlog, ending with the root
        else {
            tb.i0 = i0;
            c->tree = &tb;
            if (D.head) {                                // a head's node takes the head's estimate at its parent
                c->head_est = true;
                for (int r = 0; r < m; ++r) c->fsrc.idx[r] = (uint8_t)ts.parent[i0 + r];
            }
            rc = forward(c, D, base + i0, m, Qd, true);
            c->head_est = false;
            c->fsrc = FeatSrc{};
            c->tree = nullptr;
        }
        if (rc) return rc;
        if (c->cfg.temperature > 0.f)
            hipLaunchKernelGGL(tree_children_sample_kernel, dim3(m), dim3(AK_NT), 0, c->stream, (const float*)Qd, V, c->cfg.temperature, c->cfg.seed,
                               0u, (uint32_t)c->sq[0].round, ts, i0, c->d_hist() + base, c->d_draft());
        else
            hipLaunchKernelGGL(tree_children_kernel, dim3(m), dim3(AK_NT), 0, c->stream, (const float*)Qd, V, ts, i0, c->d_hist() + base, c->d_draft());
        LAUNCH_CHECK(c, "tree_children");
    }
    c->tshape = ts;
    c->sq[0].cur_k = k;
    c->phase = PH_TREE_DRAFTED;
    return METASD_OK;
}

int32_t metasd_verify_tree(metasd_ctx* c) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (c->phase != PH_TREE_DRAFTED) return c->fail(METASD_E_ORDER, "verify_tree: draft_tree has not been run for this round");
    const int n = c->tshape.n, base = c->sq[0].l - 1;
    TreeBlk tb{};
    tb.on = 1; tb.base = base; tb.i0 = 0;
    for (int i = 0; i < n; ++i) { tb.anc[i] = c->tanc[i]; tb.depth[i] = (uint8_t)c->tdepth[i]; }
    c->tree = &tb;
    const int rc = forward(c, c->target, base, n, c->d_P(), true);
    c->tree = nullptr;
    if (rc) return rc;
    c->phase = PH_TREE_VERIFIED;
    return METASD_OK;
}

int32_t metasd_accept_tree(metasd_ctx* c, int32_t* n_acc_out, int32_t* token_out, int32_t* path_out) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (c->phase != PH_TREE_VERIFIED) return c->fail(METASD_E_ORDER, "accept_tree: verify_tree has not been run for this round");
    const int n = c->tshape.n, V = c->target.d.vocab, l = c->sq[0].l, base = l - 1;
    if (c->cfg.temperature > 0.f) {
        hipLaunchKernelGGL(accept_tree_node_kernel, dim3(n), dim3(AK_NT), 0, c->stream, (const float*)c->d_P(), (const float*)c->d_Q(),
                           (const int32_t*)c->d_draft(), V, c->cfg.temperature, c->cfg.seed, 0u, (uint32_t)c->sq[0].round, c->tshape, c->d_tstep());
        LAUNCH_CHECK(c, "accept_tree (nodes)");
        hipLaunchKernelGGL(accept_tree_walk_kernel, dim3(1), dim3(64), 0, c->stream, (const int2*)c->d_tstep(), (const int32_t*)c->d_draft(),
                           c->tshape, c->d_res(), c->d_hist() + base);
    } else {
        int32_t* amax = reinterpret_cast<int32_t*>(c->d_cand());
        if (launch_sample(c->stream, c->d_P(), n, V, 0.f, c->cfg.seed, 0u, 0u, 0u, amax, 1, nullptr)) return c->fail(METASD_E_HIP, "launch argmax failed");
        hipLaunchKernelGGL(accept_tree_kernel, dim3(1), dim3(64), 0, c->stream, (const int32_t*)amax, (const int32_t*)c->d_draft(), c->tshape, c->d_res(),
                           c->d_hist() + base);
    }
    LAUNCH_CHECK(c, "accept_tree");
    Model& D = c->drafters[c->sq[0].cur_k];
    int rc = c->target.d.dtype == METASD_BF16 ? compact_kv<bf16_t>(c, c->target, base, TREE_MAX) : compact_kv<float>(c, c->target, base, TREE_MAX);
    if (!rc && !D.shared_kv && !D.head)                  // a head keeps nothing of the round: no rows to move
        rc = D.d.dtype == METASD_BF16 ? compact_kv<bf16_t>(c, D, base, c->tmaxdepth - 1) : compact_kv<float>(c, D, base, c->tmaxdepth - 1);
    if (rc) return rc;
    if (c->cfg.feature_heads) {                          // the target's features of the accepted nodes, from their slots to their positions
        const int Dm = c->target.d.d_model;
        hipLaunchKernelGGL(kv_compact_kernel<float>, dim3((unsigned)((Dm + 255) / 256)), dim3(256), 0, c->stream, c->d_feat(), 1, c->cfg.max_ctx, Dm,
                           base, (const int32_t*)c->d_res(), TREE_MAX, c->tshape.n);
        LAUNCH_CHECK(c, "feature rows of the accepted nodes");
    }
    if ((rc = c->fetch_results())) return rc;
    if (c->mirror<GridBar>(c->lay.bar)->abort) {
        (void)hipMemsetAsync(c->d_bar(), 0, sizeof(GridBar), c->stream);
        c->phase = PH_NONE;
        return c->fail(METASD_E_HIP, "a bounded device-side wait between workgroups timed out (split-K reduction); call metasd_set_context to start over");
    }
    const int32_t* hres = c->mirror<int32_t>(c->lay.res);
    const int32_t* htok = c->mirror<int32_t>(c->lay.draft);
    const int na = hres[0], token = hres[1];
    if (na < 0 || na > c->tmaxdepth || token < 0 || token >= V) return c->fail(METASD_E_HIP, "accept_tree: device returned n_acc %d token %d", na, token);
    for (int j = 0; j < na; ++j) {
        const int node = hres[2 + j];
        if (node < 1 || node >= n) return c->fail(METASD_E_HIP, "accept_tree: device returned path node %d", node);
        c->sq[0].hist[l + j] = htok[node];
        if (path_out) path_out[j] = node;
    }
    c->sq[0].hist[l + na] = token;
    c->sq[0].l = l + na + 1;
    c->target.kvl[0] = l + na;
    D.kvl[0] = std::min(l + na, l + c->tmaxdepth - 1);
    if (D.head) D.kvl[0] = l;                            // what a head computed from estimated features is not kept
    c->sq[0].round += 1;
    sync_shared_kv(c);
    c->phase = PH_READY;
    if (n_acc_out) *n_acc_out = na;
    if (token_out) *token_out = token;
    return METASD_OK;
}

// ---- stand-alone kernels

int32_t metasd_accept_logits(const float* P, const float* Q, const int32_t* d, int32_t rows, int32_t gamma, int32_t V,
                             float temperature, uint64_t seed, uint32_t round, uint32_t seq0, int32_t* n_acc, int32_t* token,
                             uint32_t* mask, double* bd, void* scratch, void* hip_stream) {
    if (!P || !Q || !d || !n_acc || !token || !scratch) return fail_global(METASD_E_INVALID, "accept_logits: NULL pointer");
    if (rows < 1 || rows > 65535 || gamma < 1 || gamma > 31 || !valid_vocab(V) || !(temperature >= 0.f))
        return fail_global(METASD_E_INVALID, "accept_logits: rows 1..65535, gamma 1..31, V %% 4 == 0, V <= 32768, T >= 0");
    // scratch: [rows (gamma+1)] candidates of 16 bytes, then the exchange words of the split kernel
    unsigned long long* xchg = (unsigned long long*)((char*)scratch + (size_t)rows * (gamma + 1) * 16);
    if (launch_accept((hipStream_t)hip_stream, P, Q, d, rows, gamma, V, temperature, seed, one_round(round), seq0, (int2*)scratch, bd, n_acc,
                      token, mask, nullptr, 0, xchg))
        return fail_global(METASD_E_HIP, "accept_logits: launch failed");
    return METASD_OK;
}

// Device address of `scratch` on the current device (asked for once per device, with that device current).
static int noalloc_scratch(unsigned char** out) {
    constexpr int MAX_DEV = 64;
    static std::mutex mu;
    static unsigned char* ptr[MAX_DEV] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_global(METASD_E_HIP, "accept_logits_noalloc: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEV) return fail_global(METASD_E_INVALID, "accept_logits_noalloc: device index %d not supported", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail_global(METASD_E_HIP, "accept_logits_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(e));
        ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = ptr[dev];
    return METASD_OK;
}

int32_t metasd_accept_logits_noalloc(const float* P, const float* Q, const int32_t* d, int32_t rows, int32_t gamma, int32_t V,
                                     float temperature, uint64_t seed, uint32_t round, uint32_t seq0, int32_t* n_acc,
                                     int32_t* token, uint32_t* mask, double* bd, void* hip_stream) {
    if (!P || !Q || !d || !n_acc || !token) return fail_global(METASD_E_INVALID, "accept_logits_noalloc: NULL pointer");
    if (rows < 1 || rows > 65535 || gamma < 1 || gamma > 31 || !valid_vocab(V) || !(temperature >= 0.f))
        return fail_global(METASD_E_INVALID, "accept_logits_noalloc: rows 1..65535, gamma 1..31, V %% 4 == 0, V <= 32768, T >= 0");
    const size_t items = (size_t)rows * (gamma + 1);
    if (items > METASD_ACCEPT_NOALLOC_MAX_ITEMS)
        return fail_global(METASD_E_INVALID, "accept_logits_noalloc: rows * (gamma + 1) = %zu exceeds the built-in scratch of %d items; use metasd_accept_logits with a scratch buffer of your own",
                           items, METASD_ACCEPT_NOALLOC_MAX_ITEMS);
    unsigned char* sp = nullptr;
    if (int rc = noalloc_scratch(&sp)) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    // The array keeps what the last call left.  The part this call uses is cleared by a kernel (not a memset: the call
    // may be recorded into a graph, and a replay repeats this call's launch tag, so the words of the replay before
    // must be gone).
    const unsigned n16 = (unsigned)(items * 336 / 16);
    hipLaunchKernelGGL(zero_fill_kernel, dim3((n16 + 255) / 256), dim3(256), 0, st, reinterpret_cast<uint4*>(sp), n16);
    if (hipGetLastError() != hipSuccess) return fail_global(METASD_E_HIP, "accept_logits_noalloc: launch failed");
    unsigned long long* xchg = reinterpret_cast<unsigned long long*>(sp + items * 16);
    if (launch_accept(st, P, Q, d, rows, gamma, V, temperature, seed, one_round(round), seq0, reinterpret_cast<int2*>(sp), bd, n_acc, token, mask,
                      nullptr, 0, xchg))
        return fail_global(METASD_E_HIP, "accept_logits_noalloc: launch failed");
    return METASD_OK;
}

int32_t metasd_sample_logits(const float* logits, int32_t rows, int32_t V, float temperature, uint64_t seed, uint32_t round,
                             uint32_t pos, uint32_t seq0, int32_t* tok, void* hip_stream) {
    if (!logits || !tok) return fail_global(METASD_E_INVALID, "sample_logits: NULL pointer");
    if (rows < 1 || !valid_vocab(V) || !(temperature >= 0.f)) return fail_global(METASD_E_INVALID, "sample_logits: rows >= 1, V %% 4 == 0, V <= 32768, T >= 0");
    if (launch_sample((hipStream_t)hip_stream, logits, rows, V, temperature, seed, round, pos, seq0, tok, 1, nullptr))
        return fail_global(METASD_E_HIP, "sample_logits: launch failed");
    return METASD_OK;
}

int32_t metasd_philox_words(uint64_t seed, uint32_t c0_start, int32_t n, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t* out,
                            void* hip_stream) {
    if (!out || n < 1) return fail_global(METASD_E_INVALID, "philox_words: bad argument");
    hipLaunchKernelGGL(philox_words_kernel, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)hip_stream, seed, c0_start, n, c1, c2,
                       c3, out);
    if (hipGetLastError() != hipSuccess) return fail_global(METASD_E_HIP, "philox_words: launch failed");
    return METASD_OK;
}

int32_t metasd_stream_read(const void* src, size_t bytes, uint32_t* sink, void* hip_stream) {
    if (!src || !sink || bytes < 1024 || ((uintptr_t)src & 15)) return fail_global(METASD_E_INVALID, "stream_read: bad argument");
    int dev = 0, ncu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ncu < 1)
        return fail_global(METASD_E_HIP, "stream_read: cannot query the device");
    const int grid = std::min(ncu * 4, METASD_STREAM_READ_SINK_WORDS / 4);
    hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(256), 0, (hipStream_t)hip_stream, (const u32x4*)src, bytes / 1024, sink);
    if (hipGetLastError() != hipSuccess) return fail_global(METASD_E_HIP, "stream_read: launch failed");
    return METASD_OK;
}

// ---- per-kernel timing

int32_t metasd_profile(metasd_ctx* c, int32_t max_records) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (max_records < 0 || max_records > (1 << 20)) return c->fail(METASD_E_INVALID, "profile: max_records out of range");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    while ((int)c->prof.size() < max_records) {
        metasd_ctx::ProfRec r{};
        HIP_TRY(c, hipEventCreate(&r.a));
        hipError_t e = hipEventCreate(&r.b);
        if (e != hipSuccess) { (void)hipEventDestroy(r.a); return c->fail(METASD_E_HIP, "hipEventCreate: %s", hipGetErrorString(e)); }
        c->prof.push_back(r);
    }
    c->prof_used = 0;
    c->prof_on = max_records > 0;
    return METASD_OK;
}

int32_t metasd_profile_read(metasd_ctx* c, int32_t kind, double* ms_total, int64_t* launches, double* bytes_total) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (kind < 0 || kind > 2) return c->fail(METASD_E_INVALID, "profile_read: unknown kind %d", kind);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    double ms = 0.0, by = 0.0;
    int64_t n = 0;
    for (size_t i = 0; i < c->prof_used; ++i) {
        if (c->prof[i].kind != kind) continue;
        float t = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&t, c->prof[i].a, c->prof[i].b));
        ms += t; by += c->prof[i].bytes; ++n;
    }
    if (ms_total) *ms_total = ms;
    if (launches) *launches = n;
    if (bytes_total) *bytes_total = by;
    return METASD_OK;
}

int32_t metasd_profile_shapes(metasd_ctx* c, int32_t target_only, int32_t max_rows, int32_t* n_out, int32_t* k_out, int32_t* m_out,
                              double* ms_out, int64_t* launches_out, double* bytes_out, int32_t* rows_out) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (max_rows < 1 || !n_out || !k_out || !m_out || !ms_out || !launches_out || !bytes_out || !rows_out)
        return c->fail(METASD_E_INVALID, "profile_shapes: bad argument");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    int rows = 0;
    for (size_t i = 0; i < c->prof_used; ++i) {
        const metasd_ctx::ProfRec& r = c->prof[i];
        if (r.kind != METASD_PROF_GEMM || (target_only && r.model != -1)) continue;
        int at = 0;
        while (at < rows && !(n_out[at] == r.n && k_out[at] == r.k && m_out[at] == r.m)) ++at;
        if (at == rows) {
            if (rows == max_rows) continue;               // table full: further shapes are left out
            n_out[at] = r.n; k_out[at] = r.k; m_out[at] = r.m; ms_out[at] = 0.0; launches_out[at] = 0; bytes_out[at] = 0.0;
            ++rows;
        }
        float t = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&t, r.a, r.b));
        ms_out[at] += t; launches_out[at] += 1; bytes_out[at] += r.bytes;
    }
    *rows_out = rows;
    return METASD_OK;
}

// ---- introspection

int32_t metasd_peek(metasd_ctx* c, int32_t what, void** dev_ptr_out, size_t* bytes_out) {
    if (!c) return fail_global(METASD_E_INVALID, "NULL ctx");
    if (!dev_ptr_out || !bytes_out) return c->fail(METASD_E_INVALID, "peek: NULL output");
    const size_t V = (size_t)c->target.d.vocab;
    switch (what) {
        case METASD_PEEK_P: *dev_ptr_out = c->d_P(); *bytes_out = (size_t)c->cfg.batch * (c->cfg.gamma_max + 1) * V * 4; break;
        case METASD_PEEK_Q: *dev_ptr_out = c->d_Q(); *bytes_out = (size_t)c->cfg.batch * c->cfg.gamma_max * V * 4; break;
        case METASD_PEEK_HIST: *dev_ptr_out = c->d_hist(); *bytes_out = (size_t)c->cfg.batch * c->cfg.max_ctx * 4; break;
        case METASD_PEEK_BD: *dev_ptr_out = c->d_bd(); *bytes_out = (size_t)c->cfg.batch * c->cfg.gamma_max * 8; break;
        case METASD_PEEK_FEAT:
            if (!c->cfg.feature_heads) return c->fail(METASD_E_INVALID, "peek: this context keeps no features (metasd_config.feature_heads)");
            *dev_ptr_out = c->d_feat(); *bytes_out = (size_t)c->cfg.max_ctx * c->target.d.d_model * 4; break;
        case METASD_PEEK_DRAFT: *dev_ptr_out = c->d_draft(); *bytes_out = (size_t)c->cfg.batch * (c->cfg.gamma_max + 1) * 4; break;
        default: return c->fail(METASD_E_INVALID, "peek: unknown buffer %d", what);
    }
    return METASD_OK;
}

int32_t metasd_state_seq(const metasd_ctx* c, int32_t seq, int32_t model, int32_t* l_out, int32_t* kv_len_out, int32_t* round_out) {
    if (!c || model < -1 || model >= c->cfg.K || seq < 0 || seq >= c->cfg.batch) return fail_global(METASD_E_INVALID, "state: bad argument");
    if (l_out) *l_out = c->sq[seq].l;
    if (kv_len_out) *kv_len_out = model < 0 ? c->target.kvl[seq] : c->drafters[model].kvl[seq];
    if (round_out) *round_out = c->sq[seq].round;
    return METASD_OK;
}

int32_t metasd_accept_fallbacks(const metasd_ctx* c, int64_t* count_out) {
    if (!c || !count_out) return fail_global(METASD_E_INVALID, "accept_fallbacks: bad argument");
    *count_out = c->accept_fallbacks;
    return METASD_OK;
}

int32_t metasd_state(const metasd_ctx* c, int32_t model, int32_t* l_out, int32_t* kv_len_out, int32_t* round_out) {
    return metasd_state_seq(c, 0, model, l_out, kv_len_out, round_out);
}

}  // extern "C"
