// C interface of libpql: context, argument validation, workspace layout and the launch
// sequences of the learner steps.  All device work is done by the kernels in pql_fused.hip and
// pql_chain.hip (row-tile kernels: one launch per learner step), pql_act16.hip (Actor step on 16-row
// tiles), pql_gemm.hip (LDS-tiled GEMMs, streaming weight gradients) and pql_kernels.hip (replay,
// heads, optimiser, statistics); this file only decides which problems go into which launch.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "pql_internal.h"

using namespace pql;

// ---- per-launch timing ----------------------------------------------------------------------
namespace pql {
namespace {
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> ev;      // 2 events per recorded launch
    struct Rec { int kid; double flops, bytes; };
    std::vector<Rec> recs;
    size_t cap = 0;
} g_prof;
const char* const k_gemm_mode[3] = {"nn", "nt", "tn"};
const char* const k_gemm_tile[5] = {"128x128", "64x64", "128x32", "128x64", "128x32_noise"};

// Names of the 15 (mode, tile) instances of the LDS-tiled GEMM kernel, built once (thread-safe: a function-local static).
const std::vector<std::string>& gemm_names() {
    static const std::vector<std::string> names = [] {
        std::vector<std::string> v;
        for (int k = 0; k < 15; ++k) v.push_back(std::string("gemm_grouped_") + k_gemm_mode[k / 5] + "_" + k_gemm_tile[k % 5]);
        return v;
    }();
    return names;
}
}  // namespace

const char* kernel_name(int kid) {
    if (kid == KID_GEMM + GEMM_TN * 5 + TILE_64x64) return "gemm_tn_stream_kernel";   // small weight gradients
    if (kid >= KID_GEMM && kid < KID_GEMM + 15) return gemm_names()[kid - KID_GEMM].c_str();
    switch (kid) {
        case KID_PUSH: return "push_kernel";
        case KID_SAMPLE: return "sample_kernel";
        case KID_HEAD_CRITIC: return "head_kernel_critic";
        case KID_HEAD_POLICY: return "head_kernel_policy";
        case KID_ADAM: return "adam_reduce_kernel";
        case KID_SOFT_UPDATE: return "soft_update_kernel";
        case KID_COPY: return "copy_kernel";
        case KID_FUSED_CRITIC: return "fused_critic_kernel";
        case KID_FUSED_POLICY: return "fused_policy_kernel";
        case KID_FUSED_ACT: return "fused_act_kernel";
        case KID_TRANSPOSE: return "transpose_kernel";
        case KID_ADAM_CLIP: return "adam_clip_kernel";
        case KID_OBS_STATS: return "obs_stats_chunk_kernel";
        case KID_OBS_MERGE: return "obs_stats_merge_kernel";
        case KID_NORMALIZE: return "normalize_rows_kernel";
        case KID_DIST_CRITIC: return "dist_head_kernel_critic";
        case KID_DIST_POLICY: return "dist_head_kernel_policy";
        case KID_SAC_SAMPLE: return "sac_sample_kernel";
        case KID_SAC_GRAD: return "sac_grad_kernel";
        case KID_SAC_ALPHA: return "sac_alpha_kernel";
        case KID_MFMA_PROBE: return "mfma_probe_kernel";
        case KID_LAYER_ROWTILE: return "layer_rowtile_kernel";
        case KID_NARROW_ROWTILE: return "narrow_rowtile_kernel";
        case KID_CHAIN_CRITIC: return "chain_critic_kernel";
        case KID_CHAIN_POLICY: return "chain_policy_kernel";
        case KID_CHAIN_ACT: return "chain_act_kernel";
        case KID_FUSED_ACT16: return "fused_act16_kernel";
        default: return "?";
    }
}

bool prof_active() { return g_prof.on && g_prof.recs.size() < g_prof.cap; }

ProfSlot prof_slot() {
    ProfSlot s{nullptr, nullptr, false};
    if (!prof_active()) return s;
    s.start = g_prof.ev[2 * g_prof.recs.size()];
    s.stop = g_prof.ev[2 * g_prof.recs.size() + 1];
    s.on = true;
    return s;
}

void prof_commit(const ProfSlot& s, int kid, double flops, double bytes) {
    if (s.on) g_prof.recs.push_back({kid, flops, bytes});
}
}  // namespace pql

// ---- scratch of pql_critic_update_static -------------------------------------------------------
// A device array of fixed size that takes the place of the caller's workspace.  Each GPU the library
// runs on holds one copy until the process ends.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
constexpr int STATIC_MAX_DEVICES = 64;
void* g_scratch_ptr[STATIC_MAX_DEVICES];      // per device: the address of that device's copy, once known
std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch` (looked up on the first call on that device).
hipError_t static_scratch_address(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr || (((uintptr_t)p) & 255)) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

struct pql_ctx {
    pql_config cfg;
    int L;                       // hidden layers
    int64_t T;                   // ring rows
    int64_t head, count, pushes, samples, acts, critic_t, actor_t, state_samples;
    // parameter offsets (floats) inside one actor / one critic vector: W then b per layer
    int64_t a_w[PQL_MAX_HIDDEN + 1], a_b[PQL_MAX_HIDDEN + 1], a_total;
    int64_t c_w[PQL_MAX_HIDDEN + 1], c_b[PQL_MAX_HIDDEN + 1], c_total;
    void* obs_norm;              // caller-owned device block of running observation statistics, or NULL
    float obs_eps;
    float* temperature;          // caller-owned device floats {log alpha, Adam m, Adam v, -} of the SAC variant, or NULL
    const float* temperature_v;  // the V-learner's copy of log alpha (defaults to the one above)
    float target_entropy;
    // vectors that follow an optimiser step (index 0: the critics' targets, 1: the lagged policy), or NULL
    float* track[2];
    float track_tau[2];
    // caller-owned block of transposed weights and the parameter vectors whose transposes it holds
    float* wcache;
    const float* wcache_critic;
    const float* wcache_actor;
    std::string err;
};

namespace {

constexpr size_t ALIGN_F = 64;   // workspace buffers start on 256-byte boundaries
inline size_t up(size_t x) { return (x + ALIGN_F - 1) / ALIGN_F * ALIGN_F; }

int validate_cfg(const pql_config* c) {
    if (!c) return PQL_ERR_NULL;
    if (c->obs_dim < 1 || c->act_dim < 1 || c->num_envs < 1 || c->nstep < 1) return PQL_ERR_INVALID_ARG;
    if (c->n_hidden < 1 || c->n_hidden > PQL_MAX_HIDDEN) return PQL_ERR_INVALID_ARG;
    for (int i = 0; i < c->n_hidden; ++i)
        if (c->hidden[i] < 1 || c->hidden[i] > 65536) return PQL_ERR_INVALID_ARG;
    if (c->hidden[c->n_hidden - 1] > 1024) return PQL_ERR_INVALID_ARG;   // head kernel register budget
    if (!(c->gamma > 0.f) || c->gamma > 1.f) return PQL_ERR_INVALID_ARG;
    if (c->max_batch < 1) return PQL_ERR_INVALID_ARG;
    if (c->capacity < (int64_t)c->num_envs * c->nstep) return PQL_ERR_INVALID_ARG;
    if (c->capacity / c->num_envs > 0x7fffffffLL) return PQL_ERR_INVALID_ARG;
    if ((int64_t)c->max_batch * c->act_dim > 0xffffffffLL) return PQL_ERR_INVALID_ARG;   // 32-bit element counter
    if (c->num_atoms < 0 || c->num_atoms > DIST_MAX_ATOMS) return PQL_ERR_INVALID_ARG;
    if (c->num_atoms >= 2 && !(c->v_max > c->v_min)) return PQL_ERR_INVALID_ARG;
    if (c->stochastic_policy != 0 && c->stochastic_policy != 1) return PQL_ERR_INVALID_ARG;
    // the stochastic policy is built for scalar critics; its gradient kernel keeps 2a + 1 columns of 256 rows in LDS
    if (c->stochastic_policy && (c->num_atoms >= 2 || c->act_dim > 31)) return PQL_ERR_INVALID_ARG;
    // The weight-gradient kernel addresses the rows of one wavefront's share of a split (at most a quarter of
    // the batch, when the batch is not split at all) with 32-bit byte offsets: the widest operand row
    // times that many rows must stay below 2 GiB for every batch the context may see.
    int64_t ld = c->obs_dim > c->act_dim ? c->obs_dim : c->act_dim;
    for (int i = 0; i < c->n_hidden; ++i) ld = c->hidden[i] > ld ? c->hidden[i] : ld;
    if (c->num_atoms > ld) ld = c->num_atoms;
    if (2 * (int64_t)c->act_dim > ld) ld = 2 * (int64_t)c->act_dim;
    if ((((int64_t)c->max_batch + 31) / 4 + 16) * (ld + 64) * 4 >= 0x7fffffffLL) return PQL_ERR_INVALID_ARG;
    return PQL_OK;
}

// Outputs of one critic: 1 (scalar Q) or the number of atoms of a distributional critic.
inline int critic_out(const pql_config* c) { return c->num_atoms >= 2 ? c->num_atoms : 1; }
inline bool distributional(const pql_config* c) { return c->num_atoms >= 2; }
// Outputs of the policy network: a (deterministic) or 2a (mean and log standard deviation).
inline int actor_out(const pql_config* c) { return c->stochastic_policy ? 2 * c->act_dim : c->act_dim; }

int64_t net_params(int in, const pql_config* c, int out, int64_t* w, int64_t* b) {
    int64_t off = 0;
    int prev = in;
    for (int l = 0; l <= c->n_hidden; ++l) {
        const int width = (l < c->n_hidden) ? c->hidden[l] : out;
        if (w) w[l] = off;
        off += (int64_t)prev * width;
        if (b) b[l] = off;
        off += width;
        prev = width;
    }
    return off;
}

// ---- tile choice and split-K planning -------------------------------------------------------
int choose_tile(int mode, const std::vector<GemmProb>& ps) {
    int max_n = 0, max_m = 0;
    long tiles128 = 0;
    for (const GemmProb& p : ps) {
        max_n = p.N > max_n ? p.N : max_n;
        max_m = p.M > max_m ? p.M : max_m;
        tiles128 += (long)((p.M + 127) / 128) * ((p.N + 127) / 128);
    }
    if (mode == GEMM_TN) return TILE_64x64;      // the streaming weight-gradient kernel
    if (max_n <= 32) return TILE_128x32;
    if (max_n <= 64) return TILE_64x64;
    // measured: the backward-data kernel is at its best with 64x64 tiles at every size; the forward
    // kernel gains from 128x128 tiles once there are several of them per compute unit
    if (mode == GEMM_NT) return TILE_64x64;
    return tiles128 >= 1024 ? TILE_128x128 : TILE_64x64;
}

int colsum_rows(int tile, int M) { return ((M + gemm_tile_m(tile) - 1) / gemm_tile_m(tile)) * gemm_waves_m(tile); }

// Split count for weight gradients over K batch rows with the given total of 64x64 output tiles.
// The streaming kernel keeps three workgroups per compute unit resident, so the launch runs in
// rounds of 768 workgroups and a round lasts as long as one split's rows: the smallest count within
// 2 % of the cheapest rounds x rows wins (every split costs one more slab for the reduction).
constexpr int DW_MAX_SPLITS = 32;
constexpr int DW_MIN_ROWS = 256;
int dw_max_splits(int K) {
    const int by_k = K / DW_MIN_ROWS;
    return by_k < 1 ? 1 : (by_k > DW_MAX_SPLITS ? DW_MAX_SPLITS : by_k);
}
int split_target(long tiles, int K) {
    const int smax = dw_max_splits(K);
    int best_s = 1;
    double best = 1e300;
    for (int s = 1; s <= smax; ++s) {
        const double rounds = (double)((tiles * s + 767) / 768);
        const double cost = rounds * (double)((K + s - 1) / s);
        if (cost < 0.98 * best) { best = cost; best_s = s; }
    }
    return best_s;
}

struct Layout {
    size_t hA[PQL_MAX_HIDDEN + 1], dA[PQL_MAX_HIDDEN + 1];           // index 1..L
    size_t hT[2][PQL_MAX_HIDDEN + 1], hQ[2][PQL_MAX_HIDDEN + 1], dQ[2][PQL_MAX_HIDDEN + 1];
    size_t colQ[2][PQL_MAX_HIDDEN + 1];                               // bias-grad partials of critic layer l
    size_t colA[PQL_MAX_HIDDEN + 2];                                  // bias-grad partials of actor layer l (1..L+1)
    size_t aOut, dPre, y, q[2];
    size_t p_dw[2], p_dbh[2], p_db[2], p_loss;
    size_t wT[2][PQL_MAX_HIDDEN + 1];                                 // transposed critic weights, layer l = 1..L-1
    size_t w1aT[2];                                                   // transposed action rows of the critics' first layer
    size_t waT[PQL_MAX_HIDDEN + 1];                                   // transposed policy weights, layer l = 1..L
    size_t splitk;
    size_t lgT[2], lgQ[2], p_dbo[2], woT[2];                          // distributional critics: logits, output-bias partials, W_out^T
    size_t mu2a, logp, epsb, dOut, p_sc, p_lp;                        // stochastic policy: outputs, log pi, draws, gradient, partials
    size_t sqp;                                                       // per-workgroup sums of squared gradients
    size_t xn;                                                        // standardised Actor observations
    size_t total;
};

// The row-tile fused kernels apply when every hidden layer is a multiple of 32 and at most
// FUSED_MAXW wide, the action vector fits one MFMA tile and the tile's LDS footprint fits a CU.
bool fused_ok(const pql_config* c) {
    int hmax = 0;
    for (int l = 0; l < c->n_hidden; ++l) {
        if (c->hidden[l] % 32 != 0 || c->hidden[l] > FUSED_MAXW) return false;
        hmax = c->hidden[l] > hmax ? c->hidden[l] : hmax;
    }
    const int aw = actor_out(c);                  // the policy's output columns share one 32-column tile
    if (aw > FUSED_MAX_ACT || c->obs_dim > 1024) return false;
    if (distributional(c) && hmax < 64) return false;   // the dlogits of a row tile borrow 64 columns of an activation tile
    return fused_lds_bytes(c->obs_dim, aw, hmax) <= 160 * 1024;
}
// The row-tile chain kernels take networks with a layer too wide for the kernels above (up to 512 columns),
// scalar critics and a deterministic policy, once the batch has a row tile for at least half the compute
// units (below that the LDS-tiled kernels, which spread one layer over more workgroups, are the better fit).
constexpr int CHAIN_MIN_TILES = 128;
bool chain_ok(const pql_config* c, int rows) {
    if (fused_ok(c) || distributional(c) || c->stochastic_policy) return false;
    if ((rows + FUSED_BM - 1) / FUSED_BM < CHAIN_MIN_TILES) return false;
    return chain_shape_ok(c->obs_dim, c->act_dim, c->hidden, c->n_hidden);
}
int max_hidden(const pql_config* c) {
    int hmax = 0;
    for (int l = 0; l < c->n_hidden; ++l) hmax = c->hidden[l] > hmax ? c->hidden[l] : hmax;
    return hmax;
}

inline long dw_tiles(int M, int N) { return (long)((M + 63) / 64) * ((N + 63) / 64); }

// Floats of split-K slab space that a list of (M, N) weight-gradient problems can need for any
// batch size up to K: (largest split count) x (sum of M*N).
size_t dw_slab_bound(const std::vector<std::pair<int, int>>& mn, int K) {
    size_t elems = 0;
    for (const auto& d : mn) elems += (size_t)d.first * d.second;
    return (size_t)dw_max_splits(K) * elems;
}

size_t splitk_floats(const pql_config* c, int B) {
    const int L = c->n_hidden;
    std::vector<std::pair<int, int>> critic, actor;
    for (int i = 0; i < 2; ++i) {
        critic.push_back({c->obs_dim, c->hidden[0]});
        critic.push_back({c->act_dim, c->hidden[0]});
        for (int l = 1; l < L; ++l) critic.push_back({c->hidden[l - 1], c->hidden[l]});
        if (distributional(c)) critic.push_back({c->hidden[L - 1], c->num_atoms});
    }
    actor.push_back({c->obs_dim, c->hidden[0]});
    for (int l = 1; l < L; ++l) actor.push_back({c->hidden[l - 1], c->hidden[l]});
    actor.push_back({c->hidden[L - 1], actor_out(c)});
    const size_t sc = dw_slab_bound(critic, B), sa = dw_slab_bound(actor, B);
    return sc > sa ? sc : sa;
}

void make_layout(const pql_config* c, Layout& w) {
    std::memset(&w, 0, sizeof(w));
    const int L = c->n_hidden;
    const size_t B = (size_t)c->max_batch;
    size_t off = 0;
    auto take = [&](size_t n) { const size_t o = off; off += up(n); return o; };
    const size_t crow = B / 32 + 8;                 // rows of a column-sum partial buffer
    size_t nwg = (size_t)head_workgroups((int)B);
    if (nwg < (B + FUSED_BM - 1) / FUSED_BM) nwg = (B + FUSED_BM - 1) / FUSED_BM;   // one partial row per row tile
    if (distributional(c) && nwg < (size_t)dist_head_workgroups((int)B)) nwg = (size_t)dist_head_workgroups((int)B);
    for (int l = 1; l <= L; ++l) {
        const size_t h = (size_t)c->hidden[l - 1];
        w.hA[l] = take(B * h);
        w.dA[l] = take(B * h);
        w.colA[l] = take(crow * h);
        for (int i = 0; i < 2; ++i) {
            w.hT[i][l] = take(B * h);
            w.hQ[i][l] = take(B * h);
            w.dQ[i][l] = take(B * h);
            w.colQ[i][l] = take(crow * h);
        }
    }
    w.colA[L + 1] = take(crow * (size_t)actor_out(c));
    w.aOut = take(B * c->act_dim);
    w.dPre = take(B * (size_t)actor_out(c));
    w.y = take(B);
    const size_t hl = (size_t)c->hidden[L - 1];
    for (int i = 0; i < 2; ++i) {
        w.q[i] = take(B);
        w.p_dw[i] = take(nwg * hl);
        w.p_dbh[i] = take(nwg * hl);
        w.p_db[i] = take(nwg);
    }
    w.p_loss = take(2 * nwg);
    for (int i = 0; i < 2; ++i) {
        for (int l = 1; l < L; ++l) w.wT[i][l] = take((size_t)c->hidden[l - 1] * c->hidden[l]);
        w.w1aT[i] = take((size_t)c->act_dim * c->hidden[0]);
    }
    for (int l = 1; l <= L; ++l) w.waT[l] = take((size_t)c->hidden[l - 1] * (l < L ? c->hidden[l] : actor_out(c)));
    w.splitk = take(splitk_floats(c, (int)B));
    {
        const size_t pa = (size_t)pql_actor_param_count(c), pc = 2 * (size_t)pql_critic_param_count(c);
        w.sqp = take(adam_reduce_blocks_bound(pa > pc ? pa : pc, RED_MAX_TENSORS));
    }
    w.xn = fused_ok(c) ? off : take(B * (size_t)c->obs_dim);
    if (c->stochastic_policy) {
        const size_t a2 = 2 * (size_t)c->act_dim, nblk = (B + SAC_ROWS - 1) / SAC_ROWS;
        w.mu2a = take(B * a2);
        w.logp = take(B);
        w.epsb = take(B * c->act_dim);
        w.dOut = take(B * a2);
        w.p_sc = take(nblk * a2);
        w.p_lp = take(nblk > nwg ? nblk : nwg);       // one partial per workgroup of whichever kernel writes them
    }
    if (distributional(c))
        for (int i = 0; i < 2; ++i) {
            w.lgT[i] = take(B * (size_t)c->num_atoms);
            w.lgQ[i] = take(B * (size_t)c->num_atoms);
            w.p_dbo[i] = take(nwg * (size_t)c->num_atoms);
            w.woT[i] = take((size_t)c->num_atoms * c->hidden[L - 1]);
        }
    w.total = off;
}

// Transposed weights kept between calls (pql_weight_cache_*): the same matrices the workspace holds as
// wT / w1aT / woT / waT, in a block of the caller's.
struct CacheLayout {
    size_t wT[2][PQL_MAX_HIDDEN + 1], w1aT[2], woT[2], waT[PQL_MAX_HIDDEN + 1];
    size_t total;
};

void make_cache_layout(const pql_config* c, CacheLayout& w) {
    std::memset(&w, 0, sizeof(w));
    const int L = c->n_hidden;
    size_t off = 0;
    auto take = [&](size_t n) { const size_t o = off; off += up(n); return o; };
    for (int i = 0; i < 2; ++i) {
        for (int l = 1; l < L; ++l) w.wT[i][l] = take((size_t)c->hidden[l - 1] * c->hidden[l]);
        w.w1aT[i] = take((size_t)c->act_dim * c->hidden[0]);
        w.woT[i] = take((size_t)critic_out(c) * c->hidden[L - 1]);
    }
    for (int l = 1; l <= L; ++l) w.waT[l] = take((size_t)c->hidden[l - 1] * (l < L ? c->hidden[l] : actor_out(c)));
    w.total = off;
}

inline int vec_ok(const float* p, int ld) { return ((((uintptr_t)p) & 15) == 0 && (ld % 4) == 0) ? 1 : 0; }

GemmProb prob(int M, int N, float* C, int ldc, int epi) {
    GemmProb p;
    std::memset(&p, 0, sizeof(p));
    p.M = M; p.N = N; p.C = C; p.ldc = ldc; p.epi = epi; p.splits = 1;
    return p;
}

void add_seg(GemmProb& p, const float* A, int lda, const float* Bm, int ldb, int K) {
    GemmSeg& s = p.seg[p.nseg++];
    s.A = A; s.lda = lda; s.B = Bm; s.ldb = ldb; s.K = K;
    s.vec = vec_ok(A, lda) | (vec_ok(Bm, ldb) << 1);
}

struct Err {
    pql_ctx* ctx;
    int fail(int code, const char* what) { ctx->err = what; return code; }
    int hip(hipError_t e, const char* where) {
        ctx->err = std::string(where) + ": " + hipGetErrorString(e);
        return PQL_ERR_HIP;
    }
};

// Launches a list of problems of one mode, in chunks that fit one kernel argument block.
hipError_t run(int mode, int tile, std::vector<GemmProb>& ps, const GemmNoise* nz, hipStream_t st) {
    for (size_t i = 0; i < ps.size(); i += GEMM_MAX_PROB) {
        GemmGroup g;
        std::memset(&g, 0, sizeof(g));
        if (nz) g.noise = *nz;
        g.nprob = (int)((ps.size() - i < (size_t)GEMM_MAX_PROB) ? ps.size() - i : GEMM_MAX_PROB);
        for (int k = 0; k < g.nprob; ++k) g.p[k] = ps[i + k];
        hipError_t e;
        if (mode == GEMM_NN && nz == nullptr && layer_rowtile_ok(g)) e = layer_rowtile_launch(g, st);
        else if (mode == GEMM_NN && narrow_rowtile_ok(g)) e = narrow_rowtile_launch(g, st);
        else e = gemm_launch(mode, tile, g, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Whether run(GEMM_NN, ...) sends this list through the row-tile layer kernel (then column-sum
// partials come one row per 32 batch rows).
bool takes_row_tiles(const std::vector<GemmProb>& ps) {
    if (ps.empty() || ps.size() > (size_t)GEMM_MAX_PROB) return false;
    GemmGroup g;
    std::memset(&g, 0, sizeof(g));
    g.nprob = (int)ps.size();
    for (int k = 0; k < g.nprob; ++k) g.p[k] = ps[k];
    return layer_rowtile_ok(g);
}

// The same for the narrow (action-wide) row-tile kernel.
bool takes_narrow_tiles(const std::vector<GemmProb>& ps) {
    if (ps.empty() || ps.size() > (size_t)GEMM_MAX_PROB) return false;
    GemmGroup g;
    std::memset(&g, 0, sizeof(g));
    g.nprob = (int)ps.size();
    for (int k = 0; k < g.nprob; ++k) g.p[k] = ps[k];
    return narrow_rowtile_ok(g);
}

hipError_t run_auto(int mode, std::vector<GemmProb>& ps, hipStream_t st) {
    return run(mode, choose_tile(mode, ps), ps, nullptr, st);
}

// Weight-gradient problems: assigns split counts and slab addresses, launches, and appends one
// reduction entry per problem.  `offsets[i]` is the parameter offset of problem i's tensor.
hipError_t run_dw(std::vector<GemmProb>& ps, const std::vector<int64_t>& offsets, int K, float* slab,
                  AdamArgs& ad, hipStream_t st, const std::vector<float*>* tdst = nullptr) {
    if (ps.empty()) return hipSuccess;
    long tiles = 0;
    for (const GemmProb& p : ps) tiles += dw_tiles(p.M, p.N);
    int S = split_target(tiles, K);
    const int chunk = ((K + S - 1) / S + 31) / 32 * 32;
    S = (K + chunk - 1) / chunk;
    for (size_t i = 0; i < ps.size(); ++i) {
        GemmProb& p = ps[i];
        // the kernel addresses a wavefront's rows (a quarter of a split) with 32-bit byte offsets; pql_create
        // has refused configurations that could exceed them (validate_cfg), so this cannot trigger
        const int64_t ld = p.seg[0].lda > p.seg[0].ldb ? p.seg[0].lda : p.seg[0].ldb;
        if (((int64_t)chunk / 4 + 16) * (ld + 64) * 4 >= 0x7fffffffLL) return hipErrorInvalidValue;
        p.splits = S; p.k_chunk = chunk;
        p.C = slab; p.ldc = p.N;
        p.split_stride = (int64_t)p.M * p.N;
        RedTensor& t = ad.t[ad.ntensors++];
        t.offset = offsets[i]; t.stride = p.split_stride; t.partial = slab;
        t.count = p.M * p.N; t.nparts = S;
        if (tdst != nullptr && (*tdst)[i] != nullptr) { t.tdst = (*tdst)[i]; t.trows = p.M; t.tcols = p.N; }
        slab += (size_t)S * p.M * p.N;
    }
    return run(GEMM_TN, TILE_64x64, ps, nullptr, st);
}

void red(AdamArgs& ad, int64_t offset, const float* partial, int count, int nparts, int64_t stride) {
    RedTensor& t = ad.t[ad.ntensors++];
    t.offset = offset; t.partial = partial; t.count = count; t.nparts = nparts; t.stride = stride;
}

bool adam_ok(const pql_adam& o) {
    return o.lr >= 0.f && o.beta1 >= 0.f && o.beta1 < 1.f && o.beta2 >= 0.f && o.beta2 < 1.f && o.eps >= 0.f &&
           o.max_grad_norm >= 0.f && o.max_grad_norm <= 3.0e38f;
}

void fill_adam(AdamArgs& ad, const pql_adam& o, int64_t t) {
    ad.lr = o.lr; ad.beta1 = o.beta1; ad.beta2 = o.beta2; ad.eps = o.eps;
    ad.inv_bc1 = (float)(1.0 / (1.0 - std::pow((double)o.beta1, (double)t)));
    ad.inv_bc2 = (float)(1.0 / (1.0 - std::pow((double)o.beta2, (double)t)));
}

// Forward pass of one hidden layer l (1-based) for a list of networks sharing the layer shape.
struct FwdNet {
    const float* params;     // network vector
    const int64_t* w; const int64_t* b;
    const float* in0; int ld0; int k0;   // first input segment (layer 1) / previous activations
    const float* in1; int ld1; int k1;   // optional second segment (layer 1 of a critic)
    float* out;
};

// Fills the critic part / the policy part of a block of transposed weights (layout `cl` at `dst`).
hipError_t transpose_critic_weights(const pql_ctx* c, const float* critic_params, float* dst, const CacheLayout& cl,
                                    hipStream_t st) {
    const int L = c->L, o = c->cfg.obs_dim, ad = c->cfg.act_dim, H1 = c->cfg.hidden[0];
    TransposeArgs tr;
    tr.n = 0;
    auto add = [&](const float* src, float* to, int rows, int cols) {
        TransposeArgs::Mat& mt = tr.m[tr.n++];
        mt.src = src; mt.dst = to; mt.rows = rows; mt.cols = cols;
    };
    for (int i = 0; i < 2; ++i) {
        const float* q = critic_params + i * c->c_total;
        for (int l = 1; l < L; ++l) add(q + c->c_w[l], dst + cl.wT[i][l], c->cfg.hidden[l - 1], c->cfg.hidden[l]);
        add(q + c->c_w[0] + (int64_t)o * H1, dst + cl.w1aT[i], ad, H1);
        if (distributional(&c->cfg)) add(q + c->c_w[L], dst + cl.woT[i], c->cfg.hidden[L - 1], c->cfg.num_atoms);
    }
    return transpose_launch(tr, st);
}

hipError_t transpose_actor_weights(const pql_ctx* c, const float* actor_params, float* dst, const CacheLayout& cl,
                                   hipStream_t st) {
    const int L = c->L;
    TransposeArgs tr;
    tr.n = 0;
    for (int l = 1; l <= L; ++l) {
        TransposeArgs::Mat& mt = tr.m[tr.n++];
        mt.src = actor_params + c->a_w[l]; mt.dst = dst + cl.waT[l];
        mt.rows = c->cfg.hidden[l - 1]; mt.cols = l < L ? c->cfg.hidden[l] : actor_out(&c->cfg);
    }
    return transpose_launch(tr, st);
}

}  // namespace

// =============================================================================================
extern "C" {

int32_t pql_create(const pql_config* cfg, pql_ctx** out) {
    if (!out) return PQL_ERR_NULL;
    *out = nullptr;
    const int rc = validate_cfg(cfg);
    if (rc != PQL_OK) return rc;
    pql_ctx* c = new (std::nothrow) pql_ctx();
    if (!c) return PQL_ERR_INVALID_ARG;
    c->cfg = *cfg;
    c->L = cfg->n_hidden;
    c->T = cfg->capacity / cfg->num_envs;
    c->head = c->count = c->pushes = c->samples = c->acts = c->critic_t = c->actor_t = c->state_samples = 0;
    c->obs_norm = nullptr;
    c->obs_eps = 0.f;
    c->a_total = net_params(cfg->obs_dim, cfg, actor_out(cfg), c->a_w, c->a_b);
    c->temperature = nullptr;
    c->temperature_v = nullptr;
    c->target_entropy = 0.f;
    c->track[0] = c->track[1] = nullptr;
    c->track_tau[0] = c->track_tau[1] = 0.f;
    c->wcache = nullptr;
    c->wcache_critic = c->wcache_actor = nullptr;
    c->c_total = net_params(cfg->obs_dim + cfg->act_dim, cfg, critic_out(cfg), c->c_w, c->c_b);
    *out = c;
    return PQL_OK;
}

int32_t pql_destroy(pql_ctx* ctx) {
    if (!ctx) return PQL_ERR_NULL;
    delete ctx;
    return PQL_OK;
}

int64_t pql_replay_rows(const pql_config* cfg) {
    const int rc = validate_cfg(cfg);
    return rc != PQL_OK ? rc : cfg->capacity / cfg->num_envs;
}

int64_t pql_actor_param_count(const pql_config* cfg) {
    const int rc = validate_cfg(cfg);
    return rc != PQL_OK ? rc : net_params(cfg->obs_dim, cfg, actor_out(cfg), nullptr, nullptr);
}

int64_t pql_critic_param_count(const pql_config* cfg) {
    const int rc = validate_cfg(cfg);
    return rc != PQL_OK ? rc : net_params(cfg->obs_dim + cfg->act_dim, cfg, critic_out(cfg), nullptr, nullptr);
}

int64_t pql_workspace_bytes(const pql_config* cfg) {
    const int rc = validate_cfg(cfg);
    if (rc != PQL_OK) return rc;
    Layout w;
    make_layout(cfg, w);
    return (int64_t)(w.total * sizeof(float));
}

int32_t pql_workspace_view(const pql_config* cfg, int32_t what, int64_t* offset_bytes) {
    if (!offset_bytes) return PQL_ERR_NULL;
    const int rc = validate_cfg(cfg);
    if (rc != PQL_OK) return rc;
    Layout w;
    make_layout(cfg, w);
    size_t off;
    switch (what) {
        case PQL_VIEW_TD_TARGET: off = w.y; break;
        case PQL_VIEW_Q1: off = w.q[0]; break;
        case PQL_VIEW_Q2: off = w.q[1]; break;
        default: return PQL_ERR_INVALID_ARG;
    }
    *offset_bytes = (int64_t)(off * sizeof(float));
    return PQL_OK;
}

const char* pql_last_error(const pql_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int32_t pql_get_state(const pql_ctx* c, int64_t out[8]) {
    if (!c || !out) return PQL_ERR_NULL;
    out[0] = c->head; out[1] = c->count; out[2] = c->pushes; out[3] = c->samples;
    out[4] = c->acts; out[5] = c->critic_t; out[6] = c->actor_t; out[7] = c->state_samples;
    return PQL_OK;
}

int32_t pql_set_state(pql_ctx* c, const int64_t in[8]) {
    if (!c || !in) return PQL_ERR_NULL;
    Err E{c};
    if (in[0] < 0 || in[0] >= c->T || in[1] < 0 || in[1] > c->T) return E.fail(PQL_ERR_INVALID_ARG, "ring cursor out of range");
    for (int i = 2; i < 8; ++i)
        if (in[i] < 0) return E.fail(PQL_ERR_INVALID_ARG, "negative counter");
    c->head = in[0]; c->count = in[1]; c->pushes = in[2]; c->samples = in[3];
    c->acts = in[4]; c->critic_t = in[5]; c->actor_t = in[6]; c->state_samples = in[7];
    return PQL_OK;
}

// ---------------------------------------------------------------------------------------------
int32_t pql_replay_push(pql_ctx* c, pql_replay_storage st, const float* obs, const float* act, const float* rew,
                        const float* next_obs, const float* done, void* stream) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!st.obs || !st.act || !st.rew || !st.next_obs || !st.done || !obs || !act || !rew || !next_obs || !done)
        return E.fail(PQL_ERR_NULL, "pql_replay_push: null pointer");
    const int64_t N = c->cfg.num_envs, o = c->cfg.obs_dim, a = c->cfg.act_dim;
    const int64_t base = c->head * N;
    PushArgs p;
    p.src[0] = obs;      p.dst[0] = st.obs + base * o;       p.count[0] = N * o;
    p.src[1] = act;      p.dst[1] = st.act + base * a;       p.count[1] = N * a;
    p.src[2] = rew;      p.dst[2] = st.rew + base;           p.count[2] = N;
    p.src[3] = next_obs; p.dst[3] = st.next_obs + base * o;  p.count[3] = N * o;
    p.src[4] = done;     p.dst[4] = st.done + base;          p.count[4] = N;
    hipError_t e = push_launch(p, (hipStream_t)stream);
    if (e != hipSuccess) return E.hip(e, "pql_replay_push");
    // the row copy is enqueued: the cursor covers the row from here on, whatever happens to the statistics
    c->head = (c->head + 1) % c->T;
    c->count = c->count + 1 < c->T ? c->count + 1 : c->T;
    c->pushes += 1;
    if (c->obs_norm) {
        e = obs_stats_update_launch(obs_stats_view(c->obs_norm, (int)o), obs, (int)N, (int)o, c->obs_eps, (hipStream_t)stream);
        if (e != hipSuccess) return E.hip(e, "pql_replay_push: observation statistics (the row itself was stored)");
    }
    return PQL_OK;
}

static int32_t sample_common(pql_ctx* c, pql_replay_storage st, const int64_t* idx_in, int32_t batch, pql_batch out,
                             void* stream, const char* who) {
    Err E{c};
    if (!st.obs || !st.act || !st.rew || !st.next_obs || !st.done || !out.obs || !out.act || !out.ret ||
        !out.next_obs || !out.boot || (!idx_in && !out.idx))
        return E.fail(PQL_ERR_NULL, who);
    if (batch < 0) return E.fail(PQL_ERR_INVALID_ARG, who);
    if (batch > c->cfg.max_batch) return E.fail(PQL_ERR_BATCH_TOO_LARGE, who);
    if (c->count < c->cfg.nstep) return E.fail(PQL_ERR_NOT_ENOUGH_DATA, who);
    SampleArgs a;
    a.st = st; a.out = out; a.idx_in = idx_in;
    a.batch = batch; a.o = c->cfg.obs_dim; a.a = c->cfg.act_dim; a.N = c->cfg.num_envs; a.T = (int)c->T;
    a.nstep = c->cfg.nstep; a.head = (int)c->head; a.count = (int)c->count; a.gamma = c->cfg.gamma;
    a.key0 = (uint32_t)(c->cfg.seed & 0xffffffffu); a.key1 = (uint32_t)(c->cfg.seed >> 32);
    a.ctr2 = (uint32_t)((uint64_t)c->samples & 0xffffffffu); a.ctr3 = (uint32_t)((uint64_t)c->samples >> 32);
    a.stream_id = 1u; a.only_obs = 0;
    a.nmean = a.nrstd = nullptr;
    if (c->obs_norm) {
        const ObsStatsView ov = obs_stats_view(c->obs_norm, c->cfg.obs_dim);
        a.nmean = ov.mean_f; a.nrstd = ov.rstd_f;
    }
    const hipError_t e = sample_launch(a, (hipStream_t)stream);
    if (e != hipSuccess) return E.hip(e, who);
    return PQL_OK;
}

int32_t pql_sample_nstep(pql_ctx* c, pql_replay_storage st, int32_t batch, pql_batch out, void* stream) {
    if (!c) return PQL_ERR_NULL;
    const int32_t rc = sample_common(c, st, nullptr, batch, out, stream, "pql_sample_nstep");
    if (rc == PQL_OK) c->samples += 1;
    return rc;
}

int32_t pql_sample_states(pql_ctx* c, pql_replay_storage st, int32_t batch, int64_t* idx_out, float* obs_out,
                          void* stream) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    const char* who = "pql_sample_states";
    if (!st.obs || !idx_out || !obs_out) return E.fail(PQL_ERR_NULL, who);
    if (batch < 0) return E.fail(PQL_ERR_INVALID_ARG, who);
    if (batch > c->cfg.max_batch) return E.fail(PQL_ERR_BATCH_TOO_LARGE, who);
    if (c->count < 1) return E.fail(PQL_ERR_NOT_ENOUGH_DATA, who);
    SampleArgs a;
    std::memset(&a, 0, sizeof(a));
    a.st = st; a.out.idx = idx_out; a.out.obs = obs_out;
    a.batch = batch; a.o = c->cfg.obs_dim; a.a = c->cfg.act_dim; a.N = c->cfg.num_envs; a.T = (int)c->T;
    a.nstep = 1; a.head = (int)c->head; a.count = (int)c->count; a.gamma = c->cfg.gamma;
    a.key0 = (uint32_t)(c->cfg.seed & 0xffffffffu); a.key1 = (uint32_t)(c->cfg.seed >> 32);
    a.ctr2 = (uint32_t)((uint64_t)c->state_samples & 0xffffffffu); a.ctr3 = (uint32_t)((uint64_t)c->state_samples >> 32);
    a.stream_id = 3u; a.only_obs = 1;
    if (c->obs_norm) {
        const ObsStatsView ov = obs_stats_view(c->obs_norm, c->cfg.obs_dim);
        a.nmean = ov.mean_f; a.nrstd = ov.rstd_f;
    }
    const hipError_t e = sample_launch(a, (hipStream_t)stream);
    if (e != hipSuccess) return E.hip(e, who);
    c->state_samples += 1;
    return PQL_OK;
}

int32_t pql_gather_nstep(pql_ctx* c, pql_replay_storage st, const int64_t* idx, int32_t batch, pql_batch out,
                         void* stream) {
    if (!c) return PQL_ERR_NULL;
    if (!idx) { c->err = "pql_gather_nstep: null idx"; return PQL_ERR_NULL; }
    return sample_common(c, st, idx, batch, out, stream, "pql_gather_nstep");
}

// ---------------------------------------------------------------------------------------------
// Forward passes of the policy (hidden layers), shared by act / critic update / policy update.
static hipError_t actor_hidden_forward(pql_ctx* c, const float* params, const float* obs, int B, float* ws,
                                       const Layout& w, hipStream_t st) {
    const int L = c->L;
    for (int l = 1; l <= L; ++l) {
        std::vector<GemmProb> ps;
        const int H = c->cfg.hidden[l - 1];
        GemmProb p = prob(B, H, ws + w.hA[l], H, EPI_BIAS_ELU);
        if (l == 1) add_seg(p, obs, c->cfg.obs_dim, params + c->a_w[0], H, c->cfg.obs_dim);
        else add_seg(p, ws + w.hA[l - 1], c->cfg.hidden[l - 2], params + c->a_w[l - 1], H, c->cfg.hidden[l - 2]);
        p.bias = params + c->a_b[l - 1];
        ps.push_back(p);
        const hipError_t e = run_auto(GEMM_NN, ps, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Draw selection of the stochastic policy inside the row-tile kernels (off for a deterministic policy).
static FusedSac fused_sac(const pql_ctx* c, uint32_t stream_id, int64_t call, const float* log_alpha) {
    FusedSac f;
    std::memset(&f, 0, sizeof(f));
    f.on = c->cfg.stochastic_policy ? 1 : 0;
    f.stream_id = stream_id;
    f.key0 = (uint32_t)(c->cfg.seed & 0xffffffffu); f.key1 = (uint32_t)(c->cfg.seed >> 32);
    f.ctr2 = (uint32_t)((uint64_t)call & 0xffffffffu); f.ctr3 = (uint32_t)((uint64_t)call >> 32);
    f.log_alpha = log_alpha;
    return f;
}

// Output layer of the stochastic policy (mu, raw log sigma) on top of hA[L], then one sample per row.
static hipError_t stochastic_policy_sample(pql_ctx* c, const float* params, int B, float* ws, const Layout& w, float* act,
                                           float* logp, float* eps, uint32_t stream_id, int64_t call, hipStream_t st) {
    const int L = c->L, HL = c->cfg.hidden[L - 1], ad = c->cfg.act_dim;
    std::vector<GemmProb> ps;
    GemmProb p = prob(B, 2 * ad, ws + w.mu2a, 2 * ad, EPI_BIAS);
    add_seg(p, ws + w.hA[L], HL, params + c->a_w[L], 2 * ad, HL);
    p.bias = params + c->a_b[L];
    ps.push_back(p);
    hipError_t e = run_auto(GEMM_NN, ps, st);
    if (e != hipSuccess) return e;
    SacSampleArgs sa;
    sa.B = B; sa.a = ad; sa.out2a = ws + w.mu2a; sa.act = act; sa.logp = logp; sa.eps = eps;
    sa.stream_id = stream_id;
    sa.key0 = (uint32_t)(c->cfg.seed & 0xffffffffu); sa.key1 = (uint32_t)(c->cfg.seed >> 32);
    sa.ctr2 = (uint32_t)((uint64_t)call & 0xffffffffu); sa.ctr3 = (uint32_t)((uint64_t)call >> 32);
    return sac_sample_launch(sa, st);
}

// One hidden layer of a critic as a forward problem.
static GemmProb critic_layer(pql_ctx* c, const float* params, int l, const float* s, const float* a, int lda_a,
                             const float* h_prev, float* h_out, int B) {
    const int H = c->cfg.hidden[l - 1];
    GemmProb p = prob(B, H, h_out, H, EPI_BIAS_ELU);
    if (l == 1) {
        const int o = c->cfg.obs_dim, ad = c->cfg.act_dim;
        add_seg(p, s, o, params + c->c_w[0], H, o);
        add_seg(p, a, lda_a, params + c->c_w[0] + (int64_t)o * H, H, ad);
    } else {
        add_seg(p, h_prev, c->cfg.hidden[l - 2], params + c->c_w[l - 1], H, c->cfg.hidden[l - 2]);
    }
    p.bias = params + c->c_b[l - 1];
    return p;
}

int32_t pql_actor_act(pql_ctx* c, const float* actor_params, const float* obs, int32_t num, float sigma_min,
                      float sigma_max, float* act_out, void* workspace, void* stream) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!actor_params || !obs || !act_out || !workspace) return E.fail(PQL_ERR_NULL, "pql_actor_act: null pointer");
    if (num < 1 || sigma_min < 0.f || sigma_max < 0.f) return E.fail(PQL_ERR_INVALID_ARG, "pql_actor_act: bad num/sigma");
    if (num > c->cfg.max_batch) return E.fail(PQL_ERR_BATCH_TOO_LARGE, "pql_actor_act: num > max_batch");
    if (((uintptr_t)workspace) & 255) return E.fail(PQL_ERR_ALIGNMENT, "pql_actor_act: workspace not 256-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    float* ws = (float*)workspace;
    Layout w;
    make_layout(&c->cfg, w);
    const bool chain = chain_ok(&c->cfg, num);
    if (fused_ok(&c->cfg) || chain) {
        FusedActArgs fa;
        std::memset(&fa, 0, sizeof(fa));
        fa.B = num; fa.o = c->cfg.obs_dim; fa.a = c->cfg.act_dim; fa.L = c->L; fa.hmax = max_hidden(&c->cfg);
        for (int l = 0; l < c->L; ++l) fa.H[l] = c->cfg.hidden[l];
        for (int l = 0; l <= c->L; ++l) { fa.pi.w[l] = actor_params + c->a_w[l]; fa.pi.b[l] = actor_params + c->a_b[l]; }
        fa.obs = obs; fa.act_out = act_out;
        if (c->obs_norm) {
            const ObsStatsView ov = obs_stats_view(c->obs_norm, c->cfg.obs_dim);
            fa.nmean = ov.mean_f; fa.nrstd = ov.rstd_f;
        }
        fa.noise.act_dim = c->cfg.act_dim; fa.noise.sigma_rows = num; fa.noise.sigma_min = sigma_min; fa.noise.sigma_max = sigma_max;
        fa.noise.key0 = (uint32_t)(c->cfg.seed & 0xffffffffu); fa.noise.key1 = (uint32_t)(c->cfg.seed >> 32);
        fa.noise.ctr2 = (uint32_t)((uint64_t)c->acts & 0xffffffffu); fa.noise.ctr3 = (uint32_t)((uint64_t)c->acts >> 32);
        fa.sac = fused_sac(c, 2u, c->acts, nullptr);
        // up to 4096 environments the 32-row tiles leave compute units idle: 16-row tiles where that kernel applies
        const hipError_t fe = chain ? chain_act_launch(fa, st) : (act16_ok(fa) ? fused_act16_launch(fa, st) : fused_act_launch(fa, st));
        if (fe != hipSuccess) return E.hip(fe, "pql_actor_act");
        c->acts += 1;
        return PQL_OK;
    }
    hipError_t e;
    if (c->obs_norm) {
        const ObsStatsView ov = obs_stats_view(c->obs_norm, c->cfg.obs_dim);
        e = normalize_rows_launch(obs, ov.mean_f, ov.rstd_f, ws + w.xn, num, c->cfg.obs_dim, st);
        if (e != hipSuccess) return E.hip(e, "pql_actor_act");
        obs = ws + w.xn;
    }
    e = actor_hidden_forward(c, actor_params, obs, num, ws, w, st);
    if (e != hipSuccess) return E.hip(e, "pql_actor_act");
    if (c->cfg.stochastic_policy) {     // exploration is the policy's own randomness; the sigma schedule does not apply
        e = stochastic_policy_sample(c, actor_params, num, ws, w, act_out, nullptr, nullptr, 2u, c->acts, st);
        if (e != hipSuccess) return E.hip(e, "pql_actor_act");
        c->acts += 1;
        return PQL_OK;
    }
    const int L = c->L, HL = c->cfg.hidden[L - 1], ad = c->cfg.act_dim;
    std::vector<GemmProb> ps;
    GemmProb p = prob(num, ad, act_out, ad, EPI_BIAS_TANH_NOISE);
    add_seg(p, ws + w.hA[L], HL, actor_params + c->a_w[L], ad, HL);
    p.bias = actor_params + c->a_b[L];
    ps.push_back(p);
    GemmNoise nz;
    nz.act_dim = ad; nz.sigma_rows = num; nz.sigma_min = sigma_min; nz.sigma_max = sigma_max;
    nz.key0 = (uint32_t)(c->cfg.seed & 0xffffffffu); nz.key1 = (uint32_t)(c->cfg.seed >> 32);
    nz.ctr2 = (uint32_t)((uint64_t)c->acts & 0xffffffffu); nz.ctr3 = (uint32_t)((uint64_t)c->acts >> 32);
    e = run(GEMM_NN, TILE_128x32, ps, &nz, st);
    if (e != hipSuccess) return E.hip(e, "pql_actor_act");
    c->acts += 1;
    return PQL_OK;
}

// ---------------------------------------------------------------------------------------------
// Host-side argument checks of the V-learner step (everything but the scratch buffer).
static int32_t critic_update_check(pql_ctx* c, const float* critic_params, const float* critic_target_params,
                                   const float* actor_target_params, const float* adam_m, const float* adam_v,
                                   const float* grads_out, const pql_batch& batch, int32_t B, const pql_adam& opt,
                                   const float* loss_out) {
    Err E{c};
    if (!critic_params || !critic_target_params || !actor_target_params || !adam_m || !adam_v || !grads_out ||
        !batch.obs || !batch.act || !batch.ret || !batch.next_obs || !batch.boot || !loss_out)
        return E.fail(PQL_ERR_NULL, "pql_critic_update: null pointer");
    if (B < 1 || !adam_ok(opt)) return E.fail(PQL_ERR_INVALID_ARG, "pql_critic_update: bad batch size or Adam constants");
    if (c->cfg.stochastic_policy && !c->temperature) return E.fail(PQL_ERR_NULL, "pql_critic_update: no temperature attached");
    if (B > c->cfg.max_batch) return E.fail(PQL_ERR_BATCH_TOO_LARGE, "pql_critic_update: batch > max_batch");
    return PQL_OK;
}

// The launch sequence of the V-learner step on a checked argument list; `workspace` is device
// memory of at least pql_workspace_bytes(cfg) bytes, 256-byte aligned, whoever owns it.
static int32_t critic_update_run(pql_ctx* c, float* critic_params, const float* critic_target_params,
                                 const float* actor_target_params, float* adam_m, float* adam_v, float* grads_out,
                                 pql_batch batch, int32_t B, pql_adam opt, float* loss_out, void* workspace, void* stream) {
    Err E{c};
    hipStream_t st = (hipStream_t)stream;
    float* ws = (float*)workspace;
    Layout w;
    make_layout(&c->cfg, w);
    const int L = c->L, o = c->cfg.obs_dim, ad = c->cfg.act_dim, HL = c->cfg.hidden[L - 1];
    const int64_t Pc = c->c_total;
    hipError_t e;
    const char* who = "pql_critic_update";

    AdamArgs adm;
    std::memset(&adm, 0, sizeof(adm));
    int head_parts = 0;
    const bool dist = distributional(&c->cfg);
    // Transposed weights: from the caller's cache when it holds those of this parameter vector (then the
    // optimiser kernel refreshes them at the end of the call), else transposed into the workspace here.
    const bool cached = c->wcache != nullptr && c->wcache_critic == critic_params;
    CacheLayout cl;
    make_cache_layout(&c->cfg, cl);
    auto WT = [&](int i, int l) { return cached ? c->wcache + cl.wT[i][l] : ws + w.wT[i][l]; };
    auto WOT = [&](int i) { return cached ? c->wcache + cl.woT[i] : ws + w.woT[i]; };
    const bool chain = chain_ok(&c->cfg, B);
    if (fused_ok(&c->cfg) || chain) {
        // One launch per row tile: target path, forward, heads and backward data path.
        TransposeArgs tr;
        tr.n = 0;
        FusedCriticArgs fa;
        std::memset(&fa, 0, sizeof(fa));
        fa.B = B; fa.o = o; fa.a = ad; fa.L = L; fa.nwg = (B + FUSED_BM - 1) / FUSED_BM; fa.hmax = max_hidden(&c->cfg);
        for (int l = 0; l < L; ++l) fa.H[l] = c->cfg.hidden[l];
        for (int l = 0; l <= L; ++l) {
            fa.pi.w[l] = actor_target_params + c->a_w[l]; fa.pi.b[l] = actor_target_params + c->a_b[l];
            for (int i = 0; i < 2; ++i) {
                fa.qt[i].w[l] = critic_target_params + i * Pc + c->c_w[l]; fa.qt[i].b[l] = critic_target_params + i * Pc + c->c_b[l];
                fa.q[i].w[l] = critic_params + i * Pc + c->c_w[l];        fa.q[i].b[l] = critic_params + i * Pc + c->c_b[l];
            }
        }
        for (int i = 0; i < 2; ++i) {
            for (int l = 1; l < L; ++l) {
                if (!cached) {
                    TransposeArgs::Mat& mt = tr.m[tr.n++];
                    mt.src = critic_params + i * Pc + c->c_w[l]; mt.dst = ws + w.wT[i][l];
                    mt.rows = c->cfg.hidden[l - 1]; mt.cols = c->cfg.hidden[l];
                }
                fa.wT[i][l] = WT(i, l);
            }
            for (int l = 1; l <= L; ++l) {
                fa.hQ[i][l] = ws + w.hQ[i][l]; fa.dQ[i][l] = ws + w.dQ[i][l]; fa.colQ[i][l] = ws + w.colQ[i][l];
            }
            fa.q_out[i] = ws + w.q[i];
            fa.p_dw[i] = ws + w.p_dw[i]; fa.p_dbh[i] = ws + w.p_dbh[i]; fa.p_db[i] = ws + w.p_db[i];
        }
        fa.obs = batch.obs; fa.act = batch.act; fa.ret = batch.ret; fa.next_obs = batch.next_obs; fa.boot = batch.boot;
        fa.y = ws + w.y; fa.p_loss = ws + w.p_loss;
        fa.sac = fused_sac(c, 4u, c->critic_t, c->temperature_v);
        if (dist) {
            fa.atoms = c->cfg.num_atoms; fa.v_min = c->cfg.v_min; fa.v_max = c->cfg.v_max;
            for (int i = 0; i < 2; ++i) {
                if (!cached) {
                    TransposeArgs::Mat& mt = tr.m[tr.n++];
                    mt.src = critic_params + i * Pc + c->c_w[L]; mt.dst = ws + w.woT[i]; mt.rows = HL; mt.cols = fa.atoms;
                }
                fa.woT[i] = WOT(i); fa.dlg[i] = ws + w.lgQ[i]; fa.p_dbo[i] = ws + w.p_dbo[i];
            }
        }
        if ((e = transpose_launch(tr, st)) != hipSuccess) return E.hip(e, who);
        if ((e = chain ? chain_critic_launch(fa, st) : fused_critic_launch(fa, st)) != hipSuccess) return E.hip(e, who);
        head_parts = fa.nwg;
        for (int i = 0; i < 2; ++i) {
            for (int l = 1; l < L; ++l)
                red(adm, i * Pc + c->c_b[l - 1], ws + w.colQ[i][l], c->cfg.hidden[l - 1], fa.nwg, c->cfg.hidden[l - 1]);
            if (dist) red(adm, i * Pc + c->c_b[L - 1], ws + w.colQ[i][L], HL, fa.nwg, HL);
        }
    } else {
        // 1. lagged policy pi^v on s' (hidden layers) together with the online critics on (s, a)
        for (int l = 1; l <= L; ++l) {
            std::vector<GemmProb> ps;
            const int H = c->cfg.hidden[l - 1];
            GemmProb p = prob(B, H, ws + w.hA[l], H, EPI_BIAS_ELU);
            if (l == 1) add_seg(p, batch.next_obs, o, actor_target_params + c->a_w[0], H, o);
            else add_seg(p, ws + w.hA[l - 1], c->cfg.hidden[l - 2], actor_target_params + c->a_w[l - 1], H, c->cfg.hidden[l - 2]);
            p.bias = actor_target_params + c->a_b[l - 1];
            ps.push_back(p);
            for (int i = 0; i < 2; ++i)
                ps.push_back(critic_layer(c, critic_params + i * Pc, l, batch.obs, batch.act, ad,
                                          l > 1 ? ws + w.hQ[i][l - 1] : nullptr, ws + w.hQ[i][l], B));
            if ((e = run_auto(GEMM_NN, ps, st)) != hipSuccess) return E.hip(e, who);
        }
        // 2. a' = tanh(output layer of pi^v), or a sample a' ~ pi^v(.|s') with its log-density
        if (c->cfg.stochastic_policy) {
            if ((e = stochastic_policy_sample(c, actor_target_params, B, ws, w, ws + w.aOut, ws + w.logp, nullptr, 4u,
                                              c->critic_t, st)) != hipSuccess)
                return E.hip(e, who);
        } else {
            std::vector<GemmProb> ps;
            GemmProb p = prob(B, ad, ws + w.aOut, ad, EPI_BIAS_TANH);
            add_seg(p, ws + w.hA[L], HL, actor_target_params + c->a_w[L], ad, HL);
            p.bias = actor_target_params + c->a_b[L];
            ps.push_back(p);
            if ((e = run(GEMM_NN, TILE_128x32, ps, nullptr, st)) != hipSuccess) return E.hip(e, who);
        }
        // 3. twin target critics on (s', a')
        for (int l = 1; l <= L; ++l) {
            std::vector<GemmProb> ps;
            for (int i = 0; i < 2; ++i)
                ps.push_back(critic_layer(c, critic_target_params + i * Pc, l, batch.next_obs, ws + w.aOut, ad,
                                          l > 1 ? ws + w.hT[i][l - 1] : nullptr, ws + w.hT[i][l], B));
            if ((e = run_auto(GEMM_NN, ps, st)) != hipSuccess) return E.hip(e, who);
        }
        if (dist) {
            // 4. logits of the four critics, then target distribution, projection, cross-entropy, dLoss/dlogits
            const int la = c->cfg.num_atoms;
            std::vector<GemmProb> ps;
            for (int i = 0; i < 2; ++i) {
                GemmProb pt = prob(B, la, ws + w.lgT[i], la, EPI_BIAS);
                add_seg(pt, ws + w.hT[i][L], HL, critic_target_params + i * Pc + c->c_w[L], la, HL);
                pt.bias = critic_target_params + i * Pc + c->c_b[L];
                ps.push_back(pt);
                GemmProb pq = prob(B, la, ws + w.lgQ[i], la, EPI_BIAS);
                add_seg(pq, ws + w.hQ[i][L], HL, critic_params + i * Pc + c->c_w[L], la, HL);
                pq.bias = critic_params + i * Pc + c->c_b[L];
                ps.push_back(pq);
            }
            if ((e = run_auto(GEMM_NN, ps, st)) != hipSuccess) return E.hip(e, who);
            DistHeadArgs h;
            std::memset(&h, 0, sizeof(h));
            h.B = B; h.atoms = la; h.nwg = dist_head_workgroups(B); h.v_min = c->cfg.v_min; h.v_max = c->cfg.v_max;
            for (int i = 0; i < 2; ++i) { h.logitsT[i] = ws + w.lgT[i]; h.logitsQ[i] = ws + w.lgQ[i]; h.p_db[i] = ws + w.p_dbo[i]; }
            h.ret = batch.ret; h.boot = batch.boot; h.p_loss = ws + w.p_loss;
            if ((e = dist_critic_head_launch(h, st)) != hipSuccess) return E.hip(e, who);
            head_parts = h.nwg;
            // delta of the last hidden layer through the logits layer; its column sums are that layer's bias gradient
            std::vector<GemmProb> pb;
            for (int i = 0; i < 2; ++i) {
                GemmProb p = prob(B, HL, ws + w.dQ[i][L], HL, EPI_MUL_DELU);
                add_seg(p, ws + w.lgQ[i], la, critic_params + i * Pc + c->c_w[L], la, la);
                p.aux = ws + w.hQ[i][L]; p.ldaux = HL;
                p.colsum = ws + w.colQ[i][L];
                pb.push_back(p);
            }
            const int tile = choose_tile(GEMM_NT, pb);
            if ((e = run(GEMM_NT, tile, pb, nullptr, st)) != hipSuccess) return E.hip(e, who);
            for (int i = 0; i < 2; ++i)
                red(adm, i * Pc + c->c_b[L - 1], ws + w.colQ[i][L], HL, colsum_rows(tile, B), HL);
        } else {
            // 4. heads: y, losses, output deltas, delta of the last hidden layer
            HeadArgs h;
            std::memset(&h, 0, sizeof(h));
            h.B = B; h.H = HL; h.nwg = head_workgroups(B);
            for (int i = 0; i < 2; ++i) {
                h.hT[i] = ws + w.hT[i][L]; h.wT[i] = critic_target_params + i * Pc + c->c_w[L]; h.bT[i] = critic_target_params + i * Pc + c->c_b[L];
                h.hQ[i] = ws + w.hQ[i][L]; h.wQ[i] = critic_params + i * Pc + c->c_w[L];        h.bQ[i] = critic_params + i * Pc + c->c_b[L];
                h.dQ[i] = ws + w.dQ[i][L]; h.q[i] = ws + w.q[i];
                h.p_dw[i] = ws + w.p_dw[i]; h.p_dbh[i] = ws + w.p_dbh[i]; h.p_db[i] = ws + w.p_db[i];
            }
            h.ret = batch.ret; h.boot = batch.boot; h.y = ws + w.y; h.p_loss = ws + w.p_loss;
            if (c->cfg.stochastic_policy) { h.logp_next = ws + w.logp; h.log_alpha = c->temperature_v; }
            if ((e = critic_head_launch(h, st)) != hipSuccess) return E.hip(e, who);
            head_parts = h.nwg;
        }

        // 5. backward data path: delta_{l-1} = (delta_l W_l^T) * ELU'(z_{l-1}), bias grads as column sums
        // Wide layers run on row tiles with W^T as a row-major B operand (transposed once per call);
        // the others take the LDS-tiled kernel on W itself.
        bool transposed = cached;
        for (int l = L; l >= 2; --l) {
            std::vector<GemmProb> ps, pt;
            const int Hl = c->cfg.hidden[l - 1], Hp = c->cfg.hidden[l - 2];
            for (int i = 0; i < 2; ++i) {
                GemmProb p = prob(B, Hp, ws + w.dQ[i][l - 1], Hp, EPI_MUL_DELU);
                p.aux = ws + w.hQ[i][l - 1]; p.ldaux = Hp;
                p.colsum = ws + w.colQ[i][l - 1];
                GemmProb q = p;
                add_seg(p, ws + w.dQ[i][l], Hl, critic_params + i * Pc + c->c_w[l - 1], Hl, Hl);
                add_seg(q, ws + w.dQ[i][l], Hl, WT(i, l - 1), Hp, Hl);
                ps.push_back(p); pt.push_back(q);
            }
            int parts;
            if (takes_row_tiles(pt)) {
                if (!transposed) {
                    TransposeArgs tr;
                    tr.n = 0;
                    for (int i = 0; i < 2; ++i)
                        for (int k = 1; k < L; ++k) {
                            TransposeArgs::Mat& mt = tr.m[tr.n++];
                            mt.src = critic_params + i * Pc + c->c_w[k]; mt.dst = ws + w.wT[i][k];
                            mt.rows = c->cfg.hidden[k - 1]; mt.cols = c->cfg.hidden[k];
                        }
                    if ((e = transpose_launch(tr, st)) != hipSuccess) return E.hip(e, who);
                    transposed = true;
                }
                if ((e = run(GEMM_NN, TILE_64x64, pt, nullptr, st)) != hipSuccess) return E.hip(e, who);
                parts = (B + FUSED_BM - 1) / FUSED_BM;
            } else {
                const int tile = choose_tile(GEMM_NT, ps);
                if ((e = run(GEMM_NT, tile, ps, nullptr, st)) != hipSuccess) return E.hip(e, who);
                parts = colsum_rows(tile, B);
            }
            for (int i = 0; i < 2; ++i)
                red(adm, i * Pc + c->c_b[l - 2], ws + w.colQ[i][l - 1], Hp, parts, Hp);
        }
    }
    // 6. weight gradients X^T delta (split over the batch)
    {
        std::vector<GemmProb> ps;
        std::vector<int64_t> offs;
        std::vector<float*> tds;         // where the optimiser kernel leaves the transposed copy of the updated tensor
        const bool keep_t = cached;
        for (int i = 0; i < 2; ++i) {
            for (int l = 1; l <= L; ++l) {
                const int Hl = c->cfg.hidden[l - 1];
                if (l == 1) {
                    GemmProb p = prob(o, Hl, nullptr, Hl, EPI_STORE);
                    add_seg(p, batch.obs, o, ws + w.dQ[i][1], Hl, B);
                    ps.push_back(p); offs.push_back(i * Pc + c->c_w[0]); tds.push_back(nullptr);
                    GemmProb p2 = prob(ad, Hl, nullptr, Hl, EPI_STORE);
                    add_seg(p2, batch.act, ad, ws + w.dQ[i][1], Hl, B);
                    ps.push_back(p2); offs.push_back(i * Pc + c->c_w[0] + (int64_t)o * Hl);
                    tds.push_back(keep_t ? c->wcache + cl.w1aT[i] : nullptr);
                } else {
                    const int Hp = c->cfg.hidden[l - 2];
                    GemmProb p = prob(Hp, Hl, nullptr, Hl, EPI_STORE);
                    add_seg(p, ws + w.hQ[i][l - 1], Hp, ws + w.dQ[i][l], Hl, B);
                    ps.push_back(p); offs.push_back(i * Pc + c->c_w[l - 1]);
                    tds.push_back(keep_t ? c->wcache + cl.wT[i][l - 1] : nullptr);
                }
            }
            if (dist) {
                const int la = c->cfg.num_atoms;
                GemmProb p = prob(HL, la, nullptr, la, EPI_STORE);
                add_seg(p, ws + w.hQ[i][L], HL, ws + w.lgQ[i], la, B);
                ps.push_back(p); offs.push_back(i * Pc + c->c_w[L]);
                tds.push_back(keep_t ? c->wcache + cl.woT[i] : nullptr);
            }
        }
        if ((e = run_dw(ps, offs, B, ws + w.splitk, adm, st, &tds)) != hipSuccess) return E.hip(e, who);
    }
    // 7. remaining reductions (last hidden bias, output layer) + Adam + loss scalars
    for (int i = 0; i < 2; ++i) {
        if (dist) {
            red(adm, i * Pc + c->c_b[L], ws + w.p_dbo[i], c->cfg.num_atoms, head_parts, c->cfg.num_atoms);
            continue;
        }
        red(adm, i * Pc + c->c_b[L - 1], ws + w.p_dbh[i], HL, head_parts, HL);
        red(adm, i * Pc + c->c_w[L], ws + w.p_dw[i], HL, head_parts, HL);
        red(adm, i * Pc + c->c_b[L], ws + w.p_db[i], 1, head_parts, 1);
    }
    adm.nloss = 2; adm.loss_parts = head_parts; adm.loss_scale = 1.f / (float)B;
    adm.loss_partial = ws + w.p_loss; adm.loss_out = loss_out;
    adm.theta = critic_params; adm.m = adam_m; adm.v = adam_v; adm.g = grads_out;
    adm.max_norm = opt.max_grad_norm; adm.sq_partial = ws + w.sqp; adm.norm_out = loss_out + 2;
    // what follows the step (target tracking, transposed weights for the next call) rides on the pass that
    // writes the parameters: the optimiser kernel's, or the second kernel's of a clipped step
    if (c->track[0] != nullptr && c->track_tau[0] > 0.f) { adm.track = c->track[0]; adm.tau = c->track_tau[0]; }
    fill_adam(adm, opt, c->critic_t + 1);
    if ((e = adam_reduce_launch(adm, st)) != hipSuccess) return E.hip(e, who);
    c->critic_t += 1;
    return PQL_OK;
}

int32_t pql_critic_update(pql_ctx* c, float* critic_params, const float* critic_target_params,
                          const float* actor_target_params, float* adam_m, float* adam_v, float* grads_out,
                          pql_batch batch, int32_t B, pql_adam opt, float* loss_out, void* workspace, void* stream) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!workspace) return E.fail(PQL_ERR_NULL, "pql_critic_update: null pointer");
    const int32_t rc = critic_update_check(c, critic_params, critic_target_params, actor_target_params, adam_m, adam_v,
                                           grads_out, batch, B, opt, loss_out);
    if (rc != PQL_OK) return rc;
    if (((uintptr_t)workspace) & 255) return E.fail(PQL_ERR_ALIGNMENT, "pql_critic_update: workspace not 256-byte aligned");
    return critic_update_run(c, critic_params, critic_target_params, actor_target_params, adam_m, adam_v, grads_out, batch,
                             B, opt, loss_out, workspace, stream);
}

// ---- the same step on the library's own scratch --------------------------------------------
// For callers that cannot allocate device memory (code under graph capture, tight serving loops):
// the workspace of pql_critic_update is replaced by a file-scope device array.  Every GPU holds its
// own copy of that array at its own address, looked up once per device with that device current;
// host code only ever uses the looked-up address (the array's name is a host-side stand-in here).
int64_t pql_static_scratch_bytes(void) { return (int64_t)STATIC_SCRATCH_BYTES; }

int32_t pql_critic_update_static(pql_ctx* c, float* critic_params, const float* critic_target_params,
                                 const float* actor_target_params, float* adam_m, float* adam_v, float* grads_out,
                                 pql_batch batch, int32_t B, pql_adam opt, float* loss_out, void* stream) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    const int32_t rc = critic_update_check(c, critic_params, critic_target_params, actor_target_params, adam_m, adam_v,
                                           grads_out, batch, B, opt, loss_out);
    if (rc != PQL_OK) return rc;
    Layout w;
    make_layout(&c->cfg, w);
    if (w.total * sizeof(float) > STATIC_SCRATCH_BYTES) {
        char msg[192];
        std::snprintf(msg, sizeof(msg), "pql_critic_update_static: this configuration needs %zu bytes of scratch, the static "
                      "array holds %zu (lower cfg.max_batch or use pql_critic_update)", w.total * sizeof(float),
                      (size_t)STATIC_SCRATCH_BYTES);
        return E.fail(PQL_ERR_SCRATCH_TOO_SMALL, msg);
    }
    void* ws = nullptr;
    const hipError_t e = static_scratch_address(&ws);
    if (e != hipSuccess) return E.hip(e, "pql_critic_update_static: scratch address");
    return critic_update_run(c, critic_params, critic_target_params, actor_target_params, adam_m, adam_v, grads_out, batch,
                             B, opt, loss_out, ws, stream);
}

// ---------------------------------------------------------------------------------------------
int32_t pql_actor_update(pql_ctx* c, float* actor_params, const float* critic_params, float* adam_m, float* adam_v,
                         float* grads_out, const float* obs, int32_t B, pql_adam opt, float* loss_out,
                         void* workspace, void* stream) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!actor_params || !critic_params || !adam_m || !adam_v || !grads_out || !obs || !loss_out || !workspace)
        return E.fail(PQL_ERR_NULL, "pql_actor_update: null pointer");
    if (B < 1 || !adam_ok(opt)) return E.fail(PQL_ERR_INVALID_ARG, "pql_actor_update: bad batch size or Adam constants");
    if (c->cfg.stochastic_policy && !c->temperature) return E.fail(PQL_ERR_NULL, "pql_actor_update: no temperature attached");
    if (B > c->cfg.max_batch) return E.fail(PQL_ERR_BATCH_TOO_LARGE, "pql_actor_update: batch > max_batch");
    if (((uintptr_t)workspace) & 255) return E.fail(PQL_ERR_ALIGNMENT, "pql_actor_update: workspace not 256-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    float* ws = (float*)workspace;
    Layout w;
    make_layout(&c->cfg, w);
    const int L = c->L, o = c->cfg.obs_dim, ad = c->cfg.act_dim, HL = c->cfg.hidden[L - 1], H1 = c->cfg.hidden[0];
    const int64_t Pc = c->c_total;
    hipError_t e;
    const char* who = "pql_actor_update";

    AdamArgs adm;
    std::memset(&adm, 0, sizeof(adm));
    int loss_parts = 0;
    const bool sac = c->cfg.stochastic_policy != 0;
    const int aw = actor_out(&c->cfg);                          // width of the policy's output layer
    const float* d_top = sac ? ws + w.dOut : ws + w.dPre;       // gradient at that layer
    int logp_parts = (B + SAC_ROWS - 1) / SAC_ROWS;             // partial sums of log pi (stochastic policy)
    // Transposed weights from the caller's cache where it holds those of these parameter vectors
    const bool cached_q = c->wcache != nullptr && c->wcache_critic == critic_params;
    const bool cached_a = c->wcache != nullptr && c->wcache_actor == actor_params;
    CacheLayout cl;
    make_cache_layout(&c->cfg, cl);
    auto WT = [&](int i, int l) { return cached_q ? c->wcache + cl.wT[i][l] : ws + w.wT[i][l]; };
    auto W1AT = [&](int i) { return cached_q ? c->wcache + cl.w1aT[i] : ws + w.w1aT[i]; };
    auto WOT = [&](int i) { return cached_q ? c->wcache + cl.woT[i] : ws + w.woT[i]; };
    auto WAT = [&](int l) { return cached_a ? c->wcache + cl.waT[l] : ws + w.waT[l]; };
    const bool chain = chain_ok(&c->cfg, B);
    if (fused_ok(&c->cfg) || chain) {
        TransposeArgs tr;
        tr.n = 0;
        FusedPolicyArgs fa;
        std::memset(&fa, 0, sizeof(fa));
        fa.B = B; fa.o = o; fa.a = ad; fa.L = L; fa.nwg = (B + FUSED_BM - 1) / FUSED_BM; fa.hmax = max_hidden(&c->cfg);
        for (int l = 0; l < L; ++l) fa.H[l] = c->cfg.hidden[l];
        for (int l = 0; l <= L; ++l) {
            fa.pi.w[l] = actor_params + c->a_w[l]; fa.pi.b[l] = actor_params + c->a_b[l];
            for (int i = 0; i < 2; ++i) { fa.q[i].w[l] = critic_params + i * Pc + c->c_w[l]; fa.q[i].b[l] = critic_params + i * Pc + c->c_b[l]; }
        }
        auto add_tr = [&](const float* src, float* dst, int rows, int cols) {
            TransposeArgs::Mat& mt = tr.m[tr.n++];
            mt.src = src; mt.dst = dst; mt.rows = rows; mt.cols = cols;
        };
        for (int i = 0; i < 2; ++i) {
            for (int l = 1; l < L; ++l) {
                if (!cached_q) add_tr(critic_params + i * Pc + c->c_w[l], ws + w.wT[i][l], c->cfg.hidden[l - 1], c->cfg.hidden[l]);
                fa.wT[i][l] = WT(i, l);
            }
            if (!cached_q) add_tr(critic_params + i * Pc + c->c_w[0] + (int64_t)o * H1, ws + w.w1aT[i], ad, H1);
            fa.w1aT[i] = W1AT(i);
            for (int l = 1; l <= L; ++l) fa.hQ[i][l] = ws + w.hQ[i][l];
            fa.q_out[i] = ws + w.q[i];
            if (distributional(&c->cfg)) {
                if (!cached_q) add_tr(critic_params + i * Pc + c->c_w[L], ws + w.woT[i], HL, c->cfg.num_atoms);
                fa.woT[i] = WOT(i);
            }
        }
        if (distributional(&c->cfg)) { fa.atoms = c->cfg.num_atoms; fa.v_min = c->cfg.v_min; fa.v_max = c->cfg.v_max; }
        for (int l = 1; l <= L; ++l) {
            if (!cached_a) add_tr(actor_params + c->a_w[l], ws + w.waT[l], c->cfg.hidden[l - 1], l < L ? c->cfg.hidden[l] : aw);
            fa.waT[l] = WAT(l);
            fa.hA[l] = ws + w.hA[l]; fa.dA[l] = ws + w.dA[l]; fa.colA[l] = ws + w.colA[l];
        }
        fa.colA[L + 1] = ws + w.colA[L + 1];
        fa.obs = obs; fa.dPre = const_cast<float*>(d_top); fa.p_loss = ws + w.p_loss;
        fa.sac = fused_sac(c, 5u, c->actor_t, c->temperature);
        fa.p_logp = sac ? ws + w.p_lp : nullptr;
        if ((e = transpose_launch(tr, st)) != hipSuccess) return E.hip(e, who);
        if ((e = chain ? chain_policy_launch(fa, st) : fused_policy_launch(fa, st)) != hipSuccess) return E.hip(e, who);
        loss_parts = fa.nwg;
        logp_parts = fa.nwg;
        red(adm, c->a_b[L], ws + w.colA[L + 1], aw, fa.nwg, aw);
        for (int l = 1; l <= L; ++l) red(adm, c->a_b[l - 1], ws + w.colA[l], c->cfg.hidden[l - 1], fa.nwg, c->cfg.hidden[l - 1]);
    } else {
        // 1. a = pi(s), or the reparameterised sample a = tanh(mu + sigma eps)
        if ((e = actor_hidden_forward(c, actor_params, obs, B, ws, w, st)) != hipSuccess) return E.hip(e, who);
        if (sac) {
            if ((e = stochastic_policy_sample(c, actor_params, B, ws, w, ws + w.aOut, ws + w.logp, ws + w.epsb, 5u,
                                              c->actor_t, st)) != hipSuccess)
                return E.hip(e, who);
        } else {
            std::vector<GemmProb> ps;
            GemmProb p = prob(B, ad, ws + w.aOut, ad, EPI_BIAS_TANH);
            add_seg(p, ws + w.hA[L], HL, actor_params + c->a_w[L], ad, HL);
            p.bias = actor_params + c->a_b[L];
            ps.push_back(p);
            if ((e = run(GEMM_NN, TILE_128x32, ps, nullptr, st)) != hipSuccess) return E.hip(e, who);
        }
        // 2. twin critics on (s, pi(s))
        for (int l = 1; l <= L; ++l) {
            std::vector<GemmProb> ps;
            for (int i = 0; i < 2; ++i)
                ps.push_back(critic_layer(c, critic_params + i * Pc, l, obs, ws + w.aOut, ad,
                                          l > 1 ? ws + w.hQ[i][l - 1] : nullptr, ws + w.hQ[i][l], B));
            if ((e = run_auto(GEMM_NN, ps, st)) != hipSuccess) return E.hip(e, who);
        }
        if (distributional(&c->cfg)) {
            // 3. logits, J partials from the distribution means, dJ/dlogits, delta of the last hidden layer
            const int la = c->cfg.num_atoms;
            std::vector<GemmProb> ps;
            for (int i = 0; i < 2; ++i) {
                GemmProb pq = prob(B, la, ws + w.lgQ[i], la, EPI_BIAS);
                add_seg(pq, ws + w.hQ[i][L], HL, critic_params + i * Pc + c->c_w[L], la, HL);
                pq.bias = critic_params + i * Pc + c->c_b[L];
                ps.push_back(pq);
            }
            if ((e = run_auto(GEMM_NN, ps, st)) != hipSuccess) return E.hip(e, who);
            DistHeadArgs h;
            std::memset(&h, 0, sizeof(h));
            h.B = B; h.atoms = la; h.nwg = dist_head_workgroups(B); h.v_min = c->cfg.v_min; h.v_max = c->cfg.v_max;
            for (int i = 0; i < 2; ++i) h.logitsQ[i] = ws + w.lgQ[i];
            h.p_loss = ws + w.p_loss;
            if ((e = dist_policy_head_launch(h, st)) != hipSuccess) return E.hip(e, who);
            loss_parts = h.nwg;
            std::vector<GemmProb> pb;
            for (int i = 0; i < 2; ++i) {
                GemmProb p = prob(B, HL, ws + w.dQ[i][L], HL, EPI_MUL_DELU);
                add_seg(p, ws + w.lgQ[i], la, critic_params + i * Pc + c->c_w[L], la, la);
                p.aux = ws + w.hQ[i][L]; p.ldaux = HL;
                pb.push_back(p);
            }
            if ((e = run_auto(GEMM_NT, pb, st)) != hipSuccess) return E.hip(e, who);
        } else {
            // 3. heads: J partials and the delta entering the smaller critic
            HeadArgs h;
            std::memset(&h, 0, sizeof(h));
            h.B = B; h.H = HL; h.nwg = head_workgroups(B);
            for (int i = 0; i < 2; ++i) {
                h.hQ[i] = ws + w.hQ[i][L]; h.wQ[i] = critic_params + i * Pc + c->c_w[L]; h.bQ[i] = critic_params + i * Pc + c->c_b[L];
                h.dQ[i] = ws + w.dQ[i][L]; h.q[i] = ws + w.q[i];
            }
            h.p_loss = ws + w.p_loss;
            if ((e = policy_head_launch(h, st)) != hipSuccess) return E.hip(e, who);
            loss_parts = h.nwg;
        }
        // 4. critic backward data path down to layer 1 (wide layers on row tiles with W^T as a
        //    row-major B operand, transposed once per call; the others on the LDS-tiled kernel)
        bool transposed_q = cached_q;
        for (int l = L; l >= 2; --l) {
            std::vector<GemmProb> ps, pt;
            const int Hl = c->cfg.hidden[l - 1], Hp = c->cfg.hidden[l - 2];
            for (int i = 0; i < 2; ++i) {
                GemmProb p = prob(B, Hp, ws + w.dQ[i][l - 1], Hp, EPI_MUL_DELU);
                p.aux = ws + w.hQ[i][l - 1]; p.ldaux = Hp;
                GemmProb q = p;
                add_seg(p, ws + w.dQ[i][l], Hl, critic_params + i * Pc + c->c_w[l - 1], Hl, Hl);
                add_seg(q, ws + w.dQ[i][l], Hl, WT(i, l - 1), Hp, Hl);
                ps.push_back(p); pt.push_back(q);
            }
            if (takes_row_tiles(pt)) {
                if (!transposed_q) {
                    TransposeArgs tr;
                    tr.n = 0;
                    for (int i = 0; i < 2; ++i)
                        for (int k = 1; k < L; ++k) {
                            TransposeArgs::Mat& mt = tr.m[tr.n++];
                            mt.src = critic_params + i * Pc + c->c_w[k]; mt.dst = ws + w.wT[i][k];
                            mt.rows = c->cfg.hidden[k - 1]; mt.cols = c->cfg.hidden[k];
                        }
                    if ((e = transpose_launch(tr, st)) != hipSuccess) return E.hip(e, who);
                    transposed_q = true;
                }
                if ((e = run(GEMM_NN, TILE_64x64, pt, nullptr, st)) != hipSuccess) return E.hip(e, who);
            } else {
                if ((e = run_auto(GEMM_NT, ps, st)) != hipSuccess) return E.hip(e, who);
            }
        }
        // 5. gradient w.r.t. the action input of both critics, through tanh'
        {
            std::vector<GemmProb> ps, pt;
            GemmProb p = prob(B, ad, ws + w.dPre, ad, EPI_MUL_DTANH);
            p.aux = ws + w.aOut; p.ldaux = ad;
            if (!sac) p.colsum = ws + w.colA[L + 1];
            GemmProb q = p;
            for (int i = 0; i < 2; ++i) {
                add_seg(p, ws + w.dQ[i][1], H1, critic_params + i * Pc + c->c_w[0] + (int64_t)o * H1, H1, H1);
                add_seg(q, ws + w.dQ[i][1], H1, W1AT(i), ad, H1);
            }
            ps.push_back(p); pt.push_back(q);
            int parts;
            if (takes_narrow_tiles(pt)) {      // on row tiles, with the action rows of W_1 transposed
                TransposeArgs tr;
                tr.n = 0;
                for (int i = 0; i < 2 && !cached_q; ++i) {
                    TransposeArgs::Mat& mt = tr.m[tr.n++];
                    mt.src = critic_params + i * Pc + c->c_w[0] + (int64_t)o * H1; mt.dst = ws + w.w1aT[i];
                    mt.rows = ad; mt.cols = H1;
                }
                if ((e = transpose_launch(tr, st)) != hipSuccess) return E.hip(e, who);
                if ((e = run(GEMM_NN, TILE_128x32, pt, nullptr, st)) != hipSuccess) return E.hip(e, who);
                parts = (B + FUSED_BM - 1) / FUSED_BM;
            } else {
                if ((e = run(GEMM_NT, TILE_128x32, ps, nullptr, st)) != hipSuccess) return E.hip(e, who);
                parts = colsum_rows(TILE_128x32, B);
            }
            if (!sac) red(adm, c->a_b[L], ws + w.colA[L + 1], ad, parts, ad);
        }
        if (sac) {      // add the log-density terms and split into the gradients of mu and raw log sigma
            SacGradArgs ga;
            ga.B = B; ga.a = ad; ga.d_u = ws + w.dPre; ga.act = ws + w.aOut; ga.eps = ws + w.epsb; ga.out2a = ws + w.mu2a;
            ga.logp = ws + w.logp; ga.log_alpha = c->temperature;
            ga.d_out = ws + w.dOut; ga.p_cols = ws + w.p_sc; ga.p_logp = ws + w.p_lp;
            if ((e = sac_grad_launch(ga, st)) != hipSuccess) return E.hip(e, who);
            red(adm, c->a_b[L], ws + w.p_sc, aw, (B + SAC_ROWS - 1) / SAC_ROWS, aw);
        }
        // 6. policy backward data path
        bool transposed_a = cached_a;
        for (int l = L + 1; l >= 2; --l) {
            std::vector<GemmProb> ps, pt;
            const int Hl = (l == L + 1) ? aw : c->cfg.hidden[l - 1], Hp = c->cfg.hidden[l - 2];
            GemmProb p = prob(B, Hp, ws + w.dA[l - 1], Hp, EPI_MUL_DELU);
            p.aux = ws + w.hA[l - 1]; p.ldaux = Hp;
            p.colsum = ws + w.colA[l - 1];
            GemmProb q = p;
            add_seg(p, (l == L + 1) ? d_top : ws + w.dA[l], Hl, actor_params + c->a_w[l - 1], Hl, Hl);
            add_seg(q, (l == L + 1) ? d_top : ws + w.dA[l], Hl, WAT(l - 1), Hp, Hl);
            ps.push_back(p); pt.push_back(q);
            int parts;
            if (takes_row_tiles(pt)) {
                if (!transposed_a) {
                    TransposeArgs tr;
                    tr.n = 0;
                    for (int k = 1; k <= L; ++k) {
                        TransposeArgs::Mat& mt = tr.m[tr.n++];
                        mt.src = actor_params + c->a_w[k]; mt.dst = ws + w.waT[k];
                        mt.rows = c->cfg.hidden[k - 1]; mt.cols = k < L ? c->cfg.hidden[k] : aw;
                    }
                    if ((e = transpose_launch(tr, st)) != hipSuccess) return E.hip(e, who);
                    transposed_a = true;
                }
                if ((e = run(GEMM_NN, TILE_64x64, pt, nullptr, st)) != hipSuccess) return E.hip(e, who);
                parts = (B + FUSED_BM - 1) / FUSED_BM;
            } else {
                const int tile = choose_tile(GEMM_NT, ps);
                if ((e = run(GEMM_NT, tile, ps, nullptr, st)) != hipSuccess) return E.hip(e, who);
                parts = colsum_rows(tile, B);
            }
            red(adm, c->a_b[l - 2], ws + w.colA[l - 1], Hp, parts, Hp);
        }
    }
    // 7. policy weight gradients
    {
        std::vector<GemmProb> ps;
        std::vector<int64_t> offs;
        std::vector<float*> tds;         // transposed copies of W_1 .. W_L left by the optimiser kernel
        for (int l = 1; l <= L + 1; ++l) {
            const int Hl = (l == L + 1) ? aw : c->cfg.hidden[l - 1];
            const int Hp = (l == 1) ? o : c->cfg.hidden[l - 2];
            GemmProb p = prob(Hp, Hl, nullptr, Hl, EPI_STORE);
            add_seg(p, (l == 1) ? obs : ws + w.hA[l - 1], Hp, (l == L + 1) ? d_top : ws + w.dA[l], Hl, B);
            ps.push_back(p); offs.push_back(c->a_w[l - 1]);
            tds.push_back((cached_a && l >= 2) ? c->wcache + cl.waT[l - 1] : nullptr);
        }
        if ((e = run_dw(ps, offs, B, ws + w.splitk, adm, st, &tds)) != hipSuccess) return E.hip(e, who);
    }
    adm.nloss = 1; adm.loss_parts = loss_parts; adm.loss_scale = -1.f / (float)B;
    adm.loss_partial = ws + w.p_loss; adm.loss_out = loss_out;
    adm.theta = actor_params; adm.m = adam_m; adm.v = adam_v; adm.g = grads_out;
    adm.max_norm = opt.max_grad_norm; adm.sq_partial = ws + w.sqp; adm.norm_out = loss_out + 1;
    if (c->track[1] != nullptr && c->track_tau[1] > 0.f) { adm.track = c->track[1]; adm.tau = c->track_tau[1]; }
    fill_adam(adm, opt, c->actor_t + 1);
    if ((e = adam_reduce_launch(adm, st)) != hipSuccess) return E.hip(e, who);
    if (sac) {      // temperature step on the log-densities of this batch
        SacAlphaArgs al;
        al.B = B; al.nparts = logp_parts; al.p_logp = ws + w.p_lp; al.temperature = c->temperature;
        al.loss_out = loss_out; al.target_entropy = c->target_entropy;
        al.lr = adm.lr; al.beta1 = adm.beta1; al.beta2 = adm.beta2; al.eps = adm.eps; al.inv_bc1 = adm.inv_bc1; al.inv_bc2 = adm.inv_bc2;
        if ((e = sac_alpha_launch(al, st)) != hipSuccess) return E.hip(e, who);
    }
    c->actor_t += 1;
    return PQL_OK;
}

// ---------------------------------------------------------------------------------------------
int32_t pql_profile_begin(pql_ctx* c, int32_t max_launches) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (max_launches < 1 || max_launches > (1 << 20)) return E.fail(PQL_ERR_INVALID_ARG, "pql_profile_begin: bad max_launches");
    if (g_prof.on) return E.fail(PQL_ERR_INVALID_ARG, "pql_profile_begin: already profiling");
    g_prof.ev.assign((size_t)2 * max_launches, nullptr);
    for (size_t i = 0; i < g_prof.ev.size(); ++i) {
        const hipError_t e = hipEventCreate(&g_prof.ev[i]);
        if (e != hipSuccess) {
            for (size_t k = 0; k < i; ++k) (void)hipEventDestroy(g_prof.ev[k]);
            g_prof.ev.clear();
            return E.hip(e, "pql_profile_begin");
        }
    }
    g_prof.recs.clear();
    g_prof.cap = (size_t)max_launches;
    g_prof.on = true;
    return PQL_OK;
}

int32_t pql_profile_end(pql_ctx* c, pql_kernel_stat* out, int32_t max_out, int32_t* n_out) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!out || !n_out) return E.fail(PQL_ERR_NULL, "pql_profile_end: null pointer");
    if (!g_prof.on) return E.fail(PQL_ERR_INVALID_ARG, "pql_profile_end: profiling is not on");
    g_prof.on = false;
    int32_t rc = PQL_OK;
    pql_kernel_stat acc[KID_COUNT];
    std::memset(acc, 0, sizeof(acc));
    for (size_t i = 0; i < g_prof.recs.size(); ++i) {
        hipError_t e = hipEventSynchronize(g_prof.ev[2 * i + 1]);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]);
        if (e != hipSuccess) { rc = E.hip(e, "pql_profile_end"); break; }
        pql_kernel_stat& a = acc[g_prof.recs[i].kid];
        a.launches += 1; a.total_ms += ms; a.flops += g_prof.recs[i].flops; a.bytes += g_prof.recs[i].bytes;
    }
    for (hipEvent_t ev : g_prof.ev) (void)hipEventDestroy(ev);
    g_prof.ev.clear();
    g_prof.recs.clear();
    int32_t n = 0;
    for (int k = 0; k < KID_COUNT && rc == PQL_OK; ++k) {
        if (acc[k].launches == 0) continue;
        if (n < max_out) {
            out[n] = acc[k];
            std::snprintf(out[n].name, sizeof(out[n].name), "%s", kernel_name(k));
        }
        ++n;
    }
    *n_out = n;
    return rc;
}

// ---------------------------------------------------------------------------------------------
int32_t pql_probe_mfma(pql_ctx* c, float* out, int32_t blocks, int32_t iters, void* stream) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!out) return E.fail(PQL_ERR_NULL, "pql_probe_mfma: null pointer");
    if (blocks < 1 || blocks > (1 << 20) || iters < 1 || iters > (1 << 24)) return E.fail(PQL_ERR_INVALID_ARG, "pql_probe_mfma: bad size");
    const hipError_t e = mfma_probe_launch(out, blocks, iters, (hipStream_t)stream);
    if (e != hipSuccess) return E.hip(e, "pql_probe_mfma");
    return PQL_OK;
}

// ---------------------------------------------------------------------------------------------
int32_t pql_sac_attach(pql_ctx* c, float* temperature, float target_entropy) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!c->cfg.stochastic_policy) return E.fail(PQL_ERR_INVALID_ARG, "pql_sac_attach: the policy of this context is deterministic");
    if (temperature && (((uintptr_t)temperature) & 15)) return E.fail(PQL_ERR_ALIGNMENT, "pql_sac_attach: not 16-byte aligned");
    c->temperature = temperature;
    c->temperature_v = temperature;
    c->target_entropy = target_entropy;
    return PQL_OK;
}

int32_t pql_sac_attach_lagged(pql_ctx* c, const float* log_alpha) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!c->cfg.stochastic_policy) return E.fail(PQL_ERR_INVALID_ARG, "pql_sac_attach_lagged: the policy of this context is deterministic");
    c->temperature_v = log_alpha ? log_alpha : c->temperature;
    return PQL_OK;
}

// ---------------------------------------------------------------------------------------------
int32_t pql_track_attach(pql_ctx* c, int32_t which, float* dst, float tau) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (which != PQL_TRACK_CRITIC_TARGETS && which != PQL_TRACK_LAGGED_POLICY)
        return E.fail(PQL_ERR_INVALID_ARG, "pql_track_attach: unknown vector");
    if (dst != nullptr && (!(tau >= 0.f) || tau > 1.f)) return E.fail(PQL_ERR_INVALID_ARG, "pql_track_attach: tau outside [0, 1]");
    c->track[which] = dst;
    c->track_tau[which] = dst ? tau : 0.f;
    return PQL_OK;
}

int64_t pql_weight_cache_bytes(const pql_config* cfg) {
    const int rc = validate_cfg(cfg);
    if (rc != PQL_OK) return rc;
    CacheLayout cl;
    make_cache_layout(cfg, cl);
    return (int64_t)(cl.total * sizeof(float));
}

int32_t pql_weight_cache_attach(pql_ctx* c, void* cache) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (cache && (((uintptr_t)cache) & 255)) return E.fail(PQL_ERR_ALIGNMENT, "pql_weight_cache_attach: block not 256-byte aligned");
    c->wcache = (float*)cache;
    c->wcache_critic = c->wcache_actor = nullptr;       // nothing in the block is current yet
    return PQL_OK;
}

int32_t pql_weight_cache_refresh(pql_ctx* c, const float* critic_params, const float* actor_params, void* stream) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!c->wcache) return E.fail(PQL_ERR_NULL, "pql_weight_cache_refresh: no block attached");
    CacheLayout cl;
    make_cache_layout(&c->cfg, cl);
    hipError_t e;
    c->wcache_critic = c->wcache_actor = nullptr;
    if (critic_params) {
        if ((e = transpose_critic_weights(c, critic_params, c->wcache, cl, (hipStream_t)stream)) != hipSuccess)
            return E.hip(e, "pql_weight_cache_refresh");
        c->wcache_critic = critic_params;
    }
    if (actor_params) {
        if ((e = transpose_actor_weights(c, actor_params, c->wcache, cl, (hipStream_t)stream)) != hipSuccess)
            return E.hip(e, "pql_weight_cache_refresh");
        c->wcache_actor = actor_params;
    }
    return PQL_OK;
}

// ---------------------------------------------------------------------------------------------
int64_t pql_obs_norm_bytes(const pql_config* cfg) {
    const int rc = validate_cfg(cfg);
    return rc != PQL_OK ? rc : (int64_t)obs_stats_bytes(cfg->obs_dim, cfg->num_envs);
}

int32_t pql_obs_norm_attach(pql_ctx* c, void* stats, float eps) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (stats && (((uintptr_t)stats) & 255)) return E.fail(PQL_ERR_ALIGNMENT, "pql_obs_norm_attach: block not 256-byte aligned");
    if (stats && !(eps >= 0.f && eps <= 3.0e38f)) return E.fail(PQL_ERR_INVALID_ARG, "pql_obs_norm_attach: bad eps");
    c->obs_norm = stats;
    c->obs_eps = stats ? eps : 0.f;
    return PQL_OK;
}

int32_t pql_obs_norm_reset(pql_ctx* c, void* stream) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!c->obs_norm) return E.fail(PQL_ERR_NULL, "pql_obs_norm_reset: no statistics block attached");
    const hipError_t e = obs_stats_reset_launch(obs_stats_view(c->obs_norm, c->cfg.obs_dim), c->cfg.obs_dim, c->obs_eps,
                                                (hipStream_t)stream);
    if (e != hipSuccess) return E.hip(e, "pql_obs_norm_reset");
    return PQL_OK;
}

// ---------------------------------------------------------------------------------------------
int32_t pql_adam_step(pql_ctx* c, float* params, const float* grads, float* adam_m, float* adam_v, int64_t count,
                      pql_adam opt, int64_t t, void* stream) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!params || !grads || !adam_m || !adam_v) return E.fail(PQL_ERR_NULL, "pql_adam_step: null pointer");
    if (count < 0 || count > 0x7fffffffLL || t < 1 || !adam_ok(opt) || opt.max_grad_norm != 0.f)
        return E.fail(PQL_ERR_INVALID_ARG, "pql_adam_step: bad count, step number or Adam constants");
    if (count == 0) return PQL_OK;
    AdamArgs adm;
    std::memset(&adm, 0, sizeof(adm));
    red(adm, 0, grads, (int)count, 1, 0);
    adm.theta = params; adm.m = adam_m; adm.v = adam_v; adm.g = nullptr;
    fill_adam(adm, opt, t);
    const hipError_t e = adam_reduce_launch(adm, (hipStream_t)stream);
    if (e != hipSuccess) return E.hip(e, "pql_adam_step");
    return PQL_OK;
}

// ---------------------------------------------------------------------------------------------
int32_t pql_soft_update(pql_ctx* c, const float* src, float* dst, int64_t count, float tau, void* stream) {
    if (!c) return PQL_ERR_NULL;
    Err E{c};
    if (!src || !dst) return E.fail(PQL_ERR_NULL, "pql_soft_update: null pointer");
    if (count < 0 || !(tau >= 0.f) || tau > 1.f) return E.fail(PQL_ERR_INVALID_ARG, "pql_soft_update: bad count or tau");
    const hipError_t e = soft_update_launch(src, dst, count, tau, (hipStream_t)stream);
    if (e != hipSuccess) return E.hip(e, "pql_soft_update");
    return PQL_OK;
}

}  // extern "C"
