// Internal declarations shared by the translation units of libpql.  Nothing here is part of
// the public C interface (include/pql.h).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <mutex>

#include "pql.h"

namespace pql {

// ---- optional per-launch timing (HIP events on the launch stream) ---------------------------
// Kernel classes reported by pql_profile_end.  GEMM ids are KID_GEMM + mode * 5 + tile, with
// tile 4 = the 128x32 instantiation that carries the exploration-noise epilogue.
enum KernelId : int {
    KID_GEMM = 0, KID_PUSH = 15, KID_SAMPLE = 16, KID_HEAD_CRITIC = 17, KID_HEAD_POLICY = 18,
    KID_ADAM = 19, KID_SOFT_UPDATE = 20, KID_COPY = 21, KID_FUSED_CRITIC = 22, KID_FUSED_POLICY = 23,
    KID_FUSED_ACT = 24, KID_TRANSPOSE = 25, KID_ADAM_CLIP = 26, KID_OBS_STATS = 27, KID_OBS_MERGE = 28,
    KID_NORMALIZE = 29, KID_DIST_CRITIC = 30, KID_DIST_POLICY = 31, KID_SAC_SAMPLE = 32, KID_SAC_GRAD = 33,
    KID_SAC_ALPHA = 34, KID_MFMA_PROBE = 35, KID_LAYER_ROWTILE = 36, KID_NARROW_ROWTILE = 37, KID_CHAIN_CRITIC = 38,
    KID_CHAIN_POLICY = 39, KID_CHAIN_ACT = 40, KID_FUSED_ACT16 = 41, KID_COUNT = 42
};
const char* kernel_name(int kid);
bool prof_active();
// One timed launch: when profiling is on, prof_slot() hands out an event pair that PQL_LAUNCH
// attaches to the kernel dispatch itself (the events then carry the dispatch's own begin / end
// timestamps, with no marker commands in between); prof_commit() files the launch under its
// kernel class with its algorithmic work.  All no-ops unless profiling is on.
struct ProfSlot { hipEvent_t start, stop; bool on; };
ProfSlot prof_slot();
void prof_commit(const ProfSlot& s, int kid, double flops, double bytes);

#define PQL_LAUNCH(slot, kernel, grid, block, lds, stream, ...)                                              \
    do {                                                                                                     \
        if ((slot).on)                                                                                       \
            hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, (slot).start, (slot).stop, 0, __VA_ARGS__); \
        else                                                                                                 \
            hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                               \
    } while (0)

// Largest dynamic-LDS size granted so far to one kernel, per device (the attribute belongs to the device's
// copy of the function).  The grant only grows, under a lock, so that launches of the same kernel from several
// threads with different tile sizes never see it shrink between their request and their launch.
struct LdsLimit {
    std::mutex mu;
    size_t granted[64] = {};
};
inline hipError_t set_lds_limit(const void* fn, size_t lds, LdsLimit& lim) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(lim.mu);
    if (lds <= lim.granted[dev]) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) lim.granted[dev] = lds;
    return e;
}

// ---- grouped fp32 MFMA GEMM ------------------------------------------------------------
// One launch computes several independent problems C_p = epi(sum_seg A_seg * B_seg).  A problem
// may contract over up to two K-segments (the critic's first layer reads s and a from two
// arrays; the action gradient of the policy step sums over the two critics).

enum GemmMode : int {
    GEMM_NN = 0,   // A[M][K] row-major, B[K][N] row-major              (forward:  X * W)
    GEMM_NT = 1,   // A[M][K] row-major, B stored [N][K] row-major      (backward: delta * W^T)
    GEMM_TN = 2    // A stored [K][M] row-major, B[K][N] row-major, K split across workgroups
                   //                                                    (weight grad: X^T * delta)
};

enum GemmEpilogue : int {
    EPI_STORE = 0,          // C = acc  (split-K partial sums)
    EPI_BIAS_ELU = 1,       // C = ELU(acc + bias[n])
    EPI_BIAS_TANH = 2,      // C = tanh(acc + bias[n])
    EPI_BIAS_TANH_NOISE = 3,// C = clip(tanh(acc + bias[n]) + sigma_m * eps, -1, 1)
    EPI_MUL_DELU = 4,       // C = acc * ELU'(z) with ELU'(z) recovered from aux = ELU(z)
    EPI_MUL_DTANH = 5,      // C = acc * (1 - aux^2), aux = tanh(z)
    EPI_BIAS = 6            // C = acc + bias[n]  (logits of a distributional critic)
};

struct GemmSeg {
    const float* A;
    const float* B;
    int lda, ldb;
    int K;
    int vec;                // bit 0 / bit 1: 16-byte vector loads are legal for A / B
};

struct GemmProb {
    GemmSeg seg[2];
    int nseg;
    int M, N;
    int ldc;
    float* C;
    const float* bias;
    const float* aux;
    float* colsum;          // optional per-wave-row column sums of C: [tiles_m * waves_m][N]
    int ldaux;
    int epi;
    int tiles_m, tiles_n;
    int splits, k_chunk;    // GEMM_TN only: K range of split s is [s*k_chunk, min(K,(s+1)*k_chunk))
    int tile_begin;         // first linear tile id of this problem within the launch
    int pad_;
    int64_t split_stride;   // floats between consecutive split-K partial slabs
};

constexpr int GEMM_MAX_PROB = 16;

// Exploration-noise parameters for the (single) EPI_BIAS_TANH_NOISE problem of a launch.
struct GemmNoise {
    int act_dim;            // element index = m * act_dim + n
    int sigma_rows;         // number of environments in the sigma schedule
    float sigma_min, sigma_max;
    uint32_t key0, key1, ctr2, ctr3;
};

struct GemmGroup {
    int nprob;
    int total_tiles;
    GemmNoise noise;
    GemmProb p[GEMM_MAX_PROB];
};

enum GemmTile : int { TILE_128x128 = 0, TILE_64x64 = 1, TILE_128x32 = 2, TILE_128x64 = 3 };

int gemm_tile_m(int tile);
int gemm_tile_n(int tile);
int gemm_waves_m(int tile);
// Fills tiles_m/tiles_n/tile_begin/total_tiles from M, N, splits; returns hipError.
hipError_t gemm_launch(int mode, int tile, GemmGroup& g, hipStream_t stream);
hipError_t mfma_probe_launch(float* out, int blocks, int iters, hipStream_t stream);

// ---- reduction + Adam -------------------------------------------------------------------
struct RedTensor {
    int64_t offset;         // first element in the flat parameter vector
    int64_t stride;         // floats between consecutive partials
    const float* partial;   // partial[s * stride + i], s < nparts, i < count
    int count;
    int nparts;
    int block_begin;        // first workgroup of this tensor (filled by adam_reduce_launch)
    int qlog2;              // log2 of the number of lanes that share one element's partial sum
    // Optional transposed copy of the updated parameters: the tensor read as [trows][tcols] row-major
    // goes to tdst[tcols][trows] (the B operand of the next backward products); NULL: none.
    float* tdst;
    int trows, tcols;
};

constexpr int RED_MAX_TENSORS = 48;

struct AdamArgs {
    int ntensors;
    int nloss;              // number of loss scalars (2 critic / 1 actor)
    int loss_parts;         // partials per loss scalar
    float loss_scale;       // multiplies the summed partials
    const float* loss_partial;   // [nloss][loss_parts]
    float* loss_out;
    float* theta; float* m; float* v; float* g;
    float lr, beta1, beta2, eps, inv_bc1, inv_bc2;
    // Clipping by global norm (max_norm > 0): the reduction writes the gradient to g and one
    // sum of squares per workgroup to sq_partial; a second kernel rescales and steps.
    float max_norm;
    float* sq_partial;      // at least adam_reduce_blocks(a) floats
    float* norm_out;        // receives the norm before clipping
    // Optional tracking vector (target network, lagged policy), updated in the pass that writes theta
    // (the second kernel's when the step is clipped): track[k] = tau * theta_new[k] + (1 - tau) * track[k];
    // NULL: none.
    float* track;
    float tau;
    RedTensor t[RED_MAX_TENSORS];
};

hipError_t adam_reduce_launch(const AdamArgs& a, hipStream_t stream);
// Upper bound of the reduction's workgroup count for `params` elements in `ntensors` tensors.
size_t adam_reduce_blocks_bound(size_t params, int ntensors);

// ---- output heads -----------------------------------------------------------------------
struct HeadArgs {
    int B, H;               // rows, width of the last hidden layer
    int nwg;                // workgroups launched == partial rows written
    // target critics (critic update only)
    const float* hT[2]; const float* wT[2]; const float* bT[2];
    const float* ret; const float* boot;
    // online critics
    const float* hQ[2]; const float* wQ[2]; const float* bQ[2];
    float* dQ[2];           // delta at the last hidden layer, [B][H]
    float* y; float* q[2];  // [B] each (kept for inspection)
    float* p_dw[2];         // [nwg][H]  partial sums of dL/dW_out
    float* p_dbh[2];        // [nwg][H]  partial column sums of dQ (bias grad of last hidden)
    float* p_db[2];         // [nwg]     partial sums of dL/db_out
    float* p_loss;          // [2][nwg] (critic) or [1][nwg] (policy)
    // soft target of the stochastic-policy variant: y = ret + boot * (min Q' - exp(*log_alpha) * logp_next)
    const float* logp_next; const float* log_alpha;
};

// ---- stochastic (tanh-Gaussian) policy of the SAC variant -----------------------------------
constexpr float SAC_LOG_STD_MIN = -5.f, SAC_LOG_STD_MAX = 2.f;
constexpr int SAC_ROWS = 256;           // rows per workgroup of the policy-gradient kernel
struct SacSampleArgs {
    int B, a;
    const float* out2a;     // [B][2a]: mu, raw log sigma
    float* act;             // [B][a]  tanh(mu + sigma eps)
    float* logp;            // [B] log pi(a|s), or NULL
    float* eps;             // [B][a] the draws, kept for the backward pass, or NULL
    uint32_t stream_id, key0, key1, ctr2, ctr3;
};
hipError_t sac_sample_launch(const SacSampleArgs& a, hipStream_t stream);

struct SacGradArgs {
    int B, a;
    const float* d_u;       // [B][a]: dJ/da * (1 - a^2) from the critics
    const float* act; const float* eps; const float* out2a; const float* logp;
    const float* log_alpha;
    float* d_out;           // [B][2a]: gradient at the policy's output layer
    float* p_cols;          // [nblk][2a] partial column sums of d_out (output-bias gradient)
    float* p_logp;          // [nblk] partial sums of log pi
};
hipError_t sac_grad_launch(const SacGradArgs& a, hipStream_t stream);

struct SacAlphaArgs {
    int B, nparts;
    const float* p_logp;
    float* temperature;     // log alpha, Adam m, Adam v
    float* loss_out;        // [2] <- alpha * mean log pi, [3] <- mean log pi
    float target_entropy, lr, beta1, beta2, eps, inv_bc1, inv_bc2;
};
hipError_t sac_alpha_launch(const SacAlphaArgs& a, hipStream_t stream);

// Heads of the distributional critics (PQL-D): one wavefront per row, lane = atom.
constexpr int DIST_MAX_ATOMS = 64;
struct DistHeadArgs {
    int B, atoms, nwg;
    float v_min, v_max;
    const float* logitsT[2];    // [B][atoms] target critics at (s', pi^v(s'))   (critic update only)
    float* logitsQ[2];          // [B][atoms] online critics; overwritten with dLoss/dlogits
    const float* ret; const float* boot;
    float* p_db[2];             // [nwg][atoms] partial sums of the output-bias gradient (critic update only)
    float* p_loss;              // [2][nwg] (critic) or [1][nwg] (policy)
};
hipError_t dist_critic_head_launch(const DistHeadArgs& a, hipStream_t stream);
hipError_t dist_policy_head_launch(const DistHeadArgs& a, hipStream_t stream);

hipError_t critic_head_launch(const HeadArgs& a, hipStream_t stream);
hipError_t policy_head_launch(const HeadArgs& a, hipStream_t stream);
int head_workgroups(int B);
int dist_head_workgroups(int B);

// ---- replay + elementwise ---------------------------------------------------------------
struct PushArgs {
    const float* src[5]; float* dst[5]; int64_t count[5];   // floats per field
};
double adam_bytes(const AdamArgs& a);
hipError_t push_launch(const PushArgs& a, hipStream_t stream);

struct SampleArgs {
    pql_replay_storage st; pql_batch out;
    const int64_t* idx_in;  // NULL: draw indices; else use these
    int batch, o, a, N, T, nstep;
    int head, count;
    float gamma;
    uint32_t key0, key1, ctr2, ctr3;
    const float* nmean;     // optional standardisation of s and s': (x - nmean[c]) * nrstd[c]
    const float* nrstd;
    uint32_t stream_id;     // generator stream of the draw: 1 = transitions, 3 = the P-learner's states
    int only_obs;           // 1: windows of one row, write idx and obs only
};
hipError_t sample_launch(const SampleArgs& a, hipStream_t stream);

hipError_t soft_update_launch(const float* src, float* dst, int64_t count, float tau, hipStream_t stream);
// dst <- tau * src + (1 - tau) * dst, one rounding per operation in this order everywhere it is computed
// (the stand-alone kernel and the optimiser kernel's tracking epilogue give the same bits).
__device__ inline float polyak_mix(float tau, float keep, float src, float dst) {
    return __fmaf_rn(tau, src, __fmul_rn(keep, dst));
}

// ---- running observation statistics --------------------------------------------------------
// Device block handed over by the caller (all offsets in bytes from its 256-byte aligned start):
//   double count, pad, mean[o], m2[o];  float mean_f[o], rstd_f[o];  then per-chunk partials.
constexpr int OBS_CHUNK_ROWS = 64;
struct ObsStatsView {
    double* stat;           // count, pad, mean[o], m2[o]
    float* mean_f;          // [o]
    float* rstd_f;          // [o]
    double* part;           // [nchunk][2][o]: chunk mean, chunk sum of squared deviations
};
size_t obs_stats_bytes(int o, int max_rows);
ObsStatsView obs_stats_view(void* base, int o);
hipError_t obs_stats_reset_launch(const ObsStatsView& v, int o, float eps, hipStream_t stream);
hipError_t obs_stats_update_launch(const ObsStatsView& v, const float* obs, int rows, int o, float eps, hipStream_t stream);
hipError_t normalize_rows_launch(const float* x, const float* mean_f, const float* rstd_f, float* out, int rows, int o,
                                 hipStream_t stream);

// ---- row-tile fused kernels (layers at most FUSED_MAXW wide) ------------------------------
constexpr int FUSED_BM = 32;        // batch rows per workgroup
constexpr int FUSED_MAXW = 256;     // widest hidden layer
constexpr int FUSED_MAX_ACT = 32;   // widest action vector

// Stochastic (tanh-Gaussian) policy inside the row-tile kernels: which draw to use and where alpha lives.
struct FusedSac {
    int on;
    uint32_t stream_id, key0, key1, ctr2, ctr3;
    const float* log_alpha;
};

struct FusedNet {                   // per layer l = 0..L: weights W_l[in][out] and bias b_l[out]
    const float* w[PQL_MAX_HIDDEN + 1];
    const float* b[PQL_MAX_HIDDEN + 1];
};

struct FusedCriticArgs {
    int B, o, a, L, nwg, hmax;
    int H[PQL_MAX_HIDDEN];
    FusedNet pi;                    // lagged policy pi^v
    FusedNet qt[2];                 // target critics
    FusedNet q[2];                  // online critics
    const float* wT[2][PQL_MAX_HIDDEN + 1];   // [i][l]: transpose of W_l of online critic i, l = 1..L-1
    const float *obs, *act, *ret, *next_obs, *boot;
    float* hQ[2][PQL_MAX_HIDDEN + 1];          // [i][l], l = 1..L-1: hidden activations (layer numbers from 1)
    float* dQ[2][PQL_MAX_HIDDEN + 1];          // [i][l], l = 1..L: deltas
    float* colQ[2][PQL_MAX_HIDDEN + 1];        // [i][l], l = 1..L-1: bias-gradient partials [nwg][H_l]
    float* y; float* q_out[2];
    float* p_dw[2]; float* p_dbh[2]; float* p_db[2]; float* p_loss;
    FusedSac sac;                   // on: a' is a sample of pi^v and y carries the entropy term
    // distributional critics (atoms >= 2): the last layer has `atoms` outputs
    int atoms; float v_min, v_max;
    const float* woT[2];            // transpose of the online critics' output weights: [atoms][H_L]
    float* dlg[2];                  // [B][atoms] dLoss/dlogits (for the weight-gradient GEMM)
    float* p_dbo[2];                // [nwg][atoms] partial sums of the output-bias gradient
};
hipError_t fused_critic_launch(const FusedCriticArgs& a, hipStream_t stream);
size_t fused_lds_bytes(int o, int a, int hmax);

struct FusedPolicyArgs {
    int B, o, a, L, nwg, hmax;
    int H[PQL_MAX_HIDDEN];
    FusedNet pi;                    // policy being updated
    FusedNet q[2];                  // online critics (read-only)
    const float* wT[2][PQL_MAX_HIDDEN + 1];   // [i][l]: transpose of critic W_l, l = 1..L-1
    const float* w1aT[2];                      // transpose of the action rows of critic W_0: [H_1][a]
    const float* waT[PQL_MAX_HIDDEN + 1];      // [l]: transpose of policy W_l, l = 1..L
    const float* obs;
    float* hA[PQL_MAX_HIDDEN + 1];             // [l], l = 1..L: policy activations
    float* dA[PQL_MAX_HIDDEN + 1];             // [l], l = 1..L: policy deltas
    float* colA[PQL_MAX_HIDDEN + 2];           // [l], l = 1..L+1: bias-gradient partials [nwg][width]
    float* hQ[2][PQL_MAX_HIDDEN + 1];          // [i][l], l = 1..L-1: critic activations (scratch for L > 2)
    float* dPre;                               // [B][a] (stochastic policy: [B][2a]): delta at the policy's output layer
    float* q_out[2];
    float* p_loss;                             // [nwg]
    FusedSac sac;                              // on: reparameterised sample, log-density terms in the gradient
    float* p_logp;                             // [nwg] partial sums of log pi (stochastic policy)
    int atoms; float v_min, v_max;             // distributional critics (atoms >= 2)
    const float* woT[2];                       // transpose of the critics' output weights: [atoms][H_L]
};
hipError_t fused_policy_launch(const FusedPolicyArgs& a, hipStream_t stream);

struct FusedActArgs {
    int B, o, a, L, hmax;
    int H[PQL_MAX_HIDDEN];
    FusedNet pi;
    const float* obs;
    const float* nmean;             // optional standardisation of obs
    const float* nrstd;
    float* act_out;
    GemmNoise noise;
    FusedSac sac;                   // on: the action is a sample of the policy, `noise` is unused
};
hipError_t fused_act_launch(const FusedActArgs& a, hipStream_t stream);
// The same step on 16-row tiles (pql_act16.hip), for up to 4096 environments.
bool act16_ok(const FusedActArgs& a);
hipError_t fused_act16_launch(const FusedActArgs& a, hipStream_t stream);

// Row-tile chains for networks with layers up to 512 columns wide (pql_chain.hip): same argument blocks,
// scalar critics and deterministic policy only.
bool chain_shape_ok(int o, int a, const int* H, int L);
size_t chain_lds_bytes(int o, int a, const int* H, int L);
hipError_t chain_critic_launch(const FusedCriticArgs& a, hipStream_t stream);
hipError_t chain_policy_launch(const FusedPolicyArgs& a, hipStream_t stream);
hipError_t chain_act_launch(const FusedActArgs& a, hipStream_t stream);

struct TransposeArgs {
    struct Mat { const float* src; float* dst; int rows, cols, block_begin, pad_; };
    int n;
    // most entries: policy step with PQL_MAX_HIDDEN layers and distributional critics:
    // 2 * (L - 1 + 1 + 1) critic matrices + L policy matrices = 26
    Mat m[2 * (PQL_MAX_HIDDEN + 1) + PQL_MAX_HIDDEN];
};
hipError_t transpose_launch(TransposeArgs& a, hipStream_t stream);

// Forward layers too wide for the chained kernels, on row tiles (pql_fused.hip).
bool layer_rowtile_ok(const GemmGroup& g);
hipError_t layer_rowtile_launch(GemmGroup& g, hipStream_t stream);
// Action-wide products (at most 32 columns) of the layered path on row tiles.
bool narrow_rowtile_ok(const GemmGroup& g);
hipError_t narrow_rowtile_launch(GemmGroup& g, hipStream_t stream);

}  // namespace pql
