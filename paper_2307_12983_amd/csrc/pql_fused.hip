// Row-tile fused learner kernels for networks whose layers are at most 256 wide.
//
// A workgroup (8 wavefronts) owns 32 batch rows and carries them through a whole chain of
// layers: the activations of the tile live in LDS (two ping-pong buffers), the weights are
// streamed straight from L2 into registers as the B operand of v_mfma_f32_32x32x2_f32 (each
// wavefront owns 32 output columns, lanes run along the contiguous output dimension of W, so
// every load is a coalesced 128-byte row piece), and only what a later kernel needs (activations
// and deltas for the weight-gradient GEMMs) is written to memory.  For the V-learner step this
// replaces the per-layer launches of the target policy, the twin target critics, the twin online
// critics, the output heads and the backward data path by one launch; weight gradients (a
// contraction over the whole batch) stay in the split-K GEMM kernel.
//
// Backward products delta * W^T are computed as delta * (W^T) with W^T materialised once per
// call by transpose_kernel, so that they use the same coalesced operand path.
#include "pql_rowtile.h"

namespace pql {


// LDS of one row tile: XA (state-like input), XB (action-like input), two ping-pong activation
// tiles for each of two networks, scratch for split contractions (aliased onto the second
// network's tiles when those are large enough), small per-row arrays.
struct TileMem {
    int XA, XB, H0, scratch, sm;          // offsets into smem, in floats
    int SXA, SXB, SH;
    // ping-pong tile k of network n; computed, not tabulated: a table indexed at run time would
    // live in private memory
    __device__ int Ht(int n, int k) const { return H0 + (2 * n + k) * (BMF * SH); }
};

__host__ __device__ inline int tile_floats(int o, int a, int hmax, bool with_small) {
    const int sxa = ((o + 7) & ~7) + 4, sxb = ((a + 7) & ~7) + 4, sh = hmax + 4;
    const int scratch = (2 * BMF * sh >= SCRATCH_F) ? 0 : SCRATCH_F;
    return BMF * (sxa + sxb + 4 * sh) + scratch + (with_small ? 48 * BMF : 0);
}

__device__ inline TileMem carve(int o, int a, int hmax) {
    TileMem m;
    m.SXA = ((o + 7) & ~7) + 4;
    m.SXB = ((a + 7) & ~7) + 4;
    m.SH = hmax + 4;
    m.XA = 0;
    m.XB = m.XA + BMF * m.SXA;
    m.H0 = m.XB + BMF * m.SXB;
    int p = m.H0 + 4 * BMF * m.SH;
    if (2 * BMF * m.SH >= SCRATCH_F) m.scratch = m.Ht(1, 0);
    else { m.scratch = p; p += SCRATCH_F; }
    m.sm = p;
    return m;
}

// Whether the scratch region reaches into tile k of the second network.  When it is aliased it starts at
// that network's tile 0 and is SCRATCH_F floats long: it covers tile 0 and, for tiles shorter than that,
// the head of tile 1 as well.
__device__ inline bool scratch_overlaps(const TileMem& m, int k) {
    return m.scratch == m.Ht(1, 0) && (k == 0 || BMF * m.SH < SCRATCH_F);
}

size_t fused_lds_bytes(int o, int a, int hmax) { return sizeof(float) * (size_t)tile_floats(o, a, hmax, true); }

// Hidden layers of NN equally shaped networks on the tile: layer 1 reads XA (and XB when
// a_cols > 0), later layers ping-pong between the two tiles of each network.  Returns the index of
// the tile holding the last hidden activations.  With keep_hidden, hG[n][l] (l = 1..keep_upto, L - 1 by
// default, and L with store_last) receives h_l; the flag is separate from the pointers so that no address
// derived from the kernel's argument block is ever compared (that would force a private copy of the block).
// Rows to bring into XA / XB as soon as the first layer has consumed them (their load latency then
// hides behind the remaining layers instead of standing alone before the next chain).
struct NextInputs { const float* xa; int xa_cols; const float* xb; int xb_cols; };

template <int NN>
__device__ inline int hidden_forward(const Lanes& T, const TileMem& m, const FusedNet* const (&nets)[NN], const int* Hw,
                                     int L, int o, int a_cols, bool keep_hidden, float* const* const (&hG)[NN], int r0,
                                     int B, bool store_last = false, const NextInputs* next = nullptr, int keep_upto = -1) {
    int cur = 0;
    const int kept = keep_upto < 0 ? L - 1 : keep_upto;
    for (int l = 0; l < L; ++l) {
        const int N = Hw[l];
        WideArgs<NN> w;
        w.ldw = N; w.N = N; w.epi = WIDE_BIAS_ELU; w.ldaux = 0; w.ldo = m.SH; w.ldg = N;
        const int dst = (l == 0) ? 0 : (cur ^ 1);
#pragma unroll
        for (int n = 0; n < NN; ++n) {
            if (l == 0) {
                w.in0[n] = m.XA; w.W0[n] = nets[n]->w[0];
                w.in1[n] = m.XB; w.W1[n] = nets[n]->w[0] + (size_t)o * N;
            } else {
                w.in0[n] = m.Ht(n, cur); w.W0[n] = nets[n]->w[l];
                w.in1[n] = 0; w.W1[n] = nullptr;
            }
            w.bias[n] = nets[n]->b[l]; w.aux[n] = 0;
            w.outL[n] = m.Ht(n, dst);
            w.outG[n] = (keep_hidden && (l < kept || (store_last && l == L - 1))) ? hG[n][l + 1] : nullptr;
            w.colsum[n] = nullptr;
        }
        if (l == 0) { w.ld0 = m.SXA; w.K0 = o; w.ld1 = m.SXB; w.K1 = a_cols; }
        else        { w.ld0 = m.SH; w.K0 = Hw[l - 1]; w.ld1 = 0; w.K1 = 0; }
        wide_linear<NN>(T, w, r0, B);
        cur = dst;
        __syncthreads();
        if (l == 0 && next != nullptr) {
            load_rows(T, m.XA, m.SXA, next->xa, next->xa_cols, r0, B);
            if (next->xb != nullptr) load_rows(T, m.XB, m.SXB, next->xb, next->xb_cols, r0, B);
        }
    }
    return cur;
}

// ---- stochastic policy on a tile (SAC variant) ------------------------------------------------

__device__ inline float std_normal_f(uint32_t element, const FusedSac& sc) {
    uint32_t w0, w1;
    philox4x32_10_f(element, sc.stream_id, sc.ctr2, sc.ctr3, sc.key0, sc.key1, w0, w1);
    // double precision: (w >> 8) + 0.5 needs 25 significant bits
    const double u1 = ((double)(w0 >> 8) + 0.5) * 0x1p-24;
    const double u2 = ((double)(w1 >> 8) + 0.5) * 0x1p-24;
    return (float)(sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2));
}

// After small_partial() of the policy's 2a-column output layer: element e of the 32x32 result tile
// that falls on column col < a draws eps, forms a = tanh(mu + sigma eps) and its share of log pi;
// the shares of a row (32 consecutive lanes) are added, so every lane returns the row's log pi.
// Outputs for col >= a are zero.
__device__ inline float sac_tile_sample(int scratch, int e, int a, const float* __restrict__ bias, int r0, const FusedSac& sc,
                                        int& row, int& col, float& act, float& eps, float& raw) {
    const float s = small_sum(scratch, e, row, col);
    float lp = 0.f;
    act = 0.f; eps = 0.f; raw = 0.f;
    if (col < a) {
        int r2, c2;
        const float mu = s + bias[col];
        raw = small_sum(scratch, e + a, r2, c2) + bias[col + a];
        eps = std_normal_f((uint32_t)((r0 + row) * a + col), sc);
        const float ls = fminf(fmaxf(raw, SAC_LOG_STD_MIN), SAC_LOG_STD_MAX);
        const float u = mu + expf(ls) * eps;
        const float x = -2.f * u;
        const float softplus = fmaxf(x, 0.f) + log1pf(expf(-fabsf(x)));
        lp = -0.5f * eps * eps - ls - 0.91893853320467274178f - 2.f * (0.69314718055994530942f - u - softplus);
        act = tanhf(u);
    }
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) lp += __shfl_xor(lp, o);
    return lp;
}

// ---- distributional critics on a tile (PQL-D) -------------------------------------------------
__device__ inline float wmax(float x) {
    x = fmaxf(x, dpp_move<0xB1>(x));
    x = fmaxf(x, dpp_move<0x4E>(x));
    x = fmaxf(x, dpp_move<0x141>(x));
    x = fmaxf(x, dpp_move<0x140>(x));
    return fmaxf(fmaxf(lane_value(x, 0), lane_value(x, 16)), fmaxf(lane_value(x, 32), lane_value(x, 48)));
}

// Softmax over the lanes < atoms (lane = atom): returns p and, through logp, log p (0 for idle lanes).
__device__ inline float lane_softmax_f(float logit, bool live, float& logp) {
    const float mx = wmax(live ? logit : -3.0e38f);
    const float e = live ? expf(logit - mx) : 0.f;
    const float s = wsum(e);
    logp = live ? (logit - mx) - logf(s) : 0.f;
    return e / s;
}

// Logits of two critics (atoms <= 64 columns each) from their last hidden tiles: wavefront w takes
// network (w >> 1) & 1, 32-column tile w & 1 and every second chunk of the contraction starting at
// w >> 2; the eight partial 32x32 tiles go to `scratch` (accumulator layout).  The scratch region may
// alias one of the input tiles, hence the barrier between reading and writing.
__device__ inline void dist_logit_partial(const Lanes& T, const int (&in)[2], int ld, int K, const float* const (&W)[2],
                                          int atoms, int scratch) {
    floatx16 acc[1];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][r] = 0.f;
    const int net = (T.wave >> 1) & 1, tile = T.wave & 1, kh = T.wave >> 2;
    const int n = tile * 32 + T.l32;
    const int ncol = n < atoms ? n : atoms - 1;
    const int ins[1] = {net ? in[1] : in[0]};
    const float* const ws[1] = {net ? W[1] : W[0]};
    if (tile * 32 < atoms) mac_segment<1>(acc, ins, ld, K, ws, atoms, ncol, T, kh, 2);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) smem[scratch + T.wave * 1024 + r * 64 + T.lane] = acc[0][r];
}

// Logit (before the bias) of network `net` at tile row `row`, atom k < 64, from those partial tiles.
__device__ inline float dist_logit(int scratch, int net, int row, int k) {
    const int tile = k >> 5, col = k & 31;
    const int rr = ((row >> 3) << 2) | (row & 3), half = (row >> 2) & 1;    // inverse of acc_row()
    const int e = rr * 64 + half * 32 + col;
    const int w0 = net * 2 + tile;
    return smem[scratch + w0 * 1024 + e] + smem[scratch + (w0 + 4) * 1024 + e];
}

// =============================================================================================
// V-learner step on one row tile (Algorithm 3; Section 3.2 for the lagged target policy):
// a' = pi^v(s'), t_i = Q'_i(s', a'), y = ret + boot * min(t_1, t_2); q_i = Q_i(s, a);
// loss partials, output deltas, and the deltas of every hidden layer of both critics.  The twin
// critics always run as a pair: each wavefront carries one 32-column tile of both.
// =============================================================================================
template <bool DIST>
__global__ __launch_bounds__(FT) void fused_critic_kernel(const FusedCriticArgs A) {
    Lanes T;
    T.tid = threadIdx.x; T.lane = T.tid & 63; T.wave = __builtin_amdgcn_readfirstlane(T.tid >> 6); T.l32 = T.lane & 31; T.half = T.lane >> 5;
    const int o = A.o, a = A.a, L = A.L, B = A.B;
    const bool sac = A.sac.on != 0;
    const TileMem m = carve(o, sac ? 2 * a : a, A.hmax);
    const int r0 = blockIdx.x * BMF;
    const int HL = A.H[L - 1];
    float* sm_ret = &smem[m.sm];           // [32]
    float* sm_boot = &smem[m.sm + 32];     // [32]
    float* sm_y = &smem[m.sm + 64];        // [32]
    float* sm_logp = &smem[m.sm + 96];     // [32] log pi^v(a'|s') of the sampled target action
    float* sm_red = &smem[m.sm + 128];     // [FW][4]

    // ---- target path ------------------------------------------------------------------------
    load_rows(T, m.XA, m.SXA, A.next_obs, o, r0, B);
    if (T.tid < 32) {
        const bool rv = r0 + T.tid < B;
        sm_ret[T.tid] = rv ? A.ret[r0 + T.tid] : 0.f;
        sm_boot[T.tid] = rv ? A.boot[r0 + T.tid] : 0.f;
    }
    __syncthreads();
    int cur;
    {
        const FusedNet* const nets[1] = {&A.pi};
        float* const* const hg[1] = {nullptr};
        cur = hidden_forward<1>(T, m, nets, A.H, L, o, 0, false, hg, r0, B);
    }
    const int aw = sac ? 2 * a : a;        // columns of the policy's output layer
    small_partial(T, m.Ht(0, cur), m.SH, HL, A.pi.w[L], aw, aw, m.scratch);
    __syncthreads();
    for (int e = T.tid; e < 1024; e += FT) {
        int row, col;
        if (sac) {      // a' ~ pi^v(.|s') with its log-density (soft target of the SAC variant)
            float act, eps, raw;
            const float lp = sac_tile_sample(m.scratch, e, a, A.pi.b[L], r0, A.sac, row, col, act, eps, raw);
            if (col < m.SXB - 4) smem[m.XB + row * m.SXB + col] = act;
            if (col == 0) sm_logp[row] = lp;
        } else {
            const float s = small_sum(m.scratch, e, row, col);
            if (col < m.SXB - 4) smem[m.XB + row * m.SXB + col] = col < a ? tanhf(s + A.pi.b[L][col]) : 0.f;
        }
    }
    __syncthreads();
    {
        const FusedNet* const nets[2] = {&A.qt[0], &A.qt[1]};
        float* const* const hg[2] = {nullptr, nullptr};
        const NextInputs nx = {A.obs, o, A.act, a};        // the online critics' inputs
        cur = hidden_forward<2>(T, m, nets, A.H, L, o, a, false, hg, r0, B, false, &nx);
    }
    float m_reg[BMF / FW];      // distributional critics: the projected target distribution of this wavefront's rows (lane = atom)
    const int atoms = DIST ? A.atoms : 1;
    const bool live = T.lane < atoms;
    const float dz = DIST ? (A.v_max - A.v_min) / (float)(atoms - 1) : 0.f;
    const float zk = A.v_min + (float)T.lane * dz;
    if (DIST) {
        // logits of the twin target critics, the smaller mean picks the next-state distribution, its atoms
        // move to clip(ret + boot z) and are projected back onto the support (lane k gathers atom k's mass)
        const int ins[2] = {m.Ht(0, cur), m.Ht(1, cur)};
        const float* const wo[2] = {A.qt[0].w[L], A.qt[1].w[L]};
        dist_logit_partial(T, ins, m.SH, HL, wo, atoms, m.scratch);
        __syncthreads();
        const float bt0 = live ? A.qt[0].b[L][T.lane] : 0.f, bt1 = live ? A.qt[1].b[L][T.lane] : 0.f;
#pragma unroll
        for (int rr = 0; rr < BMF / FW; ++rr) {
            const int row = T.wave * (BMF / FW) + rr;
            float unused;
            const float t0 = lane_softmax_f(dist_logit(m.scratch, 0, row, T.lane) + bt0, live, unused);
            const float t1 = lane_softmax_f(dist_logit(m.scratch, 1, row, T.lane) + bt1, live, unused);
            const float q0 = wsum(t0 * zk), q1 = wsum(t1 * zk);
            const float pn = q0 <= q1 ? t0 : t1;
            const float tz = fminf(fmaxf(sm_ret[row] + sm_boot[row] * zk, A.v_min), A.v_max);
            const float pos = (tz - A.v_min) / dz;
            float mm = 0.f;
            for (int j = 0; j < atoms; ++j) {           // j is wave-uniform: lane j's values come as scalars
                const float pos_j = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pos), j));
                const float pn_j = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pn), j));
                mm += pn_j * fminf(fmaxf(1.f - fabsf(pos_j - (float)T.lane), 0.f), 1.f);
            }
            m_reg[rr] = live ? mm : 0.f;
        }
    } else {
        {   // scalar heads of the target critics, min, TD target: one wavefront per row
            float wt0[4], wt1[4];
    #pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = T.lane + 64 * j;
                wt0[j] = c < HL ? A.qt[0].w[L][c] : 0.f;
                wt1[j] = c < HL ? A.qt[1].w[L][c] : 0.f;
            }
            const float bt0 = A.qt[0].b[L][0], bt1 = A.qt[1].b[L][0];
            const float alpha = sac ? expf(A.sac.log_alpha[0]) : 0.f;
            // all reads, then all reductions, then all results: the rows' chains (LDS read -> dot product ->
            // wave reduction) are independent and overlap instead of running one after the other
            float st[2][BMF / FW];
#pragma unroll
            for (int rr = 0; rr < BMF / FW; ++rr) {
                const int row = T.wave * (BMF / FW) + rr;
                float s0 = 0.f, s1 = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int c = T.lane + 64 * j;
                    const int cc = c < HL ? c : 0;          // idle lanes read a valid column and multiply by a zero weight
                    s0 += smem[m.Ht(0, cur) + row * m.SH + cc] * wt0[j];
                    s1 += smem[m.Ht(1, cur) + row * m.SH + cc] * wt1[j];
                }
                st[0][rr] = s0; st[1][rr] = s1;
            }
#pragma unroll
            for (int rr = 0; rr < BMF / FW; ++rr) {
                st[0][rr] = wsum(st[0][rr]) + bt0;
                st[1][rr] = wsum(st[1][rr]) + bt1;
            }
#pragma unroll
            for (int rr = 0; rr < BMF / FW; ++rr) {
                const int row = T.wave * (BMF / FW) + rr;
                if (T.lane == 0) {
                    float tq = fminf(st[0][rr], st[1][rr]);
                    if (sac) tq -= alpha * sm_logp[row];
                    const float y = sm_ret[row] + sm_boot[row] * tq;
                    sm_y[row] = y;
                    if (r0 + row < B) A.y[r0 + row] = y;
                }
            }
        }
    }
    __syncthreads();
    // ---- online critics (their inputs were loaded behind the target critics' first layer) ---------
    {
        const FusedNet* const nets[2] = {&A.q[0], &A.q[1]};
        float* const* const hg[2] = {A.hQ[0], A.hQ[1]};
        cur = hidden_forward<2>(T, m, nets, A.H, L, o, a, true, hg, r0, B, DIST);
    }
    const float invB = 1.f / (float)B;
    float loss_acc[2] = {0.f, 0.f}, db_acc[2] = {0.f, 0.f};
    float dw_acc[2][4], dbh_acc[2][4];
    if (DIST) {
        // logits of the online critics, cross-entropy against the projected target, dLoss/dlogits
        const int ins[2] = {m.Ht(0, cur), m.Ht(1, cur)};
        const float* const wo[2] = {A.q[0].w[L], A.q[1].w[L]};
        dist_logit_partial(T, ins, m.SH, HL, wo, atoms, m.scratch);
        __syncthreads();
        float dl[2][BMF / FW];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const float bq = live ? A.q[i].b[L][T.lane] : 0.f;
#pragma unroll
            for (int rr = 0; rr < BMF / FW; ++rr) {
                const int row = T.wave * (BMF / FW) + rr;
                const bool rv = r0 + row < B;
                float lp;
                const float p = lane_softmax_f(dist_logit(m.scratch, i, row, T.lane) + bq, live, lp);
                const float S = wsum(m_reg[rr]);
                const float ce = wsum(m_reg[rr] * lp);
                if (rv) loss_acc[i] -= ce;
                const float d = (rv && live) ? (p * S - m_reg[rr]) * invB : 0.f;
                dl[i][rr] = d;
                db_acc[i] += d;                         // per lane: the output-bias gradient of atom `lane`
                if (rv && live) A.dlg[i][(size_t)(r0 + row) * atoms + T.lane] = d;
            }
        }
        __syncthreads();                                // the partial tiles in scratch have been read
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int rr = 0; rr < BMF / FW; ++rr)
                smem[m.Ht(i, cur ^ 1) + (T.wave * (BMF / FW) + rr) * m.SH + T.lane] = dl[i][rr];
        smem[m.sm + 160 + (0 * FW + T.wave) * 64 + T.lane] = db_acc[0];
        smem[m.sm + 160 + (1 * FW + T.wave) * 64 + T.lane] = db_acc[1];
        // the partial tiles may have overwritten the second critic's last hidden tile: bring it back
        if (scratch_overlaps(m, cur)) load_rows(T, m.Ht(1, cur), m.SH, A.hQ[1][L], HL, r0, B);
        __syncthreads();
        // delta of the last hidden layer: (dlogits W_out^T) * ELU'(h_L), in place over h_L
        WideArgs<2> w;
        w.ld0 = m.SH; w.K0 = atoms; w.ld1 = 0; w.K1 = 0; w.ldw = HL; w.N = HL; w.epi = WIDE_MUL_DELU;
        w.ldaux = m.SH; w.ldo = m.SH; w.ldg = HL;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            w.in0[i] = m.Ht(i, cur ^ 1); w.W0[i] = A.woT[i]; w.in1[i] = 0; w.W1[i] = nullptr;
            w.bias[i] = nullptr; w.aux[i] = m.Ht(i, cur); w.outL[i] = m.Ht(i, cur);
            w.outG[i] = A.dQ[i][L];
            w.colsum[i] = A.colQ[i][L] + (size_t)blockIdx.x * HL;
        }
        wide_linear<2>(T, w, r0, B);
    } else {   // heads: q, Bellman error, output delta; delta of the last hidden layer written in place
        float wq[2][4], bq[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            bq[i] = A.q[i].b[L][0];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                wq[i][j] = (T.lane + 64 * j < HL) ? A.q[i].w[L][T.lane + 64 * j] : 0.f;
                dw_acc[i][j] = 0.f; dbh_acc[i][j] = 0.f;
            }
        }
        // phases instead of a row-by-row loop: the rows' chains are independent (see the target heads)
        float hh[2][BMF / FW][4], qv[2][BMF / FW];
#pragma unroll
        for (int rr = 0; rr < BMF / FW; ++rr) {
            const int row = T.wave * (BMF / FW) + rr;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                float sdot = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int c = T.lane + 64 * j;
                    hh[i][rr][j] = c < HL ? smem[m.Ht(i, cur) + row * m.SH + c] : 0.f;
                    sdot += hh[i][rr][j] * wq[i][j];
                }
                qv[i][rr] = sdot;
            }
        }
#pragma unroll
        for (int rr = 0; rr < BMF / FW; ++rr)
#pragma unroll
            for (int i = 0; i < 2; ++i) qv[i][rr] = wsum(qv[i][rr]) + bq[i];
        // per-lane addresses of this wavefront's first row, formed once: inside the loop the compiler
        // otherwise fetches the pointers from the argument block again before every store
        const int row_w = T.wave * (BMF / FW);
        float* gdq[2];
        float* gq[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            gdq[i] = A.dQ[i][L] + (size_t)(r0 + row_w) * (size_t)HL + T.lane;
            gq[i] = A.q_out[i] + r0 + row_w;
        }
#pragma unroll
        for (int rr = 0; rr < BMF / FW; ++rr) {
            const int row = row_w + rr;
            const bool rv = r0 + row < B;
            const float yv = sm_y[row];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int hrow = m.Ht(i, cur) + row * m.SH + T.lane;
                const float q = qv[i][rr];
                const float e = rv ? q - yv : 0.f;
                const float d = 2.f * e * invB;
                loss_acc[i] += e * e;
                db_acc[i] += d;
                if (T.lane == 0 && rv) gq[i][rr] = q;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (T.lane + 64 * j < HL) {
                        const float g = d * wq[i][j] * delu_h(hh[i][rr][j]);
                        smem[hrow + 64 * j] = g;
                        if (rv) gdq[i][(size_t)rr * (size_t)HL + 64 * j] = g;
                        dbh_acc[i][j] += g;
                        dw_acc[i][j] += d * hh[i][rr][j];
                    }
                }
            }
        }
    }
    __syncthreads();
    // backward data path: delta_{l-1} = (delta_l W_l^T) * ELU'(z_{l-1}), l = L..2 (layers from 1)
    for (int l = L; l >= 2; --l) {
        const int Hl = A.H[l - 1], Hp = A.H[l - 2];
        if (l < L || DIST) {   // h_{l-1} is no longer on chip (the dlogits took its tile): bring it back from memory
            load_rows(T, m.Ht(0, cur ^ 1), m.SH, A.hQ[0][l - 1], Hp, r0, B);
            load_rows(T, m.Ht(1, cur ^ 1), m.SH, A.hQ[1][l - 1], Hp, r0, B);
            __syncthreads();
        }
        WideArgs<2> w;
        w.ld0 = m.SH; w.K0 = Hl; w.ld1 = 0; w.K1 = 0; w.ldw = Hp; w.N = Hp; w.epi = WIDE_MUL_DELU;
        w.ldaux = m.SH; w.ldo = m.SH; w.ldg = Hp;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            w.in0[i] = m.Ht(i, cur); w.W0[i] = A.wT[i][l - 1]; w.in1[i] = 0; w.W1[i] = nullptr;
            w.bias[i] = nullptr; w.aux[i] = m.Ht(i, cur ^ 1); w.outL[i] = m.Ht(i, cur ^ 1);
            w.outG[i] = A.dQ[i][l - 1];
            w.colsum[i] = A.colQ[i][l - 1] + (size_t)blockIdx.x * Hp;
        }
        wide_linear<2>(T, w, r0, B);
        cur ^= 1;
        __syncthreads();
    }
    // ---- per-workgroup partial sums -----------------------------------------------------------
    // scratch[(arr * FW + wave) * 256 + c], arr = 0..3: dW_out(Q1), dW_out(Q2), db_L(Q1), db_L(Q2)
    if (!DIST) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = T.lane + 64 * j;
            smem[m.scratch + (0 * FW + T.wave) * 256 + c] = dw_acc[0][j];
            smem[m.scratch + (1 * FW + T.wave) * 256 + c] = dw_acc[1][j];
            smem[m.scratch + (2 * FW + T.wave) * 256 + c] = dbh_acc[0][j];
            smem[m.scratch + (3 * FW + T.wave) * 256 + c] = dbh_acc[1][j];
        }
    }
    if (T.lane == 0) {
        sm_red[T.wave * 4 + 0] = loss_acc[0]; sm_red[T.wave * 4 + 1] = loss_acc[1];
        sm_red[T.wave * 4 + 2] = db_acc[0];   sm_red[T.wave * 4 + 3] = db_acc[1];
    }
    __syncthreads();
    const int wg = blockIdx.x, nwg = gridDim.x;
    if (DIST) {
        // output-bias gradient per atom: the wavefronts' per-lane sums were left in the small region
        if (T.tid < 128) {
            const int i = T.tid >> 6, k = T.tid & 63;
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < FW; ++w) s += smem[m.sm + 160 + (i * FW + w) * 64 + k];
            if (k < atoms) A.p_dbo[i][(size_t)wg * atoms + k] = s;
        }
    } else {
        for (int e = T.tid; e < 4 * 256; e += FT) {
            const int arr = e >> 8, c = e & 255;
            if (c < HL) {
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < FW; ++w) s += smem[m.scratch + (arr * FW + w) * 256 + c];
                float* dst = arr == 0 ? A.p_dw[0] : (arr == 1 ? A.p_dw[1] : (arr == 2 ? A.p_dbh[0] : A.p_dbh[1]));
                dst[(size_t)wg * HL + c] = s;
            }
        }
    }
    if (T.tid < 4) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < FW; ++w) s += sm_red[w * 4 + T.tid];
        if (T.tid == 0) A.p_loss[wg] = s;
        if (T.tid == 1) A.p_loss[nwg + wg] = s;
        if (!DIST && T.tid == 2) A.p_db[0][wg] = s;
        if (!DIST && T.tid == 3) A.p_db[1][wg] = s;
    }
}

// =============================================================================================
// P-learner step on one row tile (Algorithm 2: maximise min_i Q_i(s, pi(s))): a = pi(s), both
// critics on (s, a), the gradient -1/B through the smaller critic down to its action input,
// through tanh' and back through the policy.  Leaves the policy's activations and deltas in
// memory for the weight-gradient GEMMs.
// =============================================================================================
template <bool DIST>
__global__ __launch_bounds__(FT) void fused_policy_kernel(const FusedPolicyArgs A) {
    Lanes T;
    T.tid = threadIdx.x; T.lane = T.tid & 63; T.wave = __builtin_amdgcn_readfirstlane(T.tid >> 6); T.l32 = T.lane & 31; T.half = T.lane >> 5;
    const int o = A.o, a = A.a, L = A.L, B = A.B;
    const bool sac = A.sac.on != 0;
    const int aw = sac ? 2 * a : a;        // columns of the policy's output layer
    const TileMem m = carve(o, aw, A.hmax);
    const int r0 = blockIdx.x * BMF;
    const int HL = A.H[L - 1], H1 = A.H[0];
    float* sm_red = &smem[m.sm + 128];     // [FW]
    const int wg = blockIdx.x;

    load_rows(T, m.XA, m.SXA, A.obs, o, r0, B);
    __syncthreads();
    int cur;
    {
        const FusedNet* const nets[1] = {&A.pi};
        float* const* const hg[1] = {A.hA};
        cur = hidden_forward<1>(T, m, nets, A.H, L, o, 0, true, hg, r0, B, true);
    }
    small_partial(T, m.Ht(0, cur), m.SH, HL, A.pi.w[L], aw, aw, m.scratch);
    __syncthreads();
    float* sm_eps = &smem[m.sm + 160];     // [32][16] draws of the reparameterised sample
    float* sm_raw = &smem[m.sm + 672];     // [32][16] raw log sigma outputs
    float logp_acc = 0.f;
    for (int e = T.tid; e < 1024; e += FT) {
        int row, col;
        if (sac) {      // a = tanh(mu + sigma eps); eps and raw are kept for the backward pass
            float act, eps, raw;
            const float lp = sac_tile_sample(m.scratch, e, a, A.pi.b[L], r0, A.sac, row, col, act, eps, raw);
            if (col < m.SXB - 4) smem[m.XB + row * m.SXB + col] = act;
            if (col < a) { sm_eps[row * 16 + col] = eps; sm_raw[row * 16 + col] = raw; }
            if (col == 0 && r0 + row < B) logp_acc += lp;
        } else {
            const float s = small_sum(m.scratch, e, row, col);
            if (col < m.SXB - 4) smem[m.XB + row * m.SXB + col] = col < a ? tanhf(s + A.pi.b[L][col]) : 0.f;
        }
    }
    __syncthreads();
    {
        // the critics' activations leave the chip only where the backward pass below reads them back: h_{L-1}
        // is still in its tile when that pass starts (unless the dlogits of distributional critics took it)
        const FusedNet* const nets[2] = {&A.q[0], &A.q[1]};
        float* const* const hg[2] = {A.hQ[0], A.hQ[1]};
        cur = hidden_forward<2>(T, m, nets, A.H, L, o, a, true, hg, r0, B, DIST, nullptr, DIST ? L - 1 : L - 2);
    }
    float loss_acc = 0.f;
    if (DIST) {
        // Q_i = mean of critic i's distribution; the smaller one receives dJ/dlogit_k = -(1/B) p_k (z_k - Q)
        const int atoms = A.atoms;
        const bool live = T.lane < atoms;
        const float zk = A.v_min + (float)T.lane * ((A.v_max - A.v_min) / (float)(atoms - 1));
        const float invB = 1.f / (float)B;
        const int ins[2] = {m.Ht(0, cur), m.Ht(1, cur)};
        const float* const wo[2] = {A.q[0].w[L], A.q[1].w[L]};
        dist_logit_partial(T, ins, m.SH, HL, wo, atoms, m.scratch);
        __syncthreads();
        const float bq0 = live ? A.q[0].b[L][T.lane] : 0.f, bq1 = live ? A.q[1].b[L][T.lane] : 0.f;
        float dl[2][BMF / FW];
#pragma unroll
        for (int rr = 0; rr < BMF / FW; ++rr) {
            const int row = T.wave * (BMF / FW) + rr;
            const bool rv = r0 + row < B;
            float unused;
            const float p0 = lane_softmax_f(dist_logit(m.scratch, 0, row, T.lane) + bq0, live, unused);
            const float p1 = lane_softmax_f(dist_logit(m.scratch, 1, row, T.lane) + bq1, live, unused);
            const float q0 = wsum(p0 * zk), q1 = wsum(p1 * zk);
            const bool pick0 = q0 <= q1;
            if (rv) loss_acc += pick0 ? q0 : q1;
            if (T.lane == 0 && rv) { A.q_out[0][r0 + row] = q0; A.q_out[1][r0 + row] = q1; }
            dl[0][rr] = (rv && live && pick0) ? -invB * p0 * (zk - q0) : 0.f;
            dl[1][rr] = (rv && live && !pick0) ? -invB * p1 * (zk - q1) : 0.f;
        }
        __syncthreads();                                // the partial tiles in scratch have been read
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int rr = 0; rr < BMF / FW; ++rr)
                smem[m.Ht(i, cur ^ 1) + (T.wave * (BMF / FW) + rr) * m.SH + T.lane] = dl[i][rr];
        if (scratch_overlaps(m, cur)) load_rows(T, m.Ht(1, cur), m.SH, A.hQ[1][L], HL, r0, B);
        __syncthreads();
        WideArgs<2> w;
        w.ld0 = m.SH; w.K0 = atoms; w.ld1 = 0; w.K1 = 0; w.ldw = HL; w.N = HL; w.epi = WIDE_MUL_DELU;
        w.ldaux = m.SH; w.ldo = m.SH; w.ldg = HL;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            w.in0[i] = m.Ht(i, cur ^ 1); w.W0[i] = A.woT[i]; w.in1[i] = 0; w.W1[i] = nullptr;
            w.bias[i] = nullptr; w.aux[i] = m.Ht(i, cur); w.outL[i] = m.Ht(i, cur);
            w.outG[i] = nullptr; w.colsum[i] = nullptr;
        }
        wide_linear<2>(T, w, r0, B);
    } else {   // heads: q_1, q_2, the smaller one receives -1/B; delta of the last hidden layer in place
        const float invB = 1.f / (float)B;
        float wq[2][4], bq[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            bq[i] = A.q[i].b[L][0];
#pragma unroll
            for (int j = 0; j < 4; ++j) wq[i][j] = (T.lane + 64 * j < HL) ? A.q[i].w[L][T.lane + 64 * j] : 0.f;
        }
        // phases instead of a row-by-row loop: the rows' chains (LDS read -> dot product -> wave reduction)
        // are independent and overlap
        float hh[2][BMF / FW][4], qv[2][BMF / FW];
#pragma unroll
        for (int rr = 0; rr < BMF / FW; ++rr) {
            const int row = T.wave * (BMF / FW) + rr;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                float sdot = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int c = T.lane + 64 * j;
                    hh[i][rr][j] = c < HL ? smem[m.Ht(i, cur) + row * m.SH + c] : 0.f;
                    sdot += hh[i][rr][j] * wq[i][j];
                }
                qv[i][rr] = sdot;
            }
        }
#pragma unroll
        for (int rr = 0; rr < BMF / FW; ++rr)
#pragma unroll
            for (int i = 0; i < 2; ++i) qv[i][rr] = wsum(qv[i][rr]) + bq[i];
#pragma unroll
        for (int rr = 0; rr < BMF / FW; ++rr) {
            const int row = T.wave * (BMF / FW) + rr;
            const bool rv = r0 + row < B;
            const float q0 = qv[0][rr], q1 = qv[1][rr];
            if (T.lane == 0 && rv) { A.q_out[0][r0 + row] = q0; A.q_out[1][r0 + row] = q1; }
            const bool pick0 = q0 <= q1;
            if (rv) loss_acc += pick0 ? q0 : q1;
            const float d[2] = {(rv && pick0) ? -invB : 0.f, (rv && !pick0) ? -invB : 0.f};
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int c = T.lane + 64 * j;
                    if (c < HL) smem[m.Ht(i, cur) + row * m.SH + c] = d[i] * wq[i][j] * delu_h(hh[i][rr][j]);
                }
        }
    }
    __syncthreads();
    // critic backward data path down to the first hidden layer (no parameter gradients here)
    for (int l = L; l >= 2; --l) {
        const int Hl = A.H[l - 1], Hp = A.H[l - 2];
        if (l < L || DIST) {
            load_rows(T, m.Ht(0, cur ^ 1), m.SH, A.hQ[0][l - 1], Hp, r0, B);
            load_rows(T, m.Ht(1, cur ^ 1), m.SH, A.hQ[1][l - 1], Hp, r0, B);
            __syncthreads();
        }
        WideArgs<2> w;
        w.ld0 = m.SH; w.K0 = Hl; w.ld1 = 0; w.K1 = 0; w.ldw = Hp; w.N = Hp; w.epi = WIDE_MUL_DELU;
        w.ldaux = m.SH; w.ldo = m.SH; w.ldg = Hp;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            w.in0[i] = m.Ht(i, cur); w.W0[i] = A.wT[i][l - 1]; w.in1[i] = 0; w.W1[i] = nullptr;
            w.bias[i] = nullptr; w.aux[i] = m.Ht(i, cur ^ 1); w.outL[i] = m.Ht(i, cur ^ 1);
            w.outG[i] = nullptr; w.colsum[i] = nullptr;
        }
        wide_linear<2>(T, w, r0, B);
        cur ^= 1;
        __syncthreads();
    }
    // gradient w.r.t. the action input, summed over both critics, through tanh'
    {
        floatx16 acc[1];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][r] = 0.f;
        const int ncol = T.l32 < a ? T.l32 : a - 1;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ins[1] = {m.Ht(i, cur)};
            const float* const ws[1] = {A.w1aT[i]};
            mac_segment<1>(acc, ins, m.SH, H1, ws, a, ncol, T, T.wave, FW);
        }
        // the scratch region may alias the second network's tiles: everyone must be done reading
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 16; ++r) smem[m.scratch + T.wave * 1024 + r * 64 + T.lane] = acc[0][r];
    }
    __syncthreads();
    const float ab = sac ? expf(A.sac.log_alpha[0]) / (float)B : 0.f;
    for (int e = T.tid; e < 1024; e += FT) {
        int row, col;
        const float s = small_sum(m.scratch, e, row, col);
        const bool rv = r0 + row < B;
        if (!sac) {
            if (col < m.SXB - 4) {
                const float ap = smem[m.XB + row * m.SXB + col];
                const float g = (col < a && rv) ? s * (1.f - ap * ap) : 0.f;
                smem[m.XB + row * m.SXB + col] = g;
                if (col < a && rv) A.dPre[(size_t)(r0 + row) * a + col] = g;
            }
        } else if (col < a) {
            // J = mean(alpha log pi - min Q): dJ/dmu = dJ/du = g + (alpha/B) 2a; dJ/draw = dJ/du sigma eps - alpha/B
            // inside the clip of log sigma, 0 outside.  This thread writes columns col (mu) and a + col (raw).
            const float ap = smem[m.XB + row * m.SXB + col];
            const float raw = sm_raw[row * 16 + col];
            const float ls = fminf(fmaxf(raw, SAC_LOG_STD_MIN), SAC_LOG_STD_MAX);
            const float dmu = rv ? s * (1.f - ap * ap) + ab * 2.f * ap : 0.f;
            const float draw = (rv && raw > SAC_LOG_STD_MIN && raw < SAC_LOG_STD_MAX) ? dmu * expf(ls) * sm_eps[row * 16 + col] - ab : 0.f;
            smem[m.XB + row * m.SXB + col] = dmu;
            smem[m.XB + row * m.SXB + a + col] = draw;
            if (rv) {
                A.dPre[(size_t)(r0 + row) * aw + col] = dmu;
                A.dPre[(size_t)(r0 + row) * aw + a + col] = draw;
            }
        } else if (col >= aw && col < m.SXB - 4) {
            smem[m.XB + row * m.SXB + col] = 0.f;
        }
    }
    __syncthreads();
    if (T.tid < aw) {      // bias gradient of the output layer: column sums of dPre over the tile
        float s = 0.f;
        for (int row = 0; row < BMF; ++row) s += smem[m.XB + row * m.SXB + T.tid];
        A.colA[L + 1][(size_t)wg * aw + T.tid] = s;
    }
    // policy backward data path: delta_L = (dPre W_out^T) * ELU'(z_L), then down the hidden layers
    int pc = 0;
    load_rows(T, m.Ht(0, pc), m.SH, A.hA[L], HL, r0, B);
    __syncthreads();
    {
        WideArgs<1> w;
        w.in0[0] = m.XB; w.W0[0] = A.waT[L]; w.ld0 = m.SXB; w.K0 = aw; w.in1[0] = 0; w.W1[0] = nullptr; w.ld1 = 0; w.K1 = 0;
        w.ldw = HL; w.N = HL; w.bias[0] = nullptr; w.aux[0] = m.Ht(0, pc); w.ldaux = m.SH; w.outL[0] = m.Ht(0, pc); w.ldo = m.SH;
        w.outG[0] = A.dA[L]; w.ldg = HL; w.colsum[0] = A.colA[L] + (size_t)wg * HL; w.epi = WIDE_MUL_DELU;
        wide_linear<1>(T, w, r0, B);
    }
    __syncthreads();
    for (int l = L; l >= 2; --l) {
        const int Hl = A.H[l - 1], Hp = A.H[l - 2];
        load_rows(T, m.Ht(0, pc ^ 1), m.SH, A.hA[l - 1], Hp, r0, B);
        __syncthreads();
        WideArgs<1> w;
        w.in0[0] = m.Ht(0, pc); w.W0[0] = A.waT[l - 1]; w.ld0 = m.SH; w.K0 = Hl; w.in1[0] = 0; w.W1[0] = nullptr; w.ld1 = 0; w.K1 = 0;
        w.ldw = Hp; w.N = Hp; w.bias[0] = nullptr; w.aux[0] = m.Ht(0, pc ^ 1); w.ldaux = m.SH; w.outL[0] = m.Ht(0, pc ^ 1); w.ldo = m.SH;
        w.outG[0] = A.dA[l - 1]; w.ldg = Hp; w.colsum[0] = A.colA[l - 1] + (size_t)wg * Hp; w.epi = WIDE_MUL_DELU;
        wide_linear<1>(T, w, r0, B);
        pc ^= 1;
        __syncthreads();
    }
    logp_acc = wsum(logp_acc);
    if (T.lane == 0) { sm_red[T.wave] = loss_acc; sm_red[FW + T.wave] = logp_acc; }
    __syncthreads();
    if (T.tid == 0) {
        float s = 0.f, lp = 0.f;
#pragma unroll
        for (int w = 0; w < FW; ++w) { s += sm_red[w]; lp += sm_red[FW + w]; }
        A.p_loss[wg] = s;
        if (sac) A.p_logp[wg] = lp;
    }
}

// =============================================================================================
// Actor step on one row tile (Section 3.3, Algorithm 1): a = clip(pi(s) + sigma_i * eps, -1, 1).
// =============================================================================================
__global__ __launch_bounds__(FT) void fused_act_kernel(const FusedActArgs A) {
    Lanes T;
    T.tid = threadIdx.x; T.lane = T.tid & 63; T.wave = __builtin_amdgcn_readfirstlane(T.tid >> 6); T.l32 = T.lane & 31; T.half = T.lane >> 5;
    const int o = A.o, a = A.a, L = A.L, B = A.B;
    const bool sac = A.sac.on != 0;
    const int aw = sac ? 2 * a : a;
    const TileMem m = carve(o, aw, A.hmax);
    const int r0 = blockIdx.x * BMF;
    load_rows(T, m.XA, m.SXA, A.obs, o, r0, B);
    if (A.nmean != nullptr) {
        // standardise the rows just loaded (by other threads: wait for them)
        __syncthreads();
        const int kp = (o + 7) & ~7;
        for (int i = T.tid; i < BMF * kp; i += FT) {
            const int row = i / kp, col = i - row * kp;
            if (col < o && r0 + row < B) {
                const int at = m.XA + row * m.SXA + col;
                smem[at] = (smem[at] - A.nmean[col]) * A.nrstd[col];
            }
        }
    }
    __syncthreads();
    const FusedNet* const nets[1] = {&A.pi};
    float* const* const hg[1] = {nullptr};
    const int cur = hidden_forward<1>(T, m, nets, A.H, L, o, 0, false, hg, r0, B);
    small_partial(T, m.Ht(0, cur), m.SH, A.H[L - 1], A.pi.w[L], aw, aw, m.scratch);
    __syncthreads();
    const GemmNoise& nz = A.noise;
    for (int e = T.tid; e < 1024; e += FT) {
        int row, col;
        if (sac) {      // the Actor of the SAC variant samples its policy
            float act, eps, raw;
            (void)sac_tile_sample(m.scratch, e, a, A.pi.b[L], r0, A.sac, row, col, act, eps, raw);
            if (col < a && r0 + row < B) A.act_out[(size_t)(r0 + row) * a + col] = act;
            continue;
        }
        const float s = small_sum(m.scratch, e, row, col);
        const int env = r0 + row;
        if (col < a && env < B) {
            uint32_t w0, w1;
            philox4x32_10_f((uint32_t)(env * a + col), 2u, nz.ctr2, nz.ctr3, nz.key0, nz.key1, w0, w1);
            // double precision: (w >> 8) + 0.5 needs 25 significant bits
            const double u1 = ((double)(w0 >> 8) + 0.5) * 0x1p-24;
            const double u2 = ((double)(w1 >> 8) + 0.5) * 0x1p-24;
            const double eps = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
            double sigma = (double)nz.sigma_min;
            if (nz.sigma_rows > 1)
                sigma += ((double)env / (double)(nz.sigma_rows - 1)) * ((double)nz.sigma_max - (double)nz.sigma_min);
            const float x = tanhf(s + A.pi.b[L][col]) + (float)(sigma * eps);
            A.act_out[(size_t)env * a + col] = fminf(fmaxf(x, -1.f), 1.f);
        }
    }
}

hipError_t fused_policy_launch(const FusedPolicyArgs& a, hipStream_t stream) {
    const size_t lds = fused_lds_bytes(a.o, a.sac.on ? 2 * a.a : a.a, a.hmax);
    static LdsLimit configured, configured_d;
    const bool dist = a.atoms >= 2;
    const hipError_t e = dist ? set_lds_limit(reinterpret_cast<const void*>(fused_policy_kernel<true>), lds, configured_d)
                              : set_lds_limit(reinterpret_cast<const void*>(fused_policy_kernel<false>), lds, configured);
    if (e != hipSuccess) return e;
    const ProfSlot ps = prof_slot();
    if (dist) PQL_LAUNCH(ps, fused_policy_kernel<true>, dim3(a.nwg), dim3(FT), lds, stream, a);
    else      PQL_LAUNCH(ps, fused_policy_kernel<false>, dim3(a.nwg), dim3(FT), lds, stream, a);
    double flops = 0.0;
    if (ps.on) {
        double pa = (double)a.o * a.H[0], pc = (double)(a.o + a.a) * a.H[0], pb = (double)a.a * a.H[0], pab = 0.0;
        for (int l = 1; l < a.L; ++l) {
            const double w = (double)a.H[l - 1] * a.H[l];
            pa += w; pc += w; pb += w; pab += w;
        }
        const double outs = a.atoms >= 2 ? (double)a.atoms : 1.0, aw = a.sac.on ? 2.0 * a.a : (double)a.a;   // critic / policy output widths
        pa += (double)a.H[a.L - 1] * aw; pab += (double)a.H[a.L - 1] * aw; pc += a.H[a.L - 1] * outs; pb += a.H[a.L - 1] * outs;
        flops = 2.0 * a.B * (pa + 2.0 * pc + 2.0 * pb + pab);
    }
    prof_commit(ps, KID_FUSED_POLICY, flops, 0.0);
    return hipGetLastError();
}

hipError_t fused_act_launch(const FusedActArgs& a, hipStream_t stream) {
    const size_t lds = fused_lds_bytes(a.o, a.sac.on ? 2 * a.a : a.a, a.hmax);
    static LdsLimit configured;
    const hipError_t e = set_lds_limit(reinterpret_cast<const void*>(fused_act_kernel), lds, configured);
    if (e != hipSuccess) return e;
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, fused_act_kernel, dim3((a.B + BMF - 1) / BMF), dim3(FT), lds, stream, a);
    double flops = 0.0;
    if (ps.on) {
        double pa = (double)a.o * a.H[0];
        for (int l = 1; l < a.L; ++l) pa += (double)a.H[l - 1] * a.H[l];
        pa += (double)a.H[a.L - 1] * a.a;
        flops = 2.0 * a.B * pa;
    }
    prof_commit(ps, KID_FUSED_ACT, flops, 0.0);
    return hipGetLastError();
}

hipError_t fused_critic_launch(const FusedCriticArgs& a, hipStream_t stream) {
    const size_t lds = fused_lds_bytes(a.o, a.sac.on ? 2 * a.a : a.a, a.hmax);
    static LdsLimit configured, configured_d;
    const bool dist = a.atoms >= 2;
    const hipError_t le = dist ? set_lds_limit(reinterpret_cast<const void*>(fused_critic_kernel<true>), lds, configured_d)
                               : set_lds_limit(reinterpret_cast<const void*>(fused_critic_kernel<false>), lds, configured);
    if (le != hipSuccess) return le;
    const ProfSlot ps = prof_slot();
    if (dist) PQL_LAUNCH(ps, fused_critic_kernel<true>, dim3(a.nwg), dim3(FT), lds, stream, a);
    else      PQL_LAUNCH(ps, fused_critic_kernel<false>, dim3(a.nwg), dim3(FT), lds, stream, a);
    // 2 flops per multiply-add of every layer the tile passes through (no weight gradients here)
    double flops = 0.0;
    if (ps.on) {
        double pa = (double)a.o * a.H[0], pc = (double)(a.o + a.a) * a.H[0], pb = 0.0;
        for (int l = 1; l < a.L; ++l) { pa += (double)a.H[l - 1] * a.H[l]; pc += (double)a.H[l - 1] * a.H[l]; pb += (double)a.H[l - 1] * a.H[l]; }
        const double outs = a.atoms >= 2 ? (double)a.atoms : 1.0;
        pa += (double)a.H[a.L - 1] * (a.sac.on ? 2.0 * a.a : (double)a.a); pc += a.H[a.L - 1] * outs; pb += a.H[a.L - 1] * outs;
        flops = 2.0 * a.B * (pa + 4.0 * pc + 2.0 * pb);
    }
    prof_commit(ps, KID_FUSED_CRITIC, flops, 0.0);
    return hipGetLastError();
}

// =============================================================================================
// One wide layer on row tiles, for networks whose layers are too wide for the chained kernels
// above: Y = act(X W + b), or delta W^T * ELU'(.) with W^T materialised by transpose_kernel, for a
// list of problems (the twin critics, the target critics and the policy share launches).  A
// workgroup stages 32 input rows in LDS once and its eight wavefronts sweep the output columns, 32
// each per pass, with the weights streamed from L2 as in the chained kernels; nothing but the input
// rows and the output tile touches memory.  Two workgroups fit a compute unit while the input tile
// stays below 80 KB (sixteen wavefronts: the kernel is held to 128 registers, and has none to
// spare: requesting the first weight chunks ahead of the input rows spilled and ran 6 % slower).
// =============================================================================================
__global__ __launch_bounds__(FT, 4) void layer_rowtile_kernel(const GemmGroup g) {
    Lanes T;
    T.tid = threadIdx.x; T.lane = T.tid & 63; T.wave = __builtin_amdgcn_readfirstlane(T.tid >> 6); T.l32 = T.lane & 31; T.half = T.lane >> 5;
    const int b = blockIdx.x;
    int pi = 0;
    for (int i = 1; i < g.nprob; ++i)
        if (b >= g.p[i].tile_begin) pi = i;
    const GemmProb& P = g.p[pi];
    // tiles_n holds the row tiles per workgroup: 2 for layers of at most 128 columns (four wavefronts
    // cover those, the other four take a second row tile), else 1
    const int RT = P.tiles_n, CW = FW / RT;
    const int rt = T.wave / CW, cw = T.wave - rt * CW;
    const int M = P.M, N = P.N;
    const int K0 = P.seg[0].K, K1 = P.nseg > 1 ? P.seg[1].K : 0;
    const int S0 = ((K0 + 7) & ~7) + 4, S1 = K1 > 0 ? ((K1 + 7) & ~7) + 4 : 0;
    const int rw = (b - P.tile_begin) * BMF * RT;
    for (int t = 0; t < RT; ++t) {
        load_rows(T, t * BMF * S0, S0, P.seg[0].A, K0, rw + t * BMF, M);
        if (K1 > 0) load_rows(T, RT * BMF * S0 + t * BMF * S1, S1, P.seg[1].A, K1, rw + t * BMF, M);
    }
    __syncthreads();
    const int r0 = rw + rt * BMF;
    if (r0 >= M) return;                 // (no barrier follows)
    const int XA = rt * BMF * S0, XB = RT * BMF * S0 + rt * BMF * S1;
    const int epi = P.epi;
    const int ldc = P.ldc, ldaux = P.ldaux;
    const int lrow = 4 * T.half;
    const bool full = r0 + BMF <= M;
    for (int n0 = cw * 32; n0 < N; n0 += 32 * CW) {
        const int n = n0 + T.l32;
        const bool n_ok = n < N;
        const int ncol = n_ok ? n : N - 1;
        const float bv = epi == EPI_MUL_DELU ? 0.f : P.bias[ncol];
        floatx16 acc[1];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][r] = 0.f;
        const int in0[1] = {XA};
        const float* const W0[1] = {P.seg[0].B};
        if (K1 > 0) {
            float bs[1][16], bf[1][16];
            const int in1[1] = {XB};
            const float* const W1[1] = {P.seg[1].B};
            prefetch_first_chunk<1>(bs, W1, K1, P.seg[1].ldb, ncol, T, 0, 1);
            prefetch_first_chunk<1>(bf, W0, K0, P.seg[0].ldb, ncol, T, 0, 1);
            mac_segment<1>(acc, in1, S1, K1, W1, P.seg[1].ldb, ncol, T, 0, 1, true, bs);
            mac_segment<1>(acc, in0, S0, K0, W0, P.seg[0].ldb, ncol, T, 0, 1, true, bf);
        } else {
            mac_segment<1>(acc, in0, S0, K0, W0, P.seg[0].ldb, ncol, T, 0, 1);
        }
        float* __restrict__ gbase = P.C + (size_t)(r0 + lrow) * (size_t)ldc + n;
        if (epi == EPI_MUL_DELU) {
            // backward data path: delta = acc * ELU'(z) with the activation read from memory; the
            // tile's column sums are one partial row of the bias gradient
            const float* __restrict__ abase = P.aux + (size_t)(r0 + lrow) * (size_t)ldaux + ncol;
            float h[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int dr = 8 * (r >> 2) + (r & 3);
                h[r] = (full || r0 + lrow + dr < M) ? abase[(size_t)dr * (size_t)ldaux] : 0.f;
            }
            float cs = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int dr = 8 * (r >> 2) + (r & 3);
                const bool rv = full || r0 + lrow + dr < M;
                const float x = rv ? acc[0][r] * delu_h(h[r]) : 0.f;
                if (n_ok && rv) gbase[(size_t)dr * (size_t)ldc] = x;
                cs += x;
            }
            if (P.colsum != nullptr) {
                cs += __shfl_xor(cs, 32);
                if (T.half == 0 && n_ok) P.colsum[(size_t)((b - P.tile_begin) * RT + rt) * (size_t)N + n] = cs;
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int dr = 8 * (r >> 2) + (r & 3);
                float x = acc[0][r] + bv;
                if (epi == EPI_BIAS_ELU) x = elu_f(x);
                if (n_ok && (full || r0 + lrow + dr < M)) gbase[(size_t)dr * (size_t)ldc] = x;
            }
        }
    }
}

// Whether a launch of X W products (B operand [K][N] row-major) can take the row-tile layer kernel:
// bias (+ ELU) epilogues, or the backward data path's ELU' epilogue with column sums (one partial
// row per 32 batch rows); dense input rows (row stride = width), enough columns to occupy the eight wavefronts, enough rows to
// fill the chip, input tiles that fit LDS, and weights within reach of a 32-bit buffer offset.
bool layer_rowtile_ok(const GemmGroup& g) {
    long wgs = 0;
    for (int i = 0; i < g.nprob; ++i) {
        const GemmProb& p = g.p[i];
        if (p.epi != EPI_BIAS_ELU && p.epi != EPI_BIAS && p.epi != EPI_MUL_DELU) return false;
        if (p.epi == EPI_MUL_DELU ? (p.aux == nullptr || p.ldaux < p.N) : (p.bias == nullptr || p.colsum != nullptr)) return false;
        if (p.nseg < 1 || p.nseg > 2 || p.ldc < p.N) return false;
        if (p.N < 128 || p.M < 1) return false;
        size_t floats = 0;
        for (int s = 0; s < p.nseg; ++s) {
            const GemmSeg& q = p.seg[s];
            if (q.K < 1 || q.lda != q.K || q.ldb < p.N) return false;
            if ((size_t)q.K * (size_t)q.ldb * sizeof(float) >= ((size_t)1 << 31)) return false;
            floats += (size_t)BMF * (size_t)(((q.K + 7) & ~7) + 4);
        }
        if (floats * sizeof(float) > 150 * 1024) return false;
        wgs += (p.M + BMF - 1) / BMF;
    }
    return wgs >= 256;
}

static size_t layer_tile_floats(const GemmProb& p) {
    size_t floats = 0;
    for (int s = 0; s < p.nseg; ++s) floats += (size_t)BMF * (size_t)(((p.seg[s].K + 7) & ~7) + 4);
    return floats;
}

hipError_t layer_rowtile_launch(GemmGroup& g, hipStream_t stream) {
    // Narrow layers (at most 128 columns) take two row tiles per workgroup, if the launch still has
    // a workgroup for every compute unit and the two input tiles fit LDS.
    long wgs2 = 0;
    bool fits2 = true;
    for (int i = 0; i < g.nprob; ++i) {
        const GemmProb& p = g.p[i];
        const int rt = p.N <= 128 ? 2 : 1;
        wgs2 += (p.M + BMF * rt - 1) / (BMF * rt);
        if (rt == 2 && 2 * layer_tile_floats(p) * sizeof(float) > 150 * 1024) fits2 = false;
    }
    const bool pair_rows = fits2 && wgs2 >= 256;
    int total = 0;
    size_t lds = 0;
    double flops = 0.0;
    for (int i = 0; i < g.nprob; ++i) {
        GemmProb& p = g.p[i];
        const int rt = (pair_rows && p.N <= 128) ? 2 : 1;
        p.tile_begin = total;
        p.tiles_m = (p.M + BMF * rt - 1) / (BMF * rt); p.tiles_n = rt; p.splits = 1; p.k_chunk = 0;
        total += p.tiles_m;
        for (int s = 0; s < p.nseg; ++s) flops += 2.0 * p.M * (double)p.N * p.seg[s].K;
        const size_t bytes = rt * layer_tile_floats(p) * sizeof(float);
        if (bytes > lds) lds = bytes;
    }
    g.total_tiles = total;
    if (total == 0) return hipSuccess;
    static LdsLimit configured;
    const hipError_t e = set_lds_limit(reinterpret_cast<const void*>(layer_rowtile_kernel), lds, configured);
    if (e != hipSuccess) return e;
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, layer_rowtile_kernel, dim3(total), dim3(FT), lds, stream, g);
    prof_commit(ps, KID_LAYER_ROWTILE, ps.on ? flops : 0.0, 0.0);
    return hipGetLastError();
}

// =============================================================================================
// Action-wide products of the layered path (at most 32 output columns): the policy's output layer
// (with the Actor's exploration noise where asked for) and the gradient with respect to the action.  One wavefront's 32 columns already cover the
// output, so the eight wavefronts of a row tile split the contraction instead (every eighth chunk
// of 32 k-values each, as in the chained kernels' narrow layers) and their partial tiles meet in
// LDS.  Segments (the twin critics' first-layer deltas) pass through the same input tile one after
// the other.  B operands are row-major [K][N].
// =============================================================================================
__global__ __launch_bounds__(FT, 2) void narrow_rowtile_kernel(const GemmGroup g) {
    Lanes T;
    T.tid = threadIdx.x; T.lane = T.tid & 63; T.wave = __builtin_amdgcn_readfirstlane(T.tid >> 6); T.l32 = T.lane & 31; T.half = T.lane >> 5;
    const int b = blockIdx.x;
    int pi = 0;
    for (int i = 1; i < g.nprob; ++i)
        if (b >= g.p[i].tile_begin) pi = i;
    const GemmProb& P = g.p[pi];
    const int part = b - P.tile_begin, r0 = part * BMF, M = P.M, N = P.N;
    int kmax = P.seg[0].K;
    if (P.nseg > 1 && P.seg[1].K > kmax) kmax = P.seg[1].K;
    const int S = ((kmax + 7) & ~7) + 4;
    // input tile; the partial tiles and the 32 x 33 output tile take its place once the products are done
    const int XA = 0, scratch = 0, red = SCRATCH_F;
    const int ncol = T.l32 < N ? T.l32 : N - 1;
    floatx16 acc[1];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][r] = 0.f;
    for (int sg = 0; sg < P.nseg; ++sg) {
        if (sg > 0) __syncthreads();                                     // the tile is reused
        load_rows(T, XA, S, P.seg[sg].A, P.seg[sg].K, r0, M);
        __syncthreads();
        const int ins[1] = {XA};
        const float* const ws[1] = {P.seg[sg].B};
        mac_segment<1>(acc, ins, S, P.seg[sg].K, ws, P.seg[sg].ldb, ncol, T, T.wave, FW);
    }
    __syncthreads();                                                     // every wavefront is done with the input tile
#pragma unroll
    for (int r = 0; r < 16; ++r) smem[scratch + T.wave * 1024 + r * 64 + T.lane] = acc[0][r];
    __syncthreads();
    const int epi = P.epi;
    for (int e = T.tid; e < 1024; e += FT) {
        int row, col;
        float x = small_sum(scratch, e, row, col);
        const bool ok = col < N && r0 + row < M;
        if (ok) {
            if (epi == EPI_MUL_DTANH) {
                const float t = P.aux[(size_t)(r0 + row) * (size_t)P.ldaux + col];
                x *= 1.f - t * t;
            } else {
                x = tanhf(x + P.bias[col]);
                if (epi == EPI_BIAS_TANH_NOISE) {
                    // Actor step (Section 3.3): a = clip(pi(s) + sigma_i * eps, -1, 1), sigma_i linear in the
                    // environment index, eps from Philox-4x32-10 (stream 2) by Box-Muller, as in fused_act_kernel
                    const GemmNoise& nz = g.noise;
                    const int env = r0 + row;
                    uint32_t w0, w1;
                    philox4x32_10_f((uint32_t)(env * nz.act_dim + col), 2u, nz.ctr2, nz.ctr3, nz.key0, nz.key1, w0, w1);
                    const double u1 = ((double)(w0 >> 8) + 0.5) * 0x1p-24;
                    const double u2 = ((double)(w1 >> 8) + 0.5) * 0x1p-24;
                    const double eps = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
                    double sigma = (double)nz.sigma_min;
                    if (nz.sigma_rows > 1)
                        sigma += ((double)env / (double)(nz.sigma_rows - 1)) * ((double)nz.sigma_max - (double)nz.sigma_min);
                    x = fminf(fmaxf(x + (float)(sigma * eps), -1.f), 1.f);
                }
            }
            P.C[(size_t)(r0 + row) * (size_t)P.ldc + col] = x;
        } else {
            x = 0.f;
        }
        smem[red + row * 33 + col] = x;
    }
    if (P.colsum != nullptr) {
        __syncthreads();
        if (T.tid < N) {
            float cs = 0.f;
            for (int row = 0; row < BMF; ++row) cs += smem[red + row * 33 + T.tid];
            P.colsum[(size_t)part * (size_t)N + T.tid] = cs;
        }
    }
}

static size_t narrow_lds_bytes(const GemmProb& p) {
    int kmax = p.seg[0].K;
    if (p.nseg > 1 && p.seg[1].K > kmax) kmax = p.seg[1].K;
    const size_t tile = (size_t)BMF * (size_t)(((kmax + 7) & ~7) + 4), tail = (size_t)SCRATCH_F + BMF * 33;
    return sizeof(float) * (tile > tail ? tile : tail);
}

// Whether a launch of X W products (B operand [K][N] row-major) can take the narrow row-tile kernel.
bool narrow_rowtile_ok(const GemmGroup& g) {
    long wgs = 0;
    for (int i = 0; i < g.nprob; ++i) {
        const GemmProb& p = g.p[i];
        if (p.epi != EPI_BIAS_TANH && p.epi != EPI_BIAS_TANH_NOISE && p.epi != EPI_MUL_DTANH) return false;
        if (p.epi == EPI_BIAS_TANH_NOISE && (g.nprob != 1 || g.noise.act_dim != p.N)) return false;
        if (p.epi == EPI_MUL_DTANH ? (p.aux == nullptr || p.ldaux < p.N) : (p.bias == nullptr || p.colsum != nullptr)) return false;
        if (p.N < 1 || p.N > 32 || p.M < 1 || p.nseg < 1 || p.nseg > 2 || p.ldc < p.N) return false;
        for (int s = 0; s < p.nseg; ++s) {
            const GemmSeg& q = p.seg[s];
            if (q.K < 1 || q.lda != q.K || q.ldb < p.N) return false;
            if ((size_t)q.K * (size_t)q.ldb * sizeof(float) >= ((size_t)1 << 31)) return false;
        }
        if (narrow_lds_bytes(p) > 150 * 1024) return false;
        wgs += (p.M + BMF - 1) / BMF;
    }
    return wgs >= 256;
}

hipError_t narrow_rowtile_launch(GemmGroup& g, hipStream_t stream) {
    int total = 0;
    size_t lds = 0;
    double flops = 0.0;
    for (int i = 0; i < g.nprob; ++i) {
        GemmProb& p = g.p[i];
        p.tile_begin = total;
        p.tiles_m = (p.M + BMF - 1) / BMF; p.tiles_n = 1; p.splits = 1; p.k_chunk = 0;
        total += p.tiles_m;
        for (int s = 0; s < p.nseg; ++s) flops += 2.0 * p.M * (double)p.N * p.seg[s].K;
        if (narrow_lds_bytes(p) > lds) lds = narrow_lds_bytes(p);
    }
    g.total_tiles = total;
    if (total == 0) return hipSuccess;
    static LdsLimit configured;
    const hipError_t e = set_lds_limit(reinterpret_cast<const void*>(narrow_rowtile_kernel), lds, configured);
    if (e != hipSuccess) return e;
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, narrow_rowtile_kernel, dim3(total), dim3(FT), lds, stream, g);
    prof_commit(ps, KID_NARROW_ROWTILE, ps.on ? flops : 0.0, 0.0);
    return hipGetLastError();
}

// =============================================================================================
// Batched 2-D transposes: dst[c][r] = src[r][c] for a list of small matrices.
// =============================================================================================
__global__ __launch_bounds__(256) void transpose_kernel(const TransposeArgs a) {
    __shared__ float tile[32][33];
    int b = blockIdx.x, mi = 0;
    for (int i = 1; i < a.n; ++i)
        if (b >= a.m[i].block_begin) mi = i;
    const TransposeArgs::Mat& M = a.m[mi];
    b -= M.block_begin;
    const int tiles_c = (M.cols + 31) / 32;
    const int tr = b / tiles_c, tc = b - tr * tiles_c;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int j = ty; j < 32; j += 8) {
        const int r = tr * 32 + j, c = tc * 32 + tx;
        tile[j][tx] = (r < M.rows && c < M.cols) ? M.src[(size_t)r * M.cols + c] : 0.f;
    }
    __syncthreads();
    for (int j = ty; j < 32; j += 8) {
        const int c = tc * 32 + j, r = tr * 32 + tx;
        if (r < M.rows && c < M.cols) M.dst[(size_t)c * M.rows + r] = tile[tx][j];
    }
}

hipError_t transpose_launch(TransposeArgs& a, hipStream_t stream) {
    int blocks = 0;
    double bytes = 0.0;
    for (int i = 0; i < a.n; ++i) {
        a.m[i].block_begin = blocks;
        blocks += ((a.m[i].rows + 31) / 32) * ((a.m[i].cols + 31) / 32);
        bytes += 8.0 * a.m[i].rows * a.m[i].cols;
    }
    if (blocks == 0) return hipSuccess;
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, transpose_kernel, dim3(blocks), dim3(256), 0, stream, a);
    prof_commit(ps, KID_TRANSPOSE, 0.0, bytes);
    return hipGetLastError();
}

}  // namespace pql
