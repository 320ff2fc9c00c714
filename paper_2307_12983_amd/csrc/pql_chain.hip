// Row-tile chain kernels for networks with layers wider than 256 columns (up to 512).
//
// As in pql_fused.hip a workgroup of eight wavefronts owns 32 batch rows and carries them through
// whole networks with the activations in LDS, so that a learner step is one launch instead of one
// per layer with a round trip through memory for every activation.  What differs: an activation tile
// of 512 columns takes 66 KB, so the twin critics cannot sit in LDS side by side.  Here the networks
// of a step pass through the tile ONE AFTER THE OTHER (policy, target critic 1, target critic 2, online
// critic 1 with its backward pass, online critic 2 with its backward pass), and the tiles of
// consecutive layers alternate between the two ends of one LDS pool: layer l reads the tile at one
// end and writes the tile at the other, so only two consecutive layers have to fit at a time (the
// input rows s are the tile "before layer 1" and are read again from memory for every network).  A
// layer of 512 columns is computed as two column halves that share the A operand (each wavefront holds
// one 32-column tile of either half: the inner loops are those of a pair of networks).
#include "pql_rowtile.h"

namespace pql {

// LDS map of a chain: [pool][XB: 32 x (a padded + 4)][small per-row arrays].  Tile t of the pool holds
// the input rows (t = 0, state columns only) or the activations of layer t; even tiles start at the
// pool's first float, odd tiles end at its last one.
struct ChainMem {
    int pool, SXA, SXB, XB, sm;
};

__host__ __device__ inline int chain_pad8(int n) { return ((n + 7) & ~7) + 4; }

// Floats of pool that the widths need: the largest pair of consecutive tiles, and room for the
// partial tiles of a contraction split over the wavefronts next to the widest tile they can follow.
__host__ __device__ inline int chain_pool_floats(int o, const int* H, int L) {
    int prev = BMF * chain_pad8(o), need = 0;
    for (int l = 0; l < L; ++l) {
        const int cur = BMF * (H[l] + 4);
        need = prev + cur > need ? prev + cur : need;
        need = cur + SCRATCH_F > need ? cur + SCRATCH_F : need;
        prev = cur;
    }
    return need;
}

constexpr int CHAIN_SMALL = 512;        // floats of per-row arrays and cross-wavefront sums behind XB

size_t chain_lds_bytes(int o, int a, const int* H, int L) {
    return sizeof(float) * ((size_t)chain_pool_floats(o, H, L) + (size_t)BMF * chain_pad8(a) + CHAIN_SMALL);
}

// Whether the chain kernels take this shape: every width a multiple of 32, at most 256 or exactly 512 (two
// column halves), the last hidden layer within the scalar heads' four columns per lane, actions within one
// 32-column tile, and the LDS map within a compute unit's 160 KB.
bool chain_shape_ok(int o, int a, const int* H, int L) {
    if (a < 1 || a > FUSED_MAX_ACT || o < 1 || o > 1024 || L < 1) return false;
    for (int l = 0; l < L; ++l)
        if (H[l] % 32 != 0 || (H[l] > 256 && H[l] != 512)) return false;
    if (H[L - 1] > 256) return false;
    return chain_lds_bytes(o, a, H, L) <= 160 * 1024;
}

__device__ inline ChainMem chain_carve(int o, int a, int pool) {
    ChainMem m;
    m.pool = pool; m.SXA = chain_pad8(o); m.SXB = chain_pad8(a);
    m.XB = pool; m.sm = pool + BMF * m.SXB;
    return m;
}

// Offset of tile t (t >= 1: activations of layer t, `width` columns; t = 0: the input rows, at 0).
__device__ inline int chain_tile(const ChainMem& m, int t, int width) { return (t & 1) ? m.pool - BMF * (width + 4) : 0; }

// One layer of one network on the tile: out[32 x N] = epi(in0 W0 (+ in1 W1)).  N <= 256: one 32-column
// tile per wavefront; N = 512: two column halves as a pair sharing the A operand.
__device__ inline void chain_layer(const Lanes& T, int in0, int ld0, int K0, const float* W0, int in1, int ld1, int K1,
                                   const float* W1, int ldw, int N, const float* bias, int aux, int ldaux, int outL, int ldo,
                                   float* outG, int ldg, float* colsum, int epi, int r0, int B) {
    if (N > 256) {
        WideArgs<2> w;
        w.ld0 = ld0; w.K0 = K0; w.ld1 = ld1; w.K1 = K1; w.ldw = ldw; w.N = 256; w.ldaux = ldaux; w.ldo = ldo; w.ldg = ldg; w.epi = epi;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            w.in0[j] = in0; w.W0[j] = W0 + 256 * j;
            w.in1[j] = in1; w.W1[j] = K1 > 0 ? W1 + 256 * j : nullptr;
            w.bias[j] = epi == WIDE_BIAS_ELU ? bias + 256 * j : nullptr;
            w.aux[j] = aux + 256 * j; w.outL[j] = outL + 256 * j;
            w.outG[j] = outG ? outG + 256 * j : nullptr;
            w.colsum[j] = colsum ? colsum + 256 * j : nullptr;
        }
        wide_linear<2, false>(T, w, r0, B);
    } else {
        WideArgs<1> w;
        w.ld0 = ld0; w.K0 = K0; w.ld1 = ld1; w.K1 = K1; w.ldw = ldw; w.N = N; w.ldaux = ldaux; w.ldo = ldo; w.ldg = ldg; w.epi = epi;
        w.in0[0] = in0; w.W0[0] = W0; w.in1[0] = in1; w.W1[0] = W1; w.bias[0] = bias; w.aux[0] = aux; w.outL[0] = outL;
        w.outG[0] = outG; w.colsum[0] = colsum;
        wide_linear<1>(T, w, r0, B);
    }
}

// Hidden layers of one network: layer 1 reads the input rows in tile 0 (and the action columns in XB when
// a_cols > 0), layer l + 1 reads tile l.  With keep, hG[l] receives h_l for l = 1..L-1 (and L with
// store_last).  Ends with a barrier; the last activations are in tile L.
__device__ inline void chain_forward(const Lanes& T, const ChainMem& m, const FusedNet& net, const int* Hw, int L, int o,
                                     int a_cols, bool keep, float* const* hG, bool store_last, int r0, int B) {
    for (int l = 0; l < L; ++l) {
        const int N = Hw[l];
        const int out = chain_tile(m, l + 1, N);
        float* og = (keep && (l < L - 1 || store_last)) ? hG[l + 1] : nullptr;
        if (l == 0)
            chain_layer(T, 0, m.SXA, o, net.w[0], m.XB, m.SXB, a_cols, net.w[0] + (size_t)o * N, N, N, net.b[0], 0, 0, out,
                        N + 4, og, N, nullptr, WIDE_BIAS_ELU, r0, B);
        else
            chain_layer(T, chain_tile(m, l, Hw[l - 1]), Hw[l - 1] + 4, Hw[l - 1], net.w[l], 0, 0, 0, nullptr, N, N, net.b[l], 0, 0,
                        out, N + 4, og, N, nullptr, WIDE_BIAS_ELU, r0, B);
        __syncthreads();
    }
}

// Backward data path of one network: tile L holds delta_L; for l = L..2,
// delta_{l-1} = (delta_l W_l^T) * ELU'(z_{l-1}) is formed in place over h_{l-1} in tile l - 1 (still on chip for
// l = L when last_on_chip, read back from hG[l - 1] otherwise).  With store, dG[l - 1] receives the deltas and
// colG[l - 1] one row of column sums (the bias gradient's partial for this row tile).  wT[l - 1] is W_l^T,
// row-major [H_l][H_{l-1}].  Ends with a barrier; delta_1 is in tile 1.
__device__ inline void chain_backward(const Lanes& T, const ChainMem& m, const float* const* wT, const int* Hw, int L,
                                      float* const* hG, bool last_on_chip, bool store, float* const* dG, float* const* colG,
                                      int wg, int r0, int B) {
    for (int l = L; l >= 2; --l) {
        const int Hl = Hw[l - 1], Hp = Hw[l - 2];
        const int tin = chain_tile(m, l, Hl), tout = chain_tile(m, l - 1, Hp);
        if (l < L || !last_on_chip) {
            load_rows(T, tout, Hp + 4, hG[l - 1], Hp, r0, B);
            __syncthreads();
        }
        chain_layer(T, tin, Hl + 4, Hl, wT[l - 1], 0, 0, 0, nullptr, Hp, Hp, nullptr, tout, Hp + 4, tout, Hp + 4,
                    store ? dG[l - 1] : nullptr, Hp, store ? colG[l - 1] + (size_t)wg * Hp : nullptr, WIDE_MUL_DELU, r0, B);
        __syncthreads();
    }
}

// Scalar output of one critic for this wavefront's four rows: q[rr] = h_L[row] . w_out + b_out, with the row's
// activations returned in hh (columns lane + 64 j).  Reads, then reductions, as independent chains.
__device__ inline void chain_head_dot(const Lanes& T, int tile, int ld, int HL, const float (&wq)[4], float bq,
                                      float (&hh)[BMF / FW][4], float (&q)[BMF / FW]) {
#pragma unroll
    for (int rr = 0; rr < BMF / FW; ++rr) {
        const int row = T.wave * (BMF / FW) + rr;
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = T.lane + 64 * j;
            hh[rr][j] = c < HL ? smem[tile + row * ld + c] : 0.f;
            s += hh[rr][j] * wq[j];
        }
        q[rr] = s;
    }
#pragma unroll
    for (int rr = 0; rr < BMF / FW; ++rr) q[rr] = wsum(q[rr]) + bq;
}

// =============================================================================================
// V-learner step on one row tile (Algorithm 3; Section 3.2 for the lagged target policy), scalar
// critics and deterministic policy: a' = pi^v(s'), t_i = Q'_i(s', a'), y = ret + boot * min(t_1, t_2);
// q_i = Q_i(s, a); loss partials, output deltas and the deltas of every hidden layer of both critics.
// =============================================================================================
__global__ __launch_bounds__(FT) void chain_critic_kernel(const FusedCriticArgs A, const int pool) {
    Lanes T;
    T.tid = threadIdx.x; T.lane = T.tid & 63; T.wave = __builtin_amdgcn_readfirstlane(T.tid >> 6); T.l32 = T.lane & 31; T.half = T.lane >> 5;
    const int o = A.o, a = A.a, L = A.L, B = A.B;
    const ChainMem m = chain_carve(o, a, pool);
    const int r0 = blockIdx.x * BMF, wg = blockIdx.x, nwg = gridDim.x;
    const int HL = A.H[L - 1], SL = HL + 4;
    const int tL = chain_tile(m, L, HL);
    float* sm_ret = &smem[m.sm];           // [32]
    float* sm_boot = &smem[m.sm + 32];     // [32]
    float* sm_y = &smem[m.sm + 64];        // [32]
    float* sm_t = &smem[m.sm + 96];        // [2][32] outputs of the target critics
    float* sm_red = &smem[m.sm + 160];     // [FW][2]

    // ---- lagged policy on s' ------------------------------------------------------------------
    load_rows(T, 0, m.SXA, A.next_obs, o, r0, B);
    if (T.tid < 32) {
        const bool rv = r0 + T.tid < B;
        sm_ret[T.tid] = rv ? A.ret[r0 + T.tid] : 0.f;
        sm_boot[T.tid] = rv ? A.boot[r0 + T.tid] : 0.f;
    }
    __syncthreads();
    chain_forward(T, m, A.pi, A.H, L, o, 0, false, nullptr, false, r0, B);
    {
        // output layer: the contraction is split over the wavefronts, whose partial tiles go to the end of the
        // pool that h_L does not occupy; a' = tanh(.) goes to XB, which lies outside the pool
        const int scr = (L & 1) ? 0 : pool - SCRATCH_F;
        small_partial(T, tL, SL, HL, A.pi.w[L], a, a, scr);
        __syncthreads();
        for (int e = T.tid; e < 1024; e += FT) {
            int row, col;
            const float s = small_sum(scr, e, row, col);
            if (col < m.SXB - 4) smem[m.XB + row * m.SXB + col] = col < a ? tanhf(s + A.pi.b[L][col]) : 0.f;
        }
        __syncthreads();                // the partial tiles have been read: the pool is free
    }
    // ---- target critics on (s', a'), one after the other ----------------------------------------
#pragma unroll 1
    for (int i = 0; i < 2; ++i) {
        load_rows(T, 0, m.SXA, A.next_obs, o, r0, B);      // tile 0 has been overwritten since the last network read it
        __syncthreads();
        chain_forward(T, m, A.qt[i], A.H, L, o, a, false, nullptr, false, r0, B);
        float wq[4], hh[BMF / FW][4], q[BMF / FW];
#pragma unroll
        for (int j = 0; j < 4; ++j) wq[j] = (T.lane + 64 * j < HL) ? A.qt[i].w[L][T.lane + 64 * j] : 0.f;
        chain_head_dot(T, tL, SL, HL, wq, A.qt[i].b[L][0], hh, q);
        if (T.lane == 0) {
#pragma unroll
            for (int rr = 0; rr < BMF / FW; ++rr) sm_t[i * 32 + T.wave * (BMF / FW) + rr] = q[rr];
        }
        __syncthreads();
    }
    if (T.tid < 32) {
        const float y = sm_ret[T.tid] + sm_boot[T.tid] * fminf(sm_t[T.tid], sm_t[32 + T.tid]);
        sm_y[T.tid] = y;
        if (r0 + T.tid < B) A.y[r0 + T.tid] = y;
    }
    // ---- online critics on (s, a): forward, head, backward data path, one after the other --------
    load_rows(T, m.XB, m.SXB, A.act, a, r0, B);
    const float invB = 1.f / (float)B;
#pragma unroll 1
    for (int i = 0; i < 2; ++i) {
        load_rows(T, 0, m.SXA, A.obs, o, r0, B);
        __syncthreads();
        chain_forward(T, m, A.q[i], A.H, L, o, a, true, A.hQ[i], false, r0, B);
        float wq[4], hh[BMF / FW][4], q[BMF / FW];
        float dw_acc[4], dbh_acc[4], loss_acc = 0.f, db_acc = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            wq[j] = (T.lane + 64 * j < HL) ? A.q[i].w[L][T.lane + 64 * j] : 0.f;
            dw_acc[j] = 0.f; dbh_acc[j] = 0.f;
        }
        chain_head_dot(T, tL, SL, HL, wq, A.q[i].b[L][0], hh, q);
        {
            const int row_w = T.wave * (BMF / FW);
            float* gdq = A.dQ[i][L] + (size_t)(r0 + row_w) * (size_t)HL + T.lane;
            float* gq = A.q_out[i] + r0 + row_w;
#pragma unroll
            for (int rr = 0; rr < BMF / FW; ++rr) {
                const int row = row_w + rr;
                const bool rv = r0 + row < B;
                const float e = rv ? q[rr] - sm_y[row] : 0.f;
                const float d = 2.f * e * invB;
                loss_acc += e * e;
                db_acc += d;
                if (T.lane == 0 && rv) gq[rr] = q[rr];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (T.lane + 64 * j < HL) {
                        const float g = d * wq[j] * delu_h(hh[rr][j]);
                        smem[tL + row * SL + T.lane + 64 * j] = g;         // delta_L in place of h_L
                        if (rv) gdq[(size_t)rr * (size_t)HL + 64 * j] = g;
                        dbh_acc[j] += g;
                        dw_acc[j] += d * hh[rr][j];
                    }
                }
            }
        }
        __syncthreads();
        chain_backward(T, m, A.wT[i], A.H, L, A.hQ[i], true, true, A.dQ[i], A.colQ[i], wg, r0, B);
        // per-workgroup partial sums of this critic's output-layer gradients (nothing in the pool is live now):
        // pool[(arr * FW + wave) * 256 + c], arr = 0: dW_out, 1: db_L
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            smem[(0 * FW + T.wave) * 256 + T.lane + 64 * j] = dw_acc[j];
            smem[(1 * FW + T.wave) * 256 + T.lane + 64 * j] = dbh_acc[j];
        }
        if (T.lane == 0) { sm_red[T.wave * 2 + 0] = loss_acc; sm_red[T.wave * 2 + 1] = db_acc; }
        __syncthreads();
        {
            const int arr = T.tid >> 8, c = T.tid & 255;
            if (c < HL) {
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < FW; ++w) s += smem[(arr * FW + w) * 256 + c];
                float* dst = arr == 0 ? A.p_dw[i] : A.p_dbh[i];
                dst[(size_t)wg * HL + c] = s;
            }
            if (T.tid < 2) {
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < FW; ++w) s += sm_red[w * 2 + T.tid];
                if (T.tid == 0) A.p_loss[i * nwg + wg] = s;
                else A.p_db[i][wg] = s;
            }
        }
        __syncthreads();
    }
}

// =============================================================================================
// P-learner step on one row tile (Algorithm 2: maximise min_i Q_i(s, pi(s))), scalar critics and
// deterministic policy: a = pi(s), both critics on (s, a) one after the other, the gradient -1/B
// through the smaller critic down to its action input, through tanh' and back through the policy.
// =============================================================================================
__global__ __launch_bounds__(FT) void chain_policy_kernel(const FusedPolicyArgs A, const int pool) {
    Lanes T;
    T.tid = threadIdx.x; T.lane = T.tid & 63; T.wave = __builtin_amdgcn_readfirstlane(T.tid >> 6); T.l32 = T.lane & 31; T.half = T.lane >> 5;
    const int o = A.o, a = A.a, L = A.L, B = A.B;
    const ChainMem m = chain_carve(o, a, pool);
    const int r0 = blockIdx.x * BMF, wg = blockIdx.x;
    const int HL = A.H[L - 1], SL = HL + 4, H1 = A.H[0];
    const int tL = chain_tile(m, L, HL);
    float* sm_q = &smem[m.sm];             // [2][32] critic outputs
    float* sm_d = &smem[m.sm + 64];        // [2][32] output deltas
    float* sm_red = &smem[m.sm + 128];     // [FW]

    // ---- a = pi(s), keeping the policy's activations for its backward pass -----------------------
    load_rows(T, 0, m.SXA, A.obs, o, r0, B);
    __syncthreads();
    chain_forward(T, m, A.pi, A.H, L, o, 0, true, A.hA, true, r0, B);
    {
        const int scr = (L & 1) ? 0 : pool - SCRATCH_F;
        small_partial(T, tL, SL, HL, A.pi.w[L], a, a, scr);
        __syncthreads();
        for (int e = T.tid; e < 1024; e += FT) {
            int row, col;
            const float s = small_sum(scr, e, row, col);
            if (col < m.SXB - 4) smem[m.XB + row * m.SXB + col] = col < a ? tanhf(s + A.pi.b[L][col]) : 0.f;
        }
        __syncthreads();
    }
    // ---- both critics on (s, a): every activation goes to memory, the backward passes read them back
    //      once the smaller critic of each row is known -------------------------------------------
#pragma unroll 1
    for (int i = 0; i < 2; ++i) {
        load_rows(T, 0, m.SXA, A.obs, o, r0, B);
        __syncthreads();
        chain_forward(T, m, A.q[i], A.H, L, o, a, true, A.hQ[i], true, r0, B);
        float wq[4], hh[BMF / FW][4], q[BMF / FW];
#pragma unroll
        for (int j = 0; j < 4; ++j) wq[j] = (T.lane + 64 * j < HL) ? A.q[i].w[L][T.lane + 64 * j] : 0.f;
        chain_head_dot(T, tL, SL, HL, wq, A.q[i].b[L][0], hh, q);
        if (T.lane == 0) {
#pragma unroll
            for (int rr = 0; rr < BMF / FW; ++rr) {
                const int row = T.wave * (BMF / FW) + rr;
                sm_q[i * 32 + row] = q[rr];
                if (r0 + row < B) A.q_out[i][r0 + row] = q[rr];
            }
        }
        __syncthreads();
    }
    float loss_acc = 0.f;
    if (T.tid < 32) {       // the gradient -1/B enters the smaller critic (ties: Q_1)
        const bool rv = r0 + T.tid < B;
        const float q0 = sm_q[T.tid], q1 = sm_q[32 + T.tid];
        const bool pick0 = q0 <= q1;
        const float invB = 1.f / (float)B;
        sm_d[T.tid] = (rv && pick0) ? -invB : 0.f;
        sm_d[32 + T.tid] = (rv && !pick0) ? -invB : 0.f;
        if (rv) loss_acc = pick0 ? q0 : q1;
    }
    loss_acc = wsum(loss_acc);          // rows 0..31 are the first 32 lanes of wavefront 0
    if (T.tid == 0) sm_red[0] = loss_acc;
    // ---- critic backward data paths down to the first hidden layer; the action gradient sums over both ----
    floatx16 gacc[1];
#pragma unroll
    for (int r = 0; r < 16; ++r) gacc[0][r] = 0.f;
    const int ncol_a = T.l32 < a ? T.l32 : a - 1;
#pragma unroll 1
    for (int i = 0; i < 2; ++i) {
        __syncthreads();                // sm_d is written; the previous network's tiles are no longer read
        load_rows(T, tL, SL, A.hQ[i][L], HL, r0, B);
        __syncthreads();
        for (int e = T.tid; e < BMF * HL; e += FT) {        // delta_L = d * w_out * ELU'(h_L), in place
            const int row = e / HL, c = e - row * HL;
            const int at = tL + row * SL + c;
            smem[at] = sm_d[i * 32 + row] * A.q[i].w[L][c] * delu_h(smem[at]);
        }
        __syncthreads();
        chain_backward(T, m, A.wT[i], A.H, L, A.hQ[i], false, false, nullptr, nullptr, wg, r0, B);
        const int ins[1] = {chain_tile(m, 1, H1)};
        const float* const ws[1] = {A.w1aT[i]};
        mac_segment<1>(gacc, ins, H1 + 4, H1, ws, a, ncol_a, T, T.wave, FW);
    }
    __syncthreads();                    // every wavefront is done with delta_1: the pool is free
    {
        const int scr = 0;
#pragma unroll
        for (int r = 0; r < 16; ++r) smem[scr + T.wave * 1024 + r * 64 + T.lane] = gacc[0][r];
        __syncthreads();
        for (int e = T.tid; e < 1024; e += FT) {
            int row, col;
            const float s = small_sum(scr, e, row, col);
            const bool rv = r0 + row < B;
            if (col < m.SXB - 4) {
                const float ap = smem[m.XB + row * m.SXB + col];
                const float g = (col < a && rv) ? s * (1.f - ap * ap) : 0.f;
                smem[m.XB + row * m.SXB + col] = g;
                if (col < a && rv) A.dPre[(size_t)(r0 + row) * a + col] = g;
            }
        }
        __syncthreads();
    }
    if (T.tid < a) {        // bias gradient of the output layer: column sums of dPre over the tile
        float s = 0.f;
        for (int row = 0; row < BMF; ++row) s += smem[m.XB + row * m.SXB + T.tid];
        A.colA[L + 1][(size_t)wg * a + T.tid] = s;
    }
    // ---- policy backward data path: delta_L = (dPre W_out^T) * ELU'(z_L), then down the hidden layers ----
    load_rows(T, tL, SL, A.hA[L], HL, r0, B);
    __syncthreads();
    chain_layer(T, m.XB, m.SXB, a, A.waT[L], 0, 0, 0, nullptr, HL, HL, nullptr, tL, SL, tL, SL, A.dA[L], HL,
                A.colA[L] + (size_t)wg * HL, WIDE_MUL_DELU, r0, B);
    __syncthreads();
    chain_backward(T, m, A.waT, A.H, L, A.hA, false, true, A.dA, A.colA, wg, r0, B);
    if (T.tid == 0) A.p_loss[wg] = sm_red[0];
}

// =============================================================================================
// Actor step on one row tile (Section 3.3, Algorithm 1): a = clip(pi(s) + sigma_i * eps, -1, 1).
// =============================================================================================
__global__ __launch_bounds__(FT) void chain_act_kernel(const FusedActArgs A, const int pool) {
    Lanes T;
    T.tid = threadIdx.x; T.lane = T.tid & 63; T.wave = __builtin_amdgcn_readfirstlane(T.tid >> 6); T.l32 = T.lane & 31; T.half = T.lane >> 5;
    const int o = A.o, a = A.a, L = A.L, B = A.B;
    const ChainMem m = chain_carve(o, a, pool);
    const int r0 = blockIdx.x * BMF;
    const int HL = A.H[L - 1];
    load_rows(T, 0, m.SXA, A.obs, o, r0, B);
    if (A.nmean != nullptr) {
        __syncthreads();                // standardise the rows just loaded (by other threads)
        const int kp = (o + 7) & ~7;
        for (int i = T.tid; i < BMF * kp; i += FT) {
            const int row = i / kp, col = i - row * kp;
            if (col < o && r0 + row < B) smem[row * m.SXA + col] = (smem[row * m.SXA + col] - A.nmean[col]) * A.nrstd[col];
        }
    }
    __syncthreads();
    chain_forward(T, m, A.pi, A.H, L, o, 0, false, nullptr, false, r0, B);
    const int scr = (L & 1) ? 0 : pool - SCRATCH_F;
    small_partial(T, chain_tile(m, L, HL), HL + 4, HL, A.pi.w[L], a, a, scr);
    __syncthreads();
    const GemmNoise& nz = A.noise;
    for (int e = T.tid; e < 1024; e += FT) {
        int row, col;
        const float s = small_sum(scr, e, row, col);
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

// ---- launches ------------------------------------------------------------------------------------

hipError_t chain_critic_launch(const FusedCriticArgs& a, hipStream_t stream) {
    if (!chain_shape_ok(a.o, a.a, a.H, a.L) || a.atoms >= 2 || a.sac.on) return hipErrorInvalidValue;
    const size_t lds = chain_lds_bytes(a.o, a.a, a.H, a.L);
    static LdsLimit configured;
    const hipError_t le = set_lds_limit(reinterpret_cast<const void*>(chain_critic_kernel), lds, configured);
    if (le != hipSuccess) return le;
    const int pool = chain_pool_floats(a.o, a.H, a.L);
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, chain_critic_kernel, dim3(a.nwg), dim3(FT), lds, stream, a, pool);
    double flops = 0.0;
    if (ps.on) {     // 2 flops per multiply-add of every layer the tile passes through (no weight gradients here)
        double pa = (double)a.o * a.H[0], pc = (double)(a.o + a.a) * a.H[0], pb = 0.0;
        for (int l = 1; l < a.L; ++l) { const double w = (double)a.H[l - 1] * a.H[l]; pa += w; pc += w; pb += w; }
        pa += (double)a.H[a.L - 1] * a.a; pc += a.H[a.L - 1]; pb += a.H[a.L - 1];
        flops = 2.0 * a.B * (pa + 4.0 * pc + 2.0 * pb);
    }
    prof_commit(ps, KID_CHAIN_CRITIC, flops, 0.0);
    return hipGetLastError();
}

hipError_t chain_policy_launch(const FusedPolicyArgs& a, hipStream_t stream) {
    if (!chain_shape_ok(a.o, a.a, a.H, a.L) || a.atoms >= 2 || a.sac.on) return hipErrorInvalidValue;
    const size_t lds = chain_lds_bytes(a.o, a.a, a.H, a.L);
    static LdsLimit configured;
    const hipError_t le = set_lds_limit(reinterpret_cast<const void*>(chain_policy_kernel), lds, configured);
    if (le != hipSuccess) return le;
    const int pool = chain_pool_floats(a.o, a.H, a.L);
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, chain_policy_kernel, dim3(a.nwg), dim3(FT), lds, stream, a, pool);
    double flops = 0.0;
    if (ps.on) {
        double pa = (double)a.o * a.H[0], pc = (double)(a.o + a.a) * a.H[0], pb = (double)a.a * a.H[0], pab = 0.0;
        for (int l = 1; l < a.L; ++l) { const double w = (double)a.H[l - 1] * a.H[l]; pa += w; pc += w; pb += w; pab += w; }
        pa += (double)a.H[a.L - 1] * a.a; pab += (double)a.H[a.L - 1] * a.a; pc += a.H[a.L - 1]; pb += a.H[a.L - 1];
        flops = 2.0 * a.B * (pa + 2.0 * pc + 2.0 * pb + pab);
    }
    prof_commit(ps, KID_CHAIN_POLICY, flops, 0.0);
    return hipGetLastError();
}

hipError_t chain_act_launch(const FusedActArgs& a, hipStream_t stream) {
    if (!chain_shape_ok(a.o, a.a, a.H, a.L) || a.sac.on) return hipErrorInvalidValue;
    const size_t lds = chain_lds_bytes(a.o, a.a, a.H, a.L);
    static LdsLimit configured;
    const hipError_t le = set_lds_limit(reinterpret_cast<const void*>(chain_act_kernel), lds, configured);
    if (le != hipSuccess) return le;
    const int pool = chain_pool_floats(a.o, a.H, a.L);
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, chain_act_kernel, dim3((a.B + BMF - 1) / BMF), dim3(FT), lds, stream, a, pool);
    double flops = 0.0;
    if (ps.on) {
        double pa = (double)a.o * a.H[0];
        for (int l = 1; l < a.L; ++l) pa += (double)a.H[l - 1] * a.H[l];
        pa += (double)a.H[a.L - 1] * a.a;
        flops = 2.0 * a.B * pa;
    }
    prof_commit(ps, KID_CHAIN_ACT, flops, 0.0);
    return hipGetLastError();
}

}  // namespace pql
