// Grouped fp32 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x2_f32) with fused epilogues.
//
// These are the dense contractions of the learner: every hidden layer of the policy and of the
// twin critics forward (X W + b, ELU / tanh), the backward data path (delta W^T times the
// activation derivative) and the weight gradients (X^T delta, reduced over the batch by
// split-K).  One launch handles a list of independent problems, so the twin critics, the target
// critics and the policy share launches.  Forward and backward-data products go through the
// LDS-tiled kernel described next when they are narrow or small (launches of wide layers with
// enough rows take the row-tile layer kernel of pql_fused.hip instead); the weight gradients,
// whose two operands are both contiguous along the MFMA's M / N dimension, go through
// gemm_tn_stream_kernel further down, which takes its fragments straight from memory.
//
// Tiling: a workgroup is 4 wavefronts of 64 lanes.  Global tiles are copied to LDS in their
// natural orientation (the contiguous dimension stays contiguous, 16-byte loads when the
// operand allows), the next tile is prefetched into registers while the current one feeds the
// matrix cores.  A 32x32x2 MFMA takes one A value and one B value per lane: lane l supplies
// A[m = l%32][k = l/32] and B[k = l/32][n = l%32] and owns, in accumulator register r,
// C[8*(r/4) + 4*(l/32) + r%4][l%32].  The k index inside a group of 8 is assigned as
// k = 4*(l/32) + i for the i-th of four consecutive MFMAs, so a lane's four A values (or B
// values) are contiguous in a k-contiguous tile and can be read with one 16-byte LDS load.
#include "pql_internal.h"

namespace pql {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int NTHREADS = 256;

// Workgroups are handed to the 8 XCDs round-robin by the hardware; renumber them so that a run
// of consecutive logical tiles (which share operand rows) lands on one XCD and shares its L2.
__device__ inline int xcd_remap(int bid, int nb) {
    const int q = nb >> 3, r = nb & 7;
    const int xcd = bid & 7, pos = bid >> 3;
    return xcd * q + (xcd < r ? xcd : r) + pos;
}

// ---- Philox-4x32-10 (Salmon et al., SC'11) and Box-Muller ---------------------------------
__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                     uint32_t& o0, uint32_t& o1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0; c1 = lo1; c2 = hi0 ^ c3 ^ k1; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    o0 = c0; o1 = c1;
}

__device__ inline float exploration_noise(const GemmNoise& nz, int m, int n) {
    uint32_t w0, w1;
    philox4x32_10((uint32_t)(m * nz.act_dim + n), 2u, nz.ctr2, nz.ctr3, nz.key0, nz.key1, w0, w1);
    // double precision: (w >> 8) + 0.5 needs 25 significant bits
    const double u1 = ((double)(w0 >> 8) + 0.5) * 0x1p-24;
    const double u2 = ((double)(w1 >> 8) + 0.5) * 0x1p-24;
    const double eps = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
    double sigma = (double)nz.sigma_min;
    if (nz.sigma_rows > 1)
        sigma += ((double)m / (double)(nz.sigma_rows - 1)) * ((double)nz.sigma_max - (double)nz.sigma_min);
    return (float)(sigma * eps);
}

// ---- global -> register tile loads ---------------------------------------------------------
// A ROWS x COLS tile whose COLS dimension is contiguous in memory, spread over 256 threads as
// float4 pieces; out-of-range elements read as zero.
template <int ROWS, int COLS>
struct TileRegs {
    static constexpr int C4 = COLS / 4;
    static constexpr int RPP = NTHREADS / C4;             // rows covered per pass
    static constexpr int NV = (ROWS * COLS) / (4 * NTHREADS);
    static_assert(NV >= 1 && ROWS % RPP == 0, "tile shape");
    float4 v[NV];

    __device__ inline void load(const float* __restrict__ src, int ld, int row0, int col0, int row_lim, int col_lim,
                                bool vec, int tid) {
        const int c = col0 + (tid % C4) * 4;
        const int r = row0 + tid / C4;
        // interior tile with aligned rows: straight 16-byte loads (uniform branch)
        if (vec && row0 + ROWS <= row_lim && col0 + COLS <= col_lim) {
            const float* p = src + (size_t)r * (size_t)ld + c;
#pragma unroll
            for (int i = 0; i < NV; ++i)
                v[i] = *reinterpret_cast<const float4*>(p + (size_t)(i * RPP) * (size_t)ld);
            return;
        }
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int rr = r + i * RPP;
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (rr < row_lim && c < col_lim) {
                const float* p = src + (size_t)rr * (size_t)ld + c;
                if (vec && c + 3 < col_lim) {
                    x = *reinterpret_cast<const float4*>(p);
                } else {
                    x.x = p[0];
                    if (c + 1 < col_lim) x.y = p[1];
                    if (c + 2 < col_lim) x.z = p[2];
                    if (c + 3 < col_lim) x.w = p[3];
                }
            }
            v[i] = x;
        }
    }

    __device__ inline void zero() {
#pragma unroll
        for (int i = 0; i < NV; ++i) v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }

    __device__ inline void store(float* tile, int stride, int tid) const {
        const int c = (tid % C4) * 4;
        const int r = tid / C4;
#pragma unroll
        for (int i = 0; i < NV; ++i)
            *reinterpret_cast<float4*>(tile + (r + i * RPP) * stride + c) = v[i];
    }
};

// One K-segment of a problem, copied to registers so that the main loop issues no descriptor
// loads.
struct SegRegs {
    const float* A;
    const float* B;
    int lda, ldb, kbeg, kend;
    bool va, vb;
};

template <int MODE, int WAVES_M, int WAVES_N, int TM, int TN, bool NOISE, int BK = 32>
__global__ __launch_bounds__(NTHREADS) void gemm_grouped_kernel(const GemmGroup g) {
    constexpr int BM = WAVES_M * TM * 32;
    constexpr int BN = WAVES_N * TN * 32;
    constexpr bool A_KC = (MODE != GEMM_TN);   // A tile k-contiguous: As[m][k]; else As[k][m]
    constexpr bool B_KC = (MODE == GEMM_NT);   // B tile k-contiguous: Bs[n][k]; else Bs[k][n]
    constexpr int KSTRIDE = BK + 4;            // row stride (floats) of a k-contiguous LDS tile
    constexpr int SA = A_KC ? KSTRIDE : BM;
    constexpr int SB = B_KC ? KSTRIDE : BN;
    constexpr int A_TILE = A_KC ? BM * SA : BK * SA;
    constexpr int B_TILE = B_KC ? BN * SB : BK * SB;
    // two LDS stages: tile t is consumed from stage t&1 while tile t+1 is written to the other
    __shared__ __attribute__((aligned(16))) float As[2][A_TILE];
    __shared__ __attribute__((aligned(16))) float Bs[2][B_TILE];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    const int bid = xcd_remap(blockIdx.x, gridDim.x);
    int pi = 0;
    for (int i = 1; i < g.nprob; ++i)
        if (bid >= g.p[i].tile_begin) pi = i;
    const GemmProb& P = g.p[pi];

    int local = bid - P.tile_begin;
    const int per_split = P.tiles_m * P.tiles_n;
    const int split = local / per_split;
    local -= split * per_split;
    const int tile_m = local / P.tiles_n, tile_n = local % P.tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int M = P.M, N = P.N;

    // K range per segment (split-K applies to single-segment problems only)
    SegRegs s0, s1;
    s0.A = P.seg[0].A; s0.B = P.seg[0].B; s0.lda = P.seg[0].lda; s0.ldb = P.seg[0].ldb;
    s0.va = (P.seg[0].vec & 1) != 0; s0.vb = (P.seg[0].vec & 2) != 0;
    s0.kbeg = 0; s0.kend = P.seg[0].K;
    if (MODE == GEMM_TN) {
        s0.kbeg = split * P.k_chunk;
        s0.kend = min(P.seg[0].K, s0.kbeg + P.k_chunk);
    }
    s1 = s0;
    int nt1 = 0;
    if (P.nseg > 1) {
        s1.A = P.seg[1].A; s1.B = P.seg[1].B; s1.lda = P.seg[1].lda; s1.ldb = P.seg[1].ldb;
        s1.va = (P.seg[1].vec & 1) != 0; s1.vb = (P.seg[1].vec & 2) != 0;
        s1.kbeg = 0; s1.kend = P.seg[1].K;
        nt1 = (s1.kend + BK - 1) / BK;
    }
    const int nt0 = (s0.kend - s0.kbeg + BK - 1) / BK;
    const int nt = nt0 + nt1;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    typedef TileRegs<A_KC ? BM : BK, A_KC ? BK : BM> RegsA;
    typedef TileRegs<B_KC ? BN : BK, B_KC ? BK : BN> RegsB;
    RegsA ra0, ra1;      // even / odd K-tiles in flight
    RegsB rb0, rb1;

    auto fetch = [&](int t, RegsA& ra, RegsB& rb) {
        if (t >= nt) { ra.zero(); rb.zero(); return; }       // the padding tile of an odd count
        const bool first = t < nt0;
        const SegRegs& S = first ? s0 : s1;
        const int k0 = first ? s0.kbeg + t * BK : (t - nt0) * BK;
        if (A_KC) ra.load(S.A, S.lda, m0, k0, M, S.kend, S.va, tid);
        else      ra.load(S.A, S.lda, k0, m0, S.kend, M, S.va, tid);
        if (B_KC) rb.load(S.B, S.ldb, n0, k0, N, S.kend, S.vb, tid);
        else      rb.load(S.B, S.ldb, k0, n0, S.kend, N, S.vb, tid);
    };

    // Operand fragments of one group of 8 k-values: lane-half h holds k = 4h + u, u = 0..3.
    auto load_frag = [&](const float* __restrict__ Asm, const float* __restrict__ Bsm, int kg, float (&a)[TM][4],
                         float (&b)[TN][4]) {
        const int kk = kg * 8 + 4 * half;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = (wm * TM + i) * 32 + l32;
            if (A_KC) {
                const float4 x = *reinterpret_cast<const float4*>(Asm + m * SA + kk);
                a[i][0] = x.x; a[i][1] = x.y; a[i][2] = x.z; a[i][3] = x.w;
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) a[i][u] = Asm[(kk + u) * SA + m];
            }
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = (wn * TN + j) * 32 + l32;
            if (B_KC) {
                const float4 x = *reinterpret_cast<const float4*>(Bsm + n * SB + kk);
                b[j][0] = x.x; b[j][1] = x.y; b[j][2] = x.z; b[j][3] = x.w;
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) b[j][u] = Bsm[(kk + u) * SB + n];
            }
        }
    };
    auto mfma_group = [&](const float (&a)[TM][4], const float (&b)[TN][4]) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][u], b[j][u], acc[i][j], 0, 0, 0);
    };

    // Every K-tile runs the full 32 k-values: the tile loads fill k beyond the segment's end with
    // zeros on both operands, so a short last tile needs no path of its own (a second path makes
    // the compiler shuttle the accumulators between register sets on every iteration).
    auto compute = [&](int t) {
        const float* Asm = As[t & 1];
        const float* Bsm = Bs[t & 1];
        float a[2][TM][4], b[2][TN][4];
        // The fragments of group kg + 1 are read from LDS while group kg feeds the matrix core: the
        // reads are spread between the MFMAs (one read after every few of them) instead of all being
        // issued, and waited for, right before their first use.
        constexpr int NMFMA = 4 * TM * TN;
        constexpr int NREAD = (A_KC ? TM : 2 * TM) + (B_KC ? TN : 2 * TN);
        constexpr int PER = NMFMA / (NREAD + 1) > 0 ? NMFMA / (NREAD + 1) : 1;
        load_frag(Asm, Bsm, 0, a[0], b[0]);
#pragma unroll
        for (int kg = 0; kg < BK / 8; ++kg) {
            if (kg + 1 < BK / 8) load_frag(Asm, Bsm, kg + 1, a[(kg + 1) & 1], b[(kg + 1) & 1]);
            mfma_group(a[kg & 1], b[kg & 1]);
            if (kg + 1 < BK / 8) {
#pragma unroll
                for (int i = 0; i < NREAD; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);    // MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // LDS read
                }
            }
            __builtin_amdgcn_sched_group_barrier(0x008, NMFMA, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Software pipeline: while tile t feeds the matrix cores from LDS stage t&1, tile t+2 is requested
    // from memory and tile t+1, requested one step earlier, moves from registers into the other stage
    // after the matrix work (a load has two steps of matrix work to arrive before it is waited for).
    // The tiles are taken in pairs with nothing conditional around the matrix work (an odd count is
    // padded with one all-zero tile): a conditional second half makes the compiler move every
    // accumulator between the accumulation registers and ordinary ones on each iteration.
    const int nt2 = (nt + 1) & ~1;
    if (nt > 0) {
        fetch(0, ra0, rb0);
        fetch(1, ra1, rb1);
        ra0.store(As[0], SA, tid);
        rb0.store(Bs[0], SB, tid);
        __syncthreads();
    }
    for (int t = 0; t < nt2; t += 2) {
        if (t + 2 < nt2) fetch(t + 2, ra0, rb0);
        compute(t);
        ra1.store(As[1], SA, tid);
        rb1.store(Bs[1], SB, tid);
        __syncthreads();
        if (t + 3 < nt2) fetch(t + 3, ra1, rb1);
        compute(t + 1);
        if (t + 2 < nt2) { ra0.store(As[0], SA, tid); rb0.store(Bs[0], SB, tid); }
        __syncthreads();
    }

    // ---- epilogue -------------------------------------------------------------------------
    const int epi = P.epi;
    float* __restrict__ C = P.C + (MODE == GEMM_TN ? (size_t)split * (size_t)P.split_stride : (size_t)0);
    const int ldc = P.ldc;
    const float* __restrict__ aux = P.aux;
    const int ldaux = P.ldaux;
    float* __restrict__ colsum = P.colsum;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + (wn * TN + j) * 32 + l32;
        const bool n_ok = n < N;
        float bias = 0.f;
        if (n_ok && (epi == EPI_BIAS_ELU || epi == EPI_BIAS_TANH || epi == EPI_BIAS_TANH_NOISE || epi == EPI_BIAS)) bias = P.bias[n];
        float csum = 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + (wm * TM + i) * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                if (!n_ok || m >= M) continue;
                float x = acc[i][j][r];
                switch (epi) {
                    // ELU: exp(x) - 1 has absolute error ~1e-7 for x <= 0, the same size as the
                    // rounding of the accumulation that produced x
                    case EPI_BIAS_ELU: x += bias; x = x > 0.f ? x : __expf(x) - 1.f; break;
                    case EPI_BIAS_TANH: x = tanhf(x + bias); break;
                    case EPI_BIAS: x += bias; break;
                    case EPI_BIAS_TANH_NOISE:
                        x = tanhf(x + bias);
                        if (NOISE) x = fminf(fmaxf(x + exploration_noise(g.noise, m, n), -1.f), 1.f);
                        break;
                    case EPI_MUL_DELU: {
                        const float h = aux[(size_t)m * ldaux + n];
                        x *= (h > 0.f ? 1.f : h + 1.f);
                        break;
                    }
                    case EPI_MUL_DTANH: {
                        const float h = aux[(size_t)m * ldaux + n];
                        x *= (1.f - h * h);
                        break;
                    }
                    default: break;
                }
                C[(size_t)m * ldc + n] = x;
                csum += x;
            }
        }
        if (colsum != nullptr) {
            csum += __shfl_xor(csum, 32);
            if (half == 0 && n_ok) colsum[(size_t)(tile_m * WAVES_M + wm) * N + n] = csum;
        }
    }
}

// ---- host side ------------------------------------------------------------------------------
int gemm_tile_m(int tile) { return tile == TILE_64x64 ? 64 : 128; }
int gemm_tile_n(int tile) { return tile == TILE_128x128 ? 128 : (tile == TILE_128x32 ? 32 : 64); }
int gemm_waves_m(int tile) { return tile == TILE_128x32 ? 4 : 2; }

// =============================================================================================
// Weight gradients of small layers, dW[M x N] = A^T B over a range of batch rows (the K dimension),
// 64 x 64 output tile per workgroup.  Both operands are row-major activations [rows x ld] whose
// contiguous dimension is the MFMA's M resp. N dimension, so the lanes of a wavefront can take
// their A and B fragments straight from memory (coalesced 128-byte row pieces through buffer
// descriptors: a scalar row offset plus one lane offset, rows past the range read as zero): no LDS
// staging and no barrier inside the loop.  The four wavefronts of a workgroup each take a quarter
// of the split's rows of the same tile (rows in chunks of 8, the next chunk requested while the
// current one feeds the matrix core); the partial tiles meet in LDS at the end.
// TM = 32-row tiles of the output per wavefront (1 for outputs of at most 32 rows).
// =============================================================================================
__device__ inline float tn_load(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
}

constexpr int TNS = 4;            // MFMA steps (2 rows each) per chunk of the streaming weight-gradient kernel

// Quarter Q of a wavefront's TM x 2 accumulator tiles: registers f in [Q * NQ, (Q + 1) * NQ), NQ = TM * 8.
template <int TM, int Q>
__device__ inline void tn_park(const floatx16 (&acc)[TM][2], float (*red)[4096], int lane) {
    constexpr int NQ = TM * 8;
#pragma unroll
    for (int f = 0; f < TM * 32; ++f) {
        const int q = f / NQ;                       // owner of this register (a constant after unrolling)
        if (q != Q) red[Q - (Q > q ? 1 : 0)][f * 64 + lane] = acc[f >> 5][(f >> 4) & 1][f & 15];
    }
}

template <int TM, int Q>
__device__ inline void tn_sum_store(const floatx16 (&acc)[TM][2], float (*red)[4096], int lane, int l32, int half,
                                    float* __restrict__ C, int M, int N, int ldc, int m0, int n0) {
    constexpr int NQ = TM * 8;
#pragma unroll
    for (int f = Q * NQ; f < (Q + 1) * NQ; ++f) {
        const int i = f >> 5, j = (f >> 4) & 1, r = f & 15;
        const int e = f * 64 + lane;
        float v = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) {               // contributions in wavefront order, whoever owns the register
            const float x = (s == Q) ? acc[i][j][r] : red[s - (s > Q ? 1 : 0)][e];
            v = (s == 0) ? x : v + x;
        }
        const int row = m0 + 32 * i + 8 * (r >> 2) + 4 * half + (r & 3);
        const int col = n0 + 32 * j + l32;
        if (row < M && col < N) C[(size_t)row * (size_t)ldc + col] = v;
    }
}

template <int TM>
__device__ inline void tn_stream_tile(const GemmProb& P, int split, int m0, int n0, float (*red)[4096]) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int K = P.seg[0].K, lda = P.seg[0].lda, ldb = P.seg[0].ldb;
    const int kb = split * P.k_chunk, ke = min(K, kb + P.k_chunk);
    const int kq = (((ke - kb + 3) >> 2) + 2 * TNS - 1) / (2 * TNS) * (2 * TNS);     // rows per wavefront, whole chunks
    const int k0 = kb + wave * kq, k1 = min(ke, k0 + kq);
    const int nch = k1 > k0 ? (k1 - k0 + 2 * TNS - 1) / (2 * TNS) : 0;
    // descriptors start at this wavefront's first row (64-bit address arithmetic; inside them 32-bit byte
    // offsets suffice) and end at its last one: the rows of a short last chunk read as zero
    const int nrows = k1 > k0 ? k1 - k0 : 0;
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(P.seg[0].A) + (size_t)k0 * (size_t)lda, 0, nrows * lda * (int)sizeof(float), 0x00020000);
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(P.seg[0].B) + (size_t)k0 * (size_t)ldb, 0, nrows * ldb * (int)sizeof(float), 0x00020000);
    // lane (l32, half) holds column l32 of row 2s + half of every step s; columns past the matrix
    // read neighbouring (finite) activations or zero and only reach output elements that are not stored
    int va[TM], vb[2];
#pragma unroll
    for (int i = 0; i < TM; ++i) va[i] = (half * lda + m0 + 32 * i + l32) * (int)sizeof(float);
#pragma unroll
    for (int j = 0; j < 2; ++j) vb[j] = (half * ldb + n0 + 32 * j + l32) * (int)sizeof(float);
    floatx16 acc[TM][2];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    float a0[TM][TNS], b0[2][TNS], a1[TM][TNS], b1[2][TNS];
    auto load = [&](int c, float (&a)[TM][TNS], float (&b)[2][TNS]) {
        const int row = 2 * TNS * (c < nch ? c : 0);          // relative to the wavefront's first row
#pragma unroll
        for (int st = 0; st < TNS; ++st) {
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i][st] = tn_load(ra, va[i], (row + 2 * st) * lda * (int)sizeof(float));
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j][st] = tn_load(rb, vb[j], (row + 2 * st) * ldb * (int)sizeof(float));
        }
    };
    auto mac = [&](const float (&a)[TM][TNS], const float (&b)[2][TNS]) {
#pragma unroll
        for (int st = 0; st < TNS; ++st)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][st], b[j][st], acc[i][j], 0, 0, 0);
    };
    if (nch > 0) {
        load(0, a0, b0);
        int left = nch, c = 0;
        // the fences keep the next chunk's requests ahead of the current chunk's MFMAs
        while (true) {
            load(c + 1, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            mac(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            if (--left == 0) break;
            ++c;
            load(c + 1, a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            mac(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            if (--left == 0) break;
            ++c;
        }
    }
    // The four partial tiles meet in LDS.  Every wavefront owns a quarter of the tile's accumulator registers
    // (flattened as f = (i * 2 + j) * 16 + r): it parks the other three quarters in LDS (slot = source wavefront,
    // skipping the owner: three slots of 64 x 64 floats), then adds the four contributions to its own quarter
    // in wavefront order and stores that part of the split's slab - all four wavefronts reduce and store.
    if (wave == 0)      tn_park<TM, 0>(acc, red, lane);
    else if (wave == 1) tn_park<TM, 1>(acc, red, lane);
    else if (wave == 2) tn_park<TM, 2>(acc, red, lane);
    else                tn_park<TM, 3>(acc, red, lane);
    __syncthreads();
    float* __restrict__ C = P.C + (size_t)split * (size_t)P.split_stride;
    if (wave == 0)      tn_sum_store<TM, 0>(acc, red, lane, l32, half, C, P.M, P.N, P.ldc, m0, n0);
    else if (wave == 1) tn_sum_store<TM, 1>(acc, red, lane, l32, half, C, P.M, P.N, P.ldc, m0, n0);
    else if (wave == 2) tn_sum_store<TM, 2>(acc, red, lane, l32, half, C, P.M, P.N, P.ldc, m0, n0);
    else                tn_sum_store<TM, 3>(acc, red, lane, l32, half, C, P.M, P.N, P.ldc, m0, n0);
}

__global__ __launch_bounds__(NTHREADS, 3) void gemm_tn_stream_kernel(const GemmGroup g) {
    __shared__ float red[3][4096];
    const int bid = xcd_remap(blockIdx.x, gridDim.x);
    int pi = 0;
    for (int i = 1; i < g.nprob; ++i)
        if (bid >= g.p[i].tile_begin) pi = i;
    const GemmProb& P = g.p[pi];
    int local = bid - P.tile_begin;
    const int per_split = P.tiles_m * P.tiles_n;
    const int split = local / per_split;
    local -= split * per_split;
    const int tile_m = local / P.tiles_n, tile_n = local % P.tiles_n;
    const int m0 = tile_m * 64, n0 = tile_n * 64;
    if (P.M - m0 <= 32) tn_stream_tile<1>(P, split, m0, n0, red);
    else                tn_stream_tile<2>(P, split, m0, n0, red);
}

template <int MODE>
static hipError_t launch_mode(int tile, const GemmGroup& g, bool noise, const ProfSlot& ps, hipStream_t stream) {
    const dim3 grid(g.total_tiles), block(NTHREADS);
    switch (tile) {
        case TILE_128x128: PQL_LAUNCH(ps, (gemm_grouped_kernel<MODE, 2, 2, 2, 2, false>), grid, block, 0, stream, g); break;
        case TILE_64x64:   PQL_LAUNCH(ps, (gemm_grouped_kernel<MODE, 2, 2, 1, 1, false>), grid, block, 0, stream, g); break;
        case TILE_128x64:  PQL_LAUNCH(ps, (gemm_grouped_kernel<MODE, 2, 2, 2, 1, false>), grid, block, 0, stream, g); break;
        default:
            if (MODE == GEMM_NN && noise)
                PQL_LAUNCH(ps, (gemm_grouped_kernel<GEMM_NN, 4, 1, 1, 1, true>), grid, block, 0, stream, g);
            else
                PQL_LAUNCH(ps, (gemm_grouped_kernel<MODE, 4, 1, 1, 1, false>), grid, block, 0, stream, g);
            break;
    }
    return hipGetLastError();
}

hipError_t gemm_launch(int mode, int tile, GemmGroup& g, hipStream_t stream) {
    const int bm = gemm_tile_m(tile), bn = gemm_tile_n(tile);
    int total = 0;
    bool noise = false;
    for (int i = 0; i < g.nprob; ++i) {
        GemmProb& p = g.p[i];
        if (p.epi == EPI_BIAS_TANH_NOISE) noise = true;
        p.tiles_m = (p.M + bm - 1) / bm;
        p.tiles_n = (p.N + bn - 1) / bn;
        if (mode != GEMM_TN) { p.splits = 1; p.k_chunk = 0; }
        p.tile_begin = total;
        total += p.tiles_m * p.tiles_n * p.splits;
    }
    g.total_tiles = total;
    if (total == 0) return hipSuccess;
    if (noise && (mode != GEMM_NN || tile != TILE_128x32)) return hipErrorInvalidValue;
    double flops = 0.0;
    const ProfSlot ps = prof_slot();
    if (ps.on)
        for (int i = 0; i < g.nprob; ++i)
            for (int s = 0; s < g.p[i].nseg; ++s) flops += 2.0 * g.p[i].M * (double)g.p[i].N * g.p[i].seg[s].K;
    hipError_t e;
    switch (mode) {
        case GEMM_NN: e = launch_mode<GEMM_NN>(tile, g, noise, ps, stream); break;
        case GEMM_NT: e = launch_mode<GEMM_NT>(tile, g, noise, ps, stream); break;
        default:      // weight gradients: always the streaming kernel on 64x64 output tiles
            if (tile != TILE_64x64) return hipErrorInvalidValue;
            PQL_LAUNCH(ps, gemm_tn_stream_kernel, dim3(g.total_tiles), dim3(NTHREADS), 0, stream, g);
            e = hipGetLastError();
            break;
    }
    prof_commit(ps, KID_GEMM + mode * 5 + (noise ? 4 : tile), flops, 0.0);
    return e;
}

// ---- achievable matrix-core rate ---------------------------------------------------------------
// Every wavefront issues `iters` rounds of four independent v_mfma_f32_32x32x2_f32 on register
// operands (no memory, no LDS): the rate the matrix cores sustain at the clock the chip holds
// under that load.  Results are stored so that the work cannot be optimised away.
__global__ __launch_bounds__(256) void mfma_probe_kernel(float* __restrict__ out, int iters) {
    floatx16 c0, c1, c2, c3;
#pragma unroll
    for (int r = 0; r < 16; ++r) { c0[r] = 0.f; c1[r] = 0.f; c2[r] = 0.f; c3[r] = 0.f; }
    float a = 1e-3f * (float)(threadIdx.x & 7), b = 1e-3f * (float)(blockIdx.x & 3);
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, a, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, a, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

hipError_t mfma_probe_launch(float* out, int blocks, int iters, hipStream_t stream) {
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, mfma_probe_kernel, dim3(blocks), dim3(256), 0, stream, out, iters);
    prof_commit(ps, KID_MFMA_PROBE, 2.0 * 32 * 32 * 2 * 4.0 * (double)iters * 4.0 * (double)blocks, 0.0);
    return hipGetLastError();
}

}  // namespace pql
