// Building blocks of the row-tile kernels (pql_fused.hip, pql_chain.hip): a workgroup of eight
// wavefronts owns 32 batch rows whose activations live in LDS; the weights are streamed from L2
// into registers as the B operand of v_mfma_f32_32x32x2_f32 (each wavefront owns 32 output
// columns; lanes run along W's contiguous output dimension).  Device code only; each translation
// unit that includes this header has its own dynamic LDS array `smem`.
#pragma once

#include "pql_internal.h"

namespace pql {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int FW = 8;                // wavefronts per workgroup
constexpr int FT = 64 * FW;          // threads per workgroup
constexpr int BMF = FUSED_BM;        // rows per workgroup (32)
constexpr int SCRATCH_F = FW * 1024; // floats of LDS scratch (one 32x32 partial tile per wavefront)

struct Lanes { int tid, lane, wave, l32, half; };

// The row tile's LDS.  Tiles are addressed as offsets (in floats) into this array rather than
// through pointers, so that every access is compiled as an LDS instruction (a generic pointer
// would turn them into flat memory operations that also wait on the global-load counter).
extern __shared__ __attribute__((aligned(16))) float smem[];

__device__ inline float elu_f(float x) { return x > 0.f ? x : __expf(x) - 1.f; }
__device__ inline float delu_h(float h) { return h > 0.f ? 1.f : h + 1.f; }   // ELU'(z) from h = ELU(z)
// Reductions over the 64 lanes of a wavefront, result in every lane; all lanes must be active.
// Data-parallel-primitive moves inside each row of 16 lanes (xor 1, xor 2, mirrored half row,
// mirrored row: after them every lane holds its row's result), then the four rows meet through
// scalar lane reads.  No LDS traffic, unlike the shuffle-based butterfly.
template <int CTRL>
__device__ inline float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
__device__ inline float lane_value(float x, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), lane));
}
__device__ inline float wsum(float x) {
    x += dpp_move<0xB1>(x);      // quad_perm [1, 0, 3, 2]
    x += dpp_move<0x4E>(x);      // quad_perm [2, 3, 0, 1]
    x += dpp_move<0x141>(x);     // row_half_mirror
    x += dpp_move<0x140>(x);     // row_mirror
    return (lane_value(x, 0) + lane_value(x, 16)) + (lane_value(x, 32) + lane_value(x, 48));
}
__device__ inline int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// Where a lane finds its B fragments (weights) of one contraction segment: W are row-major in
// memory with leading dimension ldw and K rows, the lane owns output column ncol.  The contraction
// runs in chunks of 32 k-values: nfull whole ones and, when K is no multiple of 32, a shorter tail.
// A wavefront that takes every c_step-th chunk starting at c_begin (c_step > 1 splits the
// contraction across wavefronts) first does the tail, if it is among its chunks, and then its whole
// chunks in one branch-free loop.  Every workgroup of the launch streams the same weight matrix;
// starting each workgroup at a different whole chunk (rot) spreads the simultaneous requests over
// the L2 channels instead of piling all compute units onto the same few cache lines.
// The weights are read through buffer descriptors: one vector register holds the lane's byte offset
// for every load of the segment, the row comes as a scalar offset (plain pointers cost a 64-bit
// vector address per load in flight, 60 registers for two networks), and a read outside the
// matrix returns zero instead of faulting.
template <int NN>
struct ChunkSrc {
    __amdgpu_buffer_rsrc_t r[NN];
    int K, ldw, ncol, nch, nfull, rot;
    int half4;              // 4 * (lane >> 5): the lane's first row inside a group of 8
    unsigned voff;          // byte offset of (row half4, column ncol)
    bool tail_mine;         // the short last chunk belongs to this wavefront
    int n_mine;             // whole chunks of this wavefront
};

template <int NN>
__device__ inline ChunkSrc<NN> chunk_src(const float* const (&W)[NN], int K, int ldw, int ncol, const Lanes& T,
                                         int c_begin, int c_step) {
    ChunkSrc<NN> s;
#pragma unroll
    for (int n = 0; n < NN; ++n)
        s.r[n] = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(W[n]), 0, K * ldw * (int)sizeof(float), 0x00020000);
    s.K = K; s.ldw = ldw; s.ncol = ncol;
    s.nch = (K + 31) >> 5;
    s.nfull = K >> 5;
    s.rot = s.nfull > 0 ? (int)(blockIdx.x % (unsigned)s.nfull) : 0;
    s.half4 = 4 * T.half;
    s.voff = (unsigned)(s.half4 * ldw + ncol) * (unsigned)sizeof(float);
    s.tail_mine = s.nch > s.nfull && s.nch - 1 >= c_begin && (s.nch - 1 - c_begin) % c_step == 0;
    s.n_mine = s.nfull > c_begin ? (s.nfull - c_begin + c_step - 1) / c_step : 0;
    return s;
}

__device__ inline float buf_load(__amdgpu_buffer_rsrc_t r, unsigned voff, int soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, soff, 0));
}

// The memory chunk behind whole chunk number ci of the wavefront's order.
template <int NN>
__device__ inline int rotated(const ChunkSrc<NN>& s, int ci) {
    const int cc = ci + s.rot;
    return cc >= s.nfull ? cc - s.nfull : cc;
}

// Weights of whole chunk ci (clamped to a valid one) into b: 16 loads per network, always.
template <int NN>
__device__ inline void load_full(const ChunkSrc<NN>& s, int ci, float (&b)[NN][16]) {
    const int cc = rotated(s, ci < s.nfull ? ci : 0);
    const int row_bytes = s.ldw * (int)sizeof(float);
    const int base = cc * 32 * row_bytes;
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int n = 0; n < NN; ++n) b[n][g * 4 + u] = buf_load(s.r[n], s.voff, base + (g * 8 + u) * row_bytes);
}

// Weights of the short last chunk: row indices are clamped to K - 1 (clamped rows meet zero columns
// of the input tile, whose width is padded with zeros to a multiple of 8).
template <int NN>
__device__ inline void load_tail(const ChunkSrc<NN>& s, float (&b)[NN][16]) {
    const int kbase = s.nfull * 32;
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int k = kbase + g * 8 + s.half4 + u;
            k = k < s.K ? k : s.K - 1;
            const unsigned off = (unsigned)(k * s.ldw + s.ncol) * (unsigned)sizeof(float);
#pragma unroll
            for (int n = 0; n < NN; ++n) b[n][g * 4 + u] = buf_load(s.r[n], off, 0);
        }
}

// acc[n] += in[n][32 rows x memory chunk cc] * b[n]: 16 MFMAs per network, no branches.  `in` are
// LDS tiles with row stride ld.  A operand: one 16-byte LDS read per group of 8 k-values (tile
// offsets and strides are multiples of 4 floats; indexing the array as float4 lets the compiler
// prove the alignment and emit ds_read_b128, which the stride-(width + 4) layout serves without
// bank conflicts).
template <int NN>
__device__ inline void mac_full(floatx16 (&acc)[NN], const int (&in)[NN], int ld,
                                const Lanes& T, int cc, const float (&b)[NN][16]) {
    const float4* smem4 = reinterpret_cast<const float4*>(smem);
    const int a_off4 = T.l32 * (ld >> 2) + T.half + cc * 8;
    float4 a[4][NN];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int n = 0; n < NN; ++n) a[g][n] = smem4[(in[n] >> 2) + a_off4 + g * 2];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int n = 0; n < NN; ++n) {
            acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g][n].x, b[n][g * 4 + 0], acc[n], 0, 0, 0);
            acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g][n].y, b[n][g * 4 + 1], acc[n], 0, 0, 0);
            acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g][n].z, b[n][g * 4 + 2], acc[n], 0, 0, 0);
            acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g][n].w, b[n][g * 4 + 3], acc[n], 0, 0, 0);
        }
    // Issue order: two LDS reads ahead, then four MFMAs per read (0x100 = LDS read, 0x008 = MFMA).
    // Left alone, the scheduler places every read directly before its first use.
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
    for (int i = 0; i < 4 * NN - 2; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
}

// The short last chunk: only the groups of 8 k-values that exist.
template <int NN>
__device__ inline void mac_tail(floatx16 (&acc)[NN], const int (&in)[NN], int ld,
                                const ChunkSrc<NN>& s, const Lanes& T, const float (&b)[NN][16]) {
    const float4* smem4 = reinterpret_cast<const float4*>(smem);
    const int a_off4 = T.l32 * (ld >> 2) + T.half + s.nfull * 8;
    const int ng = (s.K - s.nfull * 32 + 7) >> 3;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        if (g < ng) {
#pragma unroll
            for (int n = 0; n < NN; ++n) {
                const float4 a = smem4[(in[n] >> 2) + a_off4 + g * 2];
                acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b[n][g * 4 + 0], acc[n], 0, 0, 0);
                acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b[n][g * 4 + 1], acc[n], 0, 0, 0);
                acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b[n][g * 4 + 2], acc[n], 0, 0, 0);
                acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b[n][g * 4 + 3], acc[n], 0, 0, 0);
            }
        }
    }
}

// Requests the first chunk a later mac_segment() call with the same (W, K, ldw, ncol, c_begin,
// c_step) and use_pre = true consumes: the tail if it is the wavefront's, else its first whole chunk.
template <int NN>
__device__ inline void prefetch_first_chunk(float (&pre)[NN][16], const float* const (&W)[NN], int K, int ldw, int ncol,
                                            const Lanes& T, int c_begin, int c_step) {
    const ChunkSrc<NN> s = chunk_src<NN>(W, K, ldw, ncol, T, c_begin, c_step);
    if (s.tail_mine) load_tail<NN>(s, pre);
    else if (s.n_mine > 0) load_full<NN>(s, c_begin, pre);
}

// acc[n] += in[n][32 x K] * W[n][K x .] for NN networks at once, for the output column `ncol`
// of this lane.  The weights of the next chunk are loaded while the current one feeds the matrix
// core.  With use_pre, `pre` holds the first chunk already (prefetch_first_chunk(): its latency is
// then not paid here); a flag and a reference rather than a nullable pointer, which would keep the
// buffer in private memory.
template <int NN>
__device__ inline void mac_segment(floatx16 (&acc)[NN], const int (&in)[NN], int ld,
                                   int K, const float* const (&W)[NN], int ldw, int ncol, const Lanes& T, int c_begin,
                                   int c_step, bool use_pre, const float (&pre)[NN][16]) {
    const ChunkSrc<NN> s = chunk_src<NN>(W, K, ldw, ncol, T, c_begin, c_step);
    if (!s.tail_mine && s.n_mine == 0) return;
    float b0[NN][16], b1[NN][16];
    if (use_pre) {
#pragma unroll
        for (int n = 0; n < NN; ++n)
#pragma unroll
            for (int u = 0; u < 16; ++u) b0[n][u] = pre[n][u];
    } else if (s.tail_mine) {
        load_tail<NN>(s, b0);
    } else {
        load_full<NN>(s, c_begin, b0);
    }
    if (s.tail_mine) {
        if (s.n_mine > 0) load_full<NN>(s, c_begin, b1);
        mac_tail<NN>(acc, in, ld, s, T, b0);
        if (s.n_mine == 0) return;
#pragma unroll
        for (int n = 0; n < NN; ++n)
#pragma unroll
            for (int u = 0; u < 16; ++u) b0[n][u] = b1[n][u];
    }
    int c = c_begin, left = s.n_mine;
    // The fences keep the requests for the next chunk ahead of the MFMAs of the current one (the
    // scheduler otherwise sinks them to their first use to save registers, exposing their latency).
    while (true) {                       // b0 holds whole chunk c
        load_full<NN>(s, left > 1 ? c + c_step : c, b1);       // (a repeat at the end keeps the counters uniform)
        __builtin_amdgcn_sched_barrier(0);
        mac_full<NN>(acc, in, ld, T, rotated(s, c), b0);
        __builtin_amdgcn_sched_barrier(0);
        if (--left == 0) break;
        c += c_step;
        load_full<NN>(s, left > 1 ? c + c_step : c, b0);
        __builtin_amdgcn_sched_barrier(0);
        mac_full<NN>(acc, in, ld, T, rotated(s, c), b1);
        __builtin_amdgcn_sched_barrier(0);
        if (--left == 0) break;
        c += c_step;
    }
}

template <int NN>
__device__ inline void mac_segment(floatx16 (&acc)[NN], const int (&in)[NN], int ld,
                                   int K, const float* const (&W)[NN], int ldw, int ncol, const Lanes& T, int c_begin,
                                   int c_step) {
    float none[NN][16];
#pragma unroll
    for (int n = 0; n < NN; ++n)
#pragma unroll
        for (int u = 0; u < 16; ++u) none[n][u] = 0.f;
    mac_segment<NN>(acc, in, ld, K, W, ldw, ncol, T, c_begin, c_step, false, none);
}

enum WideEpi : int { WIDE_BIAS_ELU = 0, WIDE_MUL_DELU = 1 };

// One layer for NN networks of equal shape (the twin critics run as a pair).
template <int NN>
struct WideArgs {
    int in0[NN]; const float* W0[NN]; int ld0, K0;               // first input segment (LDS offset)
    int in1[NN]; const float* W1[NN]; int ld1, K1;               // optional second segment (K1 = 0: none)
    int ldw, N;
    const float* bias[NN];                                       // WIDE_BIAS_ELU
    int aux[NN]; int ldaux;                                      // WIDE_MUL_DELU: LDS tile of activations (offset)
    int outL[NN]; int ldo;                                       // LDS output tile (offset; may be aux, never an input)
    float* outG[NN]; int ldg;                                    // optional copy in memory
    float* colsum[NN];                                           // optional column sums over the tile's rows
    int epi;
};

// out[32 x N] (N <= 256, one 32-column tile per wavefront).  WIDE_BIAS_ELU: out = ELU(acc + bias).
// WIDE_MUL_DELU: out = acc * ELU'(.) with the activation taken from the LDS tile `aux`.  Rows
// beyond the batch are written as zero.
template <int NN, bool PRE2 = true>
__device__ inline void wide_linear(const Lanes& T, const WideArgs<NN>& w, int r0, int B) {
    const int n0 = T.wave * 32, N = w.N;
    if (n0 >= N) return;
    const int n = n0 + T.l32;
    const bool n_ok = n < N;
    const int ncol = n_ok ? n : N - 1;
    float bv[NN];
#pragma unroll
    for (int i = 0; i < NN; ++i) bv[i] = (w.epi == WIDE_BIAS_ELU) ? w.bias[i][ncol] : 0.f;   // in flight during the MFMAs
    floatx16 acc[NN];
#pragma unroll
    for (int i = 0; i < NN; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    if (w.K1 > 0 && !PRE2) {
        // two segments one after the other (for callers without the registers to hold both first chunks)
        mac_segment<NN>(acc, w.in1, w.ld1, w.K1, w.W1, w.ldw, ncol, T, 0, 1);
        mac_segment<NN>(acc, w.in0, w.ld0, w.K0, w.W0, w.ldw, ncol, T, 0, 1);
    } else if (w.K1 > 0) {
        // two segments (a critic's first layer: state columns, then action columns): the first chunks
        // of both are requested together, and the short segment runs while the long one's arrives
        float bs[NN][16], bf[NN][16];
        prefetch_first_chunk<NN>(bs, w.W1, w.K1, w.ldw, ncol, T, 0, 1);
        prefetch_first_chunk<NN>(bf, w.W0, w.K0, w.ldw, ncol, T, 0, 1);
        mac_segment<NN>(acc, w.in1, w.ld1, w.K1, w.W1, w.ldw, ncol, T, 0, 1, true, bs);
        mac_segment<NN>(acc, w.in0, w.ld0, w.K0, w.W0, w.ldw, ncol, T, 0, 1, true, bf);
    } else {
        mac_segment<NN>(acc, w.in0, w.ld0, w.K0, w.W0, w.ldw, ncol, T, 0, 1);
    }
    // Epilogue.  Row r of the accumulator sits (8 * (r / 4) + r % 4) rows below the lane's first row
    // (4 * half): offsets from per-lane bases are compile-time multiples of the strides.
    const bool full = r0 + BMF <= B;                      // uniform: every row of the tile is in the batch
    const int lrow = 4 * T.half;
#pragma unroll
    for (int i = 0; i < NN; ++i) {
        float cs = 0.f;
        const int lbase = w.outL[i] + lrow * w.ldo + n;
        const int abase = w.aux[i] + lrow * w.ldaux + ncol;
        float* __restrict__ gbase = w.outG[i] ? w.outG[i] + (size_t)(r0 + lrow) * (size_t)w.ldg + n : nullptr;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int dr = 8 * (r >> 2) + (r & 3);
            float x = acc[i][r];
            if (w.epi == WIDE_BIAS_ELU) x = elu_f(x + bv[i]);
            else x *= delu_h(smem[abase + dr * w.ldaux]);
            const bool rv = full || (r0 + lrow + dr < B);
            if (!rv) x = 0.f;
            if (n_ok) {
                smem[lbase + dr * w.ldo] = x;
                if (gbase && rv) gbase[dr * w.ldg] = x;
                cs += x;
            }
        }
        if (w.colsum[i]) {
            cs += __shfl_xor(cs, 32);
            if (T.half == 0 && n_ok) w.colsum[i][n] = cs;
        }
    }
}

// Partial products of a narrow layer (N <= 32): the contraction is split across the wavefronts,
// each leaves its 32x32 partial tile in `scratch` (accumulator layout: index r * 64 + lane).
// The caller synchronises and finishes with small_sum().
__device__ inline void small_partial(const Lanes& T, int in0, int ld0, int K0, const float* W0, int ldw, int N,
                                     int scratch) {
    floatx16 acc[1];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][r] = 0.f;
    const int ncol = T.l32 < N ? T.l32 : N - 1;
    const int ins[1] = {in0};
    const float* const ws[1] = {W0};
    mac_segment<1>(acc, ins, ld0, K0, ws, ldw, ncol, T, T.wave, FW);
#pragma unroll
    for (int r = 0; r < 16; ++r) smem[scratch + T.wave * 1024 + r * 64 + T.lane] = acc[0][r];
}

// Sum of the FW partial tiles for output element e (0..1023): returns the value and its (row, col).
__device__ inline float small_sum(int scratch, int e, int& row, int& col) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < FW; ++w) s += smem[scratch + w * 1024 + e];
    const int r = e >> 6, ln = e & 63;
    row = acc_row(r, ln >> 5);
    col = ln & 31;
    return s;
}

// Copies rows r0..r0+31 of a row-major [B][ncols] array into an LDS tile, zero-filling rows
// beyond B and the columns up to the next multiple of 8.  Four loads per thread are issued before
// the first LDS store, so a tile costs one or two memory round trips instead of one per element;
// 16-byte accesses when the row length and the base address allow it.
__device__ inline void load_rows(const Lanes& T, int dst, int stride, const float* __restrict__ src, int ncols,
                                 int r0, int B) {
    const int kp = (ncols + 7) & ~7;
    if ((ncols & 3) == 0 && (reinterpret_cast<uintptr_t>(src) & 15) == 0) {
        const int g = kp >> 2, gv = ncols >> 2;      // 16-byte granules per tile row / of them holding data
        const int total = BMF * g;
        float4* const smem4w = reinterpret_cast<float4*>(smem);
        for (int base = 0; base < total; base += 4 * FT) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + u * FT + T.tid;
                const int row = i / g, c4 = i - row * g;
                v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (i < total && c4 < gv && r0 + row < B)
                    v[u] = *reinterpret_cast<const float4*>(src + (size_t)(r0 + row) * (size_t)ncols + 4 * c4);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + u * FT + T.tid;
                const int row = i / g, c4 = i - row * g;
                if (i < total) smem4w[((dst + row * stride) >> 2) + c4] = v[u];
            }
        }
        return;
    }
    const int total = BMF * kp;
    for (int base = 0; base < total; base += 4 * FT) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = base + u * FT + T.tid;
            const int row = i / kp, col = i - row * kp;
            v[u] = 0.f;
            if (i < total && col < ncols && r0 + row < B) v[u] = src[(size_t)(r0 + row) * (size_t)ncols + col];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = base + u * FT + T.tid;
            const int row = i / kp, col = i - row * kp;
            if (i < total) smem[dst + row * stride + col] = v[u];
        }
    }
}

__device__ inline void philox4x32_10_f(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
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

}  // namespace pql
