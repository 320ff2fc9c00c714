// Actor step on 16-row tiles (Section 3.3, Algorithm 1): a = clip(pi(s) + sigma_i * eps, -1, 1).
//
// The 32-row kernel (fused_act_kernel) gives 4096 environments 128 workgroups: half of the 256 compute
// units idle, and the launch lasts as long as one workgroup needs for its tile.  Here a workgroup owns
// 16 rows, so the same environments make 256 workgroups with half the matrix work each.  The products run
// on v_mfma_f32_16x16x4_f32: each of the eight wavefronts owns 32 output columns as two 16-column tiles
// (a lane's two columns are adjacent, so its weights come as one 8-byte load per k-value), the 16 input
// rows sit in LDS, the weights stream from L2 through buffer descriptors with the row offset in the
// lane's own offset register, so that rows past the matrix (the zero padding of a short last chunk) are
// range-checked and read as zero.  Used for deterministic policies with every hidden layer a multiple of
// 32 and at most 256 wide, up to 4096 environments.
#include "pql_rowtile.h"

namespace pql {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int R16 = 16;                       // rows per workgroup
constexpr int ACT16_SCRATCH = FW * 2 * 4 * 64; // floats: one 16 x 32 partial tile per wavefront

struct Lanes16 { int tid, lane, wave, c16, kq; };

__device__ inline float2 buf_load2(__amdgpu_buffer_rsrc_t r, unsigned voff) {
    typedef unsigned int u2 __attribute__((vector_size(8)));
    const u2 v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, 0, 0);
    return make_float2(__uint_as_float(v[0]), __uint_as_float(v[1]));
}

__host__ __device__ inline int act16_pad32(int n) { return ((n + 31) & ~31) + 4; }

size_t act16_lds_bytes(int o, int hmax) {
    return sizeof(float) * ((size_t)R16 * act16_pad32(o) + 2 * (size_t)R16 * (hmax + 4) + ACT16_SCRATCH);
}

// Weights of chunk c (32 k-values) for this lane's two columns: k = 32 c + 16 g + 4 kq + i sits in b[4 g + i].
__device__ inline void act16_load(__amdgpu_buffer_rsrc_t r, unsigned lane_off, int row_bytes, int c, float2 (&b)[8]) {
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) b[g * 4 + i] = buf_load2(r, lane_off + (unsigned)((c * 32 + g * 16 + i) * row_bytes));
}

// acc[t] += in[16 x chunk c] * b: the A operand is one 16-byte LDS read per group of 16 k-values (the lane
// holds row c16, k-values 4 kq .. 4 kq + 3 of the group).
__device__ inline void act16_mac(floatx4 (&acc)[2], int in, int ld, const Lanes16& T, int c, const float2 (&b)[8]) {
    const float4* s4 = reinterpret_cast<const float4*>(smem);
#pragma unroll
    for (int g = 0; g < 2; ++g) {
        const float4 a = s4[((in + T.c16 * ld) >> 2) + c * 8 + g * 4 + T.kq];
        const float av[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], b[g * 4 + i].x, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], b[g * 4 + i].y, acc[1], 0, 0, 0);
        }
    }
}

// out[16 x N] = ELU(in[16 x K] W + bias), N a multiple of 32 and at most 256: wavefront w takes columns
// 32 w .. 32 w + 31.  The input tile is zero beyond column K up to the next multiple of 32.
__device__ inline void act16_layer(const Lanes16& T, int in, int ld, int K, const float* __restrict__ W, int N,
                                   const float* __restrict__ bias, int out, int ldo) {
    const int n0 = T.wave * 32;
    if (n0 >= N) return;
    const int ncol = n0 + 2 * T.c16;
    const __amdgpu_buffer_rsrc_t r =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(W), 0, K * N * (int)sizeof(float), 0x00020000);
    const int row_bytes = N * (int)sizeof(float);
    const unsigned lane_off = (unsigned)((4 * T.kq) * N + ncol) * (unsigned)sizeof(float);
    const float2 bv = *reinterpret_cast<const float2*>(bias + ncol);
    const int nch = (K + 31) >> 5;
    floatx4 acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
    float2 b0[8], b1[8];
    act16_load(r, lane_off, row_bytes, 0, b0);
    for (int c = 0; c < nch; c += 2) {
        if (c + 1 < nch) act16_load(r, lane_off, row_bytes, c + 1, b1);
        __builtin_amdgcn_sched_barrier(0);
        act16_mac(acc, in, ld, T, c, b0);
        __builtin_amdgcn_sched_barrier(0);
        if (c + 1 >= nch) break;
        if (c + 2 < nch) act16_load(r, lane_off, row_bytes, c + 2, b0);
        __builtin_amdgcn_sched_barrier(0);
        act16_mac(acc, in, ld, T, c + 1, b1);
        __builtin_amdgcn_sched_barrier(0);
    }
    // the lane holds rows 4 kq + rr, columns ncol (tile 0) and ncol + 1 (tile 1)
    float2* s2 = reinterpret_cast<float2*>(smem);
#pragma unroll
    for (int rr = 0; rr < 4; ++rr)
        s2[(out + (4 * T.kq + rr) * ldo + ncol) >> 1] = make_float2(elu_f(acc[0][rr] + bv.x), elu_f(acc[1][rr] + bv.y));
}

__global__ __launch_bounds__(FT) void fused_act16_kernel(const FusedActArgs A) {
    Lanes16 T;
    T.tid = threadIdx.x; T.lane = T.tid & 63; T.wave = __builtin_amdgcn_readfirstlane(T.tid >> 6); T.c16 = T.lane & 15; T.kq = T.lane >> 4;
    const int o = A.o, a = A.a, L = A.L, B = A.B;
    const int r0 = blockIdx.x * R16;
    const int SX = act16_pad32(o), SH = A.hmax + 4;
    const int XA = 0, H0 = R16 * SX, scratch = H0 + 2 * R16 * SH;
    // input rows, standardised on the way when asked for; zero beyond column o and for rows beyond the batch
    for (int i = T.tid; i < R16 * (SX - 4); i += FT) {
        const int row = i / (SX - 4), col = i - row * (SX - 4);
        float v = 0.f;
        if (col < o && r0 + row < B) {
            v = A.obs[(size_t)(r0 + row) * (size_t)o + col];
            if (A.nmean != nullptr) v = (v - A.nmean[col]) * A.nrstd[col];
        }
        smem[XA + row * SX + col] = v;
    }
    __syncthreads();
    int cur = 0;
    for (int l = 0; l < L; ++l) {
        const int N = A.H[l];
        const int dst = l == 0 ? 0 : (cur ^ 1);
        if (l == 0) act16_layer(T, XA, SX, o, A.pi.w[0], N, A.pi.b[0], H0 + dst * R16 * SH, SH);
        else        act16_layer(T, H0 + cur * R16 * SH, SH, A.H[l - 1], A.pi.w[l], N, A.pi.b[l], H0 + dst * R16 * SH, SH);
        cur = dst;
        __syncthreads();
    }
    {
        // output layer (at most 32 columns): the contraction is split over the wavefronts, every eighth chunk of
        // 32 k-values each; a lane's columns are c16 (tile 0) and 16 + c16 (tile 1), clamped into the matrix
        const int HL = A.H[L - 1], in = H0 + cur * R16 * SH;
        const float* __restrict__ W = A.pi.w[L];
        const int col0 = T.c16 < a ? T.c16 : a - 1, col1 = 16 + T.c16 < a ? 16 + T.c16 : a - 1;
        floatx4 acc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        const float4* s4 = reinterpret_cast<const float4*>(smem);
        for (int c = T.wave; c < (HL >> 5); c += FW) {
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const float4 av4 = s4[((in + T.c16 * SH) >> 2) + c * 8 + g * 4 + T.kq];
                const float av[4] = {av4.x, av4.y, av4.z, av4.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int k = c * 32 + g * 16 + 4 * T.kq + i;      // < HL: the widths are multiples of 32
                    acc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], W[(size_t)k * a + col0], acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], W[(size_t)k * a + col1], acc[1], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) smem[scratch + ((T.wave * 2 + t) * 4 + rr) * 64 + T.lane] = acc[t][rr];
    }
    __syncthreads();
    {
        // one output element per thread: row = tid / 32, column = tid % 32
        const int row = T.tid >> 5, col = T.tid & 31;
        const int t = col >> 4, lane = (row >> 2) * 16 + (col & 15), rr = row & 3;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < FW; ++w) s += smem[scratch + ((w * 2 + t) * 4 + rr) * 64 + lane];
        const int env = r0 + row;
        if (col < a && env < B) {
            const GemmNoise& nz = A.noise;
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

// Whether the 16-row kernel takes this Actor step (the caller has checked that the row-tile kernels apply at all).
bool act16_ok(const FusedActArgs& a) {
    if (a.sac.on || a.B < 1 || a.B > 256 * R16 || a.a < 1 || a.a > 32 || a.hmax > 256) return false;
    for (int l = 0; l < a.L; ++l)
        if (a.H[l] % 32 != 0 || a.H[l] > 256) return false;
    for (int l = 0; l <= a.L; ++l)                      // 8-byte loads of the lane's two weights and biases
        if ((reinterpret_cast<uintptr_t>(a.pi.w[l]) & 7) != 0 || (reinterpret_cast<uintptr_t>(a.pi.b[l]) & 7) != 0) return false;
    return act16_lds_bytes(a.o, a.hmax) <= 64 * 1024;
}

hipError_t fused_act16_launch(const FusedActArgs& a, hipStream_t stream) {
    if (!act16_ok(a)) return hipErrorInvalidValue;
    const size_t lds = act16_lds_bytes(a.o, a.hmax);
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, fused_act16_kernel, dim3((a.B + R16 - 1) / R16), dim3(FT), lds, stream, a);
    double flops = 0.0;
    if (ps.on) {
        double pa = (double)a.o * a.H[0];
        for (int l = 1; l < a.L; ++l) pa += (double)a.H[l - 1] * a.H[l];
        pa += (double)a.H[a.L - 1] * a.a;
        flops = 2.0 * a.B * pa;
    }
    prof_commit(ps, KID_FUSED_ACT16, flops, 0.0);
    return hipGetLastError();
}

}  // namespace pql
