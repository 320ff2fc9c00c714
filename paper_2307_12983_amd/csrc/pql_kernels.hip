// Bandwidth-class kernels of the learner path: replay push, index sampling + n-step gather,
// the scalar output heads of the critics (dot products, min, TD target, loss, output deltas),
// split-K reduction fused with Adam, and the Polyak target update.
#include "pql_internal.h"

namespace pql {

// =============================================================================================
// Replay push: five contiguous row copies into ring row `head` (Section 3.1 "Data Transfer";
// Algorithm 1 append / Algorithm 3 receive).
// =============================================================================================
__global__ __launch_bounds__(256) void push_kernel(const PushArgs a) {
    const int f = blockIdx.y;
    const float* __restrict__ src = a.src[f];
    float* __restrict__ dst = a.dst[f];
    const int64_t n = a.count[f];
    const bool vec = ((((uintptr_t)src) | ((uintptr_t)dst)) & 15) == 0;
    const int64_t n4 = vec ? (n >> 2) : 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = t0; i < n4; i += stride)
        reinterpret_cast<float4*>(dst)[i] = reinterpret_cast<const float4*>(src)[i];
    for (int64_t i = n4 * 4 + t0; i < n; i += stride) dst[i] = src[i];
}

hipError_t push_launch(const PushArgs& a, hipStream_t stream) {
    int64_t mx = 0;
    for (int f = 0; f < 5; ++f) mx = a.count[f] > mx ? a.count[f] : mx;
    int64_t blocks = (mx / 4 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    double bytes = 0.0;
    for (int f = 0; f < 5; ++f) bytes += 8.0 * (double)a.count[f];      // read + write
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, push_kernel, dim3((unsigned)blocks, 5), dim3(256), 0, stream, a);
    prof_commit(ps, KID_PUSH, 0.0, bytes);
    return hipGetLastError();
}

// =============================================================================================
// Index sampling + n-step gather (Section 3.1: i.i.d. batches from the GPU-resident buffer;
// Section 3: n-step returns with termination flag d).
// =============================================================================================
__device__ inline void philox4x32_10_w01(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
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

template <int G, bool VEC>
__device__ inline void copy_row(float* __restrict__ dst, const float* __restrict__ src, int n, int gl) {
    if (VEC) {
        const int n4 = n >> 2;
        for (int c = gl; c < n4; c += G) reinterpret_cast<float4*>(dst)[c] = reinterpret_cast<const float4*>(src)[c];
    } else {
        for (int c = gl; c < n; c += G) dst[c] = src[c];
    }
}

// Row copy with the standardisation (x - mu[c]) * rs[c] applied on the way (Table B.1
// "Normalized Observations": the ring keeps raw observations, batches are standardised with the
// statistics current at sampling time).
template <int G, bool VEC>
__device__ inline void copy_row_std(float* __restrict__ dst, const float* __restrict__ src, int n, int gl,
                                    const float* __restrict__ mu, const float* __restrict__ rs) {
    if (VEC) {
        const int n4 = n >> 2;
        for (int c = gl; c < n4; c += G) {
            float4 v = reinterpret_cast<const float4*>(src)[c];
            const float4 m = reinterpret_cast<const float4*>(mu)[c], r = reinterpret_cast<const float4*>(rs)[c];
            v.x = (v.x - m.x) * r.x; v.y = (v.y - m.y) * r.y; v.z = (v.z - m.z) * r.z; v.w = (v.w - m.w) * r.w;
            reinterpret_cast<float4*>(dst)[c] = v;
        }
    } else {
        for (int c = gl; c < n; c += G) dst[c] = (src[c] - mu[c]) * rs[c];
    }
}

// G lanes cooperate on one sample; the rows of s, a, s' are copied with coalesced accesses.
template <int G, bool VEC_O, bool VEC_A>
__global__ __launch_bounds__(256) void sample_kernel(const SampleArgs a) {
    const int gl = threadIdx.x % G;
    const int k = blockIdx.x * (256 / G) + threadIdx.x / G;
    if (k >= a.batch) return;

    int64_t slot;
    if (a.idx_in != nullptr) {
        slot = a.idx_in[k];
    } else {
        uint32_t w0, w1;
        philox4x32_10_w01((uint32_t)k, a.stream_id, a.ctr2, a.ctr3, a.key0, a.key1, w0, w1);
        const uint64_t u = ((uint64_t)w1 << 32) | (uint64_t)w0;
        const uint64_t V = (uint64_t)(a.count - a.nstep + 1) * (uint64_t)a.N;
        const uint64_t p = __umul64hi(u, V);
        const uint64_t j = p / (uint64_t)a.N;
        const uint64_t e = p - j * (uint64_t)a.N;
        const int64_t row = ((int64_t)a.head - (int64_t)a.count + (int64_t)j + (int64_t)a.T) % (int64_t)a.T;
        slot = row * (int64_t)a.N + (int64_t)e;
        if (gl == 0) a.out.idx[k] = slot;
    }
    if (a.only_obs) {       // Algorithm 2: the P-learner's batch is states only
        if (a.nmean != nullptr)
            copy_row_std<G, VEC_O>(a.out.obs + (size_t)k * a.o, a.st.obs + (size_t)slot * a.o, a.o, gl, a.nmean, a.nrstd);
        else
            copy_row<G, VEC_O>(a.out.obs + (size_t)k * a.o, a.st.obs + (size_t)slot * a.o, a.o, gl);
        return;
    }
    const int64_t row0 = slot / a.N;
    const int64_t env = slot - row0 * a.N;
    // slot of the window's last row (its s' is the batch's next state): index arithmetic only
    int64_t last;
    {
        int64_t r = row0 + (a.nstep - 1);
        if (r >= a.T) r -= a.T;
        last = r * (int64_t)a.N + env;
    }
    // 16-byte path with at most one granule per lane and row: the three rows' loads are issued BEFORE the
    // window's rewards and termination flags are read, so that a sample costs one memory round trip (rows,
    // rewards and flags arrive together) instead of two; the stores follow the fold
    const int no4 = a.o >> 2, na4 = a.a >> 2;
    const bool one_pass = VEC_O && VEC_A && no4 <= G && na4 <= G;
    const bool stdz = a.nmean != nullptr;
    float4 vo = make_float4(0.f, 0.f, 0.f, 0.f), vn = vo, va = vo;
    if (one_pass) {
        if (gl < no4) {
            vo = reinterpret_cast<const float4*>(a.st.obs + (size_t)slot * a.o)[gl];
            vn = reinterpret_cast<const float4*>(a.st.next_obs + (size_t)last * a.o)[gl];
        }
        if (gl < na4) va = reinterpret_cast<const float4*>(a.st.act + (size_t)slot * a.a)[gl];
    }

    // fold rewards and termination flags over the window (every lane of the group reads the
    // same addresses; lane 0 writes)
    float ret = 0.f, alive = 1.f, g = 1.f;
    for (int s = 0; s < a.nstep; ++s) {
        int64_t r = row0 + s;
        if (r >= a.T) r -= a.T;
        const int64_t at = r * (int64_t)a.N + env;
        ret += g * a.st.rew[at] * alive;
        alive *= (1.f - a.st.done[at]);
        g *= a.gamma;
    }
    if (gl == 0) {
        a.out.ret[k] = ret;
        a.out.boot[k] = g * alive;
    }
    if (one_pass) {
        if (gl < no4) {
            if (stdz) {
                const float4 mu = reinterpret_cast<const float4*>(a.nmean)[gl], rs = reinterpret_cast<const float4*>(a.nrstd)[gl];
                vo.x = (vo.x - mu.x) * rs.x; vo.y = (vo.y - mu.y) * rs.y; vo.z = (vo.z - mu.z) * rs.z; vo.w = (vo.w - mu.w) * rs.w;
                vn.x = (vn.x - mu.x) * rs.x; vn.y = (vn.y - mu.y) * rs.y; vn.z = (vn.z - mu.z) * rs.z; vn.w = (vn.w - mu.w) * rs.w;
            }
            reinterpret_cast<float4*>(a.out.obs + (size_t)k * a.o)[gl] = vo;
            reinterpret_cast<float4*>(a.out.next_obs + (size_t)k * a.o)[gl] = vn;
        }
        if (gl < na4) reinterpret_cast<float4*>(a.out.act + (size_t)k * a.a)[gl] = va;
        return;
    }
    if (VEC_O && VEC_A) {
        // 16-byte path, several granules per lane: the three rows' loads of a pass are issued together and
        // the stores follow (row after row, each copy waited for the one before it: nothing tells the
        // compiler that the batch does not alias the ring)
        const float4* __restrict__ so = reinterpret_cast<const float4*>(a.st.obs + (size_t)slot * a.o);
        const float4* __restrict__ sn = reinterpret_cast<const float4*>(a.st.next_obs + (size_t)last * a.o);
        const float4* __restrict__ sa = reinterpret_cast<const float4*>(a.st.act + (size_t)slot * a.a);
        float4* __restrict__ d_o = reinterpret_cast<float4*>(a.out.obs + (size_t)k * a.o);
        float4* __restrict__ d_n = reinterpret_cast<float4*>(a.out.next_obs + (size_t)k * a.o);
        float4* __restrict__ d_a = reinterpret_cast<float4*>(a.out.act + (size_t)k * a.a);
        const int nmax = no4 > na4 ? no4 : na4;
        for (int c = gl; c < nmax; c += G) {
            const bool po = c < no4, pa = c < na4;
            float4 xo = make_float4(0.f, 0.f, 0.f, 0.f), xn = xo, xa = xo, mu = xo, rs = make_float4(1.f, 1.f, 1.f, 1.f);
            if (po) { xo = so[c]; xn = sn[c]; }
            if (pa) xa = sa[c];
            if (po && stdz) { mu = reinterpret_cast<const float4*>(a.nmean)[c]; rs = reinterpret_cast<const float4*>(a.nrstd)[c]; }
            if (stdz) {
                xo.x = (xo.x - mu.x) * rs.x; xo.y = (xo.y - mu.y) * rs.y; xo.z = (xo.z - mu.z) * rs.z; xo.w = (xo.w - mu.w) * rs.w;
                xn.x = (xn.x - mu.x) * rs.x; xn.y = (xn.y - mu.y) * rs.y; xn.z = (xn.z - mu.z) * rs.z; xn.w = (xn.w - mu.w) * rs.w;
            }
            if (po) { d_o[c] = xo; d_n[c] = xn; }
            if (pa) d_a[c] = xa;
        }
        return;
    }
    copy_row<G, VEC_A>(a.out.act + (size_t)k * a.a, a.st.act + (size_t)slot * a.a, a.a, gl);
    if (a.nmean != nullptr) {
        copy_row_std<G, VEC_O>(a.out.obs + (size_t)k * a.o, a.st.obs + (size_t)slot * a.o, a.o, gl, a.nmean, a.nrstd);
        copy_row_std<G, VEC_O>(a.out.next_obs + (size_t)k * a.o, a.st.next_obs + (size_t)last * a.o, a.o, gl, a.nmean,
                               a.nrstd);
    } else {
        copy_row<G, VEC_O>(a.out.obs + (size_t)k * a.o, a.st.obs + (size_t)slot * a.o, a.o, gl);
        copy_row<G, VEC_O>(a.out.next_obs + (size_t)k * a.o, a.st.next_obs + (size_t)last * a.o, a.o, gl);
    }
}

template <int G>
static void sample_dispatch(const SampleArgs& a, bool vo, bool va, const ProfSlot& ps, hipStream_t stream) {
    const dim3 grid((a.batch + (256 / G) - 1) / (256 / G)), block(256);
    if (vo && va)       PQL_LAUNCH(ps, (sample_kernel<G, true, true>), grid, block, 0, stream, a);
    else if (vo)        PQL_LAUNCH(ps, (sample_kernel<G, true, false>), grid, block, 0, stream, a);
    else if (va)        PQL_LAUNCH(ps, (sample_kernel<G, false, true>), grid, block, 0, stream, a);
    else                PQL_LAUNCH(ps, (sample_kernel<G, false, false>), grid, block, 0, stream, a);
}

static inline bool al16(const void* p) { return (((uintptr_t)p) & 15) == 0; }

hipError_t sample_launch(const SampleArgs& a, hipStream_t stream) {
    if (a.batch <= 0) return hipSuccess;
    const bool vo = (a.o % 4 == 0) && al16(a.st.obs) && al16(a.out.obs) && al16(a.nmean) && al16(a.nrstd) &&
                    (a.only_obs || (al16(a.st.next_obs) && al16(a.out.next_obs)));
    const bool va = a.only_obs || ((a.a % 4 == 0) && al16(a.st.act) && al16(a.out.act));
    const int per_row = vo ? a.o / 4 : a.o;
    // per sample: read s, a, s' and n (r, d) pairs; write s, a, s', ret, boot and the index
    const double bytes = a.only_obs ? (double)a.batch * (8.0 * a.o + 8.0)
                                    : (double)a.batch * (4.0 * (2 * a.o + a.a + 2 * a.nstep) + 4.0 * (2 * a.o + a.a + 2) + 8.0);
    const ProfSlot ps = prof_slot();
    // lanes per sample: enough for one 16-byte granule per lane and row where the rows are short enough
    if (per_row <= 16)      sample_dispatch<16>(a, vo, va, ps, stream);
    else if (per_row <= 32) sample_dispatch<32>(a, vo, va, ps, stream);
    else                    sample_dispatch<64>(a, vo, va, ps, stream);
    prof_commit(ps, KID_SAMPLE, 0.0, bytes);
    return hipGetLastError();
}

// =============================================================================================
// Critic output heads.  The last critic layer has one output, so it is a dot product per row,
// done by one wavefront per row with a cross-lane reduction.  The same pass forms the TD target
// (min of the twin target critics, Algorithm 3 / Section 3.2), the squared Bellman error, the
// output delta, the delta of the last hidden layer and the partial sums of the output-layer
// gradients.
// =============================================================================================
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
__device__ inline float wave_sum(float x) {
    x += dpp_move<0xB1>(x);      // quad_perm [1, 0, 3, 2]
    x += dpp_move<0x4E>(x);      // quad_perm [2, 3, 0, 1]
    x += dpp_move<0x141>(x);     // row_half_mirror
    x += dpp_move<0x140>(x);     // row_mirror
    return (lane_value(x, 0) + lane_value(x, 16)) + (lane_value(x, 32) + lane_value(x, 48));
}

constexpr int HEAD_WAVES = 4;

// Sums the per-wave column accumulators of a workgroup through LDS and writes one partial row.
template <int NJ>
__device__ inline void block_reduce_cols(float (&acc)[NJ], float* lds, float* __restrict__ out_row, int H, int lane,
                                         int wave) {
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int c = lane + 64 * j;
        if (c < H) lds[wave * H + c] = acc[j];
    }
    __syncthreads();
    for (int c = threadIdx.x; c < H; c += 64 * HEAD_WAVES) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < HEAD_WAVES; ++w) s += lds[w * H + c];
        out_row[c] = s;
    }
}

template <int NJ, bool POLICY>
__global__ __launch_bounds__(64 * HEAD_WAVES) void head_kernel(const HeadArgs a) {
    extern __shared__ float lds[];      // HEAD_WAVES * H floats
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int H = a.H, B = a.B;
    const int gw = blockIdx.x * HEAD_WAVES + wave, nw = gridDim.x * HEAD_WAVES;

    float wq0[NJ], wq1[NJ], wt0[NJ], wt1[NJ];
    float dw0[NJ], dw1[NJ], dbh0[NJ], dbh1[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int c = lane + 64 * j;
        const bool ok = c < H;
        wq0[j] = ok ? a.wQ[0][c] : 0.f;
        wq1[j] = ok ? a.wQ[1][c] : 0.f;
        wt0[j] = (!POLICY && ok) ? a.wT[0][c] : 0.f;
        wt1[j] = (!POLICY && ok) ? a.wT[1][c] : 0.f;
        dw0[j] = dw1[j] = dbh0[j] = dbh1[j] = 0.f;
    }
    const float bq0 = a.bQ[0][0], bq1 = a.bQ[1][0];
    const float bt0 = POLICY ? 0.f : a.bT[0][0], bt1 = POLICY ? 0.f : a.bT[1][0];
    const float invB = 1.f / (float)B;
    const float alpha = (!POLICY && a.logp_next != nullptr) ? expf(a.log_alpha[0]) : 0.f;
    float loss0 = 0.f, loss1 = 0.f, db0 = 0.f, db1 = 0.f;

    for (int row = gw; row < B; row += nw) {
        const size_t base = (size_t)row * H;
        float h0[NJ], h1[NJ];
        float q0 = 0.f, q1 = 0.f, t0 = 0.f, t1 = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int c = lane + 64 * j;
            const bool ok = c < H;
            h0[j] = ok ? a.hQ[0][base + c] : 0.f;
            h1[j] = ok ? a.hQ[1][base + c] : 0.f;
            q0 += h0[j] * wq0[j];
            q1 += h1[j] * wq1[j];
            if (!POLICY) {
                t0 += (ok ? a.hT[0][base + c] : 0.f) * wt0[j];
                t1 += (ok ? a.hT[1][base + c] : 0.f) * wt1[j];
            }
        }
        q0 = wave_sum(q0) + bq0;
        q1 = wave_sum(q1) + bq1;
        float d0, d1;
        if (POLICY) {
            // maximise min(Q_1, Q_2): the gradient -1/B enters the smaller critic (ties: Q_1)
            const bool pick0 = q0 <= q1;
            loss0 += pick0 ? q0 : q1;
            d0 = pick0 ? -invB : 0.f;
            d1 = pick0 ? 0.f : -invB;
        } else {
            t0 = wave_sum(t0) + bt0;
            t1 = wave_sum(t1) + bt1;
            float tq = fminf(t0, t1);
            if (a.logp_next != nullptr) tq -= alpha * a.logp_next[row];      // soft value of the SAC variant
            const float y = a.ret[row] + a.boot[row] * tq;
            const float e0 = q0 - y, e1 = q1 - y;
            loss0 += e0 * e0;
            loss1 += e1 * e1;
            d0 = 2.f * e0 * invB;
            d1 = 2.f * e1 * invB;
            db0 += d0;
            db1 += d1;
            if (lane == 0) a.y[row] = y;
        }
        if (lane == 0) { a.q[0][row] = q0; a.q[1][row] = q1; }
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int c = lane + 64 * j;
            if (c < H) {
                const float g0 = d0 * wq0[j] * (h0[j] > 0.f ? 1.f : h0[j] + 1.f);
                const float g1 = d1 * wq1[j] * (h1[j] > 0.f ? 1.f : h1[j] + 1.f);
                a.dQ[0][base + c] = g0;
                a.dQ[1][base + c] = g1;
                if (!POLICY) {
                    dbh0[j] += g0; dbh1[j] += g1;
                    dw0[j] += d0 * h0[j]; dw1[j] += d1 * h1[j];
                }
            }
        }
    }

    const int wg = blockIdx.x, nwg = gridDim.x;
    if (!POLICY) {
        block_reduce_cols<NJ>(dw0, lds, a.p_dw[0] + (size_t)wg * H, H, lane, wave);
        block_reduce_cols<NJ>(dw1, lds, a.p_dw[1] + (size_t)wg * H, H, lane, wave);
        block_reduce_cols<NJ>(dbh0, lds, a.p_dbh[0] + (size_t)wg * H, H, lane, wave);
        block_reduce_cols<NJ>(dbh1, lds, a.p_dbh[1] + (size_t)wg * H, H, lane, wave);
    }
    // scalars: loss and output-bias gradient (identical in every lane of a wave)
    __syncthreads();
    if (lane == 0) {
        lds[wave * 4 + 0] = loss0; lds[wave * 4 + 1] = loss1;
        lds[wave * 4 + 2] = db0;   lds[wave * 4 + 3] = db1;
    }
    __syncthreads();
    if (threadIdx.x < 4) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < HEAD_WAVES; ++w) s += lds[w * 4 + threadIdx.x];
        if (threadIdx.x == 0) a.p_loss[wg] = s;
        if (!POLICY) {
            if (threadIdx.x == 1) a.p_loss[nwg + wg] = s;
            if (threadIdx.x == 2) a.p_db[0][wg] = s;
            if (threadIdx.x == 3) a.p_db[1][wg] = s;
        }
    }
}

// =============================================================================================
// Heads of the distributional critics (PQL-D: categorical distribution over fixed atoms z_k on
// [v_min, v_max], categorical projection of the n-step target, cross-entropy).  One wavefront per
// row, lane k holds atom k.
// =============================================================================================
__device__ inline float wave_max(float x) {
    x = fmaxf(x, dpp_move<0xB1>(x));
    x = fmaxf(x, dpp_move<0x4E>(x));
    x = fmaxf(x, dpp_move<0x141>(x));
    x = fmaxf(x, dpp_move<0x140>(x));
    return fmaxf(fmaxf(lane_value(x, 0), lane_value(x, 16)), fmaxf(lane_value(x, 32), lane_value(x, 48)));
}

// Softmax over the lanes < atoms: returns p_k, and log p_k through `logp` (0 / -inf-free for idle lanes).
__device__ inline float lane_softmax(float logit, bool live, float& logp) {
    const float mx = wave_max(live ? logit : -3.0e38f);
    const float e = live ? expf(logit - mx) : 0.f;
    const float s = wave_sum(e);
    logp = live ? (logit - mx) - logf(s) : 0.f;
    return e / s;
}

template <bool POLICY>
__global__ __launch_bounds__(64 * HEAD_WAVES) void dist_head_kernel(const DistHeadArgs a) {
    __shared__ float lds[HEAD_WAVES][2][64];
    __shared__ float lds_loss[HEAD_WAVES][2];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l = a.atoms, B = a.B;
    const bool live = lane < l;
    const int gw = blockIdx.x * HEAD_WAVES + wave, nw = gridDim.x * HEAD_WAVES;
    const float dz = (a.v_max - a.v_min) / (float)(l - 1);
    const float z = a.v_min + (float)lane * dz;
    const float invB = 1.f / (float)B;
    float loss0 = 0.f, loss1 = 0.f, db0 = 0.f, db1 = 0.f;

    for (int row = gw; row < B; row += nw) {
        const size_t at = (size_t)row * l + lane;
        float lp0, lp1;
        const float p0 = lane_softmax(live ? a.logitsQ[0][at] : 0.f, live, lp0);
        const float p1 = lane_softmax(live ? a.logitsQ[1][at] : 0.f, live, lp1);
        float d0, d1;
        if (POLICY) {
            // Q_i = sum_k p_ik z_k; maximise min(Q_1, Q_2): dJ/dlogit_k = -(1/B) p_k (z_k - Q) for
            // the smaller critic (ties: Q_1), 0 for the other
            const float q0 = wave_sum(p0 * z), q1 = wave_sum(p1 * z);
            const bool pick0 = q0 <= q1;
            loss0 += pick0 ? q0 : q1;
            d0 = pick0 ? -invB * p0 * (z - q0) : 0.f;
            d1 = pick0 ? 0.f : -invB * p1 * (z - q1);
        } else {
            float unused;
            const float t0 = lane_softmax(live ? a.logitsT[0][at] : 0.f, live, unused);
            const float t1 = lane_softmax(live ? a.logitsT[1][at] : 0.f, live, unused);
            const float qt0 = wave_sum(t0 * z), qt1 = wave_sum(t1 * z);
            const float pn = qt0 <= qt1 ? t0 : t1;           // next-state distribution: the smaller mean
            // atom j moves to clip(ret + boot z_j); position in units of the atom spacing
            const float tz = fminf(fmaxf(a.ret[row] + a.boot[row] * z, a.v_min), a.v_max);
            const float pos = (tz - a.v_min) / dz;
            float m = 0.f;
            for (int j = 0; j < l; ++j) {               // j is wave-uniform: lane j's values come as scalars
                const float pos_j = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pos), j));
                const float pn_j = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pn), j));
                const float wgt = 1.f - fabsf(pos_j - (float)lane);
                m += pn_j * fminf(fmaxf(wgt, 0.f), 1.f);
            }
            if (!live) m = 0.f;
            const float S = wave_sum(m);
            loss0 -= wave_sum(m * lp0);
            loss1 -= wave_sum(m * lp1);
            d0 = (p0 * S - m) * invB;
            d1 = (p1 * S - m) * invB;
            db0 += d0;
            db1 += d1;
        }
        if (live) {
            a.logitsQ[0][at] = d0;
            a.logitsQ[1][at] = d1;
        }
    }
    const int wg = blockIdx.x, nwg = gridDim.x;
    lds[wave][0][lane] = db0;
    lds[wave][1][lane] = db1;
    if (lane == 0) { lds_loss[wave][0] = loss0; lds_loss[wave][1] = loss1; }
    __syncthreads();
    if (!POLICY && threadIdx.x < 128) {
        const int i = threadIdx.x >> 6;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < HEAD_WAVES; ++w) sum += lds[w][i][lane];
        if (live) a.p_db[i][(size_t)wg * l + lane] = sum;
    }
    if (threadIdx.x < 2) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < HEAD_WAVES; ++w) sum += lds_loss[w][threadIdx.x];
        if (threadIdx.x == 0) a.p_loss[wg] = sum;
        else if (!POLICY) a.p_loss[nwg + wg] = sum;
    }
}

hipError_t dist_critic_head_launch(const DistHeadArgs& a, hipStream_t stream) {
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, dist_head_kernel<false>, dim3(a.nwg), dim3(64 * HEAD_WAVES), 0, stream, a);
    prof_commit(ps, KID_DIST_CRITIC, 0.0, 24.0 * (double)a.B * a.atoms);    // 4 logit rows read, 2 written
    return hipGetLastError();
}

hipError_t dist_policy_head_launch(const DistHeadArgs& a, hipStream_t stream) {
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, dist_head_kernel<true>, dim3(a.nwg), dim3(64 * HEAD_WAVES), 0, stream, a);
    prof_commit(ps, KID_DIST_POLICY, 0.0, 16.0 * (double)a.B * a.atoms);
    return hipGetLastError();
}

int dist_head_workgroups(int B) {
    int n = (B + HEAD_WAVES * 2 - 1) / (HEAD_WAVES * 2);   // about 2 rows per wavefront
    if (n < 1) n = 1;
    if (n > 1024) n = 1024;
    return n;
}

int head_workgroups(int B) {
    int n = (B + HEAD_WAVES * 8 - 1) / (HEAD_WAVES * 8);   // about 8 rows per wavefront
    if (n < 1) n = 1;
    if (n > 512) n = 512;
    return n;
}

template <bool POLICY>
static hipError_t head_launch(const HeadArgs& a, hipStream_t stream) {
    const dim3 grid(a.nwg), block(64 * HEAD_WAVES);
    const size_t lds = (size_t)HEAD_WAVES * (a.H > 4 ? a.H : 4) * sizeof(float);
    const int nj = (a.H + 63) / 64;
    // reads of the last hidden activations (online + target critics), write of the deltas
    const double bytes = 4.0 * (double)a.B * a.H * (POLICY ? 4.0 : 6.0);
    if (nj > 16) return hipErrorInvalidValue;
    const ProfSlot ps = prof_slot();
    if (nj <= 1)       PQL_LAUNCH(ps, (head_kernel<1, POLICY>), grid, block, lds, stream, a);
    else if (nj <= 2)  PQL_LAUNCH(ps, (head_kernel<2, POLICY>), grid, block, lds, stream, a);
    else if (nj <= 4)  PQL_LAUNCH(ps, (head_kernel<4, POLICY>), grid, block, lds, stream, a);
    else if (nj <= 8)  PQL_LAUNCH(ps, (head_kernel<8, POLICY>), grid, block, lds, stream, a);
    else               PQL_LAUNCH(ps, (head_kernel<16, POLICY>), grid, block, lds, stream, a);
    prof_commit(ps, POLICY ? KID_HEAD_POLICY : KID_HEAD_CRITIC, 0.0, bytes);
    return hipGetLastError();
}

hipError_t critic_head_launch(const HeadArgs& a, hipStream_t stream) { return head_launch<false>(a, stream); }
hipError_t policy_head_launch(const HeadArgs& a, hipStream_t stream) { return head_launch<true>(a, stream); }

// =============================================================================================
// Gradient reduction + Adam (Table B.1 "Optimizer: Adam"; Kingma & Ba, Algorithm 1).
// Each parameter's gradient is the ordered sum of its partial results (split-K slabs of the
// weight-gradient GEMMs, per-tile column sums for biases); the Adam step is applied in the
// same pass.  Block (0,0) also finalises the loss scalars.
// =============================================================================================
// A workgroup covers E = 256 / Q consecutive elements of one tensor; the Q lanes that share an
// element each sum every Q-th partial (four loads in flight), then combine through LDS in a
// fixed order, so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void adam_reduce_kernel(const AdamArgs a) {
    __shared__ float sm[256];
    const int b = blockIdx.x;
    int ti = 0;
    for (int i = 1; i < a.ntensors; ++i)
        if (b >= a.t[i].block_begin) ti = i;
    const RedTensor& T = a.t[ti];
    const int ql = T.qlog2, Q = 1 << ql, E = 256 >> ql;
    const int e = threadIdx.x & (E - 1), q = threadIdx.x >> (8 - ql);
    const int i = (b - T.block_begin) * E + e;
    const bool live = i < T.count;
    float g = 0.f;
    // the optimiser state is requested first: its latency hides behind the partial sums
    const bool step_here = live && q == 0 && !(a.max_norm > 0.f);
    const bool track = step_here && a.track != nullptr;
    float m_old = 0.f, v_old = 0.f, th_old = 0.f, tr_old = 0.f;
    if (step_here) {
        const int64_t k = T.offset + i;
        m_old = a.m[k]; v_old = a.v[k]; th_old = a.theta[k];
        if (track) tr_old = a.track[k];
    }
    if (live) {
        const float* __restrict__ p = T.partial + i;
        const size_t st = (size_t)T.stride;
        int s = q;
        for (; s + 7 * Q < T.nparts; s += 8 * Q) {      // eight loads in flight
            const float x0 = p[(size_t)s * st], x1 = p[(size_t)(s + Q) * st];
            const float x2 = p[(size_t)(s + 2 * Q) * st], x3 = p[(size_t)(s + 3 * Q) * st];
            const float x4 = p[(size_t)(s + 4 * Q) * st], x5 = p[(size_t)(s + 5 * Q) * st];
            const float x6 = p[(size_t)(s + 6 * Q) * st], x7 = p[(size_t)(s + 7 * Q) * st];
            g += ((x0 + x1) + (x2 + x3)) + ((x4 + x5) + (x6 + x7));
        }
        for (; s + 3 * Q < T.nparts; s += 4 * Q) {
            const float x0 = p[(size_t)s * st], x1 = p[(size_t)(s + Q) * st];
            const float x2 = p[(size_t)(s + 2 * Q) * st], x3 = p[(size_t)(s + 3 * Q) * st];
            g += (x0 + x1) + (x2 + x3);
        }
        for (; s < T.nparts; s += Q) g += p[(size_t)s * st];
    }
    if (Q > 1) {
        sm[threadIdx.x] = g;
        __syncthreads();
        if (q == 0)
            for (int k = 1; k < Q; ++k) g += sm[k * E + e];
    }
    const bool clip = a.max_norm > 0.f;
    if (clip) {
        // Clipping needs the norm of the whole gradient first: store g and this workgroup's sum
        // of squares; adam_clip_kernel finishes the step.
        const bool own = live && q == 0;
        if (own) a.g[T.offset + i] = g;
        const float sq = wave_sum(own ? g * g : 0.f);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = sq;
        __syncthreads();
        if (threadIdx.x == 0) a.sq_partial[b] = (sm[0] + sm[1]) + (sm[2] + sm[3]);
    } else if (step_here) {
        const int64_t k = T.offset + i;
        const float m = a.beta1 * m_old + (1.f - a.beta1) * g;
        const float v = a.beta2 * v_old + (1.f - a.beta2) * g * g;
        const float m_hat = m * a.inv_bc1;
        const float v_hat = v * a.inv_bc2;
        const float th = th_old - a.lr * m_hat / (sqrtf(v_hat) + a.eps);
        a.theta[k] = th;
        a.m[k] = m;
        a.v[k] = v;
        if (a.g != nullptr) a.g[k] = g;
        // what usually follows the step, in the same pass: the tracking vector (Polyak / hard copy) and the
        // transposed copy of the weights that the next backward products read
        if (track) a.track[k] = a.tau == 1.f ? th : polyak_mix(a.tau, 1.f - a.tau, th, tr_old);
        if (T.tdst != nullptr) {
            const int r = i / T.tcols, cc = i - r * T.tcols;
            T.tdst[(size_t)cc * (size_t)T.trows + r] = th;
        }
    }
    if (b == 0) {
        const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        if (wave < a.nloss) {
            float s = 0.f;
            for (int j = lane; j < a.loss_parts; j += 64) s += a.loss_partial[wave * a.loss_parts + j];
            s = wave_sum(s);
            if (lane == 0) a.loss_out[wave] = s * a.loss_scale;
        }
        if (!clip && threadIdx.x == 0 && a.norm_out != nullptr) *a.norm_out = 0.f;   // norm not computed
    }
}

// Second half of a clipped step (Table B.1 "Gradient Clipping"): every workgroup adds the
// per-workgroup sums of squares in the same fixed order, rescales its share of the stored
// gradient when the norm exceeds the bound, and applies Adam.
struct AdamClipArgs {
    float* theta; float* m; float* v; float* g;
    const float* sq_partial; float* norm_out;
    int64_t n; int nparts;
    float lr, beta1, beta2, eps, inv_bc1, inv_bc2, max_norm;
    // what follows the step, as in adam_reduce_kernel: tracking vector and transposed copies of some tensors
    float* track; float tau;
    int ntr;
    struct Tr { int64_t offset; float* tdst; int count, trows, tcols, pad_; } tr[RED_MAX_TENSORS];
};

__global__ __launch_bounds__(256) void adam_clip_kernel(const AdamClipArgs a) {
    __shared__ double smd[256];
    double s = 0.0;
    for (int j = threadIdx.x; j < a.nparts; j += 256) s += (double)a.sq_partial[j];
    smd[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) smd[threadIdx.x] += smd[threadIdx.x + w];
        __syncthreads();
    }
    const float norm = (float)sqrt(smd[0]);
    const float scale = norm > a.max_norm ? a.max_norm / norm : 1.f;
    if (blockIdx.x == 0 && threadIdx.x == 0) *a.norm_out = norm;
    const int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t k = base + 256 * j;
        if (k >= a.n) break;
        const float g = a.g[k] * scale;
        const float m = a.beta1 * a.m[k] + (1.f - a.beta1) * g;
        const float v = a.beta2 * a.v[k] + (1.f - a.beta2) * g * g;
        const float th = a.theta[k] - a.lr * (m * a.inv_bc1) / (sqrtf(v * a.inv_bc2) + a.eps);
        a.theta[k] = th;
        a.m[k] = m;
        a.v[k] = v;
        a.g[k] = g;
        if (a.track != nullptr) a.track[k] = a.tau == 1.f ? th : polyak_mix(a.tau, 1.f - a.tau, th, a.track[k]);
        for (int i = 0; i < a.ntr; ++i) {           // the few tensors whose transposes the next backward pass reads
            const int64_t e = k - a.tr[i].offset;
            if (e >= 0 && e < a.tr[i].count) {
                const int r = (int)e / a.tr[i].tcols, cc = (int)e - r * a.tr[i].tcols;
                a.tr[i].tdst[(size_t)cc * (size_t)a.tr[i].trows + r] = th;
            }
        }
    }
}

// Algorithmic traffic of the optimiser: read theta, g, m, v and write theta, m, v = 28 bytes per
// parameter (the partial-sum reads that replace the single read of g are not counted).
double adam_bytes(const AdamArgs& a) {
    double n = 0.0, extra = 0.0;
    for (int i = 0; i < a.ntensors; ++i) {
        n += a.t[i].count;
        if (a.t[i].tdst != nullptr) extra += 4.0 * a.t[i].count;     // the transposed copy
    }
    return (a.track != nullptr ? 36.0 : 28.0) * n + extra;           // tracking vector: one more read and write
}

hipError_t adam_reduce_launch(const AdamArgs& args, hipStream_t stream) {
    AdamArgs a = args;
    int blocks = 0;
    for (int i = 0; i < a.ntensors; ++i) {
        RedTensor& t = a.t[i];
        t.qlog2 = t.nparts <= 16 ? 0 : (t.nparts <= 64 ? 2 : 4);
        t.block_begin = blocks;
        const int E = 256 >> t.qlog2;
        blocks += (t.count + E - 1) / E;
    }
    if (blocks == 0) blocks = 1;
    const dim3 grid(blocks), block(256);
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, adam_reduce_kernel, grid, block, 0, stream, a);
    prof_commit(ps, KID_ADAM, 0.0, ps.on ? adam_bytes(a) : 0.0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !(a.max_norm > 0.f)) return e;
    AdamClipArgs c;
    c.theta = a.theta; c.m = a.m; c.v = a.v; c.g = a.g; c.sq_partial = a.sq_partial; c.norm_out = a.norm_out;
    c.n = 0;
    for (int i = 0; i < a.ntensors; ++i)
        if (a.t[i].offset + a.t[i].count > c.n) c.n = a.t[i].offset + a.t[i].count;
    c.nparts = blocks;
    c.lr = a.lr; c.beta1 = a.beta1; c.beta2 = a.beta2; c.eps = a.eps; c.inv_bc1 = a.inv_bc1; c.inv_bc2 = a.inv_bc2;
    c.max_norm = a.max_norm;
    c.track = a.track; c.tau = a.tau;
    c.ntr = 0;
    for (int i = 0; i < a.ntensors; ++i)
        if (a.t[i].tdst != nullptr) {
            AdamClipArgs::Tr& t = c.tr[c.ntr++];
            t.offset = a.t[i].offset; t.tdst = a.t[i].tdst; t.count = a.t[i].count; t.trows = a.t[i].trows; t.tcols = a.t[i].tcols;
        }
    const ProfSlot pc = prof_slot();
    PQL_LAUNCH(pc, adam_clip_kernel, dim3((unsigned)((c.n + 1023) / 1024)), block, 0, stream, c);
    prof_commit(pc, KID_ADAM_CLIP, 0.0, 32.0 * (double)c.n);   // theta, m, v, g read and written
    return hipGetLastError();
}

// The reduction handles at least 16 elements per workgroup and rounds every tensor up.
size_t adam_reduce_blocks_bound(size_t params, int ntensors) { return params / 16 + (size_t)ntensors + 1; }

// =============================================================================================
// Polyak target update (Table B.1 target update rate tau; tau = 1 is the hard policy sync of
// Section 3.2).
// =============================================================================================
__global__ __launch_bounds__(256) void soft_update_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                          int64_t n, float tau, int vec) {
    const float keep = 1.f - tau;
    const int64_t n4 = vec ? (n >> 2) : 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = t0; i < n4; i += stride) {
        const float4 s = reinterpret_cast<const float4*>(src)[i];
        float4 d = reinterpret_cast<float4*>(dst)[i];
        d.x = polyak_mix(tau, keep, s.x, d.x); d.y = polyak_mix(tau, keep, s.y, d.y);
        d.z = polyak_mix(tau, keep, s.z, d.z); d.w = polyak_mix(tau, keep, s.w, d.w);
        reinterpret_cast<float4*>(dst)[i] = d;
    }
    for (int64_t i = n4 * 4 + t0; i < n; i += stride) dst[i] = polyak_mix(tau, keep, src[i], dst[i]);
}

__global__ __launch_bounds__(256) void copy_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t n,
                                                   int vec) {
    const int64_t n4 = vec ? (n >> 2) : 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = t0; i < n4; i += stride) reinterpret_cast<float4*>(dst)[i] = reinterpret_cast<const float4*>(src)[i];
    for (int64_t i = n4 * 4 + t0; i < n; i += stride) dst[i] = src[i];
}

hipError_t soft_update_launch(const float* src, float* dst, int64_t count, float tau, hipStream_t stream) {
    if (count <= 0 || tau == 0.f) return hipSuccess;           // tau = 0 leaves dst untouched
    const int vec = (al16(src) && al16(dst)) ? 1 : 0;
    int64_t blocks = (count / 4 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 2048) blocks = 2048;
    const ProfSlot ps = prof_slot();
    if (tau == 1.f) PQL_LAUNCH(ps, copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, src, dst, count, vec);
    else PQL_LAUNCH(ps, soft_update_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, src, dst, count, tau, vec);
    prof_commit(ps, tau == 1.f ? KID_COPY : KID_SOFT_UPDATE, 0.0, (tau == 1.f ? 8.0 : 12.0) * (double)count);
    return hipGetLastError();
}

// =============================================================================================
// Running observation statistics (Table B.1 "Normalized Observations").  Per dimension the
// count, mean and sum of squared deviations of every observation pushed so far are kept in
// double; a new Actor step of N observations is merged in two launches: per chunk of rows the
// chunk mean and its sum of squared deviations (two passes over the chunk), then one workgroup
// merges the chunks into the running values in a fixed order with the pairwise update of Chan,
// Golub and LeVeque, and refreshes the fp32 mean and 1 / sqrt(var + eps) that consumers read.
// =============================================================================================
size_t obs_stats_bytes(int o, int max_rows) {
    const size_t nchunk = ((size_t)max_rows + OBS_CHUNK_ROWS - 1) / OBS_CHUNK_ROWS;
    size_t head = sizeof(double) * (2 * (size_t)o + 2) + sizeof(float) * 2 * (size_t)o;
    head = (head + 255) / 256 * 256;
    return head + sizeof(double) * nchunk * 2 * (size_t)o;
}

ObsStatsView obs_stats_view(void* base, int o) {
    ObsStatsView v;
    v.stat = (double*)base;
    v.mean_f = (float*)(v.stat + 2 * (size_t)o + 2);
    v.rstd_f = v.mean_f + o;
    size_t head = sizeof(double) * (2 * (size_t)o + 2) + sizeof(float) * 2 * (size_t)o;
    head = (head + 255) / 256 * 256;
    v.part = (double*)((char*)base + head);
    return v;
}

__global__ __launch_bounds__(256) void obs_stats_reset_kernel(ObsStatsView v, int o, float eps) {
    for (int c = threadIdx.x; c < o; c += 256) {
        v.stat[2 + c] = 0.0;
        v.stat[2 + o + c] = 0.0;
        v.mean_f[c] = 0.f;
        v.rstd_f[c] = (float)(1.0 / sqrt(1.0 + (double)eps));   // no data yet: mean 0, variance 1
    }
    if (threadIdx.x == 0) { v.stat[0] = 0.0; v.stat[1] = 0.0; }
}

__global__ __launch_bounds__(256) void obs_stats_chunk_kernel(ObsStatsView v, const float* __restrict__ x, int rows, int o) {
    __shared__ double sm[4][64];
    const int lane = threadIdx.x & 63, rg = threadIdx.x >> 6;
    const int r0 = blockIdx.x * OBS_CHUNK_ROWS;
    const int nr = rows - r0 < OBS_CHUNK_ROWS ? rows - r0 : OBS_CHUNK_ROWS;
    double* __restrict__ out = v.part + (size_t)blockIdx.x * 2 * o;
    for (int c0 = 0; c0 < o; c0 += 64) {
        const int c = c0 + lane;
        double s = 0.0;
        if (c < o)
            for (int r = rg; r < nr; r += 4) s += (double)x[(size_t)(r0 + r) * o + c];
        sm[rg][lane] = s;
        __syncthreads();
        const double mean = ((sm[0][lane] + sm[1][lane]) + (sm[2][lane] + sm[3][lane])) / (double)nr;
        __syncthreads();
        double q = 0.0;
        if (c < o)
            for (int r = rg; r < nr; r += 4) {
                const double d = (double)x[(size_t)(r0 + r) * o + c] - mean;
                q += d * d;
            }
        sm[rg][lane] = q;
        __syncthreads();
        if (rg == 0 && c < o) {
            out[c] = mean;
            out[o + c] = (sm[0][lane] + sm[1][lane]) + (sm[2][lane] + sm[3][lane]);
        }
        __syncthreads();
    }
}

// Merge of (n, mean, m2) with (nb, mb, qb): pairwise update of Chan, Golub and LeVeque.
__device__ inline void stats_merge(double& n, double& mean, double& m2, double nb, double mb, double qb) {
    if (nb <= 0.0) return;
    const double tot = n + nb, delta = mb - mean, f = nb / tot;
    mean += delta * f;
    m2 += qb + delta * delta * (n * f);
    n = tot;
}

// One workgroup; lane = column (in tiles of 64), the four wavefronts each fold a contiguous
// quarter of the chunks, then wavefront 0 folds the running values and the four quarters in order.
__global__ __launch_bounds__(256) void obs_stats_merge_kernel(ObsStatsView v, int rows, int o, float eps) {
    __shared__ double sn[4][64], smean[4][64], sm2[4][64];
    const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const double n0 = v.stat[0];
    const int nchunk = (rows + OBS_CHUNK_ROWS - 1) / OBS_CHUNK_ROWS;
    const int per = (nchunk + 3) / 4;
    const int k0 = grp * per, k1 = (k0 + per < nchunk) ? k0 + per : nchunk;
    for (int c0 = 0; c0 < o; c0 += 64) {
        const int c = c0 + lane;
        double n = 0.0, mean = 0.0, m2 = 0.0;
        if (c < o)
            for (int k = k0; k < k1; ++k) {
                const int left = rows - k * OBS_CHUNK_ROWS;
                const double nb = (double)(left < OBS_CHUNK_ROWS ? left : OBS_CHUNK_ROWS);
                stats_merge(n, mean, m2, nb, v.part[(size_t)k * 2 * o + c], v.part[(size_t)k * 2 * o + o + c]);
            }
        sn[grp][lane] = n; smean[grp][lane] = mean; sm2[grp][lane] = m2;
        __syncthreads();
        if (grp == 0 && c < o) {
            n = n0; mean = v.stat[2 + c]; m2 = v.stat[2 + o + c];
#pragma unroll
            for (int g = 0; g < 4; ++g) stats_merge(n, mean, m2, sn[g][lane], smean[g][lane], sm2[g][lane]);
            v.stat[2 + c] = mean;
            v.stat[2 + o + c] = m2;
            v.mean_f[c] = (float)mean;
            v.rstd_f[c] = (float)(1.0 / sqrt(m2 / n + (double)eps));
        }
        __syncthreads();                               // every thread has read the old count; LDS reusable
    }
    if (threadIdx.x == 0) v.stat[0] = n0 + (double)rows;
}

hipError_t obs_stats_reset_launch(const ObsStatsView& v, int o, float eps, hipStream_t stream) {
    hipLaunchKernelGGL(obs_stats_reset_kernel, dim3(1), dim3(256), 0, stream, v, o, eps);
    return hipGetLastError();
}

hipError_t obs_stats_update_launch(const ObsStatsView& v, const float* obs, int rows, int o, float eps, hipStream_t stream) {
    if (rows <= 0) return hipSuccess;
    const int nchunk = (rows + OBS_CHUNK_ROWS - 1) / OBS_CHUNK_ROWS;
    const ProfSlot p1 = prof_slot();
    PQL_LAUNCH(p1, obs_stats_chunk_kernel, dim3(nchunk), dim3(256), 0, stream, v, obs, rows, o);
    prof_commit(p1, KID_OBS_STATS, 0.0, 4.0 * (double)rows * o);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const ProfSlot p2 = prof_slot();
    PQL_LAUNCH(p2, obs_stats_merge_kernel, dim3(1), dim3(256), 0, stream, v, rows, o, eps);
    prof_commit(p2, KID_OBS_MERGE, 0.0, 16.0 * (double)nchunk * o);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void normalize_rows_kernel(const float* __restrict__ x, const float* __restrict__ mu,
                                                             const float* __restrict__ rs, float* __restrict__ out,
                                                             int64_t n, int o) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const int c = (int)(i % o);
        out[i] = (x[i] - mu[c]) * rs[c];
    }
}

hipError_t normalize_rows_launch(const float* x, const float* mean_f, const float* rstd_f, float* out, int rows, int o,
                                 hipStream_t stream) {
    const int64_t n = (int64_t)rows * o;
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, normalize_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, x, mean_f, rstd_f, out, n, o);
    prof_commit(ps, KID_NORMALIZE, 0.0, 8.0 * (double)n);
    return hipGetLastError();
}

// =============================================================================================
// Stochastic policy of the SAC variant (Section 3 / appendix "PQL for SAC"; Haarnoja et al. 2018):
// a = tanh(mu + sigma eps), log sigma = clip(raw, -5, 2),
// log pi = sum_d [-eps^2/2 - log sigma - log(2 pi)/2 - log(1 - a^2)], the last term evaluated as
// 2 (log 2 - u - softplus(-2u)).  One thread per row.
// =============================================================================================
__device__ inline float std_normal_draw(uint32_t element, uint32_t stream_id, uint32_t ctr2, uint32_t ctr3, uint32_t k0,
                                        uint32_t k1) {
    uint32_t w0, w1;
    philox4x32_10_w01(element, stream_id, ctr2, ctr3, k0, k1, w0, w1);
    // double precision: (w >> 8) + 0.5 needs 25 significant bits
    const double u1 = ((double)(w0 >> 8) + 0.5) * 0x1p-24;
    const double u2 = ((double)(w1 >> 8) + 0.5) * 0x1p-24;
    return (float)(sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2));
}

__global__ __launch_bounds__(256) void sac_sample_kernel(const SacSampleArgs a) {
    const int row = blockIdx.x * 256 + threadIdx.x;
    if (row >= a.B) return;
    const float* __restrict__ o2 = a.out2a + (size_t)row * 2 * a.a;
    float lp = 0.f;
    for (int d = 0; d < a.a; ++d) {
        const float e = std_normal_draw((uint32_t)(row * a.a + d), a.stream_id, a.ctr2, a.ctr3, a.key0, a.key1);
        const float ls = fminf(fmaxf(o2[a.a + d], SAC_LOG_STD_MIN), SAC_LOG_STD_MAX);
        const float u = o2[d] + expf(ls) * e;
        const float x = -2.f * u;
        const float softplus = fmaxf(x, 0.f) + log1pf(expf(-fabsf(x)));
        lp += -0.5f * e * e - ls - 0.91893853320467274178f - 2.f * (0.69314718055994530942f - u - softplus);
        a.act[(size_t)row * a.a + d] = tanhf(u);
        if (a.eps != nullptr) a.eps[(size_t)row * a.a + d] = e;
    }
    if (a.logp != nullptr) a.logp[row] = lp;
}

hipError_t sac_sample_launch(const SacSampleArgs& a, hipStream_t stream) {
    if (a.B <= 0) return hipSuccess;
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, sac_sample_kernel, dim3((a.B + 255) / 256), dim3(256), 0, stream, a);
    prof_commit(ps, KID_SAC_SAMPLE, 0.0, 4.0 * (double)a.B * (4.0 * a.a + 1.0));
    return hipGetLastError();
}

// Gradient at the policy's output layer: J = mean_b [alpha log pi - min Q], u = mu + sigma eps,
//   dJ/dmu = dJ/du = d_u + (alpha / B) 2 a            (d log pi / du = 2 tanh(u))
//   dJ/draw = dJ/du sigma eps - alpha / B              inside the clip, 0 outside
// plus the per-workgroup column sums of both (the output-bias gradient) and of log pi.
__global__ __launch_bounds__(SAC_ROWS) void sac_grad_kernel(const SacGradArgs a) {
    extern __shared__ float tile[];                     // [SAC_ROWS][2a + 1]
    const int row = blockIdx.x * SAC_ROWS + threadIdx.x;
    const int w2 = 2 * a.a, ld = w2 + 1;
    const float alpha = expf(a.log_alpha[0]), ab = alpha / (float)a.B;
    const bool live = row < a.B;
    for (int d = 0; d < a.a; ++d) {
        float dmu = 0.f, draw = 0.f;
        if (live) {
            const size_t at = (size_t)row * a.a + d;
            const float raw = a.out2a[(size_t)row * w2 + a.a + d];
            const float ls = fminf(fmaxf(raw, SAC_LOG_STD_MIN), SAC_LOG_STD_MAX);
            dmu = a.d_u[at] + ab * 2.f * a.act[at];
            if (raw > SAC_LOG_STD_MIN && raw < SAC_LOG_STD_MAX) draw = dmu * expf(ls) * a.eps[at] - ab;
            a.d_out[(size_t)row * w2 + d] = dmu;
            a.d_out[(size_t)row * w2 + a.a + d] = draw;
        }
        tile[threadIdx.x * ld + d] = dmu;
        tile[threadIdx.x * ld + a.a + d] = draw;
    }
    tile[threadIdx.x * ld + w2] = live ? a.logp[row] : 0.f;
    __syncthreads();
    for (int c = threadIdx.x; c <= w2; c += SAC_ROWS) {
        float s = 0.f;
        for (int r = 0; r < SAC_ROWS; ++r) s += tile[r * ld + c];
        if (c < w2) a.p_cols[(size_t)blockIdx.x * w2 + c] = s;
        else a.p_logp[blockIdx.x] = s;
    }
}

hipError_t sac_grad_launch(const SacGradArgs& a, hipStream_t stream) {
    if (a.B <= 0) return hipSuccess;
    const size_t lds = (size_t)SAC_ROWS * (2 * a.a + 1) * sizeof(float);
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, sac_grad_kernel, dim3((a.B + SAC_ROWS - 1) / SAC_ROWS), dim3(SAC_ROWS), lds, stream, a);
    prof_commit(ps, KID_SAC_GRAD, 0.0, 4.0 * (double)a.B * (7.0 * a.a + 1.0));
    return hipGetLastError();
}

// Temperature step (Table B.1 "Learnable Entropy Coefficient"): J(alpha) = -alpha mean(log pi + H),
// optimised in log alpha with Adam; also reports the entropy term of the policy objective.
__global__ __launch_bounds__(64) void sac_alpha_kernel(const SacAlphaArgs a) {
    float s = 0.f;
    for (int j = threadIdx.x; j < a.nparts; j += 64) s += a.p_logp[j];
    s = wave_sum(s);
    if (threadIdx.x == 0) {
        const float mean_logp = s / (float)a.B;
        const float la = a.temperature[0], alpha = expf(la);
        a.loss_out[2] = alpha * mean_logp;
        a.loss_out[3] = mean_logp;
        const float g = -alpha * (mean_logp + a.target_entropy);
        const float m = a.beta1 * a.temperature[1] + (1.f - a.beta1) * g;
        const float v = a.beta2 * a.temperature[2] + (1.f - a.beta2) * g * g;
        a.temperature[0] = la - a.lr * (m * a.inv_bc1) / (sqrtf(v * a.inv_bc2) + a.eps);
        a.temperature[1] = m;
        a.temperature[2] = v;
    }
}

hipError_t sac_alpha_launch(const SacAlphaArgs& a, hipStream_t stream) {
    const ProfSlot ps = prof_slot();
    PQL_LAUNCH(ps, sac_alpha_kernel, dim3(1), dim3(64), 0, stream, a);
    prof_commit(ps, KID_SAC_ALPHA, 0.0, 4.0 * (double)a.nparts);
    return hipGetLastError();
}

}  // namespace pql
