// Training-mode batch normalisation fused with the residual add and the ReLU that follow it,
// forward and backward, on NHWC tensors x[M][C] (M = N*H*W rows, channels contiguous).
//
// These layers carry no reuse: each is a stream over HBM, so the kernels are built around
// 16-byte coalesced row segments.  Thread t of a 256-thread workgroup owns the channel vector
// (t mod CV) and walks rows t/CV, t/CV + RL, ...; per-channel sums are accumulated in fp64
// registers (free in an HBM-bound kernel, and it removes the cancellation in E[x^2]-E[x]^2),
// combined through LDS, written as one partial per workgroup, and merged by a one-wave-per-
// channel kernel in a fixed order, so results are identical from run to run.
//
//   forward :  stats-partial -> finalize (mean, invstd, scale/shift) -> apply (+res, ReLU)
//   backward:  reduce-partial (sum dz, sum dz*xhat) -> finalize (dgamma, dbeta, coefficients)
//              -> apply (dx, and dz into the residual branch)
#include "common.h"

namespace dsp {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxPartialBlocks = 512;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// Layout of a workgroup over x[M][C]: CV channel vectors per row, RL row lanes.
struct RowLayout {
    int cv;   // channel vectors per row (C / VW)
    int cvb;  // channel vectors handled by one workgroup column (min(cv, 256))
    int rl;   // row lanes per workgroup (256 / cvb)
};
inline RowLayout make_layout(int C, int VW)
{
    RowLayout L;
    L.cv = C / VW;
    L.cvb = L.cv < kThreads ? L.cv : kThreads;
    L.rl = kThreads / L.cvb;
    return L;
}

// scale * x + shift as the forward pass stores it (one fused multiply-add, rounded to the storage type): the backward
// kernels that decide the ReLU from x call this too, and get the forward pass's decision
template <typename T>
__device__ inline float bn_value(float x, float scale, float shift)
{
    return to_float<T>(from_float<T>(__builtin_fmaf(x, scale, shift)));
}

// ---- per-channel sums ---------------------------------------------------------------------------
// MODE 0: s0 = sum x, s1 = sum x^2.
// MODE 1: dz = dy * [y > 0] (if RM != 0); s0 = sum dz, s1 = sum dz * (x - mean) * invstd.  RM = 1 reads the stored y;
//         RM = 2 (a batch norm without residual) forms y again from x and the forward pass's {scale, shift} with the
//         forward kernel's own expression and rounding, so the decision is the same and y is never read.
// MODE 2: out = x + dy as stored (the element-wise sum of two feature maps); s0 = sum out, s1 = sum out^2:
//         the sum layer together with the statistics pass of the batch norm that reads it.
// part[blockIdx.x][c][2]; blockIdx.y walks channel groups when C/VW > 256.
template <typename T>
struct AddOut {
    T* out;        // MODE 2: the sum
    const T* b1;   // second instance: the other operand and the sum
    T* out1;
};
template <typename T, int VW, int MODE, int RM>
__global__ __launch_bounds__(kThreads) void bn_sums_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                           const T* __restrict__ y, const float* __restrict__ mean,
                                                           const float* __restrict__ invstd, double* __restrict__ part,
                                                           int64_t M, int C, RowLayout L, int rows_per_block,
                                                           const T* __restrict__ x1, double* __restrict__ part1,
                                                           AddOut<T> add, const float* __restrict__ fcoef)
{
    // blockIdx.z = 1: the second instance of a twin launch (other tensor, same shape)
    T* __restrict__ out = add.out;
    if (blockIdx.z) {
        x = x1;
        part = part1;
        if (MODE == 2) {
            dy = add.b1;
            out = add.out1;
        }
    }
    __shared__ double red[VW][kThreads][2];  // one 16-byte pair per thread and channel, neighbouring lanes side by side: no bank conflicts
    const int tid = threadIdx.x;
    const int cvi = blockIdx.y * L.cvb + tid % L.cvb;
    const int rlane = tid / L.cvb;
    const bool active = rlane < L.rl && cvi < L.cv;
    const int c0 = cvi * VW;
    double s0[VW], s1[VW];
#pragma unroll
    for (int i = 0; i < VW; ++i) s0[i] = s1[i] = 0.0;
    float mu[VW], is[VW], fsc[VW], fsh[VW];
    if (MODE == 1 && active) {
#pragma unroll
        for (int i = 0; i < VW; ++i) {
            mu[i] = mean[c0 + i];
            is[i] = invstd[c0 + i];
            if (RM == 2) {
                fsc[i] = fcoef[c0 + i];
                fsh[i] = fcoef[C + c0 + i];
            }
        }
    }
    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r_end = r_begin + rows_per_block < M ? r_begin + rows_per_block : M;
    if (active) {
        // U rows per trip with all their loads issued before the first add: the loop is bound by load
        // latency, not by bandwidth, unless several rows are in flight per thread
        constexpr int U = 4;
        for (int64_t r = r_begin + rlane; r < r_end; r += (int64_t)U * L.rl) {
            float xv[U][VW], gv[U][VW], yv[U][VW];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t ru = r + (int64_t)u * L.rl;
                if (ru < r_end) {
                    VecIO<T, VW>::load(x + ru * C + c0, xv[u]);
                    if (MODE >= 1) VecIO<T, VW>::load(dy + ru * C + c0, gv[u]);
                    if (MODE == 1 && RM == 1) VecIO<T, VW>::load(y + ru * C + c0, yv[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (r + (int64_t)u * L.rl >= r_end) break;
#pragma unroll
                for (int i = 0; i < VW; ++i) {
                    if (MODE == 2) xv[u][i] = to_float<T>(from_float<T>(xv[u][i] + gv[u][i]));  // the value as stored
                    if (MODE == 0 || MODE == 2) {
                        s0[i] += (double)xv[u][i];
                        s1[i] += (double)xv[u][i] * (double)xv[u][i];
                    } else {
                        if (RM == 2) yv[u][i] = bn_value<T>(xv[u][i], fsc[i], fsh[i]);
                        const float dz = (RM == 0 || yv[u][i] > 0.f) ? gv[u][i] : 0.f;
                        s0[i] += (double)dz;
                        s1[i] += (double)(dz * ((xv[u][i] - mu[i]) * is[i]));
                    }
                }
                if (MODE == 2) VecIO<T, VW>::store(out + (r + (int64_t)u * L.rl) * C + c0, xv[u]);
            }
        }
    }
    // combine the row lanes of each channel vector: a fixed tree over the row lanes, all channels of the vector at once
#pragma unroll
    for (int i = 0; i < VW; ++i) {
        red[i][tid][0] = s0[i];
        red[i][tid][1] = s1[i];
    }
    __syncthreads();
    int w = 1;
    while (w < L.rl) w <<= 1;
    for (w >>= 1; w > 0; w >>= 1) {
        if (active && rlane < w && rlane + w < L.rl) {
            const int other = tid + w * L.cvb;
#pragma unroll
            for (int i = 0; i < VW; ++i) {
                red[i][tid][0] += red[i][other][0];
                red[i][tid][1] += red[i][other][1];
            }
        }
        __syncthreads();
    }
    if (active && rlane == 0) {
#pragma unroll
        for (int i = 0; i < VW; ++i) {
            double* dst = part + ((int64_t)blockIdx.x * C + c0 + i) * 2;
            dst[0] = red[i][tid][0];
            dst[1] = red[i][tid][1];
        }
    }
}

// Merging the partials.  The partials of a conv epilogue can be thousands of rows (one per row tile), so a
// workgroup of kMergeLanes x 4 threads takes 4 channels and reads whole 64-byte row segments, up to 8 loads
// in flight per thread and added in row order; then a fixed tree over the row lanes.  Returns the two sums
// of channel blockIdx.x * 4 + (threadIdx.x & 3) to the threads of row lane 0.
constexpr int kMergeLanes = 64;
typedef __attribute__((ext_vector_type(2))) double f64x2;
__device__ inline void merge_partials(const double* __restrict__ part, int nblk, int C, double (&red)[kMergeLanes][4][2],
                                      double* sa, double* sb)
{
    const int cq = threadIdx.x & 3, r = threadIdx.x >> 2;
    const int c = blockIdx.x * 4 + cq;
    double a = 0.0, b = 0.0;
    if (c < C)
        for (int k0 = r; k0 < nblk; k0 += kMergeLanes * 8) {
            f64x2 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int k = k0 + kMergeLanes * u;
                v[u] = k < nblk ? *(const f64x2*)(part + ((int64_t)k * C + c) * 2) : f64x2{0.0, 0.0};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                a += v[u][0];
                b += v[u][1];
            }
        }
    red[r][cq][0] = a;
    red[r][cq][1] = b;
    __syncthreads();
    for (int w = kMergeLanes / 2; w > 0; w >>= 1) {
        if (r < w) {
            red[r][cq][0] += red[r + w][cq][0];
            red[r][cq][1] += red[r + w][cq][1];
        }
        __syncthreads();
    }
    *sa = red[0][cq][0];
    *sb = red[0][cq][1];
}

// Forward: mean, invstd, coef = {scale, shift}.
struct BnStatOut {
    const double* part;
    float *mean, *invstd, *coef;
};
__global__ __launch_bounds__(kMergeLanes * 4) void bn_fwd_finalize_kernel(BnStatOut o0, BnStatOut o1, int nblk, int C,
                                                                          double inv_M, float eps,
                                                                          const float* __restrict__ gamma,
                                                                          const float* __restrict__ beta)
{
    __shared__ double red[kMergeLanes][4][2];
    const BnStatOut o = blockIdx.y ? o1 : o0;
    double a, b;
    merge_partials(o.part, nblk, C, red, &a, &b);
    const int c = blockIdx.x * 4 + (threadIdx.x & 3);
    if ((threadIdx.x >> 2) == 0 && c < C) {
        const double mu = a * inv_M;
        double var = b * inv_M - mu * mu;
        if (var < 0.0) var = 0.0;
        const double is = 1.0 / sqrt(var + (double)eps);
        o.mean[c] = (float)mu;
        o.invstd[c] = (float)is;
        const double sc = (double)gamma[c] * is;
        o.coef[c] = (float)sc;
        o.coef[C + c] = (float)((double)beta[c] - mu * sc);
    }
}

// Backward: dgamma, dbeta and dx = c1*dz - c2*x + c0 with
// c1 = gamma*invstd, c2 = c1*invstd*dgamma/M, c0 = c2*mean - c1*dbeta/M.
__global__ __launch_bounds__(kMergeLanes * 4) void bn_bwd_finalize_kernel(const double* __restrict__ part, int nblk, int C,
                                                                          double inv_M, const float* __restrict__ gamma,
                                                                          const float* __restrict__ mean,
                                                                          const float* __restrict__ invstd,
                                                                          float* __restrict__ dgamma,
                                                                          float* __restrict__ dbeta, float* __restrict__ coef)
{
    __shared__ double red[kMergeLanes][4][2];
    double a, b;
    merge_partials(part, nblk, C, red, &a, &b);
    const int c = blockIdx.x * 4 + (threadIdx.x & 3);
    if ((threadIdx.x >> 2) == 0 && c < C) {
        dbeta[c] = (float)a;
        dgamma[c] = (float)b;
        const double c1 = (double)gamma[c] * (double)invstd[c];
        const double c2 = c1 * (double)invstd[c] * b * inv_M;
        coef[c] = (float)c1;
        coef[C + c] = (float)c2;
        coef[2 * C + c] = (float)(c2 * (double)mean[c] - c1 * a * inv_M);
    }
}

// y = [relu](scale*x + shift [+ res]); blockIdx.y selects the instance of a twin launch
struct BnApplyIo {
    const void* x;
    const void* res;
    void* y;
    const float* coef;
};
template <typename T, int VW, bool RELU, bool HAS_RES>
__global__ __launch_bounds__(kThreads) void bn_fwd_apply_kernel(BnApplyIo io0, BnApplyIo io1, int64_t nvec, int C, int cv)
{
    const BnApplyIo io = blockIdx.y ? io1 : io0;
    const T* __restrict__ x = (const T*)io.x;
    const T* __restrict__ res = (const T*)io.res;
    T* __restrict__ y = (T*)io.y;
    const float* __restrict__ coef = io.coef;
    // channel vector of element i = i mod cv, carried along the grid-stride loop instead of divided out each trip
    const uint32_t step = gridDim.x * kThreads, step_c = step % (uint32_t)cv;
    uint32_t cvi = (blockIdx.x * kThreads + threadIdx.x) % (uint32_t)cv;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec;
         i += step, cvi = cvi + step_c >= (uint32_t)cv ? cvi + step_c - (uint32_t)cv : cvi + step_c) {
        const int c0 = (int)cvi * VW;
        float xv[VW], rv[VW], ov[VW];
        VecIO<T, VW>::load(x + i * VW, xv);
        if (HAS_RES) VecIO<T, VW>::load(res + i * VW, rv);
#pragma unroll
        for (int k = 0; k < VW; ++k) {
            float v = __builtin_fmaf(xv[k], coef[c0 + k], coef[C + c0 + k]);
            if (HAS_RES) v += rv[k];
            if (RELU) v = v > 0.f ? v : 0.f;
            ov[k] = v;
        }
        VecIO<T, VW>::store(y + i * VW, ov);
    }
}

// dz = dy*[y>0] (y as stored, or formed again from x: RM as in bn_sums_kernel);  dx = [dx_prev +] c1*dz - c2*x + c0;  dres (+)= dz.  dx_prev is dx itself (accumulate in place)
// or another tensor's gradient that reaches the same input (the shortcut of a pre-activation unit).
template <typename T, int VW, int RM, bool HAS_RES, bool RES_ACC, bool DX_ACC>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                                const T* __restrict__ y, T* dx, const T* dx_prev,
                                                                T* __restrict__ dres, const float* __restrict__ coef,
                                                                int64_t nvec, int C, int cv, const float* __restrict__ fcoef)
{
    // channel vector of element i = i mod cv, carried along the grid-stride loop instead of divided out each trip
    const uint32_t step = gridDim.x * kThreads, step_c = step % (uint32_t)cv;
    uint32_t cvi = (blockIdx.x * kThreads + threadIdx.x) % (uint32_t)cv;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec;
         i += step, cvi = cvi + step_c >= (uint32_t)cv ? cvi + step_c - (uint32_t)cv : cvi + step_c) {
        const int c0 = (int)cvi * VW;
        float gv[VW], xv[VW], yv[VW], ov[VW], rv[VW];
        VecIO<T, VW>::load(dy + i * VW, gv);
        VecIO<T, VW>::load(x + i * VW, xv);
        if (RM == 1) VecIO<T, VW>::load(y + i * VW, yv);
        if (DX_ACC) VecIO<T, VW>::load(dx_prev + i * VW, ov);
        if (HAS_RES && RES_ACC) VecIO<T, VW>::load(dres + i * VW, rv);
#pragma unroll
        for (int k = 0; k < VW; ++k) {
            if (RM == 2) yv[k] = bn_value<T>(xv[k], fcoef[c0 + k], fcoef[C + c0 + k]);
            const float dz = (RM == 0 || yv[k] > 0.f) ? gv[k] : 0.f;
            const float d = coef[c0 + k] * dz - coef[C + c0 + k] * xv[k] + coef[2 * C + c0 + k];
            ov[k] = DX_ACC ? ov[k] + d : d;
            if (HAS_RES) rv[k] = RES_ACC ? rv[k] + dz : dz;
        }
        VecIO<T, VW>::store(dx + i * VW, ov);
        if (HAS_RES) VecIO<T, VW>::store(dres + i * VW, rv);
    }
}

// ---- batch norm + ReLU + max pool in one pass (bf16) ---------------------------------------------------------
// For a batch norm whose only reader is a max pool: y = relu(scale * x + shift) is formed per window tap exactly as
// bn_fwd_apply_kernel would store it (same expression, same rounding) and never written; the pooled tensor and the
// chosen taps are the same bits the two separate kernels leave.  After the ReLU every value is a non-negative bf16, so
// values order like their bit patterns: per channel the kernel keeps one 32-bit key = value bits << 16 | (15 - tap) and
// takes the unsigned maximum, which is the largest value and, among equal ones, the first tap of the row-major window
// scan (the rule of maxpool_fwd_kernel).  A thread owns 8 consecutive channels of one output pixel; all taps of a
// window are loaded before the first is used (out-of-image taps read a clamped address and are masked out).
// Workgroup ids are dealt round-robin to the 8 XCDs; the remap gives each XCD one contiguous eighth of the output per
// grid-stride trip, so the input rows two neighbouring output rows share are fetched into one L2, once.
template <int K>
__global__ __launch_bounds__(kThreads) void bn_relu_maxpool_bf16_kernel(const bf16_t* __restrict__ x,
                                                                        const float* __restrict__ coef,
                                                                        bf16_t* __restrict__ y, uint8_t* __restrict__ arg,
                                                                        int N, int H, int W, int C, int Ho, int Wo, int k_rt,
                                                                        int stride, int pad)
{
    const int k = K ? K : k_rt;
    const uint32_t cv = (uint32_t)(C / 8);
    const uint32_t total = (uint32_t)N * Ho * Wo * cv;
    const uint32_t nb = gridDim.x, lb = (blockIdx.x & 7u) * (nb >> 3) + (blockIdx.x >> 3);
    for (uint32_t i = lb * kThreads + threadIdx.x; i < total; i += nb * kThreads) {
        const uint32_t t = i / cv;
        const int c = (int)(i - t * cv) * 8;
        const uint32_t t2 = t / (uint32_t)Wo;
        const int wo = (int)(t - t2 * Wo);
        const int n = (int)(t2 / (uint32_t)Ho), ho = (int)(t2 - (uint32_t)n * Ho);
        float sc[8], sh[8];
#pragma unroll
        for (int e = 0; e < 8; e += 4) {
            const f32x4 a = *(const f32x4*)(coef + c + e), b = *(const f32x4*)(coef + C + c + e);
            sc[e] = a.x; sc[e + 1] = a.y; sc[e + 2] = a.z; sc[e + 3] = a.w;
            sh[e] = b.x; sh[e + 1] = b.y; sh[e + 2] = b.z; sh[e + 3] = b.w;
        }
        uint32_t key[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) key[e] = 0u;
        auto tap = [&](int r, int s, u32x4 v) {
            const int hi = ho * stride + r - pad, wi = wo * stride + s - pad;
            const bool valid = (unsigned)hi < (unsigned)H && (unsigned)wi < (unsigned)W;
            const uint32_t code = (uint32_t)(15 - (r * k + s));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float lo = __builtin_fmaf(__uint_as_float(v[e] << 16), sc[2 * e], sh[2 * e]);
                float hi2 = __builtin_fmaf(__uint_as_float(v[e] & 0xffff0000u), sc[2 * e + 1], sh[2 * e + 1]);
                lo = lo > 0.f ? lo : 0.f;
                hi2 = hi2 > 0.f ? hi2 : 0.f;
                const uint32_t pk = pack_bf16x2(lo, hi2);
                const uint32_t k0 = valid ? ((pk << 16) | code) : 0u, k1 = valid ? ((pk & 0xffff0000u) | code) : 0u;
                key[2 * e] = key[2 * e] > k0 ? key[2 * e] : k0;
                key[2 * e + 1] = key[2 * e + 1] > k1 ? key[2 * e + 1] : k1;
            }
        };
        auto addr = [&](int r, int s) {
            int hi = ho * stride + r - pad, wi = wo * stride + s - pad;
            hi = hi < 0 ? 0 : (hi >= H ? H - 1 : hi);
            wi = wi < 0 ? 0 : (wi >= W ? W - 1 : wi);
            return (const u32x4*)(x + (((int64_t)n * H + hi) * W + wi) * C + c);
        };
        if (K) {
            u32x4 v[K ? K * K : 1];
#pragma unroll
            for (int r = 0; r < K; ++r)
#pragma unroll
                for (int s = 0; s < K; ++s) v[r * K + s] = *addr(r, s);
#pragma unroll
            for (int r = 0; r < K; ++r)
#pragma unroll
                for (int s = 0; s < K; ++s) tap(r, s, v[r * K + s]);
        } else {
            for (int r = 0; r < k; ++r)
                for (int s = 0; s < k; ++s) tap(r, s, *addr(r, s));
        }
        u32x4 o;
        uint32_t a0 = 0u, a1 = 0u;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o[e] = (key[2 * e] >> 16) | (key[2 * e + 1] & 0xffff0000u);
            a0 |= (15u - (key[e] & 15u)) << (8 * e);
            a1 |= (15u - (key[4 + e] & 15u)) << (8 * e);
        }
        *(u32x4*)(y + (int64_t)i * 8) = o;
        if (arg) *(u32x2*)(arg + (int64_t)i * 8) = u32x2{a0, a1};
    }
}

int plan_rows(int64_t M, const RowLayout& L, int* nblk)
{
    // every thread should see >= 4 rows (one trip of the summing loop); at most kMaxPartialBlocks workgroups
    int64_t rows = (int64_t)L.rl * 4;
    int64_t blocks = (M + rows - 1) / rows;
    if (blocks > kMaxPartialBlocks) {
        blocks = kMaxPartialBlocks;
        rows = (M + blocks - 1) / blocks;
        blocks = (M + rows - 1) / rows;
    }
    *nblk = (int)blocks;
    return (int)rows;
}

inline int apply_grid(int64_t nvec)
{
    int64_t g = (nvec + kThreads - 1) / kThreads;
    const int64_t cap = 256 * 16;
    return (int)(g < cap ? (g < 1 ? 1 : g) : cap);
}

template <typename T, int VW>
int bn_forward_t(const void* x, const void* res, void* y, const float* gamma, const float* beta, float eps, int64_t M,
                 int C, bool relu, const BnBuffers& buf, hipStream_t st, int presummed, const BnForwardTwin* tw, bool stats_only)
{
    const RowLayout L = make_layout(C, VW);
    int nblk;
    const int rows = plan_rows(M, L, &nblk);
    const unsigned ni = tw ? 2 : 1;
    const dim3 grid(nblk, ceil_div(L.cv, L.cvb), ni);
    const double tensor_bytes = (double)M * C * sizeof(T) * ni;
    if (presummed > 0) {
        nblk = presummed;
    } else {
        ProfScope ps(sizeof(T) == 2 ? "bn_stats<bf16>" : "bn_stats<fp32>", tensor_bytes, 1);
        DSP_LAUNCH(ps, (bn_sums_kernel<T, VW, 0, 0>), grid, dim3(kThreads), 0, st, (const T*)x, (const T*)nullptr,
                   (const T*)nullptr, (const float*)nullptr, (const float*)nullptr, buf.partial, M, C, L, rows,
                   (const T*)(tw ? tw->x : nullptr), tw ? tw->buf.partial : nullptr, AddOut<T>{}, (const float*)nullptr);
    }
    {
        const BnStatOut o0{buf.partial, buf.mean, buf.invstd, buf.coef};
        const BnStatOut o1 = tw ? BnStatOut{tw->buf.partial, tw->buf.mean, tw->buf.invstd, tw->buf.coef} : o0;
        ProfScope ps("bn_fwd_finalize", (double)nblk * C * 16.0 * ni, 1);
        DSP_LAUNCH(ps, bn_fwd_finalize_kernel, dim3(ceil_div(C, 4), ni), dim3(kMergeLanes * 4), 0, st, o0, o1, nblk, C,
                   1.0 / (double)M, eps, gamma, beta);
    }
    if (stats_only) {
        DSP_HIP(hipGetLastError());
        return DSP_OK;
    }
    const int64_t nvec = M * (C / VW);
    const dim3 ag(apply_grid(nvec), ni);
    const BnApplyIo io0{x, res, y, buf.coef};
    const BnApplyIo io1 = tw ? BnApplyIo{tw->x, tw->res, tw->y, tw->buf.coef} : io0;
    ProfScope ps(sizeof(T) == 2 ? "bn_apply_relu<bf16>" : "bn_apply_relu<fp32>", tensor_bytes * (res ? 3 : 2), 1);
#define BN_APPLY(R, H) \
    DSP_LAUNCH(ps, (bn_fwd_apply_kernel<T, VW, R, H>), ag, dim3(kThreads), 0, st, io0, io1, nvec, C, L.cv)
    if (relu) {
        if (res) BN_APPLY(true, true); else BN_APPLY(true, false);
    } else {
        if (res) BN_APPLY(false, true); else BN_APPLY(false, false);
    }
#undef BN_APPLY
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

template <typename T, int VW, int RM>
int bn_backward_t(const void* dy, const void* x, const void* y, void* dx, void* dres, bool racc, bool xacc,
                  const float* gamma, float* dgamma, float* dbeta, int64_t M, int C, const BnBuffers& buf, hipStream_t st,
                  const void* dx_prev, const float* fcoef)
{
    const RowLayout L = make_layout(C, VW);
    int nblk;
    const int rows = plan_rows(M, L, &nblk);
    const dim3 grid(nblk, ceil_div(L.cv, L.cvb));
    const double tensor_bytes = (double)M * C * sizeof(T);
    {
        ProfScope ps(sizeof(T) == 2 ? "bn_bwd_reduce<bf16>" : "bn_bwd_reduce<fp32>", tensor_bytes * (RM == 1 ? 3 : 2), 1);
        DSP_LAUNCH(ps, (bn_sums_kernel<T, VW, 1, RM>), grid, dim3(kThreads), 0, st, (const T*)x, (const T*)dy,
                   (const T*)y, (const float*)buf.mean, (const float*)buf.invstd, buf.partial, M, C, L, rows,
                   (const T*)nullptr, (double*)nullptr, AddOut<T>{}, fcoef);
    }
    {
        ProfScope ps("bn_bwd_finalize", (double)nblk * C * 16.0, 1);
        DSP_LAUNCH(ps, bn_bwd_finalize_kernel, dim3(ceil_div(C, 4)), dim3(kMergeLanes * 4), 0, st, (const double*)buf.partial, nblk, C,
                   1.0 / (double)M, gamma, (const float*)buf.mean, (const float*)buf.invstd, dgamma, dbeta, buf.coef);
    }
    const int64_t nvec = M * (C / VW);
    const dim3 ag(apply_grid(nvec));
    // reads dy, x (y too where the ReLU is decided from the stored output, and the old values where it accumulates);
    // writes dx (and dres)
    ProfScope ps(sizeof(T) == 2 ? "bn_bwd_apply<bf16>" : "bn_bwd_apply<fp32>",
                 tensor_bytes * (2 + (RM == 1 ? 1 : 0) + 1 + (xacc ? 1 : 0) + (dres ? 1 + (racc ? 1 : 0) : 0)), 1);
#define BN_BAPPLY(H, RA, XA)                                                                                   \
    DSP_LAUNCH(ps, (bn_bwd_apply_kernel<T, VW, (H && RM == 2) ? 1 : RM, H, RA, XA>), ag, dim3(kThreads), 0, st, \
               (const T*)dy, (const T*)x, (const T*)y, (T*)dx, (const T*)dx_prev, (T*)dres, (const float*)buf.coef,   \
               nvec, C, L.cv, fcoef)
    if (dres) {
        if (racc) { if (xacc) BN_BAPPLY(true, true, true); else BN_BAPPLY(true, true, false); }
        else      { if (xacc) BN_BAPPLY(true, false, true); else BN_BAPPLY(true, false, false); }
    } else {
        if (xacc) BN_BAPPLY(false, false, true); else BN_BAPPLY(false, false, false);
    }
#undef BN_BAPPLY
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

}  // namespace

int bn_max_partial_blocks() { return kMaxPartialBlocks; }

template <typename T, int VW>
int add_stats_t(const void* a, const void* b, void* y, int64_t M, int C, double* partial, hipStream_t st,
                const AddStatsTwin* tw)
{
    const RowLayout L = make_layout(C, VW);
    int nblk;
    const int rows = plan_rows(M, L, &nblk);
    const unsigned ni = tw ? 2 : 1;
    const dim3 grid(nblk, ceil_div(L.cv, L.cvb), ni);
    ProfScope ps("add_fwd_stats", (double)M * C * sizeof(T) * 3.0 * ni, 1);
    DSP_LAUNCH(ps, (bn_sums_kernel<T, VW, 2, 0>), grid, dim3(kThreads), 0, st, (const T*)a, (const T*)b, (const T*)nullptr,
               (const float*)nullptr, (const float*)nullptr, partial, M, C, L, rows, (const T*)(tw ? tw->a : nullptr),
               tw ? tw->partial : nullptr, (AddOut<T>{(T*)y, (const T*)(tw ? tw->b : nullptr), (T*)(tw ? tw->y : nullptr)}),
               (const float*)nullptr);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

static bool add_stats_vec(int dtype, int C) { return C % (dtype == DSP_BF16 ? 8 : 4) == 0; }

int add_stats_blocks(int dtype, int64_t M, int C)
{
    const int vw = add_stats_vec(dtype, C) ? (dtype == DSP_BF16 ? 8 : 4) : 1;
    int nblk;
    (void)plan_rows(M, make_layout(C, vw), &nblk);
    return nblk;
}

int launch_add_forward_stats(int dtype, const void* a, const void* b, void* y, int64_t M, int C, double* partial,
                             hipStream_t st, const AddStatsTwin* twin)
{
    DSP_REQUIRE(a && b && y && partial && M > 0 && C > 0, DSP_EINVAL, "add + statistics: bad argument");
    if (twin) DSP_REQUIRE(twin->a && twin->b && twin->y && twin->partial, DSP_EINVAL, "add + statistics: incomplete second instance");
    if (dtype == DSP_BF16) {
        if (add_stats_vec(dtype, C)) return add_stats_t<bf16_t, 8>(a, b, y, M, C, partial, st, twin);
        return add_stats_t<bf16_t, 1>(a, b, y, M, C, partial, st, twin);
    }
    if (add_stats_vec(dtype, C)) return add_stats_t<float, 4>(a, b, y, M, C, partial, st, twin);
    return add_stats_t<float, 1>(a, b, y, M, C, partial, st, twin);
}

int launch_bn_forward(int dtype, const void* x, const void* res, void* y, const float* gamma, const float* beta,
                      float eps, int64_t M, int C, bool relu, const BnBuffers& buf, hipStream_t st, int presummed,
                      const BnForwardTwin* twin, bool stats_only)
{
    DSP_REQUIRE(M > 0 && C > 0 && presummed >= 0, DSP_EINVAL, "bn: bad shape");
    if (twin)
        DSP_REQUIRE(twin->x && (twin->y || stats_only) && (twin->res != nullptr) == (res != nullptr), DSP_EINVAL,
                    "bn forward: incomplete second instance");
    if (dtype == DSP_BF16) {
        if (C % 8 == 0) return bn_forward_t<bf16_t, 8>(x, res, y, gamma, beta, eps, M, C, relu, buf, st, presummed, twin, stats_only);
        return bn_forward_t<bf16_t, 1>(x, res, y, gamma, beta, eps, M, C, relu, buf, st, presummed, twin, stats_only);
    }
    if (C % 4 == 0) return bn_forward_t<float, 4>(x, res, y, gamma, beta, eps, M, C, relu, buf, st, presummed, twin, stats_only);
    return bn_forward_t<float, 1>(x, res, y, gamma, beta, eps, M, C, relu, buf, st, presummed, twin, stats_only);
}

int launch_bn_apply(int dtype, const void* x, void* y, const float* coef, int64_t M, int C, bool relu, hipStream_t st)
{
    DSP_REQUIRE(M > 0 && C > 0 && x && y && coef, DSP_EINVAL, "bn apply: bad argument");
    const BnApplyIo io{x, nullptr, y, coef};
    const double bytes = (double)M * C * dtype_size(dtype) * 2;
#define BN_APPLY1(T, VW)                                                                                               \
    do {                                                                                                               \
        const int64_t nvec = M * (C / VW);                                                                             \
        ProfScope ps(sizeof(T) == 2 ? "bn_apply_relu<bf16>" : "bn_apply_relu<fp32>", bytes, 1);                        \
        if (relu) DSP_LAUNCH(ps, (bn_fwd_apply_kernel<T, VW, true, false>), dim3(apply_grid(nvec)), dim3(kThreads), 0, st, io, io, nvec, C, C / VW); \
        else DSP_LAUNCH(ps, (bn_fwd_apply_kernel<T, VW, false, false>), dim3(apply_grid(nvec)), dim3(kThreads), 0, st, io, io, nvec, C, C / VW);    \
    } while (0)
    if (dtype == DSP_BF16) {
        if (C % 8 == 0) BN_APPLY1(bf16_t, 8); else BN_APPLY1(bf16_t, 1);
    } else {
        if (C % 4 == 0) BN_APPLY1(float, 4); else BN_APPLY1(float, 1);
    }
#undef BN_APPLY1
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

bool bn_relu_maxpool_supported(int dtype, int C, int k) { return dtype == DSP_BF16 && C % 8 == 0 && k >= 1 && k <= 4; }

int launch_bn_relu_maxpool_forward(int dtype, const void* x, const float* coef, void* y, uint8_t* argmax, int N, int H, int W,
                                   int C, int k, int stride, int pad, hipStream_t st)
{
    DSP_REQUIRE(bn_relu_maxpool_supported(dtype, C, k), DSP_EINVAL, "bn + relu + max pool: bf16, channels in runs of 8, window <= 4 x 4");
    DSP_REQUIRE(x && coef && y && N > 0 && stride >= 1 && pad >= 0 && pad < k && H + 2 * pad >= k && W + 2 * pad >= k, DSP_EINVAL,
                "bn + relu + max pool: bad argument");
    DSP_REQUIRE((int64_t)N * H * W * C < (1ll << 31), DSP_EINVAL, "bn + relu + max pool: tensors of 2^31 elements or more are not supported");
    DSP_REQUIRE(((uintptr_t)x % 16) == 0 && ((uintptr_t)y % 16) == 0 && ((uintptr_t)argmax % 8) == 0 && ((uintptr_t)coef % 16) == 0,
                DSP_EINVAL, "bn + relu + max pool: unaligned tensor");
    const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
    const int64_t total = (int64_t)N * Ho * Wo * (C / 8);
    int64_t grid = (total + kThreads - 1) / kThreads;
    grid = (grid + 7) / 8 * 8;
    if (grid > 256 * 32) grid = 256 * 32;
    ProfScope ps("bn_relu_maxpool_fwd<bf16>", ((double)N * H * W * C + (double)N * Ho * Wo * C) * 2.0 + (double)N * Ho * Wo * C, 1);
    if (k == 3)
        DSP_LAUNCH(ps, (bn_relu_maxpool_bf16_kernel<3>), dim3((unsigned)grid), dim3(kThreads), 0, st, (const bf16_t*)x, coef, (bf16_t*)y,
                   argmax, N, H, W, C, Ho, Wo, k, stride, pad);
    else
        DSP_LAUNCH(ps, (bn_relu_maxpool_bf16_kernel<0>), dim3((unsigned)grid), dim3(kThreads), 0, st, (const bf16_t*)x, coef, (bf16_t*)y,
                   argmax, N, H, W, C, Ho, Wo, k, stride, pad);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_bn_backward(int dtype, const void* dy, const void* x, const void* y, void* dx, void* dres,
                       bool dres_accumulate, bool dx_accumulate, const float* gamma, float* dgamma, float* dbeta,
                       int64_t M, int C, bool relu, const BnBuffers& buf, hipStream_t st, const void* dx_add,
                       const float* fwd_coef)
{
    DSP_REQUIRE(M > 0 && C > 0, DSP_EINVAL, "bn: bad shape");
    const void* dx_prev = dx_add ? dx_add : dx;
    if (dx_add) dx_accumulate = true;
    // the ReLU of a batch norm without residual can be decided from x (no read of y) when the caller still has the
    // forward pass's {scale, shift}
    const bool from_x = relu && fwd_coef && !dres;
    DSP_REQUIRE(!relu || from_x || y, DSP_EINVAL, "bn backward: the ReLU needs the stored output");
#define BN_BWD_RM(T, VW, RM)                                                                                        \
    bn_backward_t<T, VW, RM>(dy, x, y, dx, dres, dres_accumulate, dx_accumulate, gamma, dgamma, dbeta, M, C, buf, st, \
                             dx_prev, fwd_coef)
#define BN_BWD(T, VW) (!relu ? BN_BWD_RM(T, VW, 0) : from_x ? BN_BWD_RM(T, VW, 2) : BN_BWD_RM(T, VW, 1))
    if (dtype == DSP_BF16) {
        if (C % 8 == 0) return BN_BWD(bf16_t, 8);
        return BN_BWD(bf16_t, 1);
    }
    if (C % 4 == 0) return BN_BWD(float, 4);
    return BN_BWD(float, 1);
#undef BN_BWD
#undef BN_BWD_RM
}

}  // namespace dsp
