// Small layers that close the loop of a block (max-pool, global average pool, linear head,
// softmax cross-entropy) and the fused momentum-SGD update.  None of them is a contraction worth
// the matrix cores; they are written as coalesced NHWC streams.
#include "common.h"

#include <algorithm>
#include <vector>

namespace dsp {
namespace {

constexpr int kThreads = 256;

inline int grid_for(int64_t n, int cap = 256 * 32)
{
    int64_t g = (n + kThreads - 1) / kThreads;
    if (g < 1) g = 1;
    return (int)(g < cap ? g : cap);
}

// ---- max pool ------------------------------------------------------------------------------------
// Window scan in row-major order, strict ">" so the first maximum wins; argmax keeps r*k+s.
// A thread owns VW consecutive channels of one output pixel (one 16-byte run per tap when VW > 1).
template <typename T, int VW>
__global__ __launch_bounds__(kThreads) void maxpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                               uint8_t* __restrict__ arg, int N, int H, int W, int C,
                                                               int Ho, int Wo, int k, int stride, int pad)
{
    // element counts are below 2^31 (checked by the launcher): 32-bit index arithmetic
    const uint32_t cv = (uint32_t)(C / VW);
    const uint32_t total = (uint32_t)N * Ho * Wo * cv;
    for (uint32_t i = blockIdx.x * kThreads + threadIdx.x; i < total; i += gridDim.x * kThreads) {
        uint32_t t = i / cv;
        const int c = (int)(i - t * cv) * VW;
        const uint32_t t2 = t / (uint32_t)Wo;
        const int wo = (int)(t - t2 * Wo);
        const int n = (int)(t2 / (uint32_t)Ho), ho = (int)(t2 - (uint32_t)n * Ho);
        float best[VW];
        int a[VW];
#pragma unroll
        for (int v = 0; v < VW; ++v) {
            best[v] = -INFINITY;
            a[v] = 255;
        }
        for (int r = 0; r < k; ++r)
            for (int s = 0; s < k; ++s) {
                const int hi = ho * stride + r - pad, wi = wo * stride + s - pad;
                if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                float xv[VW];
                VecIO<T, VW>::load(x + (((int64_t)n * H + hi) * W + wi) * C + c, xv);
#pragma unroll
                for (int v = 0; v < VW; ++v)
                    if (xv[v] > best[v]) {
                        best[v] = xv[v];
                        a[v] = r * k + s;
                    }
            }
        const int64_t o = (((int64_t)n * Ho + ho) * Wo + wo) * C + c;
        VecIO<T, VW>::store(y + o, best);
        if (arg)
#pragma unroll
            for (int v = 0; v < VW; ++v) arg[o + v] = (uint8_t)a[v];
    }
}

// dx[n,hi,wi,c] (+)= sum of dy over the windows whose recorded argmax is this pixel.
template <typename T, int VW, bool ACC>
__global__ __launch_bounds__(kThreads) void maxpool_bwd_kernel(const T* __restrict__ dy, const uint8_t* __restrict__ arg,
                                                               T* __restrict__ dx, int N, int H, int W, int C, int Ho,
                                                               int Wo, int k, int stride, int pad)
{
    // element counts are below 2^31 (checked by the launcher): 32-bit index arithmetic
    const uint32_t cv = (uint32_t)(C / VW);
    const uint32_t total = (uint32_t)N * H * W * cv;
    for (uint32_t i = blockIdx.x * kThreads + threadIdx.x; i < total; i += gridDim.x * kThreads) {
        uint32_t t = i / cv;
        const int c = (int)(i - t * cv) * VW;
        const uint32_t t2 = t / (uint32_t)W;
        const int wi = (int)(t - t2 * W);
        const int n = (int)(t2 / (uint32_t)H), hi = (int)(t2 - (uint32_t)n * H);
        float s[VW];
#pragma unroll
        for (int v = 0; v < VW; ++v) s[v] = 0.f;
        // windows (ho, wo) that contain this pixel: tap r = hi + pad - ho*stride in [0, k), same for columns;
        // walked with r and q ascending (ho and wo descending), the order the sums have always been taken in
        const int hn = hi + pad, wn = wi + pad;
        int ho_hi = (int)((uint32_t)hn / (uint32_t)stride), wo_hi = (int)((uint32_t)wn / (uint32_t)stride);
        const int ho_lo = hn - k + 1 > 0 ? (int)((uint32_t)(hn - k + stride) / (uint32_t)stride) : 0;
        const int wo_lo = wn - k + 1 > 0 ? (int)((uint32_t)(wn - k + stride) / (uint32_t)stride) : 0;
        if (ho_hi > Ho - 1) ho_hi = Ho - 1;
        if (wo_hi > Wo - 1) wo_hi = Wo - 1;
        for (int ho = ho_hi; ho >= ho_lo; --ho) {
            const int r = hn - ho * stride;
            for (int wo = wo_hi; wo >= wo_lo; --wo) {
                const int q = wn - wo * stride;
                const int64_t o = (((int64_t)n * Ho + ho) * Wo + wo) * C + c;
                float gv[VW];
                VecIO<T, VW>::load(dy + o, gv);
#pragma unroll
                for (int v = 0; v < VW; ++v)
                    if (arg[o + v] == r * k + q) s[v] += gv[v];
            }
        }
        const int64_t o = (((int64_t)n * H + hi) * W + wi) * C + c;
        if (ACC) {
            float old[VW];
            VecIO<T, VW>::load(dx + o, old);
#pragma unroll
            for (int v = 0; v < VW; ++v) s[v] += old[v];
        }
        VecIO<T, VW>::store(dx + o, s);
    }
}

// y[n][c] = mean over the HW positions of x[n][.][c].  A workgroup owns one image and up to 256
// channels; CW threads cover the channels (coalesced rows), 256 / CW thread rows split the positions
// and are added in row order.
template <typename T>
__global__ __launch_bounds__(kThreads) void gap_fwd_kernel(const T* __restrict__ x, float* __restrict__ y, int N, int HW,
                                                           int C, int cw)
{
    __shared__ float red[kThreads];
    const int n = blockIdx.x, c = blockIdx.y * cw + threadIdx.x % cw, row = threadIdx.x / cw, rows = kThreads / cw;
    float s = 0.f;
    if (c < C && row < rows) {
        const T* src = x + (int64_t)n * HW * C + c;
#pragma unroll 8
        for (int p = row; p < HW; p += rows) s += to_float<T>(src[(int64_t)p * C]);
    }
    red[threadIdx.x] = s;
    __syncthreads();
    if (row == 0 && c < C) {
        for (int k = 1; k < rows; ++k) s += red[k * cw + threadIdx.x];
        y[n * C + c] = s / (float)HW;
    }
}

template <typename T, bool ACC>
__global__ void gap_bwd_kernel(const float* __restrict__ dy, T* __restrict__ dx, int N, int HW, int C)
{
    const int64_t total = (int64_t)N * HW * C;
    const float inv = 1.f / (float)HW;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
        const int c = (int)(i % C), n = (int)(i / ((int64_t)HW * C));
        const float g = dy[n * C + c] * inv;
        dx[i] = from_float<T>(ACC ? to_float<T>(dx[i]) + g : g);
    }
}

// ---- linear head (fp32) ----------------------------------------------------------------------------
// z[n][j] = sum_c x[n][c] w[j][c] + bias[j]: lanes stride over c, fixed shuffle tree per output.
constexpr int kLinearJ = 8;
__global__ __launch_bounds__(kThreads) void linear_fwd_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                              const float* __restrict__ bias, float* __restrict__ z, int N,
                                                              int Cin, int Cout)
{
    // a wave forms kLinearJ outputs of one sample (x[n] is read once for all of them), the four waves of a
    // workgroup take four samples against the same rows of w; each output is summed as before: lane-strided
    // partial sums over c, then a shuffle tree
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int jblocks = (Cout + kLinearJ - 1) / kLinearJ;
    const int j0 = (int)(blockIdx.x % jblocks) * kLinearJ, n = (int)(blockIdx.x / jblocks) * (kThreads / 64) + wave;
    if (n >= N) return;
    float s[kLinearJ];
#pragma unroll
    for (int q = 0; q < kLinearJ; ++q) s[q] = 0.f;
    for (int c = lane; c < Cin; c += 64) {
        const float xv = x[n * Cin + c];
#pragma unroll
        for (int q = 0; q < kLinearJ; ++q)
            if (j0 + q < Cout) s[q] += xv * w[(j0 + q) * Cin + c];
    }
#pragma unroll
    for (int q = 0; q < kLinearJ; ++q) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s[q] += __shfl_down(s[q], off, 64);
        if (lane == 0 && j0 + q < Cout) z[n * Cout + j0 + q] = s[q] + bias[j0 + q];
    }
}

// dx[n][c] = sum_j dz[n][j] w[j][c]
__global__ void linear_bwd_x_kernel(const float* __restrict__ dz, const float* __restrict__ w, float* __restrict__ dx,
                                    int N, int Cin, int Cout)
{
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= N * Cin) return;
    const int n = i / Cin, c = i % Cin;
    float s = 0.f;
    // same order of additions as the plain loop; unrolled so that 8 rows of w are in flight per trip
#pragma unroll 8
    for (int j = 0; j < Cout; ++j) s += dz[n * Cout + j] * w[j * Cin + c];
    dx[i] = s;
}

// dw[j][c] = sum_n dz[n][j] x[n][c];  dbias[j] = sum_n dz[n][j] (column c == Cin).
// A workgroup owns one j and up to cw columns; 256 / cw thread rows split the samples and are
// added in row order.
__global__ __launch_bounds__(kThreads) void linear_bwd_w_kernel(const float* __restrict__ dz, const float* __restrict__ x,
                                                                float* __restrict__ dw, float* __restrict__ dbias, int N,
                                                                int Cin, int Cout, int cw)
{
    __shared__ float red[kThreads];
    const int j = blockIdx.x, c = blockIdx.y * cw + threadIdx.x % cw, row = threadIdx.x / cw, rows = kThreads / cw;
    float s = 0.f;
    if (c <= Cin && row < rows) {
        if (c < Cin) {
#pragma unroll 8
            for (int n = row; n < N; n += rows) s += dz[n * Cout + j] * x[n * Cin + c];
        } else {
#pragma unroll 8
            for (int n = row; n < N; n += rows) s += dz[n * Cout + j];
        }
    }
    red[threadIdx.x] = s;
    __syncthreads();
    if (row == 0 && c <= Cin) {
        for (int k = 1; k < rows; ++k) s += red[k * cw + threadIdx.x];
        if (c < Cin) dw[j * Cin + c] = s; else dbias[j] = s;
    }
}

// ---- softmax cross-entropy --------------------------------------------------------------------------
// One wave per sample: max, sum of exponentials, loss_n = log(sum) - (z_label - max),
// dz = (softmax - onehot)/N.  The mean over samples is taken by a second single-wave kernel.
__global__ __launch_bounds__(64) void softmax_ce_rows_kernel(const float* __restrict__ z,
                                                             const int32_t* __restrict__ labels,
                                                             float* __restrict__ row_loss, float* __restrict__ dz, int N,
                                                             int C)
{
    const int n = blockIdx.x, lane = threadIdx.x;
    const float* zr = z + (int64_t)n * C;
    float mx = -INFINITY;
    for (int c = lane; c < C; c += 64) mx = fmaxf(mx, zr[c]);
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    float se = 0.f;
    for (int c = lane; c < C; c += 64) se += expf(zr[c] - mx);
    for (int off = 32; off > 0; off >>= 1) se += __shfl_xor(se, off, 64);
    const int lab = labels[n];
    const float inv_n = 1.f / (float)N;
    for (int c = lane; c < C; c += 64) {
        const float p = expf(zr[c] - mx) / se;
        dz[(int64_t)n * C + c] = (p - (c == lab ? 1.f : 0.f)) * inv_n;
    }
    // a label outside [0, C) never indexes memory: its sample contributes NaN to the loss
    if (lane == 0) row_loss[n] = (lab >= 0 && lab < C) ? logf(se) - (zr[lab] - mx) : NAN;
}

__global__ __launch_bounds__(64) void mean_kernel(const float* __restrict__ v, float* __restrict__ out, int n)
{
    const int lane = threadIdx.x;
    double s = 0.0;
    for (int i = lane; i < n; i += 64) s += (double)v[i];
    for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
    if (lane == 0) *out = (float)(s / (double)n);
}

// ---- momentum SGD + shadow refresh ---------------------------------------------------------------
// Eq. (3) in velocity form: v <- beta v + G, then x <- x - alpha v for s = 0 (v^n = -(x^n - x^{n-1}) / alpha)
// and x <- x - alpha (G + beta v) for s = 1 (v^n = -(y^n - y^{n-1}) / alpha).
// v_scale = (previous step size) / (this step size) keeps the form exact across a change of alpha:
// the momentum term of Eq. (3) is a difference of iterates, not of gradients, so it is not rescaled
// by the new step size.
//
// One launch covers all parameters of a block.  The flat arrays are cut into tasks (UpdateTask):
//   flat    a run of parameters with no transposed copy (BN, linear, convs without backward-data): 16-byte
//           loads and stores of x, v, g (and 8-byte stores of the bf16 copy), 4096 elements per workgroup;
//   conv    a filter bank w[co][j], j = (r, s, ci), that also has the backward-data copy wt[ci][R-1-r][S-1-s][co]:
//           a workgroup owns a 64 x 64 tile (co, j), streams its rows with 16-byte accesses along j, keeps the new
//           values in LDS and writes the copy as 16-byte runs along co -- every global access is a coalesced run;
//   mapped  anything else (the channel-padded forward filters of a stem conv): one element per thread through
//           the index table.
template <bool UPDATE, bool NESTEROV>
__device__ inline float sgd_element(float xi, float& vi, float gi, bool decay, float lr, float momentum, float wd, float v_scale)
{
    if (!UPDATE) return xi;
    if (wd != 0.f && decay) gi += wd * xi;
    vi = momentum * (vi * v_scale) + gi;
    return xi - lr * (NESTEROV ? gi + momentum * vi : vi);
}

constexpr int kUpdFlatPerBlock = 4096;
constexpr int kUpdTile = 64;

template <typename TS, bool UPDATE, bool NESTEROV = false>
__global__ __launch_bounds__(kThreads) void sgd_update_kernel(float* __restrict__ x, float* __restrict__ v,
                                                              const float* __restrict__ g,
                                                              const UpdateTask* __restrict__ tasks, int n_tasks,
                                                              const int32_t* __restrict__ tmap,
                                                              const int32_t* __restrict__ tap_tab, bf16_t* __restrict__ wf16,
                                                              TS* __restrict__ wt, float lr, float momentum, float wd,
                                                              float v_scale)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
    __shared__ float tile[kUpdTile][kUpdTile + 1];
    int p = 0, hi = n_tasks;  // last task whose first workgroup is not after this one (block_begin ascends)
    while (hi - p > 1) {
        const int mid = (p + hi) >> 1;
        if ((int)blockIdx.x >= tasks[mid].block_begin) p = mid; else hi = mid;
    }
    const UpdateTask t = tasks[p];
    const int blk = (int)blockIdx.x - t.block_begin, tid = threadIdx.x;
    const bool decay = t.decay != 0;

    // four consecutive elements starting at i (all inside the task)
    auto quad = [&](size_t i, float (&xn)[4]) {
        f32x4 xv = *(const f32x4*)(x + i), vv = f32x4{0.f, 0.f, 0.f, 0.f}, gv = vv;
        if (UPDATE) {
            vv = *(const f32x4*)(v + i);
            gv = *(const f32x4*)(g + i);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float vi = vv[e];
            xn[e] = sgd_element<UPDATE, NESTEROV>(xv[e], vi, gv[e], decay, lr, momentum, wd, v_scale);
            vv[e] = vi;
            xv[e] = xn[e];
        }
        if (UPDATE) {
            *(f32x4*)(v + i) = vv;
            *(f32x4*)(x + i) = xv;
        }
        if (wf16) *(u32x2*)(wf16 + i) = u32x2{pack_bf16x2(xn[0], xn[1]), pack_bf16x2(xn[2], xn[3])};
    };
    auto single = [&](size_t i) -> float {
        float vi = UPDATE ? v[i] : 0.f;
        const float xn = sgd_element<UPDATE, NESTEROV>(x[i], vi, UPDATE ? g[i] : 0.f, decay, lr, momentum, wd, v_scale);
        if (UPDATE) {
            v[i] = vi;
            x[i] = xn;
        }
        if (wf16) wf16[i] = float_to_bf16(xn);
        return xn;
    };

    if (t.kind == 0) {
        const size_t base = (size_t)t.p0 + (size_t)blk * kUpdFlatPerBlock, end = (size_t)t.p0 + t.n;
        if (t.aligned) {
#pragma unroll
            for (int it = 0; it < kUpdFlatPerBlock / (kThreads * 4); ++it) {
                const size_t i = base + (size_t)it * kThreads * 4 + (size_t)tid * 4;
                if (i + 4 <= end) {
                    float xn[4];
                    quad(i, xn);
                } else {
                    for (size_t k = i; k < end; ++k) (void)single(k);
                }
            }
        } else {
            for (int it = 0; it < kUpdFlatPerBlock / kThreads; ++it) {
                const size_t i = base + (size_t)it * kThreads + tid;
                if (i < end) (void)single(i);
            }
        }
        return;
    }
    if (t.kind == 2) {
        const size_t i = (size_t)t.p0 + (size_t)blk * kThreads + tid;
        if (i < (size_t)t.p0 + t.n) {
            const float xn = single(i);
            const int32_t m = tmap[i];
            if (m >= 0) wt[m] = from_float<TS>(xn);
        }
        return;
    }
    // conv tile: rows co0 .. co0+63 of w[co][j], columns j0 .. j0+63
    const int co0 = (blk / t.tiles_j) * kUpdTile, j0 = (blk % t.tiles_j) * kUpdTile;
    {
        const int jq = tid % 16, row = tid / 16, j = j0 + 4 * jq;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int col = row + 16 * pass, co = co0 + col;
            if (co >= t.Co || j >= t.J) continue;
            const size_t i = (size_t)t.p0 + (size_t)co * t.J + j;
            float xn[4] = {0.f, 0.f, 0.f, 0.f};
            if (t.aligned && j + 4 <= t.J) {
                quad(i, xn);
            } else {
                for (int e = 0; e < 4 && j + e < t.J; ++e) xn[e] = single(i + e);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) tile[4 * jq + e][col] = xn[e];
        }
    }
    __syncthreads();
    {
        constexpr int E = 16 / (int)sizeof(TS);          // elements of the copy per 16-byte run
        constexpr int CQ = kUpdTile / E, ROWS = kThreads / CQ;
        const int cq = tid % CQ, jr = tid / CQ, co = co0 + E * cq;
#pragma unroll
        for (int pass = 0; pass < kUpdTile / ROWS; ++pass) {
            const int jl = jr + ROWS * pass, j = j0 + jl;
            if (j >= t.J || co >= t.Co) continue;
            const int ci = j % t.Ci, tap = j / t.Ci;
            // (grouped layers: the copy's rows are the input channels of all groups, its runs one group's output channels)
            const int grp = co / t.Cog;
            TS* dst = wt + (size_t)t.wt_off + (size_t)tap_tab[t.tap_tab + 2 * tap] +
                      (size_t)(grp * t.Ci + ci) * tap_tab[t.tap_tab + 2 * tap + 1] + (co - grp * t.Cog);
            if (t.wt_aligned && co + E <= t.Co) {
                float f[E];
#pragma unroll
                for (int e = 0; e < E; ++e) f[e] = tile[jl][E * cq + e];
                VecIO<TS, E>::store(dst, f);
            } else {
                for (int e = 0; e < E && co + e < t.Co; ++e) {
                    const int ge = (co + e) / t.Cog;
                    wt[(size_t)t.wt_off + (size_t)tap_tab[t.tap_tab + 2 * tap] +
                       (size_t)(ge * t.Ci + ci) * tap_tab[t.tap_tab + 2 * tap + 1] + (co + e - ge * t.Cog)] =
                        from_float<TS>(tile[jl][E * cq + e]);
                }
            }
        }
    }
}

// ---- sums of squares of a - b and of b (gradient-difference diagnostic), fixed summation order -----
__global__ __launch_bounds__(256) void diff_sumsq_partial_kernel(const float* __restrict__ a, const float* __restrict__ b,
                                                                 size_t n, double* __restrict__ partial)
{
    __shared__ double red[2][256];
    double sd = 0.0, sb = 0.0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const double bi = (double)b[i], d = (double)a[i] - bi;
        sd += d * d;
        sb += bi * bi;
    }
    red[0][threadIdx.x] = sd;
    red[1][threadIdx.x] = sb;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            red[0][threadIdx.x] += red[0][threadIdx.x + w];
            red[1][threadIdx.x] += red[1][threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        partial[2 * blockIdx.x] = red[0][0];
        partial[2 * blockIdx.x + 1] = red[1][0];
    }
}

__global__ __launch_bounds__(64) void diff_sumsq_final_kernel(const double* __restrict__ partial, int nblk,
                                                             double* __restrict__ out)
{
    if (threadIdx.x != 0) return;
    double sd = 0.0, sb = 0.0;
    for (int i = 0; i < nblk; ++i) {
        sd += partial[2 * i];
        sb += partial[2 * i + 1];
    }
    out[0] = sd;
    out[1] = sb;
}

__global__ void record_loss_kernel(const float* __restrict__ loss, float* __restrict__ history, int32_t* counter,
                                   long long capacity)
{
    const int32_t i = counter[0];
    if (i >= 0 && i < capacity) history[i] = loss[0];
    counter[0] = i + 1;
}

__global__ void spin_kernel(long long cycles)
{
    const long long t0 = wall_clock64();
    while (wall_clock64() - t0 < cycles) {}
}

}  // namespace

int launch_maxpool_forward(int dtype, const void* x, void* y, uint8_t* argmax, int N, int H, int W, int C, int k,
                           int stride, int pad, hipStream_t st)
{
    DSP_REQUIRE(k * k < 255, DSP_EINVAL, "maxpool: window too large");
    DSP_REQUIRE((int64_t)N * H * W * C < (1ll << 31), DSP_EINVAL, "maxpool: tensors of 2^31 elements or more are not supported");
    const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
    const int vw = dtype == DSP_BF16 ? 8 : 4;
    const bool vec = C % vw == 0 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)y % 16) == 0;
    const int64_t total = (int64_t)N * Ho * Wo * (vec ? C / vw : C);
    ProfScope ps("maxpool_fwd", ((double)N * H * W * C + (double)N * Ho * Wo * C) * dtype_size(dtype) + (double)N * Ho * Wo * C, 1);
#define MP_FWD(T, V) \
    DSP_LAUNCH(ps, (maxpool_fwd_kernel<T, V>), dim3(grid_for(total)), dim3(kThreads), 0, st, (const T*)x, (T*)y, argmax, N, \
               H, W, C, Ho, Wo, k, stride, pad)
    if (dtype == DSP_BF16) { if (vec) MP_FWD(bf16_t, 8); else MP_FWD(bf16_t, 1); }
    else                   { if (vec) MP_FWD(float, 4); else MP_FWD(float, 1); }
#undef MP_FWD
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_maxpool_backward(int dtype, const void* dy, const uint8_t* argmax, void* dx, bool accumulate, int N,
                            int H, int W, int C, int k, int stride, int pad, hipStream_t st)
{
    DSP_REQUIRE((int64_t)N * H * W * C < (1ll << 31), DSP_EINVAL, "maxpool: tensors of 2^31 elements or more are not supported");
    const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
    const int vw = dtype == DSP_BF16 ? 8 : 4;
    const bool vec = C % vw == 0 && ((uintptr_t)dy % 16) == 0 && ((uintptr_t)dx % 16) == 0;
    const int64_t total = (int64_t)N * H * W * (vec ? C / vw : C);
    ProfScope ps("maxpool_bwd",
                 ((double)N * Ho * Wo * C + (double)N * H * W * C * (accumulate ? 2 : 1)) * dtype_size(dtype) + (double)N * Ho * Wo * C, 1);
#define MP_BWD(T, V, A) \
    DSP_LAUNCH(ps, (maxpool_bwd_kernel<T, V, A>), dim3(grid_for(total)), dim3(kThreads), 0, st, (const T*)dy, argmax, (T*)dx, \
               N, H, W, C, Ho, Wo, k, stride, pad)
    if (dtype == DSP_BF16) {
        if (vec) { if (accumulate) MP_BWD(bf16_t, 8, true); else MP_BWD(bf16_t, 8, false); }
        else     { if (accumulate) MP_BWD(bf16_t, 1, true); else MP_BWD(bf16_t, 1, false); }
    } else {
        if (vec) { if (accumulate) MP_BWD(float, 4, true); else MP_BWD(float, 4, false); }
        else     { if (accumulate) MP_BWD(float, 1, true); else MP_BWD(float, 1, false); }
    }
#undef MP_BWD
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

// Threads that cover the channel (column) axis of a 256-thread workgroup: a power of two <= 256.
static int column_threads(int columns)
{
    int cw = 1;
    while (cw < columns && cw < kThreads) cw *= 2;
    return cw;
}

int launch_gap_forward(int dtype, const void* x, float* y, int N, int HW, int C, hipStream_t st)
{
    const int cw = column_threads(C);
    const dim3 grid(N, ceil_div(C, cw));
    ProfScope ps("gap_fwd", (double)N * HW * C * dtype_size(dtype) + 4.0 * N * C, 1);
    if (dtype == DSP_BF16)
        DSP_LAUNCH(ps, gap_fwd_kernel<bf16_t>, grid, dim3(kThreads), 0, st, (const bf16_t*)x, y, N, HW, C, cw);
    else
        DSP_LAUNCH(ps, gap_fwd_kernel<float>, grid, dim3(kThreads), 0, st, (const float*)x, y, N, HW, C, cw);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_gap_backward(int dtype, const float* dy, void* dx, bool accumulate, int N, int HW, int C, hipStream_t st)
{
    const int64_t total = (int64_t)N * HW * C;
    ProfScope ps("gap_bwd", (double)total * dtype_size(dtype) * (accumulate ? 2 : 1) + 4.0 * N * C, 1);
#define GAP_BWD(T, A) \
    DSP_LAUNCH(ps, (gap_bwd_kernel<T, A>), dim3(grid_for(total)), dim3(kThreads), 0, st, dy, (T*)dx, N, HW, C)
    if (dtype == DSP_BF16) { if (accumulate) GAP_BWD(bf16_t, true); else GAP_BWD(bf16_t, false); }
    else                   { if (accumulate) GAP_BWD(float, true); else GAP_BWD(float, false); }
#undef GAP_BWD
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_linear_forward(const float* x, const float* w, const float* bias, float* z, int N, int Cin, int Cout,
                          hipStream_t st)
{
    ProfScope ps("linear_fwd", 4.0 * ((double)N * Cin + (double)Cout * Cin + (double)N * Cout), 1);
    DSP_LAUNCH(ps, linear_fwd_kernel, dim3(ceil_div(Cout, kLinearJ) * ceil_div(N, kThreads / 64)), dim3(kThreads), 0, st, x, w,
                       bias, z, N, Cin, Cout);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_linear_backward(const float* x, const float* w, const float* dz, float* dx, float* dw, float* dbias,
                           int N, int Cin, int Cout, hipStream_t st)
{
    if (dx) {
        ProfScope ps("linear_bwd_x", 4.0 * ((double)N * Cin + (double)Cout * Cin + (double)N * Cout), 1);
        DSP_LAUNCH(ps, linear_bwd_x_kernel, dim3(ceil_div((int64_t)N * Cin, kThreads)), dim3(kThreads), 0, st, dz, w,
                   dx, N, Cin, Cout);
    }
    const int cw = column_threads(Cin + 1);
    ProfScope ps("linear_bwd_w", 4.0 * ((double)N * Cin + (double)Cout * Cin + (double)N * Cout), 1);
    DSP_LAUNCH(ps, linear_bwd_w_kernel, dim3(Cout, ceil_div(Cin + 1, cw)), dim3(kThreads), 0, st, dz, x, dw, dbias, N,
                       Cin, Cout, cw);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_softmax_ce(const float* z, const int32_t* labels, float* loss, float* dz, float* row_loss, int N, int C,
                      hipStream_t st)
{
    DSP_REQUIRE(z && labels && loss && dz && row_loss && N > 0 && C > 0, DSP_EINVAL, "softmax_ce: null buffer or empty shape");
    {
        ProfScope ps("softmax_ce_rows", 8.0 * (double)N * C, 1);
        DSP_LAUNCH(ps, softmax_ce_rows_kernel, dim3(N), dim3(64), 0, st, z, labels, row_loss, dz, N, C);
    }
    ProfScope ps("loss_mean", 4.0 * (double)N, 1);
    DSP_LAUNCH(ps, mean_kernel, dim3(1), dim3(64), 0, st, (const float*)row_loss, loss, N);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int update_plan_finish(std::vector<UpdateTask>& tasks, int dtype, int* total_blocks)
{
    int blocks = 0;
    for (UpdateTask& t : tasks) {
        t.block_begin = blocks;
        if (t.kind == 0) {
            blocks += ceil_div((int64_t)t.n, kUpdFlatPerBlock);
        } else if (t.kind == 2) {
            blocks += ceil_div((int64_t)t.n, kThreads);
        } else {
            t.tiles_j = ceil_div(t.J, kUpdTile);
            blocks += ceil_div(t.Co, kUpdTile) * t.tiles_j;
            const int E = dtype == DSP_BF16 ? 8 : 4;
            t.wt_aligned = (t.Cog % E == 0 && t.wt_off % E == 0) ? 1 : 0;  // every tap base and ci stride is a multiple of Cog
            t.aligned = (t.p0 % 4 == 0 && t.J % 4 == 0) ? 1 : 0;
        }
        if (t.kind == 0) t.aligned = (t.p0 % 4 == 0) ? 1 : 0;
    }
    *total_blocks = blocks;
    return DSP_OK;
}

template <bool UPDATE>
static int run_update(int dtype, float* x, float* v, const float* g, const UpdateTask* tasks, int n_tasks, int blocks,
                      const int32_t* tmap, const int32_t* tap_tab, void* wf16, void* wt, size_t n, float lr, float momentum,
                      float wd, hipStream_t st, bool nesterov, float v_scale)
{
    if (n == 0 || blocks == 0) return DSP_OK;
    const dim3 grid(blocks);
    // read x, v, g; write x, v, the bf16 copy (bf16 blocks) and the backward-data filter copy
    ProfScope ps(dtype == DSP_BF16 ? "sgd_update<bf16 shadows>" : "sgd_update<fp32>", UPDATE ? (double)n * 24.0 : (double)n * 8.0, 1);
#define UPD(TS, NES)                                                                                              \
    DSP_LAUNCH(ps, (sgd_update_kernel<TS, UPDATE, NES>), grid, dim3(kThreads), 0, st, x, v, g, tasks, n_tasks, tmap, \
               tap_tab, (bf16_t*)wf16, (TS*)wt, lr, momentum, wd, v_scale)
    if (dtype == DSP_BF16) { if (nesterov) UPD(bf16_t, true); else UPD(bf16_t, false); }
    else                   { if (nesterov) UPD(float, true); else UPD(float, false); }
#undef UPD
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_sgd_update(int dtype, float* x, float* v, const float* g, const UpdateTask* tasks, int n_tasks, int blocks,
                      const int32_t* tmap, const int32_t* tap_tab, void* wf16, void* wt, size_t n, float lr, float momentum,
                      float wd, hipStream_t st, bool nesterov, float v_scale)
{
    return run_update<true>(dtype, x, v, g, tasks, n_tasks, blocks, tmap, tap_tab, dtype == DSP_BF16 ? wf16 : nullptr, wt, n, lr,
                            momentum, wd, st, nesterov, v_scale);
}

int launch_refresh_shadows(int dtype, const float* x, const UpdateTask* tasks, int n_tasks, int blocks, const int32_t* tmap,
                           const int32_t* tap_tab, void* wf16, void* wt, size_t n, hipStream_t st)
{
    return run_update<false>(dtype, const_cast<float*>(x), nullptr, nullptr, tasks, n_tasks, blocks, tmap, tap_tab,
                             dtype == DSP_BF16 ? wf16 : nullptr, wt, n, 0.f, 0.f, 0.f, st, false, 1.f);
}

int launch_diff_sumsq(const float* a, const float* b, size_t n, double* partial, double* out, hipStream_t st)
{
    const int nblk = (int)std::max<size_t>(1, std::min<size_t>(kDiffSumsqBlocks, (n + 255) / 256));
    hipLaunchKernelGGL(diff_sumsq_partial_kernel, dim3(nblk), dim3(256), 0, st, a, b, n, partial);
    hipLaunchKernelGGL(diff_sumsq_final_kernel, dim3(1), dim3(64), 0, st, (const double*)partial, nblk, out);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_record_loss(const float* loss, float* history, int32_t* counter, int64_t capacity, hipStream_t st)
{
    ProfScope ps("record_loss", 12.0, 1);
    DSP_LAUNCH(ps, record_loss_kernel, dim3(1), dim3(1), 0, st, loss, history, counter, (long long)capacity);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void pad_channels_kernel(const T* __restrict__ src, T* __restrict__ dst,
                                                                int64_t pixels, int C, int Cp)
{
    const int64_t total = pixels * Cp;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
        const int c = (int)(i % Cp);
        const int64_t p = i / Cp;
        dst[i] = c < C ? src[p * C + c] : from_float<T>(0.f);
    }
}

// ---- element-wise sum of two feature maps and its backward (the gradient passes to both operands) ----
template <typename T, int VW>
__global__ __launch_bounds__(kThreads) void add_fwd_kernel(const T* __restrict__ a, const T* __restrict__ b,
                                                           T* __restrict__ y, int64_t nvec)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * kThreads) {
        float va[VW], vb[VW];
        VecIO<T, VW>::load(a + i * VW, va);
        VecIO<T, VW>::load(b + i * VW, vb);
#pragma unroll
        for (int v = 0; v < VW; ++v) va[v] += vb[v];
        VecIO<T, VW>::store(y + i * VW, va);
    }
}

// dx0 (and dx1, if given) = dy, or += dy where the buffer already holds another consumer's contribution
template <typename T, int VW>
__global__ __launch_bounds__(kThreads) void grad_pass_kernel(const T* __restrict__ dy, T* __restrict__ dx0, int acc0,
                                                             T* __restrict__ dx1, int acc1, int64_t nvec)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * kThreads) {
        float v[VW];
        VecIO<T, VW>::load(dy + i * VW, v);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            T* dx = t ? dx1 : dx0;
            if (!dx) continue;
            float o[VW];
            if (t ? acc1 : acc0) {
                VecIO<T, VW>::load(dx + i * VW, o);
#pragma unroll
                for (int k = 0; k < VW; ++k) o[k] += v[k];
            } else {
#pragma unroll
                for (int k = 0; k < VW; ++k) o[k] = v[k];
            }
            VecIO<T, VW>::store(dx + i * VW, o);
        }
    }
}

// The common case: the padded pixel is one 16-byte run (4 floats / 8 bf16).  One thread per pixel: scalar loads of
// neighbouring pixels coalesce, the store is a whole run.
template <typename T>
__global__ __launch_bounds__(kThreads) void pad_channels_run_kernel(const T* __restrict__ src, T* __restrict__ dst,
                                                                    int64_t pixels, int C)
{
    constexpr int CP = 16 / (int)sizeof(T);
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    for (int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x; p < pixels; p += (int64_t)gridDim.x * kThreads) {
        alignas(16) T v[CP];
#pragma unroll
        for (int c = 0; c < CP; ++c) v[c] = c < C ? src[p * C + c] : from_float<T>(0.f);
        *(u32x4*)(dst + p * CP) = *(const u32x4*)v;
    }
}

__global__ __launch_bounds__(kThreads) void gather_f32_kernel(const float* __restrict__ src, const int32_t* __restrict__ idx,
                                                              int32_t base, float* __restrict__ dst, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads)
        dst[i] = src[idx[i] - base];
}

// One thread per output pixel.  Its channels are the two source pixels of the cell's upper row side by side, then
// those of the lower row: each is one contiguous run of 2 * C elements in the source (a whole number of 32-bit
// words, 4-byte aligned since W is even), copied word by word; zeros behind; written as whole 16-byte runs.
template <typename T, int CP, int C>
__global__ __launch_bounds__(kThreads) void space_to_depth2_kernel(const T* __restrict__ src, T* __restrict__ dst, int N, int H,
                                                                   int W)
{
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    constexpr int WORDS = CP * (int)sizeof(T) / 4;
    constexpr int seg = 2 * C * (int)sizeof(T) / 4;  // words per row of the cell
    static_assert(2 * seg <= WORDS && WORDS % 4 == 0, "the two runs fit the padded pixel, which is whole 16-byte runs");
    const int H2 = H / 2, W2 = W / 2;
    const int64_t pixels = (int64_t)N * H2 * W2;
    const uint32_t* __restrict__ srcw = (const uint32_t*)src;
    for (int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x; p < pixels; p += (int64_t)gridDim.x * kThreads) {
        const int w2 = (int)(p % W2);
        const int64_t t = p / W2;
        const int h2 = (int)(t % H2);
        const int64_t n = t / H2;
        alignas(16) uint32_t v[WORDS];
#pragma unroll
        for (int k = 0; k < WORDS; ++k) v[k] = 0u;
        const int64_t row0 = ((n * H + 2 * h2) * W + 2 * w2) * (int64_t)seg / 2;  // word offset of the upper run
        const int64_t row1 = row0 + (int64_t)W * seg / 2;
#pragma unroll
        for (int k = 0; k < seg; ++k) {
            v[k] = srcw[row0 + k];
            v[seg + k] = srcw[row1 + k];
        }
#pragma unroll
        for (int k = 0; k < WORDS / 4; ++k) ((u32x4*)(dst + p * CP))[k] = ((const u32x4*)v)[k];
    }
}

template <typename T>
static int add_forward_t(const void* a, const void* b, void* y, int64_t n, hipStream_t st)
{
    constexpr int VW = 16 / (int)sizeof(T);
    ProfScope ps("add_fwd", (double)n * 3.0 * sizeof(T), 1);
    const bool vec = n % VW == 0 && ((uintptr_t)a % 16) == 0 && ((uintptr_t)b % 16) == 0 && ((uintptr_t)y % 16) == 0;
    if (vec)
        DSP_LAUNCH(ps, (add_fwd_kernel<T, VW>), dim3(grid_for(n / VW)), dim3(kThreads), 0, st, (const T*)a, (const T*)b,
                   (T*)y, n / VW);
    else
        DSP_LAUNCH(ps, (add_fwd_kernel<T, 1>), dim3(grid_for(n)), dim3(kThreads), 0, st, (const T*)a, (const T*)b, (T*)y, n);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_add_forward(int dtype, const void* a, const void* b, void* y, int64_t n, hipStream_t st)
{
    DSP_REQUIRE(a && b && y && n > 0, DSP_EINVAL, "add: bad argument");
    return dtype == DSP_BF16 ? add_forward_t<bf16_t>(a, b, y, n, st) : add_forward_t<float>(a, b, y, n, st);
}

template <typename T>
static int grad_pass_t(const void* dy, void* dx0, bool acc0, void* dx1, bool acc1, int64_t n, hipStream_t st)
{
    constexpr int VW = 16 / (int)sizeof(T);
    const int passes = 1 + (acc0 ? 1 : 0) + (dx1 ? 1 + (acc1 ? 1 : 0) : 0);
    ProfScope ps("add_bwd", (double)n * (1.0 + passes) * sizeof(T), 1);
    const bool vec = n % VW == 0 && ((uintptr_t)dy % 16) == 0 && ((uintptr_t)dx0 % 16) == 0 && ((uintptr_t)dx1 % 16) == 0;
    if (vec)
        DSP_LAUNCH(ps, (grad_pass_kernel<T, VW>), dim3(grid_for(n / VW)), dim3(kThreads), 0, st, (const T*)dy, (T*)dx0,
                   (int)acc0, (T*)dx1, (int)acc1, n / VW);
    else
        DSP_LAUNCH(ps, (grad_pass_kernel<T, 1>), dim3(grid_for(n)), dim3(kThreads), 0, st, (const T*)dy, (T*)dx0, (int)acc0,
                   (T*)dx1, (int)acc1, n);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_grad_pass(int dtype, const void* dy, void* dx0, bool acc0, void* dx1, bool acc1, int64_t n, hipStream_t st)
{
    DSP_REQUIRE(dy && dx0 && n > 0 && dx0 != dx1, DSP_EINVAL, "add backward: bad argument");
    return dtype == DSP_BF16 ? grad_pass_t<bf16_t>(dy, dx0, acc0, dx1, acc1, n, st)
                             : grad_pass_t<float>(dy, dx0, acc0, dx1, acc1, n, st);
}

int launch_pad_channels(int dtype, const void* src, void* dst, int64_t pixels, int C, int Cp, hipStream_t st)
{
    DSP_REQUIRE(src && dst && pixels > 0 && C > 0 && Cp >= C, DSP_EINVAL, "pad_channels: bad argument");
    ProfScope ps("pad_channels", (double)pixels * (C + Cp) * dtype_size(dtype), 1);
    if (Cp * dtype_size(dtype) == 16 && ((uintptr_t)dst % 16) == 0) {
        if (dtype == DSP_BF16)
            DSP_LAUNCH(ps, pad_channels_run_kernel<bf16_t>, dim3(grid_for(pixels)), dim3(kThreads), 0, st,
                       (const bf16_t*)src, (bf16_t*)dst, pixels, C);
        else
            DSP_LAUNCH(ps, pad_channels_run_kernel<float>, dim3(grid_for(pixels)), dim3(kThreads), 0, st, (const float*)src,
                       (float*)dst, pixels, C);
        DSP_HIP(hipGetLastError());
        return DSP_OK;
    }
    if (dtype == DSP_BF16)
        DSP_LAUNCH(ps, pad_channels_kernel<bf16_t>, dim3(grid_for(pixels * Cp)), dim3(kThreads), 0, st, (const bf16_t*)src,
                   (bf16_t*)dst, pixels, C, Cp);
    else
        DSP_LAUNCH(ps, pad_channels_kernel<float>, dim3(grid_for(pixels * Cp)), dim3(kThreads), 0, st, (const float*)src,
                   (float*)dst, pixels, C, Cp);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_gather_f32(const float* src, const int32_t* idx, int32_t base, float* dst, int64_t n, hipStream_t st)
{
    DSP_REQUIRE(src && idx && dst && n > 0, DSP_EINVAL, "gather: bad argument");
    ProfScope ps("gather_f32", (double)n * 12.0, 1);
    DSP_LAUNCH(ps, gather_f32_kernel, dim3(grid_for(n)), dim3(kThreads), 0, st, src, idx, base, dst, n);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_space_to_depth2(int dtype, const void* src, void* dst, int N, int H, int W, int C, int Cp, hipStream_t st)
{
    DSP_REQUIRE(src && dst && N > 0 && H > 0 && W > 0 && H % 2 == 0 && W % 2 == 0 && C > 0 && 4 * C <= Cp &&
                    ((uintptr_t)dst % 16) == 0 && ((uintptr_t)src % 4) == 0,
                DSP_EINVAL, "space_to_depth: bad argument");
    const int64_t pixels = (int64_t)N * (H / 2) * (W / 2);
    ProfScope ps("space_to_depth", (double)pixels * (4 * C + Cp) * dtype_size(dtype), 1);
    if (dtype == DSP_BF16 && Cp == 16 && C == 3)
        DSP_LAUNCH(ps, (space_to_depth2_kernel<bf16_t, 16, 3>), dim3(grid_for(pixels)), dim3(kThreads), 0, st, (const bf16_t*)src,
                   (bf16_t*)dst, N, H, W);
    else if (dtype == DSP_FP32 && Cp == 12 && C == 3)
        DSP_LAUNCH(ps, (space_to_depth2_kernel<float, 12, 3>), dim3(grid_for(pixels)), dim3(kThreads), 0, st, (const float*)src,
                   (float*)dst, N, H, W);
    else
        DSP_REQUIRE(false, DSP_EINVAL, "space_to_depth: %d channels padded to %d unsupported", C, Cp);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_spin(int microseconds, hipStream_t st)
{
    if (microseconds <= 0) return DSP_OK;
    // wall_clock64 ticks at 100 MHz on this family
    hipLaunchKernelGGL(spin_kernel, dim3(1), dim3(1), 0, st, (long long)microseconds * 100);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

}  // namespace dsp
