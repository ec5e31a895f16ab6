// Shared declarations of the gfx950 DSP library: status/error plumbing, storage types,
// bf16 conversion, and the launch interface between the host engine and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/dsp.h"

struct dsp_block;

namespace dsp {

// While a block is "dry" its step calls check and advance the host-side state (batch ids, update
// counter) but launch nothing: the pipeline replays the launches of that tick from a HIP graph.
void block_set_dry(dsp_block* b, bool dry);
// dsp_block_step that records `after_forward` (if not null) on the stream once the forward sweeps are issued, i.e.
// when the block's output for the block above is complete, before the backward sweep.
int block_step_event(dsp_block* b, int64_t batch_fwd, const void* d_in, void* d_out, const int32_t* d_labels, float* d_loss,
                     int64_t batch_bwd, const void* d_grad_out, void* d_grad_in, hipStream_t st, hipEvent_t after_forward);

// The block's flat fp32 parameter and gradient arrays (library layout) and their length.
struct BlockArrays {
    float* x;
    float* g;
    size_t n;
};
BlockArrays block_arrays(dsp_block* b);
// Overwrites the parameters with n floats in the library layout (device memory) and refreshes the
// storage-type copies the kernels read; ordered on st.
int block_load_params_device(dsp_block* b, const float* d_src, hipStream_t st);

// ---- error plumbing ---------------------------------------------------------------------------
void set_error(const char* fmt, ...);

#define DSP_HIP(call)                                                                      \
    do {                                                                                   \
        hipError_t e__ = (call);                                                           \
        if (e__ != hipSuccess) {                                                           \
            ::dsp::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e__), __FILE__, __LINE__); \
            return DSP_EHIP;                                                               \
        }                                                                                  \
    } while (0)

#define DSP_TRY(call)                   \
    do {                                \
        int s__ = (call);               \
        if (s__ != DSP_OK) return s__;  \
    } while (0)

#define DSP_REQUIRE(cond, status, ...)  \
    do {                                \
        if (!(cond)) {                  \
            ::dsp::set_error(__VA_ARGS__); \
            return (status);            \
        }                               \
    } while (0)

// ---- storage types ----------------------------------------------------------------------------
// bfloat16 is kept as its raw 16 bits; conversion is round-to-nearest-even (NaN stays NaN).
struct bf16_t {
    uint16_t bits;
};

__host__ __device__ inline float bf16_to_float(bf16_t v)
{
    union {
        uint32_t u;
        float f;
    } c;
    c.u = (uint32_t)v.bits << 16;
    return c.f;
}

// Round to nearest even.  On the device this is the hardware conversion (v_cvt_pk_bf16_f32), which gives the
// same bits as the integer routine below for every finite input, infinities included, and keeps NaNs NaN
// (checked on the GPU over 2^24 bit patterns with ties, denormals and values that round to infinity).
__host__ __device__ inline bf16_t float_to_bf16(float f)
{
    bf16_t r;
#if defined(__HIP_DEVICE_COMPILE__)
    r.bits = __builtin_bit_cast(uint16_t, (__bf16)f);
#else
    union {
        uint32_t u;
        float f;
    } c;
    c.f = f;
    if ((c.u & 0x7fffffffu) > 0x7f800000u) {  // NaN
        r.bits = (uint16_t)((c.u >> 16) | 0x40u);
        return r;
    }
    c.u += 0x7fffu + ((c.u >> 16) & 1u);
    r.bits = (uint16_t)(c.u >> 16);
#endif
    return r;
}

// Two values rounded to bf16 and packed into one dword (lo in bits 0-15): one instruction on the device.
__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
#else
    return (uint32_t)float_to_bf16(lo).bits | ((uint32_t)float_to_bf16(hi).bits << 16);
#endif
}

template <typename T>
__host__ __device__ inline float to_float(T v);
template <>
__host__ __device__ inline float to_float<float>(float v) { return v; }
template <>
__host__ __device__ inline float to_float<bf16_t>(bf16_t v) { return bf16_to_float(v); }

template <typename T>
__host__ __device__ inline T from_float(float v);
template <>
__host__ __device__ inline float from_float<float>(float v) { return v; }
template <>
__host__ __device__ inline bf16_t from_float<bf16_t>(float v) { return float_to_bf16(v); }

inline size_t dtype_size(int dtype) { return dtype == DSP_BF16 ? 2 : 4; }

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// ---- convolution launchers (conv_igemm.hip) -------------------------------------------------
// Geometry of one convolution y = conv(x, w): x is N x H x W x Cin (NHWC), y is N x Ho x Wo x Cout.
struct ConvShape {
    int N, H, W, Cin, Cout, R, S, stride, pad, Ho, Wo;
    int cin_real;  // > 0: only the first cin_real of the Cin input channels carry data (the rest is zero padding);
                   // used for counting the useful multiply-accumulates only
    double macs;   // > 0: the useful multiply-accumulates of the layer this problem stands for (a layer run in another
                   // form, e.g. the space-to-depth stem); used for reporting only
    int groups;    // > 1: grouped convolution -- group g maps input channels [g Cin/groups, (g+1) Cin/groups) to output
                   // channels [g Cout/groups, (g+1) Cout/groups); filters [Cout][R][S][Cin/groups].  0 and 1: ungrouped.
};

inline int conv_groups(const ConvShape& c) { return c.groups > 1 ? c.groups : 1; }
// Multiply-accumulates of the convolution as defined (taps on padding and padded channels not counted).
double conv_useful_macs(const ConvShape& c);

inline ConvShape make_conv_shape(int N, int H, int W, int Cin, int Cout, int R, int S, int stride, int pad, int groups = 1)
{
    ConvShape c{N, H, W, Cin, Cout, R, S, stride, pad, 0, 0, 0, 0.0, groups};
    c.Ho = (H + 2 * pad - R) / stride + 1;
    c.Wo = (W + 2 * pad - S) / stride + 1;
    return c;
}

// y = conv(x, w);  w in [Cout][R][S][Cin].  With column_sums != nullptr the kernel also writes partial column sums of
// y[M][Cout]: column_sums[(t*Cout + c)*2 + {0,1}] = {sum y, sum y^2} over the rows of part t, of the values as stored --
// the statistics a batch norm on y needs.  The conv_forward_row_tiles() parts cover every row once (one part per row
// tile of the kernel the shape selects, or per workgroup where a workgroup walks many tiles).
// twin != nullptr: the same launch also computes twin->y = conv(twin->x, w) (and twin->column_sums if
// column_sums is given): the forward pass of the current mini-batch and the recompute of a stale one
// share their parameters, so one launch per layer serves both.
struct ConvForwardTwin {
    const void* x;
    void* y;
    double* column_sums;
};
int launch_conv_forward(int dtype, const ConvShape& c, const void* x, const void* w, void* y, hipStream_t st,
                        double* column_sums = nullptr, const ConvForwardTwin* twin = nullptr);
int conv_forward_row_tiles(int dtype, const ConvShape& c);
// dx (+)= conv^T(dy, w);  wt in [Cin][R-1-r][S-1-s][Cout] for stride 1.  For stride 2 the copy is stored class by
// class (dgrad_classes): class (hi % 2, wi % 2) of the input pixels uses the taps r' = r0 + 2 j, s' = s0 + 2 l of the
// flipped filter, kept as [Cin][j][l][Cout] at element offset wt_off; the classes follow each other.
struct DgradClass {
    int Rc, Sc;        // taps of the class per direction (0: no tap reaches these pixels)
    int r0, s0;        // its first tap of the flipped filter
    int off_h, off_w;  // class pixel (a, b) reads source pixels (a + off_h + j, b + off_w + l)
    int Hc, Wc;        // pixels of the class per direction
    size_t wt_off;     // first element of its filters in the copy
};
void dgrad_classes(const ConvShape& c, DgradClass (&cls)[4]);
int launch_conv_backward_data(int dtype, const ConvShape& c, const void* dy, const void* wt, void* dx,
                              bool accumulate, hipStream_t st);
// dw[Cout][R][S][Cin] (float) = sum over (n, ho, wo) of dy * x;  ws holds the split partials.
// defer_reduce: write the per-slice partial sums to ws only; the caller sums them later (for all its layers
// at once, wgrad_reduce_set_*).  conv_backward_weight_slices = number of slices (1: dw is written directly).
int launch_conv_backward_weight(int dtype, const ConvShape& c, const void* x, const void* dy, float* dw, void* ws,
                                size_t ws_bytes, hipStream_t st, bool defer_reduce = false);
int conv_backward_weight_slices(int dtype, const ConvShape& c);
struct WgradReduceItem {
    const float* partials;  // [slices][n]
    float* dw;              // [n]
    size_t n;
    int slices;
};
struct WgradReduceSet;
int wgrad_reduce_set_create(const WgradReduceItem* items, int n, WgradReduceSet** out);
int wgrad_reduce_set_launch(const WgradReduceSet* s, hipStream_t st);
void wgrad_reduce_set_destroy(WgradReduceSet* s);
size_t conv_backward_weight_workspace(const ConvShape& c);

// ---- batch norm (+ residual + ReLU) launchers (bn.hip) ----------------------------------------
struct BnBuffers {
    double* partial;  // [max_blocks][C][2] partial sums
    float* mean;      // [C]
    float* invstd;    // [C]
    float* coef;      // [3*C] per-channel coefficients handed from the reduce to the apply kernel
};
int bn_max_partial_blocks();
// y = [relu]( gamma * (x - mean) * invstd + beta [+ res] ), statistics over the M rows of x[M][C].
// presummed > 0: buf.partial already holds that many per-tile column sums of x (written by the
// convolution that produced x), so the pass that sums x is skipped.
// twin != nullptr: a second instance (same shape and parameters, its own tensors and statistics
// buffers) is normalised by the same launches.
struct BnForwardTwin {
    const void* x;
    const void* res;
    void* y;
    BnBuffers buf;
    uint8_t* relu_bits;  // as the argument of launch_bn_forward, for the second instance (may be nullptr)
};
int launch_bn_forward(int dtype, const void* x, const void* res, void* y, const float* gamma, const float* beta,
                      float eps, int64_t M, int C, bool relu, const BnBuffers& buf, hipStream_t st, int presummed = 0,
                      const BnForwardTwin* twin = nullptr, bool stats_only = false, uint8_t* relu_bits = nullptr);
// relu_bits (ReLU layers whose channels come in whole 16-byte runs: bn_relu_bits_bytes() > 0 bytes): the apply kernel also
// leaves one byte per channel vector, bit k = element k of y as stored is positive.  launch_bn_backward takes the ReLU
// decision of a layer WITH residual from these bytes instead of reading y (an eighth / a sixteenth of its bytes).
size_t bn_relu_bits_bytes(int dtype, int64_t M, int C);
// stats_only: mean, invstd and buf.coef = {scale[C], shift[C]} only; y is not written (may be nullptr).  The two calls
// below finish such a layer: launch_bn_apply writes y = [relu](scale * x + shift) from those coefficients, and
// launch_bn_relu_maxpool_forward (bf16, C % 8 == 0, window k <= 4: bn_relu_maxpool_supported) writes the max pool of that
// y and the chosen taps without storing y -- the same bits launch_bn_apply + launch_maxpool_forward leave.
int launch_bn_apply(int dtype, const void* x, void* y, const float* coef, int64_t M, int C, bool relu, hipStream_t st);
bool bn_relu_maxpool_supported(int dtype, int C, int k);
int launch_bn_relu_maxpool_forward(int dtype, const void* x, const float* coef, void* y, uint8_t* argmax, int N, int H, int W,
                                   int C, int k, int stride, int pad, hipStream_t st);
// y = a + b over [M][C] (as launch_add_forward) and, in the same pass, the per-block column sums {sum y, sum y^2}
// of the stored values in partial[add_stats_blocks()][C][2]: exactly what launch_bn_forward(y, ...) would compute
// first, so the batch norm that reads y is called with presummed = add_stats_blocks().  twin: a second instance.
struct AddStatsTwin {
    const void* a;
    const void* b;
    void* y;
    double* partial;
};
int add_stats_blocks(int dtype, int64_t M, int C);
int launch_add_forward_stats(int dtype, const void* a, const void* b, void* y, int64_t M, int C, double* partial,
                             hipStream_t st, const AddStatsTwin* twin = nullptr);
// Backward of the map above given dy and the saved x, y, mean, invstd:
// dz = dy * [y > 0]; dres (+)= dz; dgamma, dbeta; dx = gamma*invstd*(dz - dbeta/M - xhat*dgamma/M).
// dx_add != nullptr: dx = dx_add + (the above) -- the gradient another consumer of the same input left in a
// buffer of its own (then dx_accumulate is ignored).
// fwd_coef != nullptr (a batch norm with ReLU and no residual): the forward pass's {scale[C], shift[C]}; the ReLU is
// then decided by forming y from x again, exactly as the forward kernel did, and y is not read (may be nullptr).
// pool != nullptr (with fwd_coef; bn_pool_backward_supported: bf16, C % 8 == 0, 3 x 3 / stride 2 / pad 1 windows over an
// even map): the batch norm's only reader is a max pool, and dy is the backward of that pool, formed on the fly from the
// pool's own output gradient and recorded taps (summed in the order and rounded to the storage type as
// launch_maxpool_backward does, so every dz is the same; the per-channel sums are taken in another order, which moves
// dgamma, dbeta and the coefficients of dx by a few units of double rounding before they become floats), without the
// pool's input gradient ever being stored.  dy is then ignored.
struct PoolGrad {
    const void* dpool;     // gradient of the pool's output, [N][Ho][Wo][C]
    const uint8_t* argmax; // the pool's recorded taps
    int H, W;              // the pool's input map = the batch norm's map (M = N * H * W)
    int k, stride, pad;
};
bool bn_pool_backward_supported(int dtype, int C, int H, int W, int k, int stride, int pad);
int launch_bn_backward(int dtype, const void* dy, const void* x, const void* y, void* dx, void* dres,
                       bool dres_accumulate, bool dx_accumulate, const float* gamma, float* dgamma, float* dbeta,
                       int64_t M, int C, bool relu, const BnBuffers& buf, hipStream_t st, const void* dx_add = nullptr,
                       const float* fwd_coef = nullptr, const PoolGrad* pool = nullptr, const uint8_t* relu_bits = nullptr);

// ---- small layers and the update (misc.hip) ---------------------------------------------------
int launch_maxpool_forward(int dtype, const void* x, void* y, uint8_t* argmax, int N, int H, int W, int C, int k,
                           int stride, int pad, hipStream_t st);
int launch_maxpool_backward(int dtype, const void* dy, const uint8_t* argmax, void* dx, bool accumulate, int N,
                            int H, int W, int C, int k, int stride, int pad, hipStream_t st);
int launch_gap_forward(int dtype, const void* x, float* y, int N, int HW, int C, hipStream_t st);
int launch_gap_backward(int dtype, const float* dy, void* dx, bool accumulate, int N, int HW, int C,
                        hipStream_t st);
int launch_linear_forward(const float* x, const float* w, const float* bias, float* z, int N, int Cin, int Cout,
                          hipStream_t st);
int launch_linear_backward(const float* x, const float* w, const float* dz, float* dx, float* dw, float* dbias,
                           int N, int Cin, int Cout, hipStream_t st);
// loss = mean_n -log softmax(z_n)[label_n];  dz = (softmax - onehot) / N;  row_loss is scratch [N].
int launch_softmax_ce(const float* z, const int32_t* labels, float* loss, float* dz, float* row_loss, int N,
                      int C, hipStream_t st);
// out[0] = sum (a_i - b_i)^2, out[1] = sum b_i^2 in fp64, same order every run; partial: 2 * kDiffSumsqBlocks doubles.
constexpr int kDiffSumsqBlocks = 256;
int launch_diff_sumsq(const float* a, const float* b, size_t n, double* partial, double* out, hipStream_t st);
// v <- momentum*v + (g + wd*x*[decay]);  x <- x - lr*v (s = 0);  the copies the kernels read are refreshed in the
// same pass: wf16[i] = bf16(x[i]) (bf16 blocks), and the backward-data filter copies in wt.  The parameters of a block
// are described as a list of tasks over the flat arrays (built once at init, kept on the device):
struct UpdateTask {
    int kind;          // 0: flat run, no copy in wt;  1: conv filters w[co][j] with the copy wt[ci][R-1-r][S-1-s][co];
                       // 2: one element per thread, copy position from the index table tmap (-1: none)
    int decay;         // weight decay applies (conv / linear weights)
    uint32_t p0, n;    // first element and length in the flat arrays
    uint32_t wt_off;   // kind 1: first element of the copy in wt
    int Co, J, Ci, R, S;  // kind 1: J = R * S * Ci (Ci: input channels of one group)
    int Cog;              // kind 1: output channels per group (= Co for an ordinary convolution); the copy of a
                          // grouped layer is wt[group * Ci + ci][..taps..][co within the group]
    int tap_tab;          // kind 1: first entry of this layer in the tap table: per tap (r * S + s) the element offset of
                          // (ci = 0, co = 0) of that tap inside the copy and the stride between consecutive ci
    int tiles_j, block_begin, aligned, wt_aligned;  // filled by update_plan_finish
};
int update_plan_finish(std::vector<UpdateTask>& tasks, int dtype, int* total_blocks);
int launch_sgd_update(int dtype, float* x, float* v, const float* g, const UpdateTask* tasks, int n_tasks, int blocks,
                      const int32_t* tmap, const int32_t* tap_tab, void* wf16, void* wt, size_t n, float lr, float momentum,
                      float wd, hipStream_t st, bool nesterov = false, float v_scale = 1.f);
// Same refresh of the copies without an update (after init / set_params).
int launch_refresh_shadows(int dtype, const float* x, const UpdateTask* tasks, int n_tasks, int blocks, const int32_t* tmap,
                           const int32_t* tap_tab, void* wf16, void* wt, size_t n, hipStream_t st);
int launch_spin(int microseconds, hipStream_t st);
// dst[p][0..Cp) = {src[p][0..C), 0...}: channel padding of an NHWC tensor (pixels rows) up to a whole 16-byte run.
// y = a + b over n elements; backward of the sum: dx0 (and dx1, unless null) = dy or += dy, one read of dy
int launch_add_forward(int dtype, const void* a, const void* b, void* y, int64_t n, hipStream_t st);
int launch_grad_pass(int dtype, const void* dy, void* dx0, bool acc0, void* dx1, bool acc1, int64_t n, hipStream_t st);
int launch_pad_channels(int dtype, const void* src, void* dst, int64_t pixels, int C, int Cp, hipStream_t st);
// dst[i] = src[idx[i] - base]: a filter gradient formed in a padded / transformed layout back into the layer's own.
int launch_gather_f32(const float* src, const int32_t* idx, int32_t base, float* dst, int64_t n, hipStream_t st);
// Space-to-depth by 2 with channel padding: dst[n][h][w][(dh * 2 + dw) * C + c] = src[n][2h + dh][2w + dw][c], channels
// 4C .. Cp-1 zero; H and W even, Cp * sizeof(T) a multiple of 16.
int launch_space_to_depth2(int dtype, const void* src, void* dst, int N, int H, int W, int C, int Cp, hipStream_t st);
// history[counter[0]] = *loss; counter[0] += 1   (one thread; keeps the loss history index on the device)
int launch_record_loss(const float* loss, float* history, int32_t* counter, int64_t capacity, hipStream_t st);

// ---- 16-byte (or single-element) loads and stores of VW consecutive elements as floats ------------
template <typename T, int VW>
struct VecIO;

template <>
struct VecIO<float, 4> {
    __device__ static inline void load(const float* p, float (&v)[4])
    {
        const float4 t = *(const float4*)p;
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    __device__ static inline void store(float* p, const float (&v)[4]) { *(float4*)p = make_float4(v[0], v[1], v[2], v[3]); }
};
template <>
struct VecIO<float, 1> {
    __device__ static inline void load(const float* p, float (&v)[1]) { v[0] = *p; }
    __device__ static inline void store(float* p, const float (&v)[1]) { *p = v[0]; }
};
template <>
struct VecIO<bf16_t, 8> {
    __device__ static inline void load(const bf16_t* p, float (&v)[8])
    {
        const uint4 t = *(const uint4*)p;
        const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static inline void store(bf16_t* p, const float (&v)[8])
    {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = pack_bf16x2(v[2 * i], v[2 * i + 1]);
        *(uint4*)p = make_uint4(w[0], w[1], w[2], w[3]);
    }
};
template <>
struct VecIO<bf16_t, 1> {
    __device__ static inline void load(const bf16_t* p, float (&v)[1]) { v[0] = bf16_to_float(*p); }
    __device__ static inline void store(bf16_t* p, const float (&v)[1]) { *p = float_to_bf16(v[0]); }
};


// n / d for n < 2^31 with precomputed mul = floor(2^32 * (2^sh - d) / d) + 1, sh = ceil(log2 d).
__device__ inline uint32_t fast_div(uint32_t n, uint32_t mul, uint32_t sh) { return (__umulhi(n, mul) + n) >> sh; }
inline void fast_div_constants(uint32_t d, uint32_t* mul, uint32_t* sh)
{
    uint32_t s = 0;
    while ((1ull << s) < d) ++s;
    *sh = s;
    *mul = (uint32_t)(((1ull << 32) * ((1ull << s) - d)) / d + 1);
}

// ---- in-situ kernel timing (block.hip) ----------------------------------------------------------
// While a profile is running (dsp_profile_start .. dsp_profile_stop) every instrumented launch goes
// through hipExtLaunchKernelGGL with a start and a stop event of its own, which the runtime fills
// from the timestamps of that kernel's dispatch packet (the same source a kernel trace uses), so a
// launch is timed exactly, on whatever stream it runs, without serialising the streams.  The pairs
// are read back and summed per kernel name at stop.  `units` is the algorithmic work of the launch:
// floating-point operations (unit_kind 0) or bytes that must cross HBM (unit_kind 1).
extern bool g_profile_on;
struct ProfScope {
    hipEvent_t start = nullptr, stop = nullptr;
    ProfScope(const char* name, double units, int unit_kind)
    {
        if (g_profile_on) begin(name, units, unit_kind);
    }
    void begin(const char* name, double units, int unit_kind);
};

// Launches `kernel`; with an active ProfScope `ps` the launch carries its own timing events.
#define DSP_LAUNCH(ps, kernel, grid, block, lds, st, ...)                                              \
    do {                                                                                               \
        if ((ps).start)                                                                                \
            hipExtLaunchKernelGGL(kernel, grid, block, lds, st, (ps).start, (ps).stop, 0, __VA_ARGS__); \
        else                                                                                           \
            hipLaunchKernelGGL(kernel, grid, block, lds, st, __VA_ARGS__);                             \
    } while (0)

}  // namespace dsp
