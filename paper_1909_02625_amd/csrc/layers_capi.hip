// Single-layer entry points of the C ABI for everything that is not a convolution: batch norm
// (+ residual + ReLU), max pool, element-wise sum, global average pool, linear head, softmax
// cross-entropy and the momentum update.  They launch exactly the kernels the block engine launches
// for such a layer, on caller-owned tensors, so that each kernel can be checked against the layer's
// definition on identical stored inputs (no block, no schedule around it).
#include "common.h"

using namespace dsp;

namespace {

bool dtype_ok(int32_t dtype) { return dtype == DSP_FP32 || dtype == DSP_BF16; }

// Layout of the batch-norm workspace: [partial sums: max(bn_max_partial_blocks(), 1) * C pairs of doubles][coef: 3 * C floats]
size_t bn_partial_bytes(int32_t C) { return (size_t)bn_max_partial_blocks() * (size_t)C * 2 * sizeof(double); }
size_t bn_ws_bytes(int32_t C) { return bn_partial_bytes(C) + (size_t)3 * C * sizeof(float); }

}  // namespace

extern "C" {

int dsp_bn_workspace_bytes(int32_t C, size_t* bytes)
{
    DSP_REQUIRE(bytes && C > 0, DSP_EINVAL, "dsp_bn_workspace_bytes: bad argument");
    *bytes = bn_ws_bytes(C);
    return DSP_OK;
}

int dsp_bn_forward(int32_t dtype, const void* d_x, const void* d_res, void* d_y, const float* d_gamma, const float* d_beta,
                   float eps, int64_t M, int32_t C, int32_t relu, float* d_mean, float* d_invstd, void* d_workspace,
                   size_t workspace_bytes, void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_x && d_y && d_gamma && d_beta && d_mean && d_invstd && d_workspace, DSP_EINVAL,
                "dsp_bn_forward: bad argument");
    DSP_REQUIRE(M > 0 && C > 0 && eps > 0.f && M * (int64_t)C < (1ll << 31), DSP_EINVAL, "dsp_bn_forward: bad shape");
    DSP_REQUIRE(workspace_bytes >= bn_ws_bytes(C) && ((uintptr_t)d_workspace % 16) == 0, DSP_EINVAL,
                "dsp_bn_forward: workspace too small or not 16-byte aligned (%zu < %zu)", workspace_bytes, bn_ws_bytes(C));
    BnBuffers buf{(double*)d_workspace, d_mean, d_invstd, (float*)((char*)d_workspace + bn_partial_bytes(C))};
    return launch_bn_forward(dtype, d_x, d_res, d_y, d_gamma, d_beta, eps, M, C, relu != 0, buf, (hipStream_t)stream);
}

int dsp_bn_backward(int32_t dtype, const void* d_dy, const void* d_x, const void* d_y, void* d_dx, void* d_dres,
                    int32_t dres_accumulate, int32_t dx_accumulate, const float* d_gamma, const float* d_mean,
                    const float* d_invstd, float* d_dgamma, float* d_dbeta, int64_t M, int32_t C, int32_t relu,
                    void* d_workspace, size_t workspace_bytes, void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_dy && d_x && d_dx && d_gamma && d_mean && d_invstd && d_dgamma && d_dbeta && d_workspace,
                DSP_EINVAL, "dsp_bn_backward: bad argument");
    DSP_REQUIRE(!relu || d_y, DSP_EINVAL, "dsp_bn_backward: the ReLU mask needs the layer output y");
    DSP_REQUIRE(M > 0 && C > 0 && M * (int64_t)C < (1ll << 31), DSP_EINVAL, "dsp_bn_backward: bad shape");
    DSP_REQUIRE(workspace_bytes >= bn_ws_bytes(C) && ((uintptr_t)d_workspace % 16) == 0, DSP_EINVAL,
                "dsp_bn_backward: workspace too small or not 16-byte aligned (%zu < %zu)", workspace_bytes, bn_ws_bytes(C));
    BnBuffers buf{(double*)d_workspace, const_cast<float*>(d_mean), const_cast<float*>(d_invstd),
                  (float*)((char*)d_workspace + bn_partial_bytes(C))};
    return launch_bn_backward(dtype, d_dy, d_x, d_y, d_dx, d_dres, dres_accumulate != 0, dx_accumulate != 0, d_gamma, d_dgamma,
                              d_dbeta, M, C, relu != 0, buf, (hipStream_t)stream);
}

int dsp_bn_relu_bits_bytes(int32_t dtype, int64_t M, int32_t C, size_t* bytes)
{
    DSP_REQUIRE(bytes && dtype_ok(dtype) && M > 0 && C > 0, DSP_EINVAL, "dsp_bn_relu_bits_bytes: bad argument");
    *bytes = bn_relu_bits_bytes(dtype, M, C);
    return DSP_OK;
}

int dsp_bn_forward_bits(int32_t dtype, const void* d_x, const void* d_res, void* d_y, const float* d_gamma, const float* d_beta,
                        float eps, int64_t M, int32_t C, float* d_mean, float* d_invstd, uint8_t* d_relu_bits, void* d_workspace,
                        size_t workspace_bytes, void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_x && d_y && d_gamma && d_beta && d_mean && d_invstd && d_relu_bits && d_workspace, DSP_EINVAL,
                "dsp_bn_forward_bits: bad argument");
    DSP_REQUIRE(M > 0 && C > 0 && eps > 0.f && M * (int64_t)C < (1ll << 31), DSP_EINVAL, "dsp_bn_forward_bits: bad shape");
    DSP_REQUIRE(bn_relu_bits_bytes(dtype, M, C) > 0, DSP_EINVAL, "dsp_bn_forward_bits: channels must come in whole 16-byte runs");
    DSP_REQUIRE(workspace_bytes >= bn_ws_bytes(C) && ((uintptr_t)d_workspace % 16) == 0, DSP_EINVAL,
                "dsp_bn_forward_bits: workspace too small or not 16-byte aligned (%zu < %zu)", workspace_bytes, bn_ws_bytes(C));
    BnBuffers buf{(double*)d_workspace, d_mean, d_invstd, (float*)((char*)d_workspace + bn_partial_bytes(C))};
    return launch_bn_forward(dtype, d_x, d_res, d_y, d_gamma, d_beta, eps, M, C, true, buf, (hipStream_t)stream, 0, nullptr, false,
                             d_relu_bits);
}

int dsp_bn_backward_bits(int32_t dtype, const void* d_dy, const void* d_x, const uint8_t* d_relu_bits, void* d_dx, void* d_dres,
                         int32_t dres_accumulate, int32_t dx_accumulate, const float* d_gamma, const float* d_mean,
                         const float* d_invstd, float* d_dgamma, float* d_dbeta, int64_t M, int32_t C, void* d_workspace,
                         size_t workspace_bytes, void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_dy && d_x && d_relu_bits && d_dx && d_gamma && d_mean && d_invstd && d_dgamma && d_dbeta &&
                    d_workspace, DSP_EINVAL, "dsp_bn_backward_bits: bad argument");
    DSP_REQUIRE(M > 0 && C > 0 && M * (int64_t)C < (1ll << 31), DSP_EINVAL, "dsp_bn_backward_bits: bad shape");
    DSP_REQUIRE(bn_relu_bits_bytes(dtype, M, C) > 0, DSP_EINVAL, "dsp_bn_backward_bits: channels must come in whole 16-byte runs");
    DSP_REQUIRE(workspace_bytes >= bn_ws_bytes(C) && ((uintptr_t)d_workspace % 16) == 0, DSP_EINVAL,
                "dsp_bn_backward_bits: workspace too small or not 16-byte aligned (%zu < %zu)", workspace_bytes, bn_ws_bytes(C));
    BnBuffers buf{(double*)d_workspace, const_cast<float*>(d_mean), const_cast<float*>(d_invstd),
                  (float*)((char*)d_workspace + bn_partial_bytes(C))};
    return launch_bn_backward(dtype, d_dy, d_x, nullptr, d_dx, d_dres, dres_accumulate != 0, dx_accumulate != 0, d_gamma, d_dgamma,
                              d_dbeta, M, C, true, buf, (hipStream_t)stream, nullptr, nullptr, nullptr, d_relu_bits);
}

int dsp_bn_relu_backward_from_x(int32_t dtype, const void* d_dy, const void* d_x, const float* d_scale_shift, void* d_dx,
                                int32_t dx_accumulate, const float* d_gamma, const float* d_mean, const float* d_invstd,
                                float* d_dgamma, float* d_dbeta, int64_t M, int32_t C, void* d_workspace, size_t workspace_bytes,
                                void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_dy && d_x && d_scale_shift && d_dx && d_gamma && d_mean && d_invstd && d_dgamma && d_dbeta &&
                    d_workspace, DSP_EINVAL, "dsp_bn_relu_backward_from_x: bad argument");
    DSP_REQUIRE(M > 0 && C > 0 && M * (int64_t)C < (1ll << 31), DSP_EINVAL, "dsp_bn_relu_backward_from_x: bad shape");
    DSP_REQUIRE(workspace_bytes >= bn_ws_bytes(C) && ((uintptr_t)d_workspace % 16) == 0, DSP_EINVAL,
                "dsp_bn_relu_backward_from_x: workspace too small or not 16-byte aligned (%zu < %zu)", workspace_bytes, bn_ws_bytes(C));
    BnBuffers buf{(double*)d_workspace, const_cast<float*>(d_mean), const_cast<float*>(d_invstd),
                  (float*)((char*)d_workspace + bn_partial_bytes(C))};
    return launch_bn_backward(dtype, d_dy, d_x, nullptr, d_dx, nullptr, false, dx_accumulate != 0, d_gamma, d_dgamma, d_dbeta, M, C,
                              true, buf, (hipStream_t)stream, nullptr, d_scale_shift);
}

int dsp_bn_relu_maxpool_backward(int32_t dtype, const void* d_dpool, const uint8_t* d_argmax, const void* d_x,
                                 const float* d_scale_shift, void* d_dx, int32_t dx_accumulate, const float* d_gamma,
                                 const float* d_mean, const float* d_invstd, float* d_dgamma, float* d_dbeta, int32_t N, int32_t H,
                                 int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad, void* d_workspace,
                                 size_t workspace_bytes, void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_dpool && d_argmax && d_x && d_scale_shift && d_dx && d_gamma && d_mean && d_invstd && d_dgamma &&
                    d_dbeta && d_workspace, DSP_EINVAL, "dsp_bn_relu_maxpool_backward: bad argument");
    DSP_REQUIRE(N > 0 && H > 0 && W > 0 && C > 0 && k > 0 && stride > 0 && pad >= 0 && pad < k && H + 2 * pad >= k && W + 2 * pad >= k &&
                    (int64_t)N * H * W * C < (1ll << 31), DSP_EINVAL, "dsp_bn_relu_maxpool_backward: bad shape");
    DSP_REQUIRE(bn_pool_backward_supported(dtype, C, H, W, k, stride, pad), DSP_EINVAL,
                "dsp_bn_relu_maxpool_backward: bf16 tensors with channels in runs of 8, 3 x 3 windows at stride 2 and pad 1 over an even map only");
    DSP_REQUIRE(workspace_bytes >= bn_ws_bytes(C) && ((uintptr_t)d_workspace % 16) == 0, DSP_EINVAL,
                "dsp_bn_relu_maxpool_backward: workspace too small or not 16-byte aligned (%zu < %zu)", workspace_bytes, bn_ws_bytes(C));
    BnBuffers buf{(double*)d_workspace, const_cast<float*>(d_mean), const_cast<float*>(d_invstd),
                  (float*)((char*)d_workspace + bn_partial_bytes(C))};
    const PoolGrad pg{d_dpool, d_argmax, H, W, k, stride, pad};
    return launch_bn_backward(dtype, nullptr, d_x, nullptr, d_dx, nullptr, false, dx_accumulate != 0, d_gamma, d_dgamma, d_dbeta,
                              (int64_t)N * H * W, C, true, buf, (hipStream_t)stream, nullptr, d_scale_shift, &pg);
}

int dsp_bn_relu_maxpool_forward(int32_t dtype, const void* d_x, const float* d_gamma, const float* d_beta, float eps, int32_t N,
                                int32_t H, int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad, void* d_pool,
                                uint8_t* d_argmax, float* d_mean, float* d_invstd, float* d_scale_shift, void* d_workspace,
                                size_t workspace_bytes, void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_x && d_gamma && d_beta && d_pool && d_argmax && d_mean && d_invstd && d_scale_shift && d_workspace,
                DSP_EINVAL, "dsp_bn_relu_maxpool_forward: bad argument");
    DSP_REQUIRE(N > 0 && H > 0 && W > 0 && C > 0 && eps > 0.f && k > 0 && stride > 0 && pad >= 0 && pad < k && H + 2 * pad >= k &&
                    W + 2 * pad >= k && (int64_t)N * H * W * C < (1ll << 31), DSP_EINVAL, "dsp_bn_relu_maxpool_forward: bad shape");
    DSP_REQUIRE(bn_relu_maxpool_supported(dtype, C, k), DSP_EINVAL,
                "dsp_bn_relu_maxpool_forward: bf16 tensors with channels in runs of 8 and windows up to 4 x 4 only");
    DSP_REQUIRE(workspace_bytes >= bn_ws_bytes(C) && ((uintptr_t)d_workspace % 16) == 0 && ((uintptr_t)d_scale_shift % 16) == 0,
                DSP_EINVAL, "dsp_bn_relu_maxpool_forward: workspace too small, or workspace / d_scale_shift not 16-byte aligned");
    BnBuffers buf{(double*)d_workspace, d_mean, d_invstd, d_scale_shift};
    DSP_TRY(launch_bn_forward(dtype, d_x, nullptr, nullptr, d_gamma, d_beta, eps, (int64_t)N * H * W, C, true, buf,
                              (hipStream_t)stream, 0, nullptr, /*stats_only=*/true));
    return launch_bn_relu_maxpool_forward(dtype, d_x, d_scale_shift, d_pool, d_argmax, N, H, W, C, k, stride, pad, (hipStream_t)stream);
}

int dsp_maxpool_forward(int32_t dtype, const void* d_x, void* d_y, uint8_t* d_argmax, int32_t N, int32_t H, int32_t W,
                        int32_t C, int32_t k, int32_t stride, int32_t pad, void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_x && d_y && d_argmax, DSP_EINVAL, "dsp_maxpool_forward: bad argument");
    DSP_REQUIRE(N > 0 && H > 0 && W > 0 && C > 0 && k > 0 && stride > 0 && pad >= 0 && pad < k && H + 2 * pad >= k &&
                    W + 2 * pad >= k, DSP_EINVAL, "dsp_maxpool_forward: bad shape");
    return launch_maxpool_forward(dtype, d_x, d_y, d_argmax, N, H, W, C, k, stride, pad, (hipStream_t)stream);
}

int dsp_maxpool_backward(int32_t dtype, const void* d_dy, const uint8_t* d_argmax, void* d_dx, int32_t accumulate, int32_t N,
                         int32_t H, int32_t W, int32_t C, int32_t k, int32_t stride, int32_t pad, void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_dy && d_dx && d_argmax, DSP_EINVAL, "dsp_maxpool_backward: bad argument");
    DSP_REQUIRE(N > 0 && H > 0 && W > 0 && C > 0 && k > 0 && stride > 0 && pad >= 0 && pad < k && H + 2 * pad >= k &&
                    W + 2 * pad >= k, DSP_EINVAL, "dsp_maxpool_backward: bad shape");
    return launch_maxpool_backward(dtype, d_dy, d_argmax, d_dx, accumulate != 0, N, H, W, C, k, stride, pad, (hipStream_t)stream);
}

int dsp_add_forward(int32_t dtype, const void* d_a, const void* d_b, void* d_y, int64_t n, void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_a && d_b && d_y && n > 0, DSP_EINVAL, "dsp_add_forward: bad argument");
    return launch_add_forward(dtype, d_a, d_b, d_y, n, (hipStream_t)stream);
}

int dsp_add_backward(int32_t dtype, const void* d_dy, void* d_da, int32_t da_accumulate, void* d_db, int32_t db_accumulate,
                     int64_t n, void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_dy && d_da && n > 0 && d_da != d_db, DSP_EINVAL, "dsp_add_backward: bad argument");
    return launch_grad_pass(dtype, d_dy, d_da, da_accumulate != 0, d_db, db_accumulate != 0, n, (hipStream_t)stream);
}

int dsp_gap_forward(int32_t dtype, const void* d_x, float* d_y, int32_t N, int32_t HW, int32_t C, void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_x && d_y && N > 0 && HW > 0 && C > 0, DSP_EINVAL, "dsp_gap_forward: bad argument");
    return launch_gap_forward(dtype, d_x, d_y, N, HW, C, (hipStream_t)stream);
}

int dsp_gap_backward(int32_t dtype, const float* d_dy, void* d_dx, int32_t accumulate, int32_t N, int32_t HW, int32_t C,
                     void* stream)
{
    DSP_REQUIRE(dtype_ok(dtype) && d_dy && d_dx && N > 0 && HW > 0 && C > 0, DSP_EINVAL, "dsp_gap_backward: bad argument");
    return launch_gap_backward(dtype, d_dy, d_dx, accumulate != 0, N, HW, C, (hipStream_t)stream);
}

int dsp_linear_forward(const float* d_x, const float* d_w, const float* d_bias, float* d_z, int32_t N, int32_t cin, int32_t cout,
                       void* stream)
{
    DSP_REQUIRE(d_x && d_w && d_bias && d_z && N > 0 && cin > 0 && cout > 0, DSP_EINVAL, "dsp_linear_forward: bad argument");
    return launch_linear_forward(d_x, d_w, d_bias, d_z, N, cin, cout, (hipStream_t)stream);
}

int dsp_linear_backward(const float* d_x, const float* d_w, const float* d_dz, float* d_dx, float* d_dw, float* d_dbias,
                        int32_t N, int32_t cin, int32_t cout, void* stream)
{
    DSP_REQUIRE(d_x && d_w && d_dz && d_dw && d_dbias && N > 0 && cin > 0 && cout > 0, DSP_EINVAL,
                "dsp_linear_backward: bad argument");
    return launch_linear_backward(d_x, d_w, d_dz, d_dx, d_dw, d_dbias, N, cin, cout, (hipStream_t)stream);
}

int dsp_softmax_ce(const float* d_z, const int32_t* d_labels, float* d_loss, float* d_dz, float* d_row_loss, int32_t N,
                   int32_t C, void* stream)
{
    return launch_softmax_ce(d_z, d_labels, d_loss, d_dz, d_row_loss, N, C, (hipStream_t)stream);
}

}  // extern "C"
