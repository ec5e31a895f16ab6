// Host engine of one DSP block: layer graph, device buffers, the stored-input ring M_k, the
// forward / recompute+backward / update sequence of Section 3.2-3.3 of the paper, and the C ABI.
//
// Per block, per tick (in this order, all asynchronous on the caller's stream):
//   forward(a)              f_k on the newest mini-batch with the live parameters; its input is
//                           kept in ring slot a mod (1+m_k+p_{k-1}); nothing else is kept.
//   recompute_backward(b)   b = a - m_k: f_k again on the stored input with the SAME live
//                           parameters (Eq. (5)), keeping conv inputs / BN statistics / ReLU
//                           outputs in the workspace, then the reverse sweep.
//   param_update            v <- beta v + G, x <- x - alpha v; shadow weight copies refreshed.
// There is exactly one live copy of the parameters (no weight stashing); "stale" only means
// that m_k updates happen between the forward and the backward of one mini-batch.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <map>
#include <new>
#include <string>
#include <mutex>
#include <vector>

#include "common.h"

namespace dsp {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// ---- in-situ kernel timing ------------------------------------------------------------------------
bool g_profile_on = false;
namespace {
struct ProfRec {
    const char* name;
    double units;
    int unit_kind;
};
std::vector<hipEvent_t> g_prof_events;  // 2 per launch
std::vector<ProfRec> g_prof_recs;
size_t g_prof_capacity = 0;
struct ProfAgg {
    std::string name;
    int64_t launches = 0;
    double ms = 0, units = 0;
    int unit_kind = 0;
};
std::vector<ProfAgg> g_prof_result;
}  // namespace

std::mutex g_prof_mu;  // launches come from one host thread per block

void ProfScope::begin(const char* name, double units, int unit_kind)
{
    std::lock_guard<std::mutex> lock(g_prof_mu);
    if (g_prof_recs.size() >= g_prof_capacity) return;  // profile full: later launches go untimed
    const size_t slot = g_prof_recs.size();
    g_prof_recs.push_back({name, units, unit_kind});
    start = g_prof_events[2 * slot];
    stop = g_prof_events[2 * slot + 1];
}

struct Tensor {
    int N = 0, C = 0, H = 1, W = 1;
    bool is_float = false;  // tensors behind a global average pool are fp32 whatever the block dtype
    size_t elems = 0;
    void* act = nullptr;
    void* grad = nullptr;
    size_t bytes(int dtype) const { return elems * (is_float ? 4 : dtype_size(dtype)); }
};

struct Layer {
    dsp_layer_desc d;
    ConvShape cs;
    size_t p0 = 0, p1 = 0;  // offsets of (w | gamma | W) and (beta | bias) in the parameter arrays
    size_t wt_off = 0;      // offset of the backward-data filter copy
    float* mean = nullptr;
    float* invstd = nullptr;
    // bn whose only reader is the max pool right behind it (pool_fused), and that pool (bn_fused = the bn's index): the
    // pool kernel forms the batch norm's output on the fly, which is then never stored
    bool pool_fused = false;
    int bn_fused = -1;
    // conv: backward-data is issued right after that of layer dgrad_after (see the block's init), not in its own turn
    int dgrad_after = -1;
    bool pool_bwd = false;  // such a bn whose backward kernels also form the pool's input gradient on the fly (never stored)
    uint8_t* relu_bits = nullptr;  // bn with residual + ReLU: sign bytes of the output the primary forward pass left (the backward sweep reads them instead of the output)
    float* fcoef = nullptr;  // bn: {scale[C], shift[C]} of the last forward pass over the primary buffers (the backward sweep decides the ReLU with them)
    uint8_t* argmax = nullptr;
    bool in0_grad = true;  // form the gradient w.r.t. in0
    bool in1_grad = true;
    bool in0_acc = false;  // add to (true) or overwrite (false) the gradient buffer of in0
    bool in1_acc = false;
    // add: this operand's gradient is not copied -- its only other consumer, a batch norm, adds the sum's
    // gradient itself (dx_add_from of that layer), or the operand has no other consumer and its producer
    // reads the sum's gradient directly (grad_alias of the block)
    bool in0_skip = false, in1_skip = false;
    int dx_add_from = -1;  // bn: layer whose output gradient is added to this layer's input gradient
    // conv: the next layer is a batch norm of this output, so the conv kernel also leaves the per-tile
    // column sums in the block's partial-sum buffer; bn: number of such tiles (0 = sum x itself)
    int sum_tiles = 0;
    // A conv on the data input whose channel count is no whole 16-byte run (the 3-channel stem): the
    // input is copied into a channel-padded buffer and the layer runs as a conv over cin_pad channels
    // (cs describes that padded problem).  Its forward filters live, padded with zeros, in the block's
    // filter-copy area (this layer needs no backward-data copy), kept up to date by the update kernel.
    // A 7x7 / stride 2 / pad 3 stem on even-sized images runs in space-to-depth form instead (s2d): the 2x2 cells of
    // the input become 4 * cin channels (padded to cin_pad) of a half-size image, on which the layer is a 4x4 / stride
    // 1 convolution with padding 2 above / left and 1 below / right -- tap r of the 7x7 filter is tap (r - 3) >> 1
    // (+ 2) and cell row (r - 3) & 1 -- i.e. 4 * 4 * cin_pad = 256 multiplications per output instead of
    // 7 * 7 * 8 = 392 of the channel-padded form, and half the bytes of padded input.
    int cin_pad = 0;
    bool s2d = false;
    int in_h = 0, in_w = 0;   // s2d: size of the layer's real input
    void* xpad = nullptr;     // padded input of the pass the backward sweep belongs to
    float* dw_pad = nullptr;  // filter gradient in the padded layout
    size_t wg_off = 0, wg_bytes = 0;  // conv: this layer's region of the partial-gradient workspace
};

}  // namespace dsp

using namespace dsp;

// A second set of the buffers a forward pass writes (activations, batch-norm statistics and scratch,
// pooling indices), so that the forward pass of the current mini-batch can run on another stream
// while the recompute / backward of a stale one uses the primary set.
struct ForwardLane {
    std::vector<void*> act;
    std::vector<float*> mean, invstd;
    std::vector<uint8_t*> argmax;
    std::vector<void*> xpad;
    double* bn_partial = nullptr;
    float* bn_coef = nullptr;
};

struct dsp_block {
    dsp_block_desc desc;
    std::vector<Layer> layers;
    std::vector<Tensor> T;
    Tensor input;
    int out_idx = -1;   // tensor that is h_{k+1}
    int loss_idx = -1;  // softmax_ce layer, if any
    int dtype = DSP_FP32;

    size_t nP = 0;
    float *x = nullptr, *v = nullptr, *g = nullptr;
    int32_t* tmap = nullptr;        // index table of the filter copies that are no plain transposition (padded stem filters)
    UpdateTask* upd_tasks = nullptr;  // how the update kernel walks the flat arrays (device copy)
    int32_t* tap_tab = nullptr;       // per conv layer and tap: where that tap's filters sit in the backward-data copy
    int upd_n_tasks = 0, upd_blocks = 0;
    void* wf16 = nullptr;  // bf16 copy of x in the same layout (bf16 blocks only)
    void* wt = nullptr;    // backward-data filter copies [cin][R-1-r][S-1-s][cout] in the storage type
    size_t wt_elems = 0;
    std::vector<int32_t> perm;  // library index -> layer-order index

    int ring_entries = 1;
    char* ring = nullptr;
    size_t slot_bytes = 0;
    std::vector<int64_t> slot_version;

    float* dz_ring = nullptr;  // loss gradient of the last 1+m_k mini-batches (last block only)
    size_t dz_elems = 0;
    float* row_loss = nullptr;
    float* loss_sink = nullptr;

    float last_lr = 0.f;  // step size of the latest update (the velocity is stored in its units)
    void* wgrad_ws = nullptr;  // per-slice partial weight gradients, one region per conv layer
    size_t wgrad_ws_bytes = 0;
    WgradReduceSet* wgrad_set = nullptr;  // sums all regions in one launch at the end of the backward sweep
    double* bn_partial = nullptr;
    float* bn_coef = nullptr;
    size_t bn_partial_elems = 0;
    int bn_max_c = 1;
    ForwardLane* fwd_lane = nullptr;  // set by dsp_block_enable_forward_lane

    size_t ring_bytes = 0, ws_bytes = 0, param_bytes = 0;
    std::vector<void*> allocs;
    std::vector<int> grad_alias;  // per tensor: the sum layer whose output gradient is also this tensor's (-1: its own buffer)

    int64_t version = 0, next_fwd = 0, next_bwd = 0;
    bool pending = false;
    bool dry = false;  // advance the host-side state only: the launches of this tick are replayed from a HIP graph
};

namespace dsp {

static int dev_alloc(dsp_block* b, void** p, size_t bytes, size_t* counter)
{
    if (bytes == 0) bytes = 16;
    hipError_t e = hipMalloc(p, bytes);
    if (e != hipSuccess) {
        set_error("hipMalloc(%zu) failed: %s", bytes, hipGetErrorString(e));
        return DSP_ENOMEM;
    }
    b->allocs.push_back(*p);
    if (counter) *counter += bytes;
    return DSP_OK;
}

static const void* weights_for_forward(const dsp_block* b, const Layer& L)
{
    return b->dtype == DSP_BF16 ? (const void*)((const bf16_t*)b->wf16 + L.p0) : (const void*)(b->x + L.p0);
}
static const void* weights_for_dgrad(const dsp_block* b, const Layer& L)
{
    return b->dtype == DSP_BF16 ? (const void*)((const bf16_t*)b->wt + L.wt_off) : (const void*)((const float*)b->wt + L.wt_off);
}

static int build_graph(dsp_block* b)
{
    const dsp_block_desc& d = b->desc;
    DSP_REQUIRE(d.n_layers > 0 && d.layers != nullptr, DSP_EINVAL, "block: no layers");
    DSP_REQUIRE(d.N > 0 && d.C > 0 && d.H > 0 && d.W > 0, DSP_EINVAL, "block: bad input shape");
    DSP_REQUIRE(d.dtype == DSP_FP32 || d.dtype == DSP_BF16, DSP_EINVAL, "block: bad dtype");
    DSP_REQUIRE(d.K >= 1 && d.k >= 0 && d.k < d.K, DSP_EINVAL, "block: bad k/K");
    DSP_REQUIRE(d.m_k >= 0 && d.p_prev >= 0, DSP_EINVAL, "block: m_k and p_prev must be >= 0");
    DSP_REQUIRE(d.bn_eps > 0.f, DSP_EINVAL, "block: bn_eps must be > 0");
    b->dtype = d.dtype;
    b->input.N = d.N; b->input.C = d.C; b->input.H = d.H; b->input.W = d.W;
    b->input.elems = (size_t)d.N * d.C * d.H * d.W;
    b->layers.resize(d.n_layers);
    b->T.resize(d.n_layers);
    size_t poff = 0, wtoff = 0;
    for (int i = 0; i < d.n_layers; ++i) {
        Layer& L = b->layers[i];
        L.d = d.layers[i];
        DSP_REQUIRE(L.d.in0 >= -1 && L.d.in0 < i, DSP_EINVAL, "layer %d: in0 must name an earlier tensor", i);
        const Tensor& s = L.d.in0 < 0 ? b->input : b->T[L.d.in0];
        Tensor& t = b->T[i];
        t.N = s.N;
        switch (L.d.op) {
        case DSP_OP_CONV:
            DSP_REQUIRE(!s.is_float && s.C == L.d.cin && L.d.cout > 0 && L.d.r > 0 && L.d.s > 0 && L.d.stride > 0 &&
                            L.d.pad >= 0, DSP_EINVAL, "layer %d: conv shape mismatch", i);
            DSP_REQUIRE(L.d.groups >= 0 && L.d.groups < 65536 && L.d.cin % (L.d.groups > 1 ? L.d.groups : 1) == 0 &&
                            L.d.cout % (L.d.groups > 1 ? L.d.groups : 1) == 0,
                        DSP_EINVAL, "layer %d: %d groups do not divide the channels", i, L.d.groups);
        {
            const int run = 16 / (int)dtype_size(d.dtype);
            const int G = L.d.groups > 1 ? L.d.groups : 1;
            int cin = L.d.cin;
            if (L.d.in0 < 0 && !d.needs_input_grad && cin % run != 0 && G == 1) {
                L.s2d = L.d.r == 7 && L.d.s == 7 && L.d.stride == 2 && L.d.pad == 3 && s.H % 2 == 0 && s.W % 2 == 0 &&
                        s.H >= 8 && s.W >= 8 && cin == 3;
                L.cin_pad = ((L.s2d ? 4 * cin : cin) + run - 1) / run * run;
                cin = L.cin_pad;
            }
            if (L.s2d) {
                const ConvShape real = make_conv_shape(s.N, s.H, s.W, L.d.cin, L.d.cout, 7, 7, 2, 3);
                L.in_h = s.H;
                L.in_w = s.W;
                L.cs = make_conv_shape(s.N, s.H / 2, s.W / 2, cin, L.d.cout, 4, 4, 1, 2);
                L.cs.Ho = real.Ho;   // = H / 2: one row / column of padding less below / right than above / left
                L.cs.Wo = real.Wo;
                L.cs.macs = conv_useful_macs(real);
            } else {
                L.cs = make_conv_shape(s.N, s.H, s.W, cin, L.d.cout, L.d.r, L.d.s, L.d.stride, L.d.pad, G);
                if (L.cin_pad) L.cs.cin_real = L.d.cin;
            }
            DSP_REQUIRE(L.cs.Ho > 0 && L.cs.Wo > 0, DSP_EINVAL, "layer %d: empty conv output", i);
            t.C = L.d.cout; t.H = L.cs.Ho; t.W = L.cs.Wo;
            L.p0 = poff;
            poff += (size_t)L.d.cout * (L.d.cin / G) * L.d.r * L.d.s;
            L.wt_off = wtoff;
            wtoff += (size_t)L.d.cout * (cin / G) * L.cs.R * L.cs.S;
            break;
        }
        case DSP_OP_BN:
            DSP_REQUIRE(!s.is_float && s.C == L.d.cin, DSP_EINVAL, "layer %d: bn channel mismatch", i);
            DSP_REQUIRE(L.d.in1 == -2 || (L.d.in1 >= -1 && L.d.in1 < i), DSP_EINVAL, "layer %d: bad residual", i);
            if (L.d.in1 != -2) {
                const Tensor& r = L.d.in1 < 0 ? b->input : b->T[L.d.in1];
                DSP_REQUIRE(!r.is_float && r.C == s.C && r.H == s.H && r.W == s.W, DSP_EINVAL,
                            "layer %d: residual shape mismatch", i);
            }
            t.C = s.C; t.H = s.H; t.W = s.W;
            L.p0 = poff; L.p1 = poff + s.C;
            poff += 2 * (size_t)s.C;
            break;
        case DSP_OP_ADD: {
            DSP_REQUIRE(!s.is_float && L.d.in1 >= -1 && L.d.in1 < i, DSP_EINVAL, "layer %d: add needs two earlier feature maps", i);
            const Tensor& r = L.d.in1 < 0 ? b->input : b->T[L.d.in1];
            DSP_REQUIRE(!r.is_float && r.C == s.C && r.H == s.H && r.W == s.W, DSP_EINVAL, "layer %d: add shape mismatch", i);
            t.C = s.C; t.H = s.H; t.W = s.W;
            break;
        }
        case DSP_OP_MAXPOOL:
            DSP_REQUIRE(!s.is_float && L.d.r > 0 && L.d.stride > 0 && L.d.pad >= 0 && L.d.pad < L.d.r, DSP_EINVAL,
                        "layer %d: bad maxpool", i);
            t.C = s.C;
            t.H = (s.H + 2 * L.d.pad - L.d.r) / L.d.stride + 1;
            t.W = (s.W + 2 * L.d.pad - L.d.r) / L.d.stride + 1;
            DSP_REQUIRE(t.H > 0 && t.W > 0, DSP_EINVAL, "layer %d: empty maxpool output", i);
            break;
        case DSP_OP_GAP:
            DSP_REQUIRE(!s.is_float, DSP_EINVAL, "layer %d: gap input must be a feature map", i);
            t.C = s.C; t.H = 1; t.W = 1; t.is_float = true;
            break;
        case DSP_OP_LINEAR:
            DSP_REQUIRE(s.is_float && s.C == L.d.cin && L.d.cout > 0, DSP_EINVAL, "layer %d: linear shape mismatch", i);
            t.C = L.d.cout; t.H = 1; t.W = 1; t.is_float = true;
            L.p0 = poff; L.p1 = poff + (size_t)L.d.cin * L.d.cout;
            poff += (size_t)L.d.cin * L.d.cout + L.d.cout;
            break;
        case DSP_OP_SOFTMAX_CE:
            DSP_REQUIRE(s.is_float && i == d.n_layers - 1 && d.k == d.K - 1, DSP_EINVAL,
                        "layer %d: softmax_ce must close the last block", i);
            t.C = 1; t.H = 1; t.W = 1; t.is_float = true;
            b->loss_idx = i;
            break;
        default:
            DSP_REQUIRE(false, DSP_EINVAL, "layer %d: unknown op %d", i, L.d.op);
        }
        t.elems = (size_t)t.N * t.C * t.H * t.W;
    }
    b->out_idx = b->loss_idx >= 0 ? b->layers[b->loss_idx].d.in0 : d.n_layers - 1;
    DSP_REQUIRE(b->out_idx >= 0, DSP_EINVAL, "block: the loss needs a producing layer");
    b->nP = poff;
    b->wt_elems = wtoff;

    // every tensor must be consumed (or be the block output); decide overwrite vs accumulate for
    // each gradient buffer by walking the layers in backward order
    std::vector<char> written(d.n_layers + 1, 0);  // index t+1
    for (int i = d.n_layers - 1; i >= 0; --i) {
        Layer& L = b->layers[i];
        if (L.d.op == DSP_OP_SOFTMAX_CE) { written[L.d.in0 + 1] = 1; continue; }
        if (i != b->out_idx) DSP_REQUIRE(written[i + 1], DSP_EINVAL, "layer %d: output is never used", i);
        L.in0_grad = !(L.d.in0 < 0 && !d.needs_input_grad);
        if (L.in0_grad) { L.in0_acc = written[L.d.in0 + 1]; written[L.d.in0 + 1] = 1; }
        if ((L.d.op == DSP_OP_BN && L.d.in1 != -2) || L.d.op == DSP_OP_ADD) {
            L.in1_grad = !(L.d.in1 < 0 && !d.needs_input_grad);
            if (L.in1_grad) { L.in1_acc = written[L.d.in1 + 1]; written[L.d.in1 + 1] = 1; }
        } else {
            L.in1_grad = false;
        }
    }
    if (d.needs_input_grad) DSP_REQUIRE(written[0], DSP_EINVAL, "block: the input never reaches a layer");

    // The backward of a sum hands its gradient to both operands unchanged.  Two cases need no copy:
    // the operand has no other consumer (its producer reads the sum's gradient in place), or its only
    // other consumer is an earlier batch norm reading it as in0, which then forms
    // (its own input gradient) + (the sum's gradient) in one pass instead of accumulating onto a copy.
    b->grad_alias.assign(d.n_layers, -1);
    {
        std::vector<std::vector<std::pair<int, int>>> consumers(d.n_layers + 1);  // tensor t+1 -> (layer, operand)
        for (int i = 0; i < d.n_layers; ++i) {
            const Layer& L = b->layers[i];
            if (L.d.op == DSP_OP_SOFTMAX_CE) continue;
            consumers[L.d.in0 + 1].push_back({i, 0});
            if ((L.d.op == DSP_OP_BN && L.d.in1 != -2) || L.d.op == DSP_OP_ADD) consumers[L.d.in1 + 1].push_back({i, 1});
        }
        // A tensor read by two convolutions, the later one (in layer order) a 1x1 / stride-2 projection: its backward-data
        // reaches only one pixel in four, and as the first writer of the gradient buffer it would have to fill the other
        // three quarters with zeros.  It is issued after the other convolution's backward-data instead and accumulates
        // onto it: one sparse launch instead of four.
        for (int t = -1; t < d.n_layers; ++t) {  // -1: the block input
            const auto& cs = consumers[t + 1];
            if (cs.size() != 2 || cs[0].second != 0 || cs[1].second != 0) continue;
            const int lo = cs[0].first < cs[1].first ? cs[0].first : cs[1].first, hi = cs[0].first + cs[1].first - lo;
            Layer& J = b->layers[lo];
            Layer& Lh = b->layers[hi];
            if (J.d.op != DSP_OP_CONV || Lh.d.op != DSP_OP_CONV || !J.in0_grad || !Lh.in0_grad) continue;
            if (!(Lh.d.stride == 2 && Lh.d.r == 1 && Lh.d.s == 1) || Lh.in0_acc || !J.in0_acc) continue;
            Lh.in0_acc = true;
            J.in0_acc = false;
            Lh.dgrad_after = lo;
        }
        for (int i = 0; i + 1 < d.n_layers; ++i) {
            Layer& L = b->layers[i];
            Layer& nx = b->layers[i + 1];
            if (L.d.op == DSP_OP_BN && L.d.relu && L.d.in1 == -2 && i != b->out_idx && L.d.in0 >= 0 && nx.d.op == DSP_OP_MAXPOOL &&
                nx.d.in0 == i && consumers[i + 1].size() == 1 && bn_relu_maxpool_supported(b->dtype, L.d.cin, nx.d.r)) {
                L.pool_fused = true;
                nx.bn_fused = i;
                L.pool_bwd = L.in0_grad && nx.in0_grad && bn_pool_backward_supported(b->dtype, L.d.cin, b->T[i].H, b->T[i].W, nx.d.r, nx.d.stride, nx.d.pad);
            }
        }
        for (int i = 0; i < d.n_layers; ++i) {
            Layer& L = b->layers[i];
            if (L.d.op != DSP_OP_ADD || L.d.in0 == L.d.in1) continue;
            for (int o = 0; o < 2; ++o) {
                const int t = o ? L.d.in1 : L.d.in0;
                const bool has_grad = o ? L.in1_grad : L.in0_grad, acc = o ? L.in1_acc : L.in0_acc;
                if (!has_grad || acc || t == b->out_idx) continue;
                const auto& cs = consumers[t + 1];
                if (cs.size() == 1 && t >= 0) {
                    b->grad_alias[t] = i;
                    (o ? L.in1_skip : L.in0_skip) = true;
                } else if (cs.size() == 2) {
                    const std::pair<int, int> other = cs[0].first == i ? cs[1] : cs[0];
                    Layer& J = b->layers[other.first];
                    if (J.d.op == DSP_OP_BN && other.second == 0 && other.first < i && J.in0_grad && J.in0_acc &&
                        J.dx_add_from < 0) {
                        J.dx_add_from = i;
                        (o ? L.in1_skip : L.in0_skip) = true;
                    }
                }
            }
        }
    }

    // parameter index maps and the update kernel's task list
    b->perm.resize(b->nP);
    std::vector<int32_t> tmap(b->nP, -1);
    std::vector<UpdateTask> tasks;
    std::vector<int32_t> tap_tab;
    auto flat_task = [&](size_t p0, size_t n, bool decay) {
        if (n == 0) return;
        if (!tasks.empty() && tasks.back().kind == 0 && tasks.back().decay == (decay ? 1 : 0) &&
            (size_t)tasks.back().p0 + tasks.back().n == p0) {
            tasks.back().n += (uint32_t)n;
            return;
        }
        UpdateTask t{};
        t.kind = 0; t.decay = decay ? 1 : 0; t.p0 = (uint32_t)p0; t.n = (uint32_t)n;
        tasks.push_back(t);
    };
    for (int i = 0; i < d.n_layers; ++i) {
        const Layer& L = b->layers[i];
        if (L.d.op == DSP_OP_CONV) {
            const int G = conv_groups(L.cs), Cog = L.d.cout / G;
            const int Co = L.d.cout, Ci = L.d.cin / G, R = L.d.r, S = L.d.s;  // Ci: input channels of one group
            const size_t n = (size_t)Co * R * S * Ci;
            for (int co = 0; co < Co; ++co)
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s)
                        for (int ci = 0; ci < Ci; ++ci) {
                            const size_t lib = L.p0 + (((size_t)co * R + r) * S + s) * Ci + ci;
                            b->perm[lib] = (int32_t)(L.p0 + (((size_t)co * Ci + ci) * R + r) * S + s);
                            if (L.s2d) {
                                const int ur = r - 3, us = s - 3;  // offsets from the centre tap; >> and & floor towards -inf
                                const int ta = (ur >> 1) + 2, tb = (us >> 1) + 2, cell = (ur & 1) * 2 + (us & 1);
                                tmap[lib] = (int32_t)(L.wt_off + (((size_t)co * 4 + ta) * 4 + tb) * L.cin_pad + cell * Ci + ci);
                            } else if (L.cin_pad)
                                tmap[lib] = (int32_t)(L.wt_off + (((size_t)co * R + r) * S + s) * L.cin_pad + ci);
                        }
            if (L.cin_pad) {
                UpdateTask t{};
                t.kind = 2; t.decay = 1; t.p0 = (uint32_t)L.p0; t.n = (uint32_t)n;
                tasks.push_back(t);
            } else if (L.in0_grad) {
                UpdateTask t{};
                t.kind = 1; t.decay = 1; t.p0 = (uint32_t)L.p0; t.n = (uint32_t)n; t.wt_off = (uint32_t)L.wt_off;
                t.Co = Co; t.Ci = Ci; t.R = R; t.S = S; t.J = R * S * Ci; t.Cog = Cog;
                t.tap_tab = (int)tap_tab.size();
                DgradClass cls[4];
                if (L.d.stride == 2) dgrad_classes(L.cs, cls);
                for (int r = 0; r < R; ++r)
                    for (int s = 0; s < S; ++s) {
                        const int rf = R - 1 - r, sf = S - 1 - s;  // tap of the flipped filter
                        if (L.d.stride == 2) {
                            const int padh = R - 1 - L.d.pad, padw = S - 1 - L.d.pad;
                            const int ph = ((padh - rf) % 2 + 2) % 2, pw = ((padw - sf) % 2 + 2) % 2;
                            const DgradClass& k = cls[ph * 2 + pw];
                            const int jj = (rf - k.r0) / 2, ll = (sf - k.s0) / 2;
                            tap_tab.push_back((int32_t)(k.wt_off + ((size_t)jj * k.Sc + ll) * Cog));
                            tap_tab.push_back((int32_t)((size_t)k.Rc * k.Sc * Cog));
                        } else {
                            tap_tab.push_back((int32_t)(((size_t)rf * S + sf) * Cog));
                            tap_tab.push_back((int32_t)((size_t)R * S * Cog));
                        }
                    }
                tasks.push_back(t);
            } else {
                flat_task(L.p0, n, true);
            }
        } else if (L.d.op == DSP_OP_BN) {
            for (size_t j = 0; j < 2 * (size_t)L.d.cin; ++j) b->perm[L.p0 + j] = (int32_t)(L.p0 + j);
            flat_task(L.p0, 2 * (size_t)L.d.cin, false);
        } else if (L.d.op == DSP_OP_LINEAR) {
            const size_t nw = (size_t)L.d.cin * L.d.cout;
            for (size_t j = 0; j < nw + L.d.cout; ++j) b->perm[L.p0 + j] = (int32_t)(L.p0 + j);
            flat_task(L.p0, nw, true);
            flat_task(L.p0 + nw, (size_t)L.d.cout, false);
        }
    }
    DSP_TRY(update_plan_finish(tasks, b->dtype, &b->upd_blocks));
    b->upd_n_tasks = (int)tasks.size();
    DSP_REQUIRE(b->nP < (1ull << 31), DSP_EINVAL, "block: too many parameters");

    // device buffers
    const size_t esz = dtype_size(b->dtype);
    DSP_TRY(dev_alloc(b, (void**)&b->x, b->nP * 4, &b->param_bytes));
    DSP_TRY(dev_alloc(b, (void**)&b->v, b->nP * 4, &b->param_bytes));
    DSP_TRY(dev_alloc(b, (void**)&b->g, b->nP * 4, &b->param_bytes));
    DSP_TRY(dev_alloc(b, (void**)&b->upd_tasks, tasks.size() * sizeof(UpdateTask), &b->param_bytes));
    if (!tasks.empty())
        DSP_HIP(hipMemcpy(b->upd_tasks, tasks.data(), tasks.size() * sizeof(UpdateTask), hipMemcpyHostToDevice));
    DSP_TRY(dev_alloc(b, (void**)&b->tap_tab, tap_tab.size() * sizeof(int32_t), &b->param_bytes));
    if (!tap_tab.empty())
        DSP_HIP(hipMemcpy(b->tap_tab, tap_tab.data(), tap_tab.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    DSP_TRY(dev_alloc(b, (void**)&b->tmap, b->nP * 4, &b->param_bytes));
    DSP_TRY(dev_alloc(b, &b->wt, b->wt_elems * esz, &b->param_bytes));
    DSP_HIP(hipMemset(b->wt, 0, b->wt_elems * esz ? b->wt_elems * esz : 16));  // the zero channels of padded filters stay zero
    if (b->dtype == DSP_BF16) DSP_TRY(dev_alloc(b, &b->wf16, b->nP * 2, &b->param_bytes));
    if (b->nP) {
        DSP_HIP(hipMemcpy(b->tmap, tmap.data(), b->nP * 4, hipMemcpyHostToDevice));
        DSP_HIP(hipMemset(b->v, 0, b->nP * 4));
        DSP_HIP(hipMemset(b->g, 0, b->nP * 4));
    }

    b->ring_entries = 1 + d.m_k + d.p_prev;
    b->slot_bytes = (b->input.elems * esz + 255) / 256 * 256;
    DSP_TRY(dev_alloc(b, (void**)&b->ring, b->slot_bytes * b->ring_entries, &b->ring_bytes));
    b->slot_version.assign(b->ring_entries, -1);

    int max_c = 1;
    size_t ws = 0;
    for (int i = 0; i < d.n_layers; ++i) {
        Layer& L = b->layers[i];
        Tensor& t = b->T[i];
        if (L.d.op == DSP_OP_SOFTMAX_CE) continue;
        if (!L.pool_fused) DSP_TRY(dev_alloc(b, &t.act, t.bytes(b->dtype), &b->ws_bytes));
        if ((i != b->out_idx || b->loss_idx >= 0) && !L.pool_bwd) DSP_TRY(dev_alloc(b, &t.grad, t.bytes(b->dtype), &b->ws_bytes));
        if (L.d.op == DSP_OP_BN) {
            DSP_TRY(dev_alloc(b, (void**)&L.mean, (size_t)L.d.cin * 4, &b->ws_bytes));
            DSP_TRY(dev_alloc(b, (void**)&L.invstd, (size_t)L.d.cin * 4, &b->ws_bytes));
            DSP_TRY(dev_alloc(b, (void**)&L.fcoef, (size_t)L.d.cin * 8, &b->ws_bytes));
            if (L.d.relu && L.d.in1 != -2) {
                const size_t nb = bn_relu_bits_bytes(b->dtype, (int64_t)t.N * t.H * t.W, t.C);
                if (nb) DSP_TRY(dev_alloc(b, (void**)&L.relu_bits, nb, &b->ws_bytes));
            }
            if (L.d.cin > max_c) max_c = L.d.cin;
        }
        if (L.d.op == DSP_OP_MAXPOOL) DSP_TRY(dev_alloc(b, (void**)&L.argmax, t.elems, &b->ws_bytes));
        if (L.cin_pad) {
            DSP_TRY(dev_alloc(b, &L.xpad, (size_t)L.cs.N * L.cs.H * L.cs.W * L.cin_pad * esz, &b->ws_bytes));
            DSP_TRY(dev_alloc(b, (void**)&L.dw_pad, (size_t)L.cs.Cout * L.cs.R * L.cs.S * L.cin_pad * 4, &b->ws_bytes));
        }
        if (L.d.op == DSP_OP_CONV) {
            L.wg_off = ws;
            L.wg_bytes = (conv_backward_weight_workspace(L.cs) + 255) & ~(size_t)255;
            ws += L.wg_bytes;
        }
    }
    b->wgrad_ws_bytes = ws;
    DSP_TRY(dev_alloc(b, &b->wgrad_ws, ws, &b->ws_bytes));
    {
        std::vector<WgradReduceItem> items;
        for (Layer& L : b->layers) {
            if (L.d.op != DSP_OP_CONV) continue;
            float* dw = L.cin_pad ? L.dw_pad : b->g + L.p0;
            items.push_back(WgradReduceItem{(const float*)((char*)b->wgrad_ws + L.wg_off), dw,
                                            (size_t)L.cs.Cout * L.cs.R * L.cs.S * (L.cs.Cin / conv_groups(L.cs)),
                                            conv_backward_weight_slices(b->dtype, L.cs)});
        }
        DSP_TRY(wgrad_reduce_set_create(items.data(), (int)items.size(), &b->wgrad_set));
    }
    size_t partial_elems = (size_t)bn_max_partial_blocks() * max_c;
    for (int i = 0; i + 1 < d.n_layers; ++i) {
        Layer& L = b->layers[i];
        Layer& nx = b->layers[i + 1];
        if (nx.d.op != DSP_OP_BN || nx.d.in0 != i) continue;
        if (L.d.op == DSP_OP_ADD) {
            // the sum layer of a pre-activation unit also leaves the column sums of its output for the next unit's BN
            const Tensor& t = b->T[i];
            L.sum_tiles = nx.sum_tiles = add_stats_blocks(b->dtype, (int64_t)t.N * t.H * t.W, t.C);
            const size_t e = (size_t)L.sum_tiles * t.C;
            if (e > partial_elems) partial_elems = e;
            continue;
        }
        if (L.d.op != DSP_OP_CONV) continue;
        L.sum_tiles = nx.sum_tiles = conv_forward_row_tiles(b->dtype, L.cs);
        const size_t e = (size_t)L.sum_tiles * L.d.cout;
        if (e > partial_elems) partial_elems = e;
    }
    b->bn_partial_elems = partial_elems;
    b->bn_max_c = max_c;
    DSP_TRY(dev_alloc(b, (void**)&b->bn_partial, partial_elems * 2 * sizeof(double), &b->ws_bytes));
    DSP_TRY(dev_alloc(b, (void**)&b->bn_coef, (size_t)3 * max_c * 4, &b->ws_bytes));
    DSP_TRY(dev_alloc(b, (void**)&b->loss_sink, 4, &b->ws_bytes));
    if (b->loss_idx >= 0) {
        const Tensor& z = b->T[b->out_idx];
        b->dz_elems = z.elems;
        DSP_TRY(dev_alloc(b, (void**)&b->dz_ring, z.elems * 4 * (1 + d.m_k), &b->ws_bytes));
        DSP_TRY(dev_alloc(b, (void**)&b->row_loss, (size_t)z.N * 4, &b->ws_bytes));
    }
    return DSP_OK;
}

static int upload_params(dsp_block* b, const float* h, float* dst)
{
    std::vector<float> lib(b->nP);
    for (size_t i = 0; i < b->nP; ++i) lib[i] = h[b->perm[i]];
    if (b->nP) DSP_HIP(hipMemcpy(dst, lib.data(), b->nP * 4, hipMemcpyHostToDevice));
    return DSP_OK;
}

static int download_params(dsp_block* b, const float* src, float* h)
{
    std::vector<float> lib(b->nP);
    DSP_HIP(hipDeviceSynchronize());
    if (b->nP) DSP_HIP(hipMemcpy(lib.data(), src, b->nP * 4, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < b->nP; ++i) h[b->perm[i]] = lib[i];
    return DSP_OK;
}

// One forward pass: where it reads its input, where the block output goes (nullptr: the lane's own
// buffer) and which buffer set it writes (nullptr: the primary set, the one the backward sweep reads).
struct ForwardPass {
    const ForwardLane* lane;
    const void* in;
    void* out_override;
};

// f_k with the live parameters.  `twin` != nullptr runs a second pass (a recompute: no loss) through
// the same launches wherever the layer kernels take two instances, else right after the first.
static int run_forward(dsp_block* b, const ForwardPass& P, const ForwardPass* twin, const int32_t* labels, float* loss,
                       float* dz_slot, hipStream_t st)
{
    const int n = (int)b->layers.size();
    for (int i = 0; i < n; ++i) {
        Layer& L = b->layers[i];
        const Tensor& s = L.d.in0 < 0 ? b->input : b->T[L.d.in0];
        // the block output lives in out_override when one is given (only the loss may read it back)
        auto act_of = [&](const ForwardPass& p, int t) -> void* {
            if (t == b->out_idx && p.out_override) return p.out_override;
            return p.lane ? p.lane->act[t] : b->T[t].act;
        };
        auto src_of = [&](const ForwardPass& p, int t) -> const void* { return t < 0 ? p.in : act_of(p, t); };
        auto bn_buffers = [&](const ForwardPass& p) {
            return BnBuffers{p.lane ? p.lane->bn_partial : b->bn_partial, p.lane ? p.lane->mean[i] : L.mean,
                             p.lane ? p.lane->invstd[i] : L.invstd, p.lane ? p.lane->bn_coef : L.fcoef};
        };
        const int passes = twin ? 2 : 1;
        switch (L.d.op) {
        case DSP_OP_CONV: {
            auto conv_src = [&](const ForwardPass& p) -> const void* {
                return L.cin_pad ? (p.lane ? p.lane->xpad[i] : L.xpad) : src_of(p, L.d.in0);
            };
            if (L.cin_pad)
                for (int q = 0; q < passes; ++q) {
                    const ForwardPass& p = q ? *twin : P;
                    if (L.s2d)
                        DSP_TRY(launch_space_to_depth2(b->dtype, p.in, const_cast<void*>(conv_src(p)), L.cs.N, L.in_h, L.in_w,
                                                       L.d.cin, L.cin_pad, st));
                    else
                        DSP_TRY(launch_pad_channels(b->dtype, p.in, const_cast<void*>(conv_src(p)),
                                                    (int64_t)L.cs.N * L.cs.H * L.cs.W, L.d.cin, L.cin_pad, st));
                }
            ConvForwardTwin tw{};
            if (twin) tw = ConvForwardTwin{conv_src(*twin), act_of(*twin, i), L.sum_tiles > 0 ? bn_buffers(*twin).partial : nullptr};
            DSP_TRY(launch_conv_forward(b->dtype, L.cs, conv_src(P), L.cin_pad ? weights_for_dgrad(b, L) : weights_for_forward(b, L),
                                        act_of(P, i), st, L.sum_tiles > 0 ? bn_buffers(P).partial : nullptr,
                                        twin ? &tw : nullptr));
            break;
        }
        case DSP_OP_BN: {
            BnForwardTwin tw{};
            if (twin)
                tw = BnForwardTwin{src_of(*twin, L.d.in0), L.d.in1 == -2 ? nullptr : src_of(*twin, L.d.in1), act_of(*twin, i),
                                   bn_buffers(*twin), twin->lane ? nullptr : L.relu_bits};
            DSP_TRY(launch_bn_forward(b->dtype, src_of(P, L.d.in0), L.d.in1 == -2 ? nullptr : src_of(P, L.d.in1),
                                      act_of(P, i), b->x + L.p0, b->x + L.p1, b->desc.bn_eps, (int64_t)s.N * s.H * s.W, s.C,
                                      L.d.relu != 0, bn_buffers(P), st, L.sum_tiles, twin ? &tw : nullptr, L.pool_fused,
                                      P.lane ? nullptr : L.relu_bits));
            break;
        }
        case DSP_OP_ADD:
            if (L.sum_tiles > 0) {  // the next layer is a batch norm on this sum: leave its column sums as well
                AddStatsTwin tw{};
                if (twin) tw = AddStatsTwin{src_of(*twin, L.d.in0), src_of(*twin, L.d.in1), act_of(*twin, i), bn_buffers(*twin).partial};
                DSP_TRY(launch_add_forward_stats(b->dtype, src_of(P, L.d.in0), src_of(P, L.d.in1), act_of(P, i),
                                                 (int64_t)s.N * s.H * s.W, s.C, bn_buffers(P).partial, st, twin ? &tw : nullptr));
                break;
            }
            for (int q = 0; q < passes; ++q) {
                const ForwardPass& p = q ? *twin : P;
                DSP_TRY(launch_add_forward(b->dtype, src_of(p, L.d.in0), src_of(p, L.d.in1), act_of(p, i),
                                           (int64_t)s.N * s.H * s.W * s.C, st));
            }
            break;
        case DSP_OP_MAXPOOL:
            for (int q = 0; q < passes; ++q) {
                const ForwardPass& p = q ? *twin : P;
                uint8_t* am = p.lane ? p.lane->argmax[i] : L.argmax;
                if (L.bn_fused >= 0) {
                    // the batch norm in front left only its coefficients (no other batch norm has run since)
                    const Layer& B = b->layers[L.bn_fused];
                    DSP_TRY(launch_bn_relu_maxpool_forward(b->dtype, src_of(p, B.d.in0), p.lane ? p.lane->bn_coef : B.fcoef, act_of(p, i),
                                                           am, s.N, s.H, s.W, s.C, L.d.r, L.d.stride, L.d.pad, st));
                    continue;
                }
                DSP_TRY(launch_maxpool_forward(b->dtype, src_of(p, L.d.in0), act_of(p, i), am, s.N, s.H, s.W, s.C, L.d.r, L.d.stride,
                                               L.d.pad, st));
            }
            break;
        case DSP_OP_GAP:
            for (int q = 0; q < passes; ++q) {
                const ForwardPass& p = q ? *twin : P;
                DSP_TRY(launch_gap_forward(b->dtype, src_of(p, L.d.in0), (float*)act_of(p, i), s.N, s.H * s.W, s.C, st));
            }
            break;
        case DSP_OP_LINEAR:
            for (int q = 0; q < passes; ++q) {
                const ForwardPass& p = q ? *twin : P;
                DSP_TRY(launch_linear_forward((const float*)src_of(p, L.d.in0), b->x + L.p0, b->x + L.p1, (float*)act_of(p, i),
                                              s.N, L.d.cin, L.d.cout, st));
            }
            break;
        case DSP_OP_SOFTMAX_CE:
            // the loss and its gradient belong to the forward pass (Eq. (5), third line); a recompute
            // (labels == nullptr, and always the twin) reuses the gradient stored then and must not touch them
            if (labels) {
                DSP_REQUIRE(loss && dz_slot, DSP_EINVAL, "softmax_ce: missing loss buffers");
                DSP_TRY(launch_softmax_ce((const float*)src_of(P, L.d.in0), labels, loss, dz_slot, b->row_loss, s.N, s.C, st));
            }
            break;
        }
    }
    return DSP_OK;
}

// Reverse sweep over the tensors left by run_forward (all in the workspace).
static int run_backward(dsp_block* b, const void* in, const void* gout, void* gin, hipStream_t st)
{
    const int n = (int)b->layers.size();
    auto grad_of = [&](int t) -> void* { return t < 0 ? gin : b->T[t].grad; };
    for (int i = n - 1; i >= 0; --i) {
        Layer& L = b->layers[i];
        if (L.d.op == DSP_OP_SOFTMAX_CE) continue;
        const Tensor& s = L.d.in0 < 0 ? b->input : b->T[L.d.in0];
        const void* src = L.d.in0 < 0 ? in : b->T[L.d.in0].act;
        auto dy_of = [&](int layer) -> const void* {  // the buffer that holds the gradient of a layer's output
            int t = layer;
            while (t != b->out_idx && b->grad_alias[t] >= 0) t = b->grad_alias[t];
            return (t == b->out_idx) ? gout : b->T[t].grad;
        };
        const void* dy = dy_of(i);
        switch (L.d.op) {
        case DSP_OP_CONV:
            // per-slice partial sums only; they are summed for all layers after the sweep
            DSP_TRY(launch_conv_backward_weight(b->dtype, L.cs, L.cin_pad ? L.xpad : src, dy,
                                                L.cin_pad ? L.dw_pad : b->g + L.p0, (char*)b->wgrad_ws + L.wg_off,
                                                L.wg_bytes, st, /*defer_reduce=*/true));
            if (L.in0_grad && L.dgrad_after < 0)
                DSP_TRY(launch_conv_backward_data(b->dtype, L.cs, dy, weights_for_dgrad(b, L), grad_of(L.d.in0), L.in0_acc, st));
            for (int j = i + 1; j < n; ++j) {  // the projection that waited for this layer's backward-data
                Layer& Pj = b->layers[j];
                if (Pj.d.op == DSP_OP_CONV && Pj.dgrad_after == i)
                    DSP_TRY(launch_conv_backward_data(b->dtype, Pj.cs, dy_of(j), weights_for_dgrad(b, Pj), grad_of(Pj.d.in0), true, st));
            }
            break;
        case DSP_OP_BN: {
            BnBuffers buf{b->bn_partial, L.mean, L.invstd, b->bn_coef};
            void* dres = L.in1_grad ? grad_of(L.d.in1) : nullptr;
            DSP_REQUIRE(L.in0_grad, DSP_EINVAL, "bn directly on the data input is not supported");
            const void* dx_add = nullptr;
            if (L.dx_add_from >= 0) {
                int t = L.dx_add_from;
                while (t != b->out_idx && b->grad_alias[t] >= 0) t = b->grad_alias[t];
                dx_add = (t == b->out_idx) ? gout : b->T[t].grad;
            }
            PoolGrad pg{};
            if (L.pool_bwd) {  // dy is the backward of the pool behind this layer, formed inside the kernels
                const Layer& Pl = b->layers[i + 1];
                pg = PoolGrad{dy_of(i + 1), Pl.argmax, s.H, s.W, Pl.d.r, Pl.d.stride, Pl.d.pad};
                dy = nullptr;
            }
            DSP_TRY(launch_bn_backward(b->dtype, dy, src, b->T[i].act, grad_of(L.d.in0), dres, L.in1_acc, L.in0_acc,
                                       b->x + L.p0, b->g + L.p0, b->g + L.p1, (int64_t)s.N * s.H * s.W, s.C,
                                       L.d.relu != 0, buf, st, dx_add,
                                       L.d.in1 == -2 ? L.fcoef : nullptr, L.pool_bwd ? &pg : nullptr, L.relu_bits));
            break;
        }
        case DSP_OP_ADD: {
            // both operands in one launch (dy is read once); the same tensor on both sides would need in0 before
            // in1, the order in which the overwrite / accumulate flags were decided, so it takes two launches
            const int64_t n_el = (int64_t)s.N * s.H * s.W * s.C;
            void* d0 = (L.in0_grad && !L.in0_skip) ? grad_of(L.d.in0) : nullptr;
            void* d1 = (L.in1_grad && !L.in1_skip) ? grad_of(L.d.in1) : nullptr;
            if (d0 && d1 && d0 != d1) {
                DSP_TRY(launch_grad_pass(b->dtype, dy, d0, L.in0_acc, d1, L.in1_acc, n_el, st));
            } else {
                if (d0) DSP_TRY(launch_grad_pass(b->dtype, dy, d0, L.in0_acc, nullptr, false, n_el, st));
                if (d1) DSP_TRY(launch_grad_pass(b->dtype, dy, d1, L.in1_acc, nullptr, false, n_el, st));
            }
            break;
        }
        case DSP_OP_MAXPOOL:
            if (L.in0_grad && !(L.bn_fused >= 0 && b->layers[L.bn_fused].pool_bwd))
                DSP_TRY(launch_maxpool_backward(b->dtype, dy, L.argmax, grad_of(L.d.in0), L.in0_acc, s.N, s.H, s.W, s.C,
                                                L.d.r, L.d.stride, L.d.pad, st));
            break;
        case DSP_OP_GAP:
            if (L.in0_grad)
                DSP_TRY(launch_gap_backward(b->dtype, (const float*)dy, grad_of(L.d.in0), L.in0_acc, s.N, s.H * s.W, s.C, st));
            break;
        case DSP_OP_LINEAR:
            DSP_REQUIRE(!L.in0_acc, DSP_EINVAL, "linear input with several consumers is not supported");
            DSP_TRY(launch_linear_backward((const float*)src, b->x + L.p0, (const float*)dy,
                                           L.in0_grad ? (float*)grad_of(L.d.in0) : nullptr, b->g + L.p0, b->g + L.p1,
                                           s.N, L.d.cin, L.d.cout, st));
            break;
        }
    }
    DSP_TRY(wgrad_reduce_set_launch(b->wgrad_set, st));
    for (Layer& L : b->layers)
        if (L.d.op == DSP_OP_CONV && L.cin_pad)
            DSP_TRY(launch_gather_f32(L.dw_pad, b->tmap + L.p0, (int32_t)L.wt_off, b->g + L.p0,
                                      (int64_t)L.d.cout * L.d.r * L.d.s * L.d.cin, st));
    return DSP_OK;
}

void block_set_dry(dsp_block* b, bool dry) { b->dry = dry; }

BlockArrays block_arrays(dsp_block* b) { return BlockArrays{b->x, b->g, b->nP}; }

int block_load_params_device(dsp_block* b, const float* d_src, hipStream_t st)
{
    if (b->nP == 0) return DSP_OK;
    DSP_HIP(hipMemcpyAsync(b->x, d_src, b->nP * 4, hipMemcpyDeviceToDevice, st));
    return launch_refresh_shadows(b->dtype, b->x, b->upd_tasks, b->upd_n_tasks, b->upd_blocks, b->tmap, b->tap_tab, b->wf16, b->wt, b->nP, st);
}

}  // namespace dsp

// ================================================================================================
extern "C" {

int dsp_block_init(const dsp_block_desc* desc, const float* h_params, size_t n_params, dsp_block** out)
{
    DSP_REQUIRE(desc && out, DSP_EINVAL, "dsp_block_init: null argument");
    *out = nullptr;
    dsp_block* b = new (std::nothrow) dsp_block();
    DSP_REQUIRE(b, DSP_ENOMEM, "dsp_block_init: out of host memory");
    b->desc = *desc;
    int rc = build_graph(b);
    if (rc == DSP_OK && n_params != b->nP) {
        set_error("dsp_block_init: expected %zu parameters, got %zu", b->nP, n_params);
        rc = DSP_EINVAL;
    }
    if (rc == DSP_OK && b->nP && !h_params) {
        set_error("dsp_block_init: null parameters");
        rc = DSP_EINVAL;
    }
    if (rc == DSP_OK) rc = upload_params(b, h_params, b->x);
    if (rc == DSP_OK) rc = launch_refresh_shadows(b->dtype, b->x, b->upd_tasks, b->upd_n_tasks, b->upd_blocks, b->tmap, b->tap_tab, b->wf16, b->wt, b->nP, nullptr);
    if (rc == DSP_OK && hipDeviceSynchronize() != hipSuccess) {
        set_error("dsp_block_init: device synchronisation failed");
        rc = DSP_EHIP;
    }
    b->desc.layers = nullptr;  // the caller's array is not kept
    if (rc != DSP_OK) {
        dsp_block_destroy(b);
        return rc;
    }
    *out = b;
    return DSP_OK;
}

int dsp_block_destroy(dsp_block* b)
{
    if (!b) return DSP_OK;
    (void)hipDeviceSynchronize();
    for (void* p : b->allocs) (void)hipFree(p);
    wgrad_reduce_set_destroy(b->wgrad_set);
    delete b->fwd_lane;
    delete b;
    return DSP_OK;
}

int dsp_block_enable_forward_lane(dsp_block* b)
{
    DSP_REQUIRE(b, DSP_EINVAL, "dsp_block_enable_forward_lane: null block");
    DSP_REQUIRE(b->desc.m_k > 0, DSP_EINVAL,
                "dsp_block_enable_forward_lane: with m_k = 0 the backward reuses the forward's activations");
    if (b->fwd_lane) return DSP_OK;
    ForwardLane* ln = new (std::nothrow) ForwardLane();
    DSP_REQUIRE(ln, DSP_ENOMEM, "dsp_block_enable_forward_lane: out of host memory");
    const int n = (int)b->layers.size();
    ln->act.assign(n, nullptr);
    ln->mean.assign(n, nullptr);
    ln->invstd.assign(n, nullptr);
    ln->argmax.assign(n, nullptr);
    ln->xpad.assign(n, nullptr);
    int rc = DSP_OK;
    for (int i = 0; i < n && rc == DSP_OK; ++i) {
        const Layer& L = b->layers[i];
        const Tensor& t = b->T[i];
        if (L.d.op == DSP_OP_SOFTMAX_CE) continue;
        if (!L.pool_fused) rc = dev_alloc(b, &ln->act[i], t.bytes(b->dtype), &b->ws_bytes);
        if (rc == DSP_OK && L.d.op == DSP_OP_BN) {
            rc = dev_alloc(b, (void**)&ln->mean[i], (size_t)L.d.cin * 4, &b->ws_bytes);
            if (rc == DSP_OK) rc = dev_alloc(b, (void**)&ln->invstd[i], (size_t)L.d.cin * 4, &b->ws_bytes);
        }
        if (rc == DSP_OK && L.d.op == DSP_OP_MAXPOOL) rc = dev_alloc(b, (void**)&ln->argmax[i], t.elems, &b->ws_bytes);
        if (rc == DSP_OK && L.cin_pad)
            rc = dev_alloc(b, &ln->xpad[i], (size_t)L.cs.N * L.cs.H * L.cs.W * L.cin_pad * dtype_size(b->dtype), &b->ws_bytes);
    }
    if (rc == DSP_OK) rc = dev_alloc(b, (void**)&ln->bn_partial, b->bn_partial_elems * 2 * sizeof(double), &b->ws_bytes);
    if (rc == DSP_OK) rc = dev_alloc(b, (void**)&ln->bn_coef, (size_t)3 * b->bn_max_c * 4, &b->ws_bytes);
    if (rc != DSP_OK) {
        delete ln;  // the device buffers stay on the block's list and are freed with it
        return rc;
    }
    b->fwd_lane = ln;
    return DSP_OK;
}

int dsp_block_input_slot(dsp_block* b, int64_t batch_id, void** d_slot)
{
    DSP_REQUIRE(b && d_slot && batch_id >= 0, DSP_EINVAL, "dsp_block_input_slot: bad argument");
    *d_slot = b->ring + (size_t)(batch_id % b->ring_entries) * b->slot_bytes;
    return DSP_OK;
}

}  // extern "C"

namespace dsp {

// Checks and host-side state of a forward call; stores the input into its ring slot.
struct ForwardCall {
    void* slot;
    float* dz;
    float* loss;
};
static int forward_begin(dsp_block* b, int64_t batch_id, const void* d_in, const int32_t* d_labels, float* d_loss,
                         hipStream_t st, ForwardCall* fc, const char* who)
{
    const int m = b->desc.m_k;
    DSP_REQUIRE(batch_id == b->next_fwd, DSP_ESTATE, "%s: expected mini-batch %lld, got %lld", who, (long long)b->next_fwd,
                (long long)batch_id);
    const int64_t due = batch_id - m;  // backward that must have been done before this forward
    DSP_REQUIRE(!b->pending && b->next_bwd == (due > 0 ? due : 0), DSP_ESTATE,
                "%s: the previous tick's backward/update has not been issued", who);
    DSP_REQUIRE(b->loss_idx < 0 || d_labels, DSP_EINVAL, "%s: the last block needs labels", who);
    const int slot = (int)(batch_id % b->ring_entries);
    fc->slot = b->ring + (size_t)slot * b->slot_bytes;
    fc->dz = b->loss_idx >= 0 ? b->dz_ring + (size_t)(batch_id % (1 + m)) * b->dz_elems : nullptr;
    fc->loss = d_loss ? d_loss : b->loss_sink;
    b->slot_version[slot] = b->version;
    b->next_fwd = batch_id + 1;
    if (!b->dry && d_in != fc->slot)
        DSP_HIP(hipMemcpyAsync(fc->slot, d_in, b->input.elems * dtype_size(b->dtype), hipMemcpyDeviceToDevice, st));
    return DSP_OK;
}

// Checks and host-side state of a recompute + backward call.
struct BackwardCall {
    void* slot;
    const void* gout;
};
static int backward_begin(dsp_block* b, int64_t batch_id, const void* d_grad_out, void* d_grad_in, BackwardCall* bc,
                          const char* who)
{
    const int m = b->desc.m_k;
    DSP_REQUIRE(!b->pending && batch_id == b->next_bwd && batch_id == b->next_fwd - 1 - m, DSP_ESTATE,
                "%s: mini-batch %lld is not due (next backward %lld, latest forward %lld, m_k %d)", who, (long long)batch_id,
                (long long)b->next_bwd, (long long)b->next_fwd - 1, m);
    DSP_REQUIRE(b->loss_idx >= 0 || d_grad_out, DSP_EINVAL, "%s: no error gradient", who);
    DSP_REQUIRE(!b->desc.needs_input_grad || d_grad_in, DSP_EINVAL, "%s: no room for G_h", who);
    const int slot = (int)(batch_id % b->ring_entries);
    bc->slot = b->ring + (size_t)slot * b->slot_bytes;
    bc->gout = d_grad_out;
    if (b->loss_idx >= 0 && !d_grad_out) bc->gout = b->dz_ring + (size_t)(batch_id % (1 + m)) * b->dz_elems;
    b->next_bwd = batch_id + 1;
    b->pending = true;
    return DSP_OK;
}

}  // namespace dsp

extern "C" {

int dsp_block_forward(dsp_block* b, int64_t batch_id, const void* d_in, void* d_out, const int32_t* d_labels,
                      float* d_loss, void* stream)
{
    DSP_REQUIRE(b && d_in, DSP_EINVAL, "dsp_block_forward: null argument");
    hipStream_t st = (hipStream_t)stream;
    ForwardCall fc;
    DSP_TRY(forward_begin(b, batch_id, d_in, d_labels, d_loss, st, &fc, "dsp_block_forward"));
    if (b->dry) return DSP_OK;
    const Tensor& o = b->T[b->out_idx];
    if (b->desc.m_k == 0) {
        // this forward is also the "recompute" of the backward that follows: keep everything
        DSP_TRY(run_forward(b, ForwardPass{nullptr, fc.slot, nullptr}, nullptr, d_labels, fc.loss, fc.dz, st));
        if (d_out) DSP_HIP(hipMemcpyAsync(d_out, o.act, o.bytes(b->dtype), hipMemcpyDeviceToDevice, st));
    } else {
        // the activations are thrown away (the backward of this mini-batch recomputes them); d_out == nullptr
        // (a last block whose output nobody takes) leaves the output in the lane's own buffer
        DSP_TRY(run_forward(b, ForwardPass{b->fwd_lane, fc.slot, d_out}, nullptr, d_labels, fc.loss, fc.dz, st));
    }
    return DSP_OK;
}

int dsp_block_recompute_backward(dsp_block* b, int64_t batch_id, const void* d_grad_out, void* d_grad_in, void* stream)
{
    DSP_REQUIRE(b, DSP_EINVAL, "dsp_block_recompute_backward: null block");
    hipStream_t st = (hipStream_t)stream;
    BackwardCall bc;
    DSP_TRY(backward_begin(b, batch_id, d_grad_out, d_grad_in, &bc, "dsp_block_recompute_backward"));
    if (b->dry) return DSP_OK;
    if (b->desc.m_k > 0)
        DSP_TRY(run_forward(b, ForwardPass{nullptr, bc.slot, nullptr}, nullptr, nullptr, b->loss_sink, nullptr, st));
    DSP_TRY(run_backward(b, bc.slot, bc.gout, d_grad_in, st));
    return DSP_OK;
}

int dsp_block_step(dsp_block* b, int64_t batch_fwd, const void* d_in, void* d_out, const int32_t* d_labels, float* d_loss,
                   int64_t batch_bwd, const void* d_grad_out, void* d_grad_in, void* stream)
{
    return block_step_event(b, batch_fwd, d_in, d_out, d_labels, d_loss, batch_bwd, d_grad_out, d_grad_in, (hipStream_t)stream,
                            nullptr);
}

}  // extern "C"

int dsp::block_step_event(dsp_block* b, int64_t batch_fwd, const void* d_in, void* d_out, const int32_t* d_labels, float* d_loss,
                     int64_t batch_bwd, const void* d_grad_out, void* d_grad_in, hipStream_t st, hipEvent_t after_forward)
{
    DSP_REQUIRE(b && d_in, DSP_EINVAL, "dsp_block_step: null argument");
    if (b->desc.m_k > 0 && !b->fwd_lane && !b->dry) DSP_TRY(dsp_block_enable_forward_lane(b));
    ForwardCall fc;
    BackwardCall bc;
    DSP_TRY(forward_begin(b, batch_fwd, d_in, d_labels, d_loss, st, &fc, "dsp_block_step"));
    DSP_TRY(backward_begin(b, batch_bwd, d_grad_out, d_grad_in, &bc, "dsp_block_step"));
    if (b->dry) return DSP_OK;
    if (b->desc.m_k == 0) {
        const Tensor& o = b->T[b->out_idx];
        DSP_TRY(run_forward(b, ForwardPass{nullptr, fc.slot, nullptr}, nullptr, d_labels, fc.loss, fc.dz, st));
        if (d_out) DSP_HIP(hipMemcpyAsync(d_out, o.act, o.bytes(b->dtype), hipMemcpyDeviceToDevice, st));
    } else {
        // forward of batch_fwd (lane buffers, output to d_out) and recompute of batch_bwd (primary buffers)
        // in one sweep: the two passes use the same parameters
        const ForwardPass recompute{nullptr, bc.slot, nullptr};
        DSP_TRY(run_forward(b, ForwardPass{b->fwd_lane, fc.slot, d_out}, &recompute, d_labels, fc.loss, fc.dz, st));
    }
    if (after_forward) DSP_HIP(hipEventRecord(after_forward, st));
    DSP_TRY(run_backward(b, bc.slot, bc.gout, d_grad_in, st));
    return DSP_OK;
}

extern "C" {

int dsp_param_update_sum(dsp_block* b, float lr, float momentum, int32_t s, float weight_decay, void* stream)
{
    DSP_REQUIRE(b, DSP_EINVAL, "dsp_param_update: null block");
    DSP_REQUIRE(s == 0 || s == 1, DSP_EINVAL, "dsp_param_update: s = %d (only s = 0 and s = 1 are built)", (int)s);
    DSP_REQUIRE(lr >= 0.f, DSP_EINVAL, "dsp_param_update: negative step size");
    DSP_REQUIRE(b->pending, DSP_ESTATE, "dsp_param_update: no pending gradient");
    DSP_REQUIRE(!(lr == 0.f && momentum != 0.f && b->last_lr > 0.f), DSP_EINVAL,
                "dsp_param_update: step size 0 after updates that carry momentum (Eq. (3) would still move x by "
                "momentum * (x^n - x^{n-1}); the velocity form cannot)");
    b->pending = false;
    b->version += 1;
    // the stored velocity is in units of the step size of the update that wrote it
    float v_scale = 1.f;
    if (lr > 0.f) {
        if (b->last_lr > 0.f && b->last_lr != lr) v_scale = b->last_lr / lr;
        b->last_lr = lr;
    }
    if (b->dry) return DSP_OK;
    DSP_TRY(launch_sgd_update(b->dtype, b->x, b->v, b->g, b->upd_tasks, b->upd_n_tasks, b->upd_blocks, b->tmap, b->tap_tab, b->wf16, b->wt,
                              b->nP, lr, momentum, weight_decay, (hipStream_t)stream, s == 1, v_scale));
    return DSP_OK;
}

int dsp_param_update(dsp_block* b, float lr, float momentum, float weight_decay, void* stream)
{
    return dsp_param_update_sum(b, lr, momentum, 0, weight_decay, stream);
}

int dsp_block_query(const dsp_block* b, int64_t out[8])
{
    DSP_REQUIRE(b && out, DSP_EINVAL, "dsp_block_query: null argument");
    out[0] = b->version;
    out[1] = b->next_fwd;
    out[2] = b->next_bwd;
    out[3] = b->ring_entries;
    out[4] = b->pending ? 1 : 0;
    out[5] = (int64_t)b->nP;
    const bool stored = b->next_bwd < b->next_fwd;
    const int slot = (int)(b->next_bwd % b->ring_entries);
    out[6] = stored ? b->slot_version[slot] : -1;
    out[7] = stored ? slot : -1;
    return DSP_OK;
}

int dsp_block_output_shape(const dsp_block* b, int32_t out[5])
{
    DSP_REQUIRE(b && out, DSP_EINVAL, "dsp_block_output_shape: null argument");
    const Tensor& o = b->T[b->out_idx];
    out[0] = o.N; out[1] = o.C; out[2] = o.H; out[3] = o.W; out[4] = o.is_float ? 1 : 0;
    return DSP_OK;
}

int dsp_block_input_shape(const dsp_block* b, int32_t out[5])
{
    DSP_REQUIRE(b && out, DSP_EINVAL, "dsp_block_input_shape: null argument");
    out[0] = b->input.N; out[1] = b->input.C; out[2] = b->input.H; out[3] = b->input.W; out[4] = b->dtype;
    return DSP_OK;
}

int dsp_block_memory(const dsp_block* b, size_t* ring_bytes, size_t* workspace_bytes, size_t* param_bytes)
{
    DSP_REQUIRE(b, DSP_EINVAL, "dsp_block_memory: null block");
    if (ring_bytes) *ring_bytes = b->ring_bytes;
    if (workspace_bytes) *workspace_bytes = b->ws_bytes;
    if (param_bytes) *param_bytes = b->param_bytes;
    return DSP_OK;
}

int dsp_block_get_params(dsp_block* b, float* h_dst, size_t n)
{
    DSP_REQUIRE(b && h_dst && n == b->nP, DSP_EINVAL, "dsp_block_get_params: bad argument");
    return download_params(b, b->x, h_dst);
}
int dsp_block_set_params(dsp_block* b, const float* h_src, size_t n)
{
    DSP_REQUIRE(b && h_src && n == b->nP, DSP_EINVAL, "dsp_block_set_params: bad argument");
    DSP_HIP(hipDeviceSynchronize());
    DSP_TRY(upload_params(b, h_src, b->x));
    DSP_TRY(launch_refresh_shadows(b->dtype, b->x, b->upd_tasks, b->upd_n_tasks, b->upd_blocks, b->tmap, b->tap_tab, b->wf16, b->wt, b->nP, nullptr));
    DSP_HIP(hipDeviceSynchronize());
    return DSP_OK;
}
int dsp_block_get_momentum(dsp_block* b, float* h_dst, size_t n)
{
    DSP_REQUIRE(b && h_dst && n == b->nP, DSP_EINVAL, "dsp_block_get_momentum: bad argument");
    return download_params(b, b->v, h_dst);
}
int dsp_block_set_momentum(dsp_block* b, const float* h_src, size_t n)
{
    DSP_REQUIRE(b && h_src && n == b->nP, DSP_EINVAL, "dsp_block_set_momentum: bad argument");
    DSP_HIP(hipDeviceSynchronize());
    return upload_params(b, h_src, b->v);
}
int dsp_block_get_grads(dsp_block* b, float* h_dst, size_t n)
{
    DSP_REQUIRE(b && h_dst && n == b->nP, DSP_EINVAL, "dsp_block_get_grads: bad argument");
    return download_params(b, b->g, h_dst);
}

int dsp_block_get_activation(dsp_block* b, int32_t layer, void* h_dst, size_t bytes)
{
    DSP_REQUIRE(b && h_dst && layer >= 0 && layer < (int)b->layers.size(), DSP_EINVAL, "dsp_block_get_activation: bad argument");
    const Tensor& t = b->T[layer];
    const Layer& L = b->layers[layer];
    DSP_REQUIRE(t.act != nullptr || L.pool_fused, DSP_EINVAL, "dsp_block_get_activation: layer %d keeps no output", (int)layer);
    DSP_REQUIRE(bytes == t.bytes(b->dtype), DSP_EINVAL, "dsp_block_get_activation: layer %d holds %zu bytes, not %zu", (int)layer,
                t.bytes(b->dtype), bytes);
    DSP_HIP(hipDeviceSynchronize());
    if (L.pool_fused) {
        // the pool kernel formed this output on the fly; it is written out here, from the stored input and the forward
        // pass's coefficients, by the kernel that stores it where the two layers run apart
        const Tensor& s = b->T[L.d.in0];
        void* tmp = nullptr;
        DSP_HIP(hipMalloc(&tmp, bytes));
        int rc = launch_bn_apply(b->dtype, s.act, tmp, L.fcoef, (int64_t)s.N * s.H * s.W, s.C, true, nullptr);
        if (rc == DSP_OK && hipDeviceSynchronize() != hipSuccess) rc = DSP_EHIP;
        if (rc == DSP_OK && hipMemcpy(h_dst, tmp, bytes, hipMemcpyDeviceToHost) != hipSuccess) rc = DSP_EHIP;
        (void)hipFree(tmp);
        return rc;
    }
    DSP_HIP(hipMemcpy(h_dst, t.act, bytes, hipMemcpyDeviceToHost));
    return DSP_OK;
}

int dsp_block_get_pool_argmax(dsp_block* b, int32_t layer, uint8_t* h_dst, size_t bytes)
{
    DSP_REQUIRE(b && h_dst && layer >= 0 && layer < (int)b->layers.size(), DSP_EINVAL, "dsp_block_get_pool_argmax: bad argument");
    const Layer& L = b->layers[layer];
    DSP_REQUIRE(L.d.op == DSP_OP_MAXPOOL && L.argmax, DSP_EINVAL, "dsp_block_get_pool_argmax: layer %d is no max pool", (int)layer);
    DSP_REQUIRE(bytes == b->T[layer].elems, DSP_EINVAL, "dsp_block_get_pool_argmax: layer %d holds %zu bytes, not %zu", (int)layer,
                b->T[layer].elems, bytes);
    DSP_HIP(hipDeviceSynchronize());
    DSP_HIP(hipMemcpy(h_dst, L.argmax, bytes, hipMemcpyDeviceToHost));
    return DSP_OK;
}

// ---- single-layer entry points ---------------------------------------------------------------------
int dsp_grouped_conv_forward(int32_t dtype, const void* d_x, const void* d_w, void* d_y, int32_t N, int32_t H, int32_t W,
                             int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride, int32_t pad, int32_t groups,
                             void* stream)
{
    DSP_REQUIRE(d_x && d_w && d_y && (dtype == DSP_FP32 || dtype == DSP_BF16), DSP_EINVAL, "dsp_conv_forward: bad argument");
    DSP_REQUIRE(N > 0 && H > 0 && W > 0 && cin > 0 && cout > 0 && r > 0 && s > 0 && stride > 0 && pad >= 0 && groups > 0,
                DSP_EINVAL, "dsp_conv_forward: bad shape");
    return launch_conv_forward(dtype, make_conv_shape(N, H, W, cin, cout, r, s, stride, pad, groups), d_x, d_w, d_y,
                               (hipStream_t)stream);
}

int dsp_grouped_conv_backward_data(int32_t dtype, const void* d_dy, const void* d_wt, void* d_dx, int32_t N, int32_t H,
                                   int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride, int32_t pad,
                                   int32_t groups, int32_t accumulate, void* stream)
{
    DSP_REQUIRE(d_dy && d_wt && d_dx && (dtype == DSP_FP32 || dtype == DSP_BF16), DSP_EINVAL, "dsp_conv_backward_data: bad argument");
    DSP_REQUIRE(N > 0 && H > 0 && W > 0 && cin > 0 && cout > 0 && r > 0 && s > 0 && stride > 0 && pad >= 0 && groups > 0,
                DSP_EINVAL, "dsp_conv_backward_data: bad shape");
    return launch_conv_backward_data(dtype, make_conv_shape(N, H, W, cin, cout, r, s, stride, pad, groups), d_dy, d_wt, d_dx,
                                     accumulate != 0, (hipStream_t)stream);
}

int dsp_grouped_conv_backward_weight(int32_t dtype, const void* d_x, const void* d_dy, float* d_dw, int32_t N, int32_t H,
                                     int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride, int32_t pad,
                                     int32_t groups, void* d_workspace, size_t workspace_bytes, void* stream)
{
    DSP_REQUIRE(d_x && d_dy && d_dw && (dtype == DSP_FP32 || dtype == DSP_BF16), DSP_EINVAL, "dsp_conv_backward_weight: bad argument");
    DSP_REQUIRE(N > 0 && H > 0 && W > 0 && cin > 0 && cout > 0 && r > 0 && s > 0 && stride > 0 && pad >= 0 && groups > 0,
                DSP_EINVAL, "dsp_conv_backward_weight: bad shape");
    return launch_conv_backward_weight(dtype, make_conv_shape(N, H, W, cin, cout, r, s, stride, pad, groups), d_x, d_dy, d_dw,
                                       d_workspace, workspace_bytes, (hipStream_t)stream);
}

int dsp_grouped_conv_workspace_bytes(int32_t N, int32_t H, int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s,
                                     int32_t stride, int32_t pad, int32_t groups, size_t* bytes)
{
    DSP_REQUIRE(bytes && N > 0 && H > 0 && W > 0 && cin > 0 && cout > 0 && r > 0 && s > 0 && stride > 0 && pad >= 0 &&
                    groups > 0 && cin % groups == 0 && cout % groups == 0,
                DSP_EINVAL, "dsp_conv_workspace_bytes: bad argument");
    const ConvShape c = make_conv_shape(N, H, W, cin, cout, r, s, stride, pad, groups);
    DSP_REQUIRE(c.Ho > 0 && c.Wo > 0, DSP_EINVAL, "dsp_conv_workspace_bytes: empty output");
    *bytes = conv_backward_weight_workspace(c);
    return DSP_OK;
}

int dsp_conv_forward(int32_t dtype, const void* d_x, const void* d_w, void* d_y, int32_t N, int32_t H, int32_t W,
                     int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride, int32_t pad, void* stream)
{
    return dsp_grouped_conv_forward(dtype, d_x, d_w, d_y, N, H, W, cin, cout, r, s, stride, pad, 1, stream);
}

int dsp_conv_backward_data(int32_t dtype, const void* d_dy, const void* d_wt, void* d_dx, int32_t N, int32_t H,
                           int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride, int32_t pad,
                           int32_t accumulate, void* stream)
{
    return dsp_grouped_conv_backward_data(dtype, d_dy, d_wt, d_dx, N, H, W, cin, cout, r, s, stride, pad, 1, accumulate, stream);
}

int dsp_conv_backward_weight(int32_t dtype, const void* d_x, const void* d_dy, float* d_dw, int32_t N, int32_t H,
                             int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s, int32_t stride, int32_t pad,
                             void* d_workspace, size_t workspace_bytes, void* stream)
{
    return dsp_grouped_conv_backward_weight(dtype, d_x, d_dy, d_dw, N, H, W, cin, cout, r, s, stride, pad, 1, d_workspace,
                                            workspace_bytes, stream);
}

int dsp_conv_workspace_bytes(int32_t N, int32_t H, int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s,
                             int32_t stride, int32_t pad, size_t* bytes)
{
    return dsp_grouped_conv_workspace_bytes(N, H, W, cin, cout, r, s, stride, pad, 1, bytes);
}

// ---- in-situ kernel timing ---------------------------------------------------------------------------
}  // extern "C"
__global__ void dsp_profile_window_begin() {}
__global__ void dsp_profile_window_end() {}
extern "C" {

int dsp_profile_start(int32_t max_launches)
{
    DSP_REQUIRE(max_launches > 0 && max_launches <= (1 << 20), DSP_EINVAL, "dsp_profile_start: bad max_launches");
    DSP_REQUIRE(!g_profile_on, DSP_ESTATE, "dsp_profile_start: a profile is already running");
    while (g_prof_events.size() < 2 * (size_t)max_launches) {
        hipEvent_t e;
        DSP_HIP(hipEventCreate(&e));
        g_prof_events.push_back(e);
    }
    g_prof_recs.clear();
    g_prof_recs.reserve(max_launches);
    g_prof_capacity = max_launches;
    g_prof_result.clear();
    DSP_HIP(hipDeviceSynchronize());
    hipLaunchKernelGGL(dsp_profile_window_begin, dim3(1), dim3(1), 0, nullptr);
    DSP_HIP(hipDeviceSynchronize());
    g_profile_on = true;
    return DSP_OK;
}

int dsp_profile_stop(int32_t* n_kernels)
{
    DSP_REQUIRE(g_profile_on, DSP_ESTATE, "dsp_profile_stop: no profile is running");
    g_profile_on = false;
    DSP_HIP(hipDeviceSynchronize());
    hipLaunchKernelGGL(dsp_profile_window_end, dim3(1), dim3(1), 0, nullptr);
    DSP_HIP(hipDeviceSynchronize());
    std::map<std::string, size_t> index;
    for (size_t i = 0; i < g_prof_recs.size(); ++i) {
        float ms = 0.f;
        DSP_HIP(hipEventElapsedTime(&ms, g_prof_events[2 * i], g_prof_events[2 * i + 1]));
        auto it = index.find(g_prof_recs[i].name);
        if (it == index.end()) {
            it = index.emplace(g_prof_recs[i].name, g_prof_result.size()).first;
            g_prof_result.push_back(ProfAgg());
            g_prof_result.back().name = g_prof_recs[i].name;
            g_prof_result.back().unit_kind = g_prof_recs[i].unit_kind;
        }
        ProfAgg& a = g_prof_result[it->second];
        a.launches += 1;
        a.ms += ms;
        a.units += g_prof_recs[i].units;
    }
    if (n_kernels) *n_kernels = (int32_t)g_prof_result.size();
    return DSP_OK;
}

int dsp_profile_get(int32_t i, char* name, size_t name_len, int64_t* launches, double* total_ms, double* total_units,
                    int32_t* unit_kind)
{
    DSP_REQUIRE(i >= 0 && (size_t)i < g_prof_result.size(), DSP_EINVAL, "dsp_profile_get: index out of range");
    const ProfAgg& a = g_prof_result[i];
    if (name && name_len) snprintf(name, name_len, "%s", a.name.c_str());
    if (launches) *launches = a.launches;
    if (total_ms) *total_ms = a.ms;
    if (total_units) *total_units = a.units;
    if (unit_kind) *unit_kind = a.unit_kind;
    return DSP_OK;
}

const char* dsp_strerror(int status)
{
    switch (status) {
    case DSP_OK: return "ok";
    case DSP_EINVAL: return "invalid argument, descriptor or schedule";
    case DSP_ESTATE: return "call out of pipeline order";
    case DSP_ENOMEM: return "out of memory";
    case DSP_EHIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

const char* dsp_last_error(void) { return dsp::g_err; }

#ifndef DSP_BUILD_ID
#define DSP_BUILD_ID "unknown"
#endif
const char* dsp_build_id(void) { return DSP_BUILD_ID; }

}  // extern "C"
