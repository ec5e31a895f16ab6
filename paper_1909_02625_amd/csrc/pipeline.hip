// DSP(p; m) over K blocks on K HIP streams of one GPU (Section 3.3 and Appendix A of the paper):
// the integer schedule (pure host code) and the tick driver.
//
// Queues as device rings: M_k and P_{k-1} share one ring of 1+m_k+p_{k-1} slots inside block k
// (block k-1 writes h_k straight into the slot block k will read p_{k-1} ticks later and again,
// for the backward, m_k ticks after that); Q_k is a ring of 1+q_k gradient slots owned here.
// Which mini-batch a block touches depends only on the tick number, so results do not depend
// on timing; streams only have to respect "a slot is written one tick or more before it is
// read, and read before it is rewritten", which waiting for both neighbours' previous tick gives.
#include <new>
#include <vector>

#include "common.h"

using namespace dsp;

namespace {

int validate_schedule(int K, const int32_t* p, const int32_t* m, int32_t* q)
{
    DSP_REQUIRE(K >= 1 && p && m, DSP_EINVAL, "schedule: K >= 1 and p, m required");
    bool all_zero = true;
    for (int k = 0; k < K; ++k) all_zero = all_zero && p[k] == 0 && m[k] == 0;
    if (q) q[0] = 0;
    if (all_zero) {
        if (q) for (int k = 0; k < K; ++k) q[k] = 0;
        return DSP_OK;
    }
    DSP_REQUIRE(p[K - 1] == 0, DSP_EINVAL, "schedule: p_{K-1} must be 0");
    DSP_REQUIRE(m[K - 1] >= 0, DSP_EINVAL, "schedule: m_{K-1} must be >= 0");
    for (int k = 0; k < K - 1; ++k) {
        DSP_REQUIRE(p[k] > 0, DSP_EINVAL, "schedule: p_%d must be > 0", k);
        DSP_REQUIRE(m[k] > 0, DSP_EINVAL, "schedule: m_%d must be > 0", k);
    }
    for (int k = 1; k < K; ++k) {
        const int qk = m[k - 1] - p[k - 1] - m[k];
        DSP_REQUIRE(qk > 0, DSP_EINVAL, "schedule: q_%d = m_%d - p_%d - m_%d = %d must be > 0", k, k - 1, k - 1, k, qk);
        if (q) q[k] = qk;
    }
    return DSP_OK;
}

}  // namespace

struct dsp_pipeline {
    int K = 0;
    bool serial = false;  // all-zero schedule: ordinary backpropagation, one stream
    std::vector<dsp_block*> blocks;
    std::vector<int32_t> p, m, q, P;  // P[k] = sum_{j<k} p_j
    float lr = 0, momentum = 0, wd = 0;
    std::vector<hipStream_t> streams;
    std::vector<hipEvent_t> done[2];  // done[tau % 2][k]: block k finished tick tau
    hipEvent_t in_ready = nullptr, in_copied = nullptr;
    std::vector<char*> qring;         // Q_k, k >= 1
    std::vector<size_t> qslot_bytes;
    int32_t* labels = nullptr;
    int label_slots = 1, N = 0;
    float* losses = nullptr;
    int64_t max_ticks = 0, tau = 0;
    std::vector<int32_t> delay_us;
    std::vector<void*> allocs;
};

extern "C" {

int dsp_schedule_validate(int32_t K, const int32_t* p, const int32_t* m, int32_t* q)
{
    return validate_schedule(K, p, m, q);
}

int dsp_schedule_index(int32_t K, const int32_t* p, const int32_t* m, int32_t k, int64_t tau, int64_t out[7])
{
    std::vector<int32_t> q(K > 0 ? K : 1);
    DSP_TRY(validate_schedule(K, p, m, q.data()));
    DSP_REQUIRE(k >= 0 && k < K && tau >= 0 && out, DSP_EINVAL, "dsp_schedule_index: bad k, tau or out");
    int64_t P = 0;
    for (int j = 0; j < k; ++j) P += p[j];
    const int64_t a = tau - P >= 0 ? tau - P : -1;
    const int64_t b = (a >= 0 && a - m[k] >= 0) ? a - m[k] : -1;
    const int64_t ring = 1 + m[k] + (k > 0 ? p[k - 1] : 0);
    out[0] = a;
    out[1] = b;
    out[2] = b > 0 ? b : 0;
    out[3] = a >= 0 ? a % ring : -1;
    out[4] = b >= 0 ? b % ring : -1;
    out[5] = (b >= 0 && k > 0) ? b % (1 + q[k]) : -1;
    out[6] = (b >= 0 && k < K - 1) ? b % (1 + q[k + 1]) : -1;
    return DSP_OK;
}

int dsp_schedule_queue_elems(int32_t K, const int32_t* p, const int32_t* m, const int64_t* h_elems, int64_t* total)
{
    std::vector<int32_t> q(K > 0 ? K : 1);
    DSP_TRY(validate_schedule(K, p, m, q.data()));
    DSP_REQUIRE(h_elems && total, DSP_EINVAL, "dsp_schedule_queue_elems: null argument");
    int64_t t = 0;
    for (int k = 0; k < K; ++k) {
        t += (int64_t)(1 + m[k] + (k > 0 ? p[k - 1] : 0)) * h_elems[k];
        if (k > 0) t += (int64_t)(1 + q[k]) * h_elems[k];
    }
    *total = t;
    return DSP_OK;
}

int dsp_pipeline_destroy(dsp_pipeline* pl)
{
    if (!pl) return DSP_OK;
    (void)hipDeviceSynchronize();
    for (hipStream_t s : pl->streams) (void)hipStreamDestroy(s);
    for (int i = 0; i < 2; ++i)
        for (hipEvent_t e : pl->done[i]) (void)hipEventDestroy(e);
    if (pl->in_ready) (void)hipEventDestroy(pl->in_ready);
    if (pl->in_copied) (void)hipEventDestroy(pl->in_copied);
    for (void* a : pl->allocs) (void)hipFree(a);
    delete pl;
    return DSP_OK;
}

static int pipeline_build(dsp_pipeline* pl, dsp_block* const* blocks)
{
    const int K = pl->K;
    int64_t info[8];
    int32_t shape[5], prev_out[5] = {0, 0, 0, 0, 0};
    int dtype0 = 0;
    for (int k = 0; k < K; ++k) {
        DSP_REQUIRE(blocks[k], DSP_EINVAL, "dsp_pipeline_init: null block %d", k);
        dsp_block* b = blocks[k];
        DSP_TRY(dsp_block_input_shape(b, shape));
        if (k == 0) dtype0 = shape[4];
        DSP_REQUIRE(shape[4] == dtype0, DSP_EINVAL, "dsp_pipeline_init: block %d has another dtype", k);
        if (k > 0)
            DSP_REQUIRE(prev_out[4] == 0 && shape[0] == prev_out[0] && shape[1] == prev_out[1] && shape[2] == prev_out[2] &&
                            shape[3] == prev_out[3],
                        DSP_EINVAL, "dsp_pipeline_init: block %d does not take the output of block %d", k, k - 1);
        DSP_TRY(dsp_block_output_shape(b, prev_out));
        DSP_TRY(dsp_block_query(b, info));
        const int want = 1 + pl->m[k] + (k > 0 ? pl->p[k - 1] : 0);
        DSP_REQUIRE(info[3] == want, DSP_EINVAL, "dsp_pipeline_init: block %d has a ring of %lld entries, DSP(p;m) needs %d",
                    k, (long long)info[3], want);
        DSP_REQUIRE(info[1] == 0 && info[2] == 0, DSP_ESTATE, "dsp_pipeline_init: block %d has already been stepped", k);
        pl->blocks.push_back(b);
    }
    for (int k = 0; k < K; ++k) {
        hipStream_t s;
        DSP_HIP(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        pl->streams.push_back(s);
        for (int i = 0; i < 2; ++i) {
            hipEvent_t e;
            DSP_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
            pl->done[i].push_back(e);
        }
    }
    DSP_HIP(hipEventCreateWithFlags(&pl->in_ready, hipEventDisableTiming));
    DSP_HIP(hipEventCreateWithFlags(&pl->in_copied, hipEventDisableTiming));
    // Q_k holds G_{h_k}: same bytes as block k's input slot.
    pl->qring.assign(K, nullptr);
    pl->qslot_bytes.assign(K, 0);
    for (int k = 1; k < K; ++k) {
        DSP_TRY(dsp_block_output_shape(pl->blocks[k - 1], shape));
        size_t bytes = (size_t)shape[0] * shape[1] * shape[2] * shape[3] * 4;  // upper bound (fp32)
        bytes = (bytes + 255) / 256 * 256;
        void* ptr;
        hipError_t e = hipMalloc(&ptr, bytes * (1 + pl->q[k]));
        DSP_REQUIRE(e == hipSuccess, DSP_ENOMEM, "dsp_pipeline_init: hipMalloc failed: %s", hipGetErrorString(e));
        pl->allocs.push_back(ptr);
        pl->qring[k] = (char*)ptr;
        pl->qslot_bytes[k] = bytes;
    }
    DSP_TRY(dsp_block_output_shape(pl->blocks[0], shape));
    pl->N = shape[0];
    pl->label_slots = pl->P[K - 1] + K;
    void* ptr;
    hipError_t e = hipMalloc(&ptr, (size_t)pl->label_slots * pl->N * 4);
    DSP_REQUIRE(e == hipSuccess, DSP_ENOMEM, "dsp_pipeline_init: hipMalloc failed: %s", hipGetErrorString(e));
    pl->allocs.push_back(ptr);
    pl->labels = (int32_t*)ptr;
    e = hipMalloc(&ptr, (size_t)(pl->max_ticks + 1) * 4);
    DSP_REQUIRE(e == hipSuccess, DSP_ENOMEM, "dsp_pipeline_init: hipMalloc failed: %s", hipGetErrorString(e));
    pl->allocs.push_back(ptr);
    pl->losses = (float*)ptr;
    DSP_HIP(hipMemset(pl->losses, 0, (size_t)(pl->max_ticks + 1) * 4));
    DSP_HIP(hipDeviceSynchronize());
    return DSP_OK;
}

int dsp_pipeline_init(int32_t K, dsp_block* const* blocks, const int32_t* p, const int32_t* m, float lr,
                      float momentum, float weight_decay, int64_t max_ticks, dsp_pipeline** out)
{
    DSP_REQUIRE(out && blocks && max_ticks > 0, DSP_EINVAL, "dsp_pipeline_init: bad argument");
    *out = nullptr;
    std::vector<int32_t> q(K > 0 ? K : 1);
    DSP_TRY(validate_schedule(K, p, m, q.data()));
    dsp_pipeline* pl = new (std::nothrow) dsp_pipeline();
    DSP_REQUIRE(pl, DSP_ENOMEM, "dsp_pipeline_init: out of host memory");
    pl->K = K;
    pl->p.assign(p, p + K);
    pl->m.assign(m, m + K);
    pl->q = q;
    pl->P.assign(K, 0);
    for (int k = 1; k < K; ++k) pl->P[k] = pl->P[k - 1] + p[k - 1];
    pl->serial = true;
    for (int k = 0; k < K; ++k) pl->serial = pl->serial && p[k] == 0 && m[k] == 0;
    if (K == 1) pl->serial = false;
    pl->lr = lr;
    pl->momentum = momentum;
    pl->wd = weight_decay;
    pl->max_ticks = max_ticks;
    pl->delay_us.assign(K, 0);
    const int rc = pipeline_build(pl, blocks);
    if (rc != DSP_OK) {
        dsp_pipeline_destroy(pl);
        return rc;
    }
    *out = pl;
    return DSP_OK;
}

int dsp_pipeline_set_delay(dsp_pipeline* pl, int32_t k, int32_t microseconds)
{
    DSP_REQUIRE(pl && k >= 0 && k < pl->K && microseconds >= 0 && microseconds <= 1000000, DSP_EINVAL,
                "dsp_pipeline_set_delay: bad argument");
    pl->delay_us[k] = microseconds;
    return DSP_OK;
}

int dsp_pipeline_step(dsp_pipeline* pl, const void* d_batch, const int32_t* d_labels, float* h_loss,
                      int64_t* loss_batch_id, void* stream)
{
    DSP_REQUIRE(pl && d_batch, DSP_EINVAL, "dsp_pipeline_step: null argument");
    DSP_REQUIRE(pl->tau < pl->max_ticks, DSP_ESTATE, "dsp_pipeline_step: max_ticks (%lld) reached", (long long)pl->max_ticks);
    const int K = pl->K;
    const int64_t tau = pl->tau;
    const int cur = (int)(tau & 1), prev = cur ^ 1;
    hipStream_t user = (hipStream_t)stream;

    // the data source: copy the mini-batch into block 0's ring slot and the labels into the label ring
    hipStream_t s0 = pl->streams[0];
    DSP_HIP(hipEventRecord(pl->in_ready, user));
    DSP_HIP(hipStreamWaitEvent(s0, pl->in_ready, 0));
    // (the mini-batch itself is copied into block 0's ring slot by dsp_block_forward, on stream 0)
    if (d_labels)
        DSP_HIP(hipMemcpyAsync(pl->labels + (size_t)(tau % pl->label_slots) * pl->N, d_labels, (size_t)pl->N * 4,
                               hipMemcpyDeviceToDevice, s0));

    auto block_tick = [&](int k, hipStream_t st, bool do_fwd, bool do_bwd) -> int {
        const int64_t a = tau - pl->P[k];
        if (a < 0) return DSP_OK;
        dsp_block* b = pl->blocks[k];
        const int64_t bb = a - pl->m[k];
        if (do_fwd) {
            const void* in;
            if (k == 0) {
                in = d_batch;  // copied into the ring by the block itself
            } else {
                void* sl;
                DSP_TRY(dsp_block_input_slot(b, a, &sl));
                in = sl;
            }
            void* out = nullptr;
            if (k < K - 1) DSP_TRY(dsp_block_input_slot(pl->blocks[k + 1], a, &out));
            const int32_t* lab = pl->labels + (size_t)(a % pl->label_slots) * pl->N;
            DSP_TRY(dsp_block_forward(b, a, in, out, k == K - 1 ? lab : nullptr, k == K - 1 ? pl->losses + a : nullptr, st));
            if (k == 0) {
                DSP_HIP(hipEventRecord(pl->in_copied, st));
                DSP_HIP(hipStreamWaitEvent(user, pl->in_copied, 0));
            }
        }
        if (do_bwd && bb >= 0) {
            const void* gout = k < K - 1 ? pl->qring[k + 1] + (size_t)(bb % (1 + pl->q[k + 1])) * pl->qslot_bytes[k + 1] : nullptr;
            void* gin = k > 0 ? pl->qring[k] + (size_t)(bb % (1 + pl->q[k])) * pl->qslot_bytes[k] : nullptr;
            DSP_TRY(dsp_block_recompute_backward(b, bb, gout, gin, st));
            DSP_TRY(dsp_param_update(b, pl->lr, pl->momentum, pl->wd, st));
        }
        return DSP_OK;
    };

    if (pl->serial) {
        // ordinary backpropagation: forward up the chain, backward down the chain, one stream
        for (int k = 0; k < K; ++k) DSP_TRY(block_tick(k, s0, true, false));
        for (int k = K - 1; k >= 0; --k) DSP_TRY(block_tick(k, s0, false, true));
    } else {
        for (int k = 0; k < K; ++k) {
            hipStream_t st = pl->streams[k];
            // Neighbours' previous tick: the slots this block reads were written then or earlier, and
            // the slots it writes were last read then or earlier.  (The labels of the mini-batch the
            // last block sees now were copied on stream 0 P_{K-1} >= K-1 ticks ago, which this chain
            // of waits orders; the label ring has P_{K-1}+K slots so a slot is not refilled too early.)
            if (tau > 0) {
                if (k > 0) DSP_HIP(hipStreamWaitEvent(st, pl->done[prev][k - 1], 0));
                if (k < K - 1) DSP_HIP(hipStreamWaitEvent(st, pl->done[prev][k + 1], 0));
            }
            if (pl->delay_us[k] > 0) DSP_TRY(launch_spin(pl->delay_us[k], st));
            DSP_TRY(block_tick(k, st, true, true));
            DSP_HIP(hipEventRecord(pl->done[cur][k], st));
        }
    }
    pl->tau = tau + 1;

    const int64_t a_last = tau - pl->P[K - 1];
    if (loss_batch_id) *loss_batch_id = a_last >= 0 ? a_last : -1;
    if (h_loss) {
        *h_loss = 0.f;
        if (a_last >= 0) {
            hipStream_t sl = pl->serial ? s0 : pl->streams[K - 1];
            DSP_HIP(hipStreamSynchronize(sl));
            DSP_HIP(hipMemcpy(h_loss, pl->losses + a_last, 4, hipMemcpyDeviceToHost));
        }
    }
    return DSP_OK;
}

int dsp_pipeline_sync(dsp_pipeline* pl)
{
    DSP_REQUIRE(pl, DSP_EINVAL, "dsp_pipeline_sync: null pipeline");
    for (hipStream_t s : pl->streams) DSP_HIP(hipStreamSynchronize(s));
    return DSP_OK;
}

int dsp_pipeline_losses(dsp_pipeline* pl, float* h_dst, int64_t n, int64_t* n_available)
{
    DSP_REQUIRE(pl, DSP_EINVAL, "dsp_pipeline_losses: null pipeline");
    int64_t avail = pl->tau - pl->P[pl->K - 1];
    if (avail < 0) avail = 0;
    if (n_available) *n_available = avail;
    if (n > 0) {
        DSP_REQUIRE(h_dst && n <= avail, DSP_EINVAL, "dsp_pipeline_losses: %lld requested, %lld available", (long long)n,
                    (long long)avail);
        DSP_TRY(dsp_pipeline_sync(pl));
        DSP_HIP(hipMemcpy(h_dst, pl->losses, (size_t)n * 4, hipMemcpyDeviceToHost));
    }
    return DSP_OK;
}

int dsp_pipeline_ticks(const dsp_pipeline* pl, int64_t* ticks)
{
    DSP_REQUIRE(pl && ticks, DSP_EINVAL, "dsp_pipeline_ticks: null argument");
    *ticks = pl->tau;
    return DSP_OK;
}

}  // extern "C"
