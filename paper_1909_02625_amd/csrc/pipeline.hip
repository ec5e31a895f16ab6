// DSP(p; m) over K blocks on K HIP streams of one GPU (Section 3.3 and Appendix A of the paper):
// the integer schedule (pure host code) and the tick driver.
//
// Queues as device rings: M_k and P_{k-1} share one ring of 1+m_k+p_{k-1} slots inside block k
// (block k-1 writes h_k straight into the slot block k will read p_{k-1} ticks later and again,
// for the backward, m_k ticks after that); Q_k is a ring of 1+q_k gradient slots owned here.
// Which mini-batch a block touches depends only on the tick number, so results do not depend
// on timing; streams only have to respect "a slot is written before it is read, and read before
// it is rewritten".  With rings of exactly those sizes a slot is rewritten one tick after its last
// read, so every block waits for both neighbours' previous tick.  Blocks built with spare ring
// entries (p_prev larger than p_{k-1}) give the queues between two blocks that much slack: the
// producer may then run 1+spare ticks ahead of the consumer's last read, the consumer needs what the
// producer wrote p_{k-1} (activations) or q_k (gradients) ticks ago, and each block waits for the
// nearer of the two per neighbour -- a block that is late for a tick no longer holds up the others
// at once (the role Section 6 of the paper gives to the FIFO queues under stragglers).
//
// Steady-state ticks are launch-bound on small layers (hundreds of kernels of a few microseconds).
// By default the K chains are issued kernel by kernel from K host threads.  Optionally
// (dsp_pipeline_set_graph_replay) each tick of a full pipeline is captured into a HIP graph -- one
// per phase of the ring rotation, lcm(ring sizes) of them -- with the K block chains as parallel
// branches, and later ticks of the same phase replay that graph with a single launch while the
// blocks' host-side state is advanced without launching.
#include <atomic>
#include <condition_variable>
#include <memory>
#include <mutex>
#include <new>
#include <numeric>
#include <string>
#include <thread>
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
    // all p_k = 0 with stale backward passes: the forward-locked schedule of the features-replay comparison
    // (Section 6); otherwise every p_k below the last block must be positive (Appendix A)
    bool locked = true;
    for (int k = 0; k < K; ++k) locked = locked && p[k] == 0;
    for (int k = 0; k < K - 1; ++k) {
        DSP_REQUIRE(locked || p[k] > 0, DSP_EINVAL, "schedule: p_%d must be > 0 (or every p_k = 0)", k);
        DSP_REQUIRE(m[k] > 0, DSP_EINVAL, "schedule: m_%d must be > 0", k);
    }
    for (int k = 1; k < K; ++k) {
        const int qk = m[k - 1] - p[k - 1] - m[k];
        DSP_REQUIRE(qk > 0, DSP_EINVAL, "schedule: q_%d = m_%d - p_%d - m_%d = %d must be > 0", k, k - 1, k - 1, k, qk);
        if (q) q[k] = qk;
    }
    return DSP_OK;
}

constexpr int kMaxGraphs = 128;

// One host thread per block stream: a tick is a few hundred kernel launches of a few microseconds of
// host time each, so issuing the K chains from K threads keeps the launch rate off the critical path.
struct Worker {
    std::thread th;
    std::mutex mu;
    std::condition_variable cv;
    bool has_job = false, finished = false, quit = false;
    int64_t tau = 0;
    int rc = DSP_OK;
    std::string err;
};

}  // namespace

struct dsp_pipeline {
    int K = 0;
    bool serial = false;  // all-zero schedule: ordinary backpropagation, one stream
    // every p_k = 0 but the backward passes are stale (the features-replay schedule): the forward passes of a tick
    // form one chain through the blocks (block k+1 reads what block k wrote in the same tick); recompute, backward and
    // update of the K blocks still run side by side
    bool fwd_locked = false;
    std::unique_ptr<std::atomic<int64_t>[]> fwd_issued;  // fwd_issued[k] = ticks whose forward-done event block k has recorded
    std::vector<dsp_block*> blocks;
    std::vector<int32_t> p, m, q, P;  // P[k] = sum_{j<k} p_j
    float lr = 0, momentum = 0, wd = 0;
    int sum_s = 0;        // Eq. (3): 0 heavy ball, 1 Nesterov
    int eager_ticks = 0;  // ticks to run unrecorded (the update after a step-size change rescales the velocity once)
    std::vector<hipStream_t> streams;
    std::vector<int32_t> spare;       // spare[k], k >= 1: entries beyond the minimum in the two queues between blocks k-1 and k
    std::vector<int32_t> qn;          // entries of Q_k = 1 + q_k + spare[k]
    std::vector<int32_t> wait_dn, wait_up;  // block k waits for tick tau - wait_dn[k] of block k-1 and tau - wait_up[k] of block k+1
    int ev_depth = 2;                 // ticks of history the done events keep (1 + the longest wait distance)
    std::vector<std::vector<hipEvent_t>> done;  // done[tau % ev_depth][k]: block k finished tick tau
    // Forward streams: a block with m_k > 0 runs forward(a) here while its main stream runs
    // recompute + backward(a - m_k); the update (main stream) waits for both.
    std::vector<hipStream_t> fstreams;
    std::vector<hipEvent_t> fdone[2];  // fdone[tau % 2][k]: block k finished the forward pass of tick tau
    std::vector<char> fwd_split;       // block k uses its forward stream
    bool use_twin = true;  // forward(a) and recompute(a - m_k) of a block share their launches (dsp_block_step)
    bool use_fwd_streams = false;  // measured slower on this GPU: a fifth and sixth stream cost more than the overlap gains
    std::vector<hipEvent_t> join;     // graph capture: branch k joins stream 0
    hipEvent_t in_ready = nullptr, in_copied = nullptr, fork = nullptr;
    std::vector<char*> qring;         // Q_k, k >= 1
    std::vector<size_t> qslot_bytes;
    int32_t* labels = nullptr;
    int label_slots = 1, N = 0;
    size_t in_bytes = 0;
    float* losses = nullptr;     // loss of mini-batch i at losses[i]
    float* loss_tmp = nullptr;   // loss of the tick in flight
    int32_t* loss_count = nullptr;
    int64_t max_ticks = 0, tau = 0;
    std::vector<int32_t> delay_us;
    std::vector<void*> allocs;
    // launch threads for blocks 1..K-1 (block 0 is issued by the caller's thread)
    std::vector<Worker*> workers;
    int device = 0;
    bool use_threads = true;
    bool single_stream = false;  // issue all K chains on stream 0 from the caller's thread (no overlap between kernels)
    // graph replay (off by default: on this runtime replaying a few hundred nodes costs more host time
    // than issuing them from K threads)
    bool use_graphs = false;
    int period = 0;      // ticks after which every ring is back in the same position (0: too long, no graphs)
    int64_t fill = 0;    // first tick at which every block runs forward, backward and update
    std::vector<hipGraphExec_t> graphs;
    // Gradient-difference diagnostic (Lemma 1, Section 5.4): a second, all-zero-schedule pipeline over
    // blocks of the same architecture re-runs each mini-batch as ordinary backpropagation at the
    // parameters every block held when it ran the forward pass of that mini-batch.
    dsp_pipeline* probe = nullptr;
    std::vector<float*> xsnap, gstash;      // per block: rings of parameter snapshots / DSP gradients, by mini-batch
    std::vector<int> xsnap_n, gstash_n;     // their entry counts
    int32_t* probe_labels = nullptr;        // labels of the last 1 + m_0 mini-batches
    double* probe_partial = nullptr;
    double* probe_out = nullptr;            // [K][2]
    int64_t probe_batch = -1;               // mini-batch of the latest result
    std::vector<double> probe_diff, probe_ref;
};

static int run_block_tick(dsp_pipeline* pl, int k, int64_t tau);

static void worker_main(dsp_pipeline* pl, int k)
{
    Worker* w = pl->workers[k];
    (void)hipSetDevice(pl->device);
    std::unique_lock<std::mutex> lk(w->mu);
    for (;;) {
        w->cv.wait(lk, [&] { return w->has_job || w->quit; });
        if (w->quit) return;
        w->has_job = false;
        const int64_t tau = w->tau;
        lk.unlock();
        const int rc = run_block_tick(pl, k, tau);
        lk.lock();
        w->rc = rc;
        w->err = rc == DSP_OK ? "" : dsp_last_error();
        w->finished = true;
        w->cv.notify_all();
    }
}

static void stop_workers(dsp_pipeline* pl)
{
    for (Worker* w : pl->workers) {
        if (!w) continue;
        {
            std::lock_guard<std::mutex> g(w->mu);
            w->quit = true;
        }
        w->cv.notify_all();
        if (w->th.joinable()) w->th.join();
        delete w;
    }
    pl->workers.clear();
}

static void drop_graphs(dsp_pipeline* pl)
{
    bool synced = false;
    for (hipGraphExec_t& g : pl->graphs)
        if (g) {
            if (!synced) (void)hipDeviceSynchronize();  // a replay of it may still be running
            synced = true;
            (void)hipGraphExecDestroy(g);
            g = nullptr;
        }
}

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

int dsp_schedule_waits(int32_t K, const int32_t* p, const int32_t* m, const int32_t* spare, int32_t* wait_down,
                       int32_t* wait_up, int32_t* label_slots)
{
    std::vector<int32_t> q(K > 0 ? K : 1);
    DSP_TRY(validate_schedule(K, p, m, q.data()));
    DSP_REQUIRE(wait_down && wait_up, DSP_EINVAL, "dsp_schedule_waits: null argument");
    DSP_REQUIRE(!spare || spare[0] == 0, DSP_EINVAL, "dsp_schedule_waits: block 0 has no queue below it (spare[0] must be 0)");
    // The nearer of "what I read was written then" (p_{k-1} ticks ago by the block below, q_{k+1} by the
    // block above) and "what I overwrite was last read then" (1 + spare ticks ago).
    int64_t labels = K, P = 0;
    for (int k = 0; k < K; ++k) {
        const int sk = spare ? spare[k] : 0, su = (spare && k < K - 1) ? spare[k + 1] : 0;
        DSP_REQUIRE(sk >= 0 && sk <= 64, DSP_EINVAL, "dsp_schedule_waits: spare[%d] = %d outside 0..64", k, sk);
        wait_down[k] = (k > 0 && p[k - 1] > 0) ? std::min(p[k - 1], 1 + sk) : 0;
        wait_up[k] = (k < K - 1 && q[k + 1] > 0) ? std::min(q[k + 1], 1 + su) : 0;
        labels += sk;
        if (k < K - 1) P += p[k];
    }
    // Labels copied at tick tau are read by the last block P_{K-1} ticks later; the copy of tick tau runs
    // after block 0's tick tau-1, hence after the last block's tick tau - 1 - (sum of the upward waits),
    // which is tick tau - K - (all spare entries) or later.
    if (label_slots) *label_slots = (int32_t)(P + labels);
    return DSP_OK;
}

int dsp_pipeline_destroy(dsp_pipeline* pl)
{
    if (!pl) return DSP_OK;
    stop_workers(pl);
    (void)hipDeviceSynchronize();
    drop_graphs(pl);
    for (hipStream_t s : pl->streams) (void)hipStreamDestroy(s);
    for (hipStream_t s : pl->fstreams) (void)hipStreamDestroy(s);
    for (auto& row : pl->done)
        for (hipEvent_t e : row) (void)hipEventDestroy(e);
    for (int i = 0; i < 2; ++i)
        for (hipEvent_t e : pl->fdone[i]) (void)hipEventDestroy(e);
    for (hipEvent_t e : pl->join) (void)hipEventDestroy(e);
    if (pl->in_ready) (void)hipEventDestroy(pl->in_ready);
    if (pl->in_copied) (void)hipEventDestroy(pl->in_copied);
    if (pl->fork) (void)hipEventDestroy(pl->fork);
    for (void* a : pl->allocs) (void)hipFree(a);
    delete pl;
    return DSP_OK;
}

static int pl_alloc(dsp_pipeline* pl, void** p, size_t bytes)
{
    hipError_t e = hipMalloc(p, bytes ? bytes : 16);
    DSP_REQUIRE(e == hipSuccess, DSP_ENOMEM, "dsp_pipeline_init: hipMalloc(%zu) failed: %s", bytes, hipGetErrorString(e));
    pl->allocs.push_back(*p);
    return DSP_OK;
}

static int pipeline_build(dsp_pipeline* pl, dsp_block* const* blocks)
{
    const int K = pl->K;
    int64_t info[8];
    int32_t shape[5], prev_out[5] = {0, 0, 0, 0, 0};
    int dtype0 = 0;
    int64_t period = 1;
    for (int k = 0; k < K; ++k) {
        DSP_REQUIRE(blocks[k], DSP_EINVAL, "dsp_pipeline_init: null block %d", k);
        dsp_block* b = blocks[k];
        DSP_TRY(dsp_block_input_shape(b, shape));
        if (k == 0) {
            dtype0 = shape[4];
            pl->N = shape[0];
            pl->in_bytes = (size_t)shape[0] * shape[1] * shape[2] * shape[3] * dtype_size(dtype0);
        }
        DSP_REQUIRE(shape[4] == dtype0, DSP_EINVAL, "dsp_pipeline_init: block %d has another dtype", k);
        if (k > 0)
            DSP_REQUIRE(prev_out[4] == 0 && shape[0] == prev_out[0] && shape[1] == prev_out[1] && shape[2] == prev_out[2] &&
                            shape[3] == prev_out[3],
                        DSP_EINVAL, "dsp_pipeline_init: block %d does not take the output of block %d", k, k - 1);
        DSP_TRY(dsp_block_output_shape(b, prev_out));
        DSP_TRY(dsp_block_query(b, info));
        const int want = 1 + pl->m[k] + (k > 0 ? pl->p[k - 1] : 0);
        DSP_REQUIRE(k > 0 ? info[3] >= want : info[3] == want, DSP_EINVAL,
                    "dsp_pipeline_init: block %d has a ring of %lld entries, DSP(p;m) needs %d%s", k, (long long)info[3], want,
                    k > 0 ? " or more" : "");
        DSP_REQUIRE(info[3] - want <= 64, DSP_EINVAL, "dsp_pipeline_init: block %d has more than 64 spare ring entries", k);
        DSP_REQUIRE(info[1] == 0 && info[2] == 0, DSP_ESTATE, "dsp_pipeline_init: block %d has already been stepped", k);
        pl->blocks.push_back(b);
        pl->spare[k] = (int32_t)(info[3] - want);
        pl->qn[k] = k > 0 ? 1 + pl->q[k] + pl->spare[k] : 1;
        period = std::lcm(period, (int64_t)info[3]);
        period = std::lcm(period, (int64_t)(1 + pl->m[k]));  // the last block's loss-gradient ring
        if (k > 0) period = std::lcm(period, (int64_t)pl->qn[k]);
        if (period > kMaxGraphs) period = kMaxGraphs + 1;
        const int64_t full = pl->P[k] + pl->m[k];
        if (full > pl->fill) pl->fill = full;
    }
    // How far back each block has to look at its neighbours (an all-zero schedule runs on one stream and
    // never waits), and how many mini-batches of labels are kept.
    int32_t label_slots = 1;
    DSP_TRY(dsp_schedule_waits(K, pl->p.data(), pl->m.data(), pl->spare.data(), pl->wait_dn.data(), pl->wait_up.data(),
                               &label_slots));
    for (int k = 0; k < K; ++k) pl->ev_depth = std::max(pl->ev_depth, 1 + std::max(pl->wait_dn[k], pl->wait_up[k]));
    pl->done.assign(pl->ev_depth, std::vector<hipEvent_t>());
    for (int k = 0; k < K; ++k) {
        hipStream_t s;
        DSP_HIP(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        pl->streams.push_back(s);
        DSP_HIP(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        pl->fstreams.push_back(s);
        for (int i = 0; i < pl->ev_depth; ++i) {
            hipEvent_t e;
            DSP_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
            pl->done[i].push_back(e);
        }
        for (int i = 0; i < 2; ++i) {
            hipEvent_t e;
            DSP_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
            pl->fdone[i].push_back(e);
        }
        hipEvent_t e;
        DSP_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        pl->join.push_back(e);
    }
    DSP_HIP(hipEventCreateWithFlags(&pl->in_ready, hipEventDisableTiming));
    DSP_HIP(hipEventCreateWithFlags(&pl->in_copied, hipEventDisableTiming));
    DSP_HIP(hipEventCreateWithFlags(&pl->fork, hipEventDisableTiming));
    // Q_k holds G_{h_k}: same bytes as block k's input slot.
    pl->qring.assign(K, nullptr);
    pl->qslot_bytes.assign(K, 0);
    for (int k = 1; k < K; ++k) {
        DSP_TRY(dsp_block_output_shape(pl->blocks[k - 1], shape));
        size_t bytes = (size_t)shape[0] * shape[1] * shape[2] * shape[3] * 4;  // upper bound (fp32)
        bytes = (bytes + 255) / 256 * 256;
        void* ptr;
        DSP_TRY(pl_alloc(pl, &ptr, bytes * pl->qn[k]));
        pl->qring[k] = (char*)ptr;
        pl->qslot_bytes[k] = bytes;
    }
    pl->label_slots = label_slots;
    period = std::lcm(period, (int64_t)pl->label_slots);
    pl->period = (pl->serial || pl->fwd_locked || period > kMaxGraphs) ? 0 : (int)period;
    pl->graphs.assign(pl->period, nullptr);
    void* ptr;
    DSP_TRY(pl_alloc(pl, &ptr, (size_t)pl->label_slots * pl->N * 4));
    pl->labels = (int32_t*)ptr;
    DSP_TRY(pl_alloc(pl, &ptr, (size_t)(pl->max_ticks + 1) * 4));
    pl->losses = (float*)ptr;
    DSP_TRY(pl_alloc(pl, &ptr, 16));
    pl->loss_tmp = (float*)ptr;
    pl->loss_count = (int32_t*)ptr + 2;
    DSP_HIP(hipMemset(pl->losses, 0, (size_t)(pl->max_ticks + 1) * 4));
    DSP_HIP(hipMemset(pl->loss_tmp, 0, 16));
    DSP_HIP(hipDeviceSynchronize());
    DSP_HIP(hipGetDevice(&pl->device));
    pl->fwd_split.assign(K, 0);
    pl->workers.assign(K, nullptr);
    if (!pl->serial)
        for (int k = 1; k < K; ++k) {
            pl->workers[k] = new (std::nothrow) Worker();
            DSP_REQUIRE(pl->workers[k], DSP_ENOMEM, "dsp_pipeline_init: out of host memory");
            pl->workers[k]->th = std::thread(worker_main, pl, k);
        }
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
    pl->fwd_locked = !pl->serial && K > 1;
    for (int k = 0; k < K; ++k) pl->fwd_locked = pl->fwd_locked && p[k] == 0;
    pl->fwd_issued.reset(new std::atomic<int64_t>[K]);
    for (int k = 0; k < K; ++k) pl->fwd_issued[k].store(0);
    pl->lr = lr;
    pl->momentum = momentum;
    pl->wd = weight_decay;
    pl->max_ticks = max_ticks;
    pl->delay_us.assign(K, 0);
    pl->spare.assign(K, 0);
    pl->qn.assign(K, 1);
    pl->wait_dn.assign(K, 1);
    pl->wait_up.assign(K, 1);
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
    if (pl->delay_us[k] != microseconds) drop_graphs(pl);  // the delay kernel is part of the captured ticks
    pl->delay_us[k] = microseconds;
    return DSP_OK;
}

int dsp_pipeline_set_optimizer(dsp_pipeline* pl, float lr, float momentum, int32_t s, float weight_decay)
{
    DSP_REQUIRE(pl, DSP_EINVAL, "dsp_pipeline_set_optimizer: null pipeline");
    DSP_REQUIRE(s == 0 || s == 1, DSP_EINVAL, "dsp_pipeline_set_optimizer: s = %d (only s = 0 and s = 1 are built)", (int)s);
    DSP_REQUIRE(lr >= 0.f, DSP_EINVAL, "dsp_pipeline_set_optimizer: negative step size");
    pl->lr = lr;
    pl->momentum = momentum;
    pl->sum_s = s;
    pl->wd = weight_decay;
    drop_graphs(pl);  // recorded ticks hold the old constants
    pl->eager_ticks = 1;
    return DSP_OK;
}

int dsp_pipeline_attach_gradient_probe(dsp_pipeline* pl, dsp_pipeline* probe)
{
    DSP_REQUIRE(pl && probe && pl != probe, DSP_EINVAL, "dsp_pipeline_attach_gradient_probe: bad argument");
    DSP_REQUIRE(pl->tau == 0 && probe->tau == 0 && !pl->probe, DSP_ESTATE,
                "dsp_pipeline_attach_gradient_probe: must be called once, before the first step of either pipeline");
    DSP_REQUIRE(!pl->serial && pl->K >= 2, DSP_EINVAL, "dsp_pipeline_attach_gradient_probe: the pipeline has no staleness to measure");
    DSP_REQUIRE(probe->serial && probe->K == pl->K && probe->N == pl->N && probe->in_bytes == pl->in_bytes, DSP_EINVAL,
                "dsp_pipeline_attach_gradient_probe: the probe must be an all-zero-schedule pipeline over the same K blocks");
    DSP_REQUIRE(probe->lr == 0.f, DSP_EINVAL, "dsp_pipeline_attach_gradient_probe: the probe must have step size 0");
    DSP_REQUIRE(probe->max_ticks >= pl->max_ticks, DSP_EINVAL, "dsp_pipeline_attach_gradient_probe: probe max_ticks too small");
    const int K = pl->K;
    for (int k = 0; k < K; ++k)
        DSP_REQUIRE(block_arrays(pl->blocks[k]).n == block_arrays(probe->blocks[k]).n, DSP_EINVAL,
                    "dsp_pipeline_attach_gradient_probe: block %d has another parameter count in the probe", k);
    // block 0 is the last to finish a mini-batch: b forwarded at tick b + P_k is needed until tick b + m_0
    const int horizon = pl->m[0];
    pl->xsnap.assign(K, nullptr);
    pl->gstash.assign(K, nullptr);
    pl->xsnap_n.assign(K, 0);
    pl->gstash_n.assign(K, 0);
    for (int k = 0; k < K; ++k) {
        const size_t n = block_arrays(pl->blocks[k]).n;
        pl->xsnap_n[k] = horizon - pl->P[k] + 1;
        pl->gstash_n[k] = horizon - pl->P[k] - pl->m[k] + 1;
        DSP_REQUIRE(pl->xsnap_n[k] >= 1 && pl->gstash_n[k] >= 1, DSP_EINVAL, "dsp_pipeline_attach_gradient_probe: schedule");
        DSP_TRY(pl_alloc(pl, (void**)&pl->xsnap[k], n * 4 * pl->xsnap_n[k]));
        DSP_TRY(pl_alloc(pl, (void**)&pl->gstash[k], n * 4 * pl->gstash_n[k]));
    }
    DSP_TRY(pl_alloc(pl, (void**)&pl->probe_labels, (size_t)pl->N * 4 * (horizon + 1)));
    DSP_TRY(pl_alloc(pl, (void**)&pl->probe_partial, sizeof(double) * 2 * kDiffSumsqBlocks));
    DSP_TRY(pl_alloc(pl, (void**)&pl->probe_out, sizeof(double) * 2 * K));
    pl->probe_diff.assign(K, 0.0);
    pl->probe_ref.assign(K, 0.0);
    pl->probe = probe;
    return DSP_OK;
}

int dsp_pipeline_gradient_difference(dsp_pipeline* pl, int64_t* batch_id, double* diff_sumsq, double* bp_sumsq)
{
    DSP_REQUIRE(pl && batch_id && diff_sumsq && bp_sumsq, DSP_EINVAL, "dsp_pipeline_gradient_difference: null argument");
    DSP_REQUIRE(pl->probe, DSP_ESTATE, "dsp_pipeline_gradient_difference: no probe attached");
    *batch_id = pl->probe_batch;
    for (int k = 0; k < pl->K; ++k) {
        diff_sumsq[k] = pl->probe_batch >= 0 ? pl->probe_diff[k] : 0.0;
        bp_sumsq[k] = pl->probe_batch >= 0 ? pl->probe_ref[k] : 0.0;
    }
    return DSP_OK;
}

int dsp_pipeline_set_graph_replay(dsp_pipeline* pl, int32_t enable)
{
    DSP_REQUIRE(pl, DSP_EINVAL, "dsp_pipeline_set_graph_replay: null pipeline");
    pl->use_graphs = enable != 0;
    return DSP_OK;
}

int dsp_pipeline_set_forward_streams(dsp_pipeline* pl, int32_t enable)
{
    DSP_REQUIRE(pl, DSP_EINVAL, "dsp_pipeline_set_forward_streams: null pipeline");
    DSP_REQUIRE(pl->tau == 0, DSP_ESTATE, "dsp_pipeline_set_forward_streams: the pipeline has already been stepped");
    DSP_REQUIRE(!enable || pl->ev_depth == 2, DSP_EINVAL,
                "dsp_pipeline_set_forward_streams: not with spare queue entries (its waits are one tick deep)");
    DSP_REQUIRE(!enable || !pl->fwd_locked, DSP_EINVAL, "dsp_pipeline_set_forward_streams: not with a forward-locked schedule");
    pl->use_fwd_streams = enable != 0;
    return DSP_OK;
}

int dsp_pipeline_set_twin_launches(dsp_pipeline* pl, int32_t enable)
{
    DSP_REQUIRE(pl, DSP_EINVAL, "dsp_pipeline_set_twin_launches: null pipeline");
    pl->use_twin = enable != 0;
    drop_graphs(pl);  // recorded ticks contain the other kind of launches
    return DSP_OK;
}

int dsp_pipeline_set_single_stream(dsp_pipeline* pl, int32_t enable)
{
    DSP_REQUIRE(pl, DSP_EINVAL, "dsp_pipeline_set_single_stream: null pipeline");
    DSP_REQUIRE(!enable || !pl->use_fwd_streams, DSP_EINVAL, "dsp_pipeline_set_single_stream: not together with forward streams");
    // work already issued on the K streams must not be overtaken by what follows on stream 0, and vice versa
    DSP_TRY(dsp_pipeline_sync(pl));
    pl->single_stream = enable != 0;
    return DSP_OK;
}

int dsp_pipeline_set_launch_threads(dsp_pipeline* pl, int32_t enable)
{
    DSP_REQUIRE(pl, DSP_EINVAL, "dsp_pipeline_set_launch_threads: null pipeline");
    pl->use_threads = enable != 0;
    return DSP_OK;
}

// The three parts of block k's tick tau.  Forward of mini-batch a = tau - P_k:
static int tick_forward(dsp_pipeline* pl, int k, int64_t tau, hipStream_t st, bool dry)
{
    const int K = pl->K;
    const int64_t a = tau - pl->P[k];
    if (a < 0) return DSP_OK;
    dsp_block* b = pl->blocks[k];
    void* in;
    DSP_TRY(dsp_block_input_slot(b, a, &in));  // block 0: filled by the data source copy of this tick
    void* out = nullptr;
    if (k < K - 1) DSP_TRY(dsp_block_input_slot(pl->blocks[k + 1], a, &out));
    const int32_t* lab = pl->labels + (size_t)(a % pl->label_slots) * pl->N;
    const bool last = k == K - 1;
    DSP_TRY(dsp_block_forward(b, a, in, out, last ? lab : nullptr, last ? pl->loss_tmp : nullptr, st));
    if (last && !dry) DSP_TRY(launch_record_loss(pl->loss_tmp, pl->losses, pl->loss_count, pl->max_ticks + 1, st));
    return DSP_OK;
}

// recompute + backward of mini-batch a - m_k (nothing while the pipeline fills):
static int tick_backward(dsp_pipeline* pl, int k, int64_t tau, hipStream_t st, bool* did)
{
    const int K = pl->K;
    const int64_t bb = tau - pl->P[k] - pl->m[k];
    *did = bb >= 0;
    if (bb < 0) return DSP_OK;
    const void* gout = k < K - 1 ? pl->qring[k + 1] + (size_t)(bb % pl->qn[k + 1]) * pl->qslot_bytes[k + 1] : nullptr;
    void* gin = k > 0 ? pl->qring[k] + (size_t)(bb % pl->qn[k]) * pl->qslot_bytes[k] : nullptr;
    return dsp_block_recompute_backward(pl->blocks[k], bb, gout, gin, st);
}

// Both of the above through dsp_block_step (same results, one launch per layer for the two forward
// sweeps).  *fused = false if the tick has only one of the two parts; nothing is issued then.
static int tick_step(dsp_pipeline* pl, int k, int64_t tau, hipStream_t st, bool dry, bool* fused, hipEvent_t after_forward = nullptr)
{
    const int K = pl->K;
    const int64_t a = tau - pl->P[k], bb = a - pl->m[k];
    *fused = pl->use_twin && pl->m[k] > 0 && bb >= 0;
    if (!*fused) return DSP_OK;
    dsp_block* b = pl->blocks[k];
    void* in;
    DSP_TRY(dsp_block_input_slot(b, a, &in));
    void* out = nullptr;
    if (k < K - 1) DSP_TRY(dsp_block_input_slot(pl->blocks[k + 1], a, &out));
    const int32_t* lab = pl->labels + (size_t)(a % pl->label_slots) * pl->N;
    const bool last = k == K - 1;
    const void* gout = k < K - 1 ? pl->qring[k + 1] + (size_t)(bb % pl->qn[k + 1]) * pl->qslot_bytes[k + 1] : nullptr;
    void* gin = k > 0 ? pl->qring[k] + (size_t)(bb % pl->qn[k]) * pl->qslot_bytes[k] : nullptr;
    DSP_TRY(block_step_event(b, a, in, out, last ? lab : nullptr, last ? pl->loss_tmp : nullptr, bb, gout, gin, st, after_forward));
    if (last && !dry) DSP_TRY(launch_record_loss(pl->loss_tmp, pl->losses, pl->loss_count, pl->max_ticks + 1, st));
    return DSP_OK;
}

// and the update that consumes that gradient.
static int tick_update(dsp_pipeline* pl, int k, hipStream_t st)
{
    return dsp_param_update_sum(pl->blocks[k], pl->lr, pl->momentum, pl->sum_s, pl->wd, st);
}

// All of it on one stream.
static int block_tick(dsp_pipeline* pl, int k, int64_t tau, hipStream_t st, bool do_fwd, bool do_bwd, bool dry = false)
{
    if (do_fwd && do_bwd) {
        bool fused;
        DSP_TRY(tick_step(pl, k, tau, st, dry, &fused));
        if (fused) return tick_update(pl, k, st);
    }
    if (do_fwd) DSP_TRY(tick_forward(pl, k, tau, st, dry));
    if (do_bwd) {
        bool did;
        DSP_TRY(tick_backward(pl, k, tau, st, &did));
        if (did) DSP_TRY(tick_update(pl, k, st));
    }
    return DSP_OK;
}

// The chain of block k at tick tau, issued kernel by kernel on the block's own stream(s).
static int run_block_tick(dsp_pipeline* pl, int k, int64_t tau)
{
    const int K = pl->K;
    const int R = pl->ev_depth;
    const int cur = (int)(tau % R), prev = (int)((tau + R - 1) % R);
    const int fcur = (int)(tau & 1), fprev = fcur ^ 1;
    const bool split = pl->fwd_split[k] != 0;
    hipStream_t sb = pl->single_stream ? pl->streams[0] : pl->streams[k];
    hipStream_t sf = split ? pl->fstreams[k] : sb;
    // The neighbours' tick wait_dn / wait_up back (the previous tick unless the queues have spare
    // entries): the slots this block reads were written then or earlier, and the slots it writes
    // were last read then or earlier.  Every host thread has issued that tick (ticks are issued
    // one at a time), so its event already stands for it.  (The labels of the mini-batch the
    // last block sees now were copied on stream 0 P_{K-1} >= K-1 ticks ago, which this chain
    // of waits orders; the label ring is long enough that a slot is not refilled too early.)
    if (k > 0 && pl->wait_dn[k] > 0 && tau >= pl->wait_dn[k]) DSP_HIP(hipStreamWaitEvent(sb, pl->done[(tau - pl->wait_dn[k]) % R][k - 1], 0));
    if (k < K - 1 && pl->wait_up[k] > 0 && tau >= pl->wait_up[k]) DSP_HIP(hipStreamWaitEvent(sb, pl->done[(tau - pl->wait_up[k]) % R][k + 1], 0));
    if (tau > 0) {
        if (split) {
            DSP_HIP(hipStreamWaitEvent(sf, pl->done[prev][k], 0));                       // its own last update
            if (k > 0) DSP_HIP(hipStreamWaitEvent(sf, pl->fdone[fprev][k - 1], 0));       // its input
            if (k < K - 1) DSP_HIP(hipStreamWaitEvent(sf, pl->done[prev][k + 1], 0));     // the slot its output goes to
        }
    }
    if (split && k == 0) DSP_HIP(hipStreamWaitEvent(sf, pl->in_copied, 0));  // the mini-batch of this tick
    if (pl->delay_us[k] > 0) {
        DSP_TRY(launch_spin(pl->delay_us[k], sb));
        if (split) DSP_TRY(launch_spin(pl->delay_us[k], sf));
    }
    if (pl->fwd_locked) {
        // This tick's forward pass of the block below produced the input (and, being later on that stream than its
        // previous tick, also stands for everything this block overwrites having been read).  Its host thread
        // records that event some time during this tick: wait until it has.
        if (k > 0) {
            while (pl->fwd_issued[k - 1].load(std::memory_order_acquire) <= tau) std::this_thread::yield();
            DSP_HIP(hipStreamWaitEvent(sb, pl->fdone[fcur][k - 1], 0));
        }
        bool fused = false;
        int rc = tick_step(pl, k, tau, sb, false, &fused, pl->fdone[fcur][k]);
        if (rc == DSP_OK && fused) {
            pl->fwd_issued[k].store(tau + 1, std::memory_order_release);
            rc = tick_update(pl, k, sb);
        } else if (rc == DSP_OK) {
            rc = tick_forward(pl, k, tau, sb, false);
            if (rc == DSP_OK && hipEventRecord(pl->fdone[fcur][k], sb) != hipSuccess) rc = DSP_EHIP;
            pl->fwd_issued[k].store(tau + 1, std::memory_order_release);
            bool did = false;
            if (rc == DSP_OK) rc = tick_backward(pl, k, tau, sb, &did);
            if (rc == DSP_OK && did) rc = tick_update(pl, k, sb);
        }
        if (rc != DSP_OK) {
            pl->fwd_issued[k].store(tau + 1, std::memory_order_release);  // never leave the block above spinning
            return rc;
        }
        DSP_HIP(hipEventRecord(pl->done[cur][k], sb));
        return DSP_OK;
    }
    if (!split) {
        DSP_TRY(block_tick(pl, k, tau, sb, true, true));
        DSP_HIP(hipEventRecord(pl->fdone[fcur][k], sb));
        DSP_HIP(hipEventRecord(pl->done[cur][k], sb));
        return DSP_OK;
    }
    DSP_TRY(tick_forward(pl, k, tau, sf, false));
    DSP_HIP(hipEventRecord(pl->fdone[fcur][k], sf));
    bool did;
    DSP_TRY(tick_backward(pl, k, tau, sb, &did));
    if (did) {
        if (split) DSP_HIP(hipStreamWaitEvent(sb, pl->fdone[fcur][k], 0));  // the forward pass has read the parameters
        DSP_TRY(tick_update(pl, k, sb));
    } else if (split) {
        DSP_HIP(hipStreamWaitEvent(sb, pl->fdone[fcur][k], 0));  // keep done[cur][k] meaning "everything of this tick"
    }
    DSP_HIP(hipEventRecord(pl->done[cur][k], sb));
    return DSP_OK;
}

// All K block chains of tick tau: kernel by kernel (one stream and one host thread per block), or
// recorded into a graph capture.
static int issue_tick(dsp_pipeline* pl, int64_t tau, bool capturing)
{
    const int K = pl->K;
    hipStream_t s0 = pl->streams[0];
    if (!capturing) {
        const bool threads = pl->use_threads && K > 1 && !pl->single_stream;
        if (threads)
            for (int k = 1; k < K; ++k) {
                Worker* w = pl->workers[k];
                {
                    std::lock_guard<std::mutex> g(w->mu);
                    w->tau = tau;
                    w->finished = false;
                    w->has_job = true;
                }
                w->cv.notify_all();
            }
        int rc = run_block_tick(pl, 0, tau);
        std::string err = rc == DSP_OK ? "" : dsp_last_error();
        for (int k = 1; k < K; ++k) {
            int rk;
            if (threads) {
                Worker* w = pl->workers[k];
                std::unique_lock<std::mutex> lk(w->mu);
                w->cv.wait(lk, [&] { return w->finished; });
                rk = w->rc;
                if (rk != DSP_OK && rc == DSP_OK) err = w->err;
            } else {
                rk = run_block_tick(pl, k, tau);
                if (rk != DSP_OK && rc == DSP_OK) err = dsp_last_error();
            }
            if (rc == DSP_OK) rc = rk;
        }
        if (rc != DSP_OK) set_error("%s", err.c_str());
        return rc;
    }
    DSP_HIP(hipEventRecord(pl->fork, s0));
    for (int k = 1; k < K; ++k) DSP_HIP(hipStreamWaitEvent(pl->streams[k], pl->fork, 0));
    for (int k = 0; k < K; ++k) {
        hipStream_t st = pl->streams[k];
        if (pl->delay_us[k] > 0) DSP_TRY(launch_spin(pl->delay_us[k], st));
        DSP_TRY(block_tick(pl, k, tau, st, true, true));
    }
    if (capturing)
        for (int k = 1; k < K; ++k) {
            DSP_HIP(hipEventRecord(pl->join[k], pl->streams[k]));
            DSP_HIP(hipStreamWaitEvent(s0, pl->join[k], 0));
        }
    return DSP_OK;
}

// Gradient-difference diagnostic, part 1: before tick tau is issued, keep the parameters every block is
// about to run the forward pass of mini-batch tau - P_k with (the tick's update comes last) and the labels.
static int probe_before_tick(dsp_pipeline* pl, int64_t tau, const int32_t* d_labels, hipStream_t user)
{
    DSP_REQUIRE(d_labels, DSP_EINVAL, "dsp_pipeline_step: the gradient probe needs labels");
    DSP_TRY(dsp_pipeline_sync(pl));
    DSP_HIP(hipStreamSynchronize(user));
    for (int k = 0; k < pl->K; ++k) {
        const int64_t a = tau - pl->P[k];
        if (a < 0) continue;
        const BlockArrays A = block_arrays(pl->blocks[k]);
        DSP_HIP(hipMemcpy(pl->xsnap[k] + (size_t)(a % pl->xsnap_n[k]) * A.n, A.x, A.n * 4, hipMemcpyDeviceToDevice));
    }
    DSP_HIP(hipMemcpy(pl->probe_labels + (size_t)(tau % (pl->m[0] + 1)) * pl->N, d_labels, (size_t)pl->N * 4,
                      hipMemcpyDeviceToDevice));
    return DSP_OK;
}

// Part 2: after tick tau, keep the DSP gradients it formed; block 0's is the last one of its mini-batch b,
// which is then re-run as ordinary backpropagation through the probe blocks at the kept parameters.
static int probe_after_tick(dsp_pipeline* pl, int64_t tau)
{
    const int K = pl->K;
    DSP_TRY(dsp_pipeline_sync(pl));
    for (int k = 0; k < K; ++k) {
        const int64_t bb = tau - pl->P[k] - pl->m[k];
        if (bb < 0) continue;
        const BlockArrays A = block_arrays(pl->blocks[k]);
        DSP_HIP(hipMemcpy(pl->gstash[k] + (size_t)(bb % pl->gstash_n[k]) * A.n, A.g, A.n * 4, hipMemcpyDeviceToDevice));
    }
    const int64_t b = tau - pl->m[0];
    if (b < 0) return DSP_OK;
    dsp_pipeline* pr = pl->probe;
    for (int k = 0; k < K; ++k) {
        const BlockArrays A = block_arrays(pr->blocks[k]);
        DSP_TRY(block_load_params_device(pr->blocks[k], pl->xsnap[k] + (size_t)(b % pl->xsnap_n[k]) * A.n, nullptr));
    }
    DSP_HIP(hipDeviceSynchronize());
    void* slot0;
    DSP_TRY(dsp_block_input_slot(pl->blocks[0], b, &slot0));  // still holds h_0(b): block 0 just recomputed from it
    DSP_TRY(dsp_pipeline_step(pr, slot0, pl->probe_labels + (size_t)(b % (pl->m[0] + 1)) * pl->N, nullptr, nullptr, nullptr));
    DSP_TRY(dsp_pipeline_sync(pr));
    for (int k = 0; k < K; ++k) {
        const BlockArrays A = block_arrays(pr->blocks[k]);
        DSP_TRY(launch_diff_sumsq(pl->gstash[k] + (size_t)(b % pl->gstash_n[k]) * A.n, A.g, A.n, pl->probe_partial,
                                  pl->probe_out + 2 * k, nullptr));
    }
    std::vector<double> out(2 * K);
    DSP_HIP(hipMemcpy(out.data(), pl->probe_out, sizeof(double) * 2 * K, hipMemcpyDeviceToHost));
    for (int k = 0; k < K; ++k) {
        pl->probe_diff[k] = out[2 * k];
        pl->probe_ref[k] = out[2 * k + 1];
    }
    pl->probe_batch = b;
    return DSP_OK;
}

int dsp_pipeline_step(dsp_pipeline* pl, const void* d_batch, const int32_t* d_labels, float* h_loss,
                      int64_t* loss_batch_id, void* stream)
{
    DSP_REQUIRE(pl && d_batch, DSP_EINVAL, "dsp_pipeline_step: null argument");
    DSP_REQUIRE(pl->tau < pl->max_ticks, DSP_ESTATE, "dsp_pipeline_step: max_ticks (%lld) reached", (long long)pl->max_ticks);
    const int K = pl->K;
    const int64_t tau = pl->tau;
    const int R = pl->ev_depth;
    const int cur = (int)(tau % R), prev = (int)((tau + R - 1) % R);
    hipStream_t user = (hipStream_t)stream;
    hipStream_t s0 = pl->streams[0];

    if (tau == 0 && pl->use_fwd_streams && !pl->serial)
        for (int k = 0; k < K; ++k)
            if (pl->m[k] > 0) {
                DSP_TRY(dsp_block_enable_forward_lane(pl->blocks[k]));
                pl->fwd_split[k] = 1;
            }
    if (pl->probe) DSP_TRY(probe_before_tick(pl, tau, d_labels, user));
    const bool graph_tick = pl->use_graphs && pl->period > 0 && !g_profile_on && tau > pl->fill && pl->eager_ticks == 0 &&
                            !pl->probe && !pl->single_stream;
    if (pl->eager_ticks > 0 && tau > pl->fill) pl->eager_ticks -= 1;
    const int phase = graph_tick ? (int)(tau % pl->period) : 0;

    // the data source: copy the mini-batch into block 0's ring slot and the labels into the label ring
    DSP_HIP(hipEventRecord(pl->in_ready, user));
    DSP_HIP(hipStreamWaitEvent(s0, pl->in_ready, 0));
    if (tau > 0 && !pl->serial) {
        // block 0's slot for this tick is free (its own earlier ticks ran on this stream); a graph tick
        // starts only after every stream has finished the previous tick, any other after the tick of block 1
        // that block 0 is about to wait for anyway
        if (graph_tick)
            for (int k = 1; k < K; ++k) DSP_HIP(hipStreamWaitEvent(s0, pl->done[prev][k], 0));
        else if (K > 1 && pl->wait_up[0] > 0 && tau >= pl->wait_up[0])
            DSP_HIP(hipStreamWaitEvent(s0, pl->done[(tau - pl->wait_up[0]) % R][1], 0));
    }
    void* slot0;
    DSP_TRY(dsp_block_input_slot(pl->blocks[0], tau, &slot0));
    DSP_HIP(hipMemcpyAsync(slot0, d_batch, pl->in_bytes, hipMemcpyDeviceToDevice, s0));
    if (d_labels)
        DSP_HIP(hipMemcpyAsync(pl->labels + (size_t)(tau % pl->label_slots) * pl->N, d_labels, (size_t)pl->N * 4,
                               hipMemcpyDeviceToDevice, s0));
    DSP_HIP(hipEventRecord(pl->in_copied, s0));
    DSP_HIP(hipStreamWaitEvent(user, pl->in_copied, 0));

    if (pl->serial) {
        // ordinary backpropagation: forward up the chain, backward down the chain, one stream (a delayed block
        // holds the whole chain up, as a slow device does in model-parallel backpropagation)
        for (int k = 0; k < K; ++k) {
            if (pl->delay_us[k] > 0) DSP_TRY(launch_spin(pl->delay_us[k], s0));
            DSP_TRY(block_tick(pl, k, tau, s0, true, false));
        }
        for (int k = K - 1; k >= 0; --k) DSP_TRY(block_tick(pl, k, tau, s0, false, true));
    } else if (!graph_tick) {
        DSP_TRY(issue_tick(pl, tau, false));
    } else {
        if (!pl->graphs[phase]) {
            // record this tick once; its launches are replayed whenever the rings are in this position again
            hipGraph_t graph = nullptr;
            DSP_HIP(hipStreamBeginCapture(s0, hipStreamCaptureModeRelaxed));
            const int rc = issue_tick(pl, tau, true);
            const hipError_t e = hipStreamEndCapture(s0, &graph);
            if (rc != DSP_OK && graph) (void)hipGraphDestroy(graph);
            DSP_TRY(rc);
            DSP_REQUIRE(e == hipSuccess && graph, DSP_EHIP, "dsp_pipeline_step: graph capture failed: %s", hipGetErrorString(e));
            hipGraphExec_t exec = nullptr;
            const hipError_t e2 = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
            (void)hipGraphDestroy(graph);
            DSP_REQUIRE(e2 == hipSuccess && exec, DSP_EHIP, "dsp_pipeline_step: graph instantiation failed: %s",
                        hipGetErrorString(e2));
            pl->graphs[phase] = exec;
        } else {
            // advance every block's host-side state exactly as the recorded launches would
            for (int k = 0; k < K; ++k) block_set_dry(pl->blocks[k], true);
            int rc = DSP_OK;
            for (int k = 0; k < K && rc == DSP_OK; ++k) rc = block_tick(pl, k, tau, nullptr, true, true, true);
            for (int k = 0; k < K; ++k) block_set_dry(pl->blocks[k], false);
            DSP_TRY(rc);
        }
        DSP_HIP(hipGraphLaunch(pl->graphs[phase], s0));
        for (int k = 0; k < K; ++k) {
            DSP_HIP(hipEventRecord(pl->done[cur][k], s0));
            DSP_HIP(hipEventRecord(pl->fdone[tau & 1][k], s0));
        }
    }
    pl->tau = tau + 1;
    if (pl->probe) DSP_TRY(probe_after_tick(pl, tau));

    const int64_t a_last = tau - pl->P[K - 1];
    if (loss_batch_id) *loss_batch_id = a_last >= 0 ? a_last : -1;
    if (h_loss) {
        *h_loss = 0.f;
        if (a_last >= 0) {
            hipStream_t sl = (pl->serial || graph_tick || pl->single_stream) ? s0 : (pl->fwd_split[K - 1] ? pl->fstreams[K - 1] : pl->streams[K - 1]);
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
    for (hipStream_t s : pl->fstreams) DSP_HIP(hipStreamSynchronize(s));
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
