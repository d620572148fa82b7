// Host side of libtw that is not tied to one kernel: status strings, device
// queries, the event pool, the token split and the overlap launch.
#include <algorithm>
#include <mutex>
#include <vector>

#include "tw_internal.h"

namespace tw {

static thread_local int g_last_hip_error = 0;
static thread_local const char *g_last_hip_where = "";

tw_status hip_fail(hipError_t e, const char *where)
{
    g_last_hip_error = static_cast<int>(e);
    g_last_hip_where = where;
    (void)hipGetLastError();  // clear the sticky per-thread error so later calls start clean
    return TW_ERR_HIP;
}

static std::mutex g_mu;
static int g_cu_count[kMaxDevices];  // 0 = not queried yet

tw_status current_cu_count(int *cu_count)
{
    int dev = 0;
    TW_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice, "tw_host.hip: device id out of range");
    {
        std::lock_guard<std::mutex> lk(g_mu);
        if (g_cu_count[dev] > 0) {
            *cu_count = g_cu_count[dev];
            return TW_OK;
        }
    }
    int n = 0;
    TW_HIP(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
    if (n <= 0) return hip_fail(hipErrorInvalidDevice, "tw_host.hip: the device reports no compute units");
    std::lock_guard<std::mutex> lk(g_mu);
    g_cu_count[dev] = n;
    *cu_count = n;
    return TW_OK;
}

tw_status allow_dynamic_lds(const void *kernel, int bytes, std::atomic<int> *done)
{
    int dev = 0;
    TW_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice, "tw_host.hip: device id out of range");
    if (done[dev].load(std::memory_order_acquire)) return TW_OK;
    TW_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    done[dev].store(1, std::memory_order_release);
    return TW_OK;
}

// Events are only used as stream-ordering markers: recorded on one stream and
// waited on by another within the same call. A wait refers to the record that
// precedes it, so an event can be recorded again once its wait has been
// enqueued. Each host thread draws from a ring of its own (per device): between
// one thread's record and its wait no other thread can record the same event,
// whatever the interleaving, and a call uses far fewer events than a ring holds,
// so a call never meets its own event twice. A thread that ends hands its events
// to a spare list for later threads; nothing is destroyed (the runtime may
// already be shutting down when the last thread-local is torn down).
static constexpr int kEventRing = 16;  // most events one call records: 5 (tw_weave_layer, ordered)
static std::vector<hipEvent_t> *g_spare_events[kMaxDevices];  // leaked on purpose, guarded by g_mu

struct EventRing {
    hipEvent_t ev[kMaxDevices][kEventRing];
    unsigned char made[kMaxDevices];  // events created so far on that device
    unsigned char next[kMaxDevices];
    EventRing() : ev(), made(), next() {}
    ~EventRing()
    {
        std::lock_guard<std::mutex> lk(g_mu);
        for (int d = 0; d < kMaxDevices; ++d) {
            if (!made[d]) continue;
            if (!g_spare_events[d]) g_spare_events[d] = new std::vector<hipEvent_t>();
            for (int i = 0; i < made[d]; ++i) g_spare_events[d]->push_back(ev[d][i]);
        }
    }
};
static thread_local EventRing t_ring;

tw_status borrow_event(hipEvent_t *ev)
{
    int dev = 0;
    TW_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice, "tw_host.hip: device id out of range");
    EventRing &r = t_ring;
    const int i = r.next[dev];
    r.next[dev] = static_cast<unsigned char>((i + 1) % kEventRing);
    if (i >= r.made[dev]) {  // slots fill in order, so i == made
        hipEvent_t e = nullptr;
        {
            std::lock_guard<std::mutex> lk(g_mu);
            std::vector<hipEvent_t> *spare = g_spare_events[dev];
            if (spare && !spare->empty()) {
                e = spare->back();
                spare->pop_back();
            }
        }
        if (!e) {
            const hipError_t err = hipEventCreateWithFlags(&e, hipEventDisableTiming);
            if (err != hipSuccess) {
                r.next[dev] = static_cast<unsigned char>(i);  // the slot stays empty
                return hip_fail(err, "tw_host.hip: hipEventCreateWithFlags");
            }
        }
        r.ev[dev][i] = e;
        r.made[dev] = static_cast<unsigned char>(i + 1);
    }
    *ev = r.ev[dev][i];
    return TW_OK;
}

// `child` waits for everything enqueued on `from` so far.
static tw_status stream_wait_stream(hipStream_t child, hipStream_t from)
{
    hipEvent_t ev;
    TW_TRY(borrow_event(&ev));
    TW_HIP(hipEventRecord(ev, from));
    TW_HIP(hipStreamWaitEvent(child, ev, 0));
    return TW_OK;
}

}  // namespace tw

using namespace tw;

extern "C" {

int tw_device_cu_count(void)
{
    int n = 0;
    return current_cu_count(&n) == TW_OK ? n : -1;
}

const char *tw_status_str(tw_status s)
{
    switch (s) {
    case TW_OK: return "ok";
    case TW_ERR_NULL: return "a required pointer is NULL";
    case TW_ERR_SHAPE: return "a size is out of range";
    case TW_ERR_ALIGN: return "a data pointer is not 16-byte aligned";
    case TW_ERR_ALIAS: return "buffers overlap in a way that is not allowed";
    case TW_ERR_UNSUPPORTED: return "no kernel for this request";
    case TW_ERR_SPLIT: return "bad split row or cuts, or identical streams";
    case TW_ERR_HIP: return "a HIP call failed (see tw_last_hip_error)";
    }
    return "unknown status";
}

const char *tw_version(void) { return "libtw 0.2 (gfx950)"; }

int tw_last_hip_error(void) { return g_last_hip_error; }

const char *tw_last_hip_error_where(void) { return g_last_hip_where; }

int64_t tw_split_point(int64_t N, int64_t multiple)
{
    if (N <= 0) return 0;
    if (multiple <= 0) multiple = 1;
    if (multiple >= N) return N;  // the first multiple at or above N/2 is already >= N
    const int64_t half = N / 2 + (N & 1);
    const int64_t blocks = half / multiple + (half % multiple != 0);
    const int64_t k = blocks * multiple;  // < half + multiple < 2N: no overflow
    return k < N ? k : N;
}

tw_status tw_split_launch(const tw_fused_args *args, int64_t split_row, void *stream_a,
                          void *stream_b, void *parent, int parent_is_set, int join)
{
    if (!args) return TW_ERR_NULL;
    TW_TRY(validate_fused(*args));
    if (split_row < 0 || split_row > args->N) return TW_ERR_SPLIT;
    const bool has_a = split_row > 0, has_b = split_row < args->N;
    if (has_a && has_b && stream_a == stream_b) return TW_ERR_SPLIT;
    if (!has_a && !has_b) return TW_OK;

    hipStream_t sa = static_cast<hipStream_t>(stream_a), sb = static_cast<hipStream_t>(stream_b);
    hipStream_t sp = static_cast<hipStream_t>(parent);
    if (parent_is_set) {
        hipEvent_t fork;
        TW_TRY(borrow_event(&fork));
        TW_HIP(hipEventRecord(fork, sp));
        if (has_a && sa != sp) TW_HIP(hipStreamWaitEvent(sa, fork, 0));
        if (has_b && sb != sp) TW_HIP(hipStreamWaitEvent(sb, fork, 0));
    }
    if (has_a) TW_TRY(launch_fused(*args, 0, split_row, nullptr, 0, sa));
    if (has_b) TW_TRY(launch_fused(*args, split_row, args->N, nullptr, 0, sb));
    if (parent_is_set && join) {
        if (has_a && sa != sp) TW_TRY(stream_wait_stream(sp, sa));
        if (has_b && sb != sp) TW_TRY(stream_wait_stream(sp, sb));
    }
    return TW_OK;
}

tw_status tw_overlap_launch(const tw_fused_args *fused, const tw_gemm_args *gemm,
                            void *stream_comm, void *stream_compute, void *parent,
                            int parent_is_set, int join)
{
    if (!fused && !gemm) return TW_ERR_NULL;
    if (fused) TW_TRY(validate_fused(*fused));
    if (gemm) TW_TRY(validate_gemm(*gemm));
    if (fused && gemm && stream_comm == stream_compute) return TW_ERR_SPLIT;

    hipStream_t sc = static_cast<hipStream_t>(stream_comm);
    hipStream_t sx = static_cast<hipStream_t>(stream_compute);
    hipStream_t sp = static_cast<hipStream_t>(parent);
    if (parent_is_set) {
        hipEvent_t fork;
        TW_TRY(borrow_event(&fork));
        TW_HIP(hipEventRecord(fork, sp));
        if (fused && sc != sp) TW_HIP(hipStreamWaitEvent(sc, fork, 0));
        if (gemm && sx != sp) TW_HIP(hipStreamWaitEvent(sx, fork, 0));
    }
    // Budgeted mode: the few workgroups of the fused kernel go first, they take
    // their compute units and the GEMM's workgroups are placed on what is left.
    // Shared mode: the GEMM goes first and takes one slot on every compute unit;
    // the small fused workgroups then fill in beside it (launched first, they
    // would pile up five to a compute unit and keep the GEMM out until done).
    const bool gemm_first = fused && gemm && fused->cu_budget == TW_CU_SHARED;
    if (gemm && gemm_first) TW_TRY(launch_gemm(*gemm, sx, fused != nullptr));
    if (fused && fused->N > 0) TW_TRY(launch_fused(*fused, 0, fused->N, nullptr, 0, sc));
    if (gemm && !gemm_first) TW_TRY(launch_gemm(*gemm, sx, fused != nullptr));
    if (parent_is_set && join) {
        if (fused && sc != sp) TW_TRY(stream_wait_stream(sp, sc));
        if (gemm && sx != sp) TW_TRY(stream_wait_stream(sp, sx));
    }
    return TW_OK;
}

// ---- one woven layer boundary: G1 -> F -> G2 over two token splits ----

static tw_gemm_args rows_of(const tw_gemm_args &g, int64_t r0, int64_t r1)
{
    tw_gemm_args s = g;
    s.A = static_cast<const char *>(g.A) + r0 * g.K * 2;
    s.C = static_cast<char *>(g.C) + r0 * g.N * 2;
    s.M = r1 - r0;
    return s;
}

// Which schedule a split layer boundary takes. The ordered schedule never lets
// two GEMMs compete but puts three cross-stream waits (15-20 us each) on the
// critical path; the chains put none there. Measured on MI355X in shared mode on
// the two boundaries of a 70B-class layer (K1 = 1024, N2 = 3584 and K1 = 3584,
// N2 = 1280; H = 8192, P = 8) for T = 256 ... 16384: the chains are level to 13 %
// faster at every token count on the first and up to 8192 tokens on the second,
// and 2.5 % slower only at 16384 tokens on the second (a narrow G2 that the
// chains let compete with a long G1). A fused kernel confined to a CU budget
// keeps the ordered schedule: the GEMMs' budget leaves its compute units free
// only while no two GEMMs overlap.
static bool takes_chains(const tw_layer_args &layer, int cus)
{
    if (layer.schedule != TW_WEAVE_AUTO) return layer.schedule == TW_WEAVE_CHAINS;
    const tw_fused_args &f = layer.fused;
    return !(f.cu_budget > 0 && f.cu_budget < cus);
}

int tw_weave_schedule(int64_t T, int64_t K1, int64_t H, int P, int64_t N2, int fused_cu_budget, int schedule,
                      int cus)
{
    if (T < 0 || K1 < 0 || H < 1 || P < 1 || N2 < 0 || cus < 1) return -1;
    if (schedule != TW_WEAVE_AUTO && schedule != TW_WEAVE_ORDERED && schedule != TW_WEAVE_CHAINS) return -1;
    tw_layer_args layer = {};
    layer.schedule = schedule;
    layer.fused.N = T;
    layer.fused.H = H;
    layer.fused.P = P;
    layer.fused.cu_budget = fused_cu_budget;
    return takes_chains(layer, cus) ? TW_WEAVE_CHAINS : TW_WEAVE_ORDERED;
}

// Checks shared by every way of launching a layer boundary; on TW_OK with T > 0
// *g1 and *g2 are the two GEMMs over all T rows.
static tw_status validate_layer(const tw_layer_args *layer, void *stream_compute, void *stream_comm, tw_gemm_args *g1,
                                tw_gemm_args *g2)
{
    if (!layer) return TW_ERR_NULL;
    const tw_fused_args &f = layer->fused;
    TW_TRY(validate_fused(f));
    const int64_t T = f.N;
    if (stream_compute == stream_comm) return TW_ERR_SPLIT;
    if (layer->K1 < 0 || layer->N2 < 0) return TW_ERR_SHAPE;
    if (layer->schedule != TW_WEAVE_AUTO && layer->schedule != TW_WEAVE_ORDERED &&
        layer->schedule != TW_WEAVE_CHAINS)
        return TW_ERR_UNSUPPORTED;
    if (T == 0) return TW_OK;
    *g1 = {layer->X1, layer->W1, const_cast<void *>(f.partials[0]), T, f.H, layer->K1, TW_B_NK, layer->gemm_cu_budget};
    *g2 = {f.out, layer->W2, layer->Y, T, layer->N2, f.H, TW_B_NK, layer->gemm_cu_budget};
    TW_TRY(validate_gemm(*g1));
    TW_TRY(validate_gemm(*g2));
    // Y is written while the other split's fused kernel may still be running:
    // it must not touch anything that kernel reads or writes, nor G1's operands
    const uint64_t y_bytes = uint64_t(T) * uint64_t(layer->N2) * 2, t_bytes = uint64_t(T) * uint64_t(f.H) * 2;
    if (ranges_overlap(layer->Y, y_bytes, f.residual, t_bytes) ||
        ranges_overlap(layer->Y, y_bytes, f.residual_out, t_bytes) ||
        ranges_overlap(layer->Y, y_bytes, f.weight, uint64_t(f.H) * 2) ||
        ranges_overlap(layer->Y, y_bytes, layer->X1, uint64_t(T) * uint64_t(layer->K1) * 2) ||
        ranges_overlap(layer->Y, y_bytes, layer->W1, uint64_t(f.H) * uint64_t(layer->K1) * 2))
        return TW_ERR_ALIAS;
    for (int p = 0; p < f.P; ++p)
        if (ranges_overlap(layer->Y, y_bytes, f.partials[p], t_bytes)) return TW_ERR_ALIAS;
    // G1 writes partials[0] before the fused kernel runs: it must not be one of
    // G1's own inputs (checked above) nor the weights of either GEMM
    const uint64_t w2_bytes = uint64_t(layer->N2) * uint64_t(f.H) * 2;
    if (ranges_overlap(f.partials[0], t_bytes, layer->W2, w2_bytes)) return TW_ERR_ALIAS;
    // one split's fused kernel writes out / residual_out while the other
    // split's G1 reads X1 and W1 and the first split's G2 reads W2
    const void *f_outs[2] = {f.out, f.residual_out};
    for (const void *o : f_outs)
        if (ranges_overlap(o, t_bytes, layer->X1, uint64_t(T) * uint64_t(layer->K1) * 2) ||
            ranges_overlap(o, t_bytes, layer->W1, uint64_t(f.H) * uint64_t(layer->K1) * 2) ||
            ranges_overlap(o, t_bytes, layer->W2, w2_bytes))
            return TW_ERR_ALIAS;
    return TW_OK;
}

// Rows [lo, mid) and [mid, hi) of the boundary as one woven pair of splits, the
// first on sx, the second on sc (mid == hi: rows [lo, hi) as one chain on sx).
static tw_status weave_pair(const tw_fused_args &f, const tw_gemm_args &g1, const tw_gemm_args &g2, bool chains,
                            bool stagger, int64_t lo, int64_t mid, int64_t hi, hipStream_t sx, hipStream_t sc)
{
    if (mid >= hi) {
        TW_TRY(launch_gemm(rows_of(g1, lo, hi), sx, false));
        TW_TRY(launch_fused(f, lo, hi, nullptr, 0, sx));
        return launch_gemm(rows_of(g2, lo, hi), sx, false);
    }
    if (chains) {
        // one chain per split. Where both chains start from the same point (the first
        // pair of a call that forks from a parent) the second is held back until the
        // first split's G1 is done, so that the two run out of step: one's fused kernel
        // beside the other's GEMM. Chains that are already running (a call without a
        // parent: the next boundary of a train; later pairs of a list of cuts) are out
        // of step as they are, and holding the second back at every boundary cost 3-4 %
        // of a boundary on trains of eight.
        // The first GEMM of the first chain and the last of the second have no fused
        // kernel of this pair beside them (the one runs before any, the other after
        // both): they take the tile shape of a GEMM launched on its own.
        TW_TRY(launch_gemm(rows_of(g1, lo, mid), sx, false));
        if (stagger) {
            hipEvent_t g1a_done;
            TW_TRY(borrow_event(&g1a_done));
            TW_HIP(hipEventRecord(g1a_done, sx));
            TW_HIP(hipStreamWaitEvent(sc, g1a_done, 0));
        }
        TW_TRY(launch_fused(f, lo, mid, nullptr, 0, sx));
        TW_TRY(launch_gemm(rows_of(g2, lo, mid), sx, true));
        TW_TRY(launch_gemm(rows_of(g1, mid, hi), sc, true));
        TW_TRY(launch_fused(f, mid, hi, nullptr, 0, sc));
        return launch_gemm(rows_of(g2, mid, hi), sc, false);
    }
    // compute stream: both G1 first, so the second split's projection is what
    // runs next to the first split's fused kernel
    const int64_t cuts[3] = {lo, mid, hi};
    hipEvent_t g1_done[2], f_done[2];
    for (int s = 0; s < 2; ++s) {
        TW_TRY(launch_gemm(rows_of(g1, cuts[s], cuts[s + 1]), sx, true));
        TW_TRY(borrow_event(&g1_done[s]));
        TW_HIP(hipEventRecord(g1_done[s], sx));
    }
    for (int s = 0; s < 2; ++s) {
        TW_HIP(hipStreamWaitEvent(sc, g1_done[s], 0));
        TW_TRY(launch_fused(f, cuts[s], cuts[s + 1], nullptr, 0, sc));
        TW_TRY(borrow_event(&f_done[s]));
        TW_HIP(hipEventRecord(f_done[s], sc));
        TW_HIP(hipStreamWaitEvent(sx, f_done[s], 0));
        TW_TRY(launch_gemm(rows_of(g2, cuts[s], cuts[s + 1]), sx, true));
    }
    return TW_OK;
}

tw_status tw_weave_layer_cuts(const tw_layer_args *layer, const int64_t *cuts, int n_cuts, void *stream_compute,
                              void *stream_comm, void *parent, int parent_is_set, int join)
{
    tw_gemm_args g1, g2;
    TW_TRY(validate_layer(layer, stream_compute, stream_comm, &g1, &g2));
    const tw_fused_args &f = layer->fused;
    const int64_t T = f.N;
    if (n_cuts < 0 || n_cuts > TW_MAX_CUTS) return TW_ERR_SPLIT;
    if (n_cuts > 0 && !cuts) return TW_ERR_NULL;
    for (int i = 0; i < n_cuts; ++i)
        if (cuts[i] <= (i ? cuts[i - 1] : 0) || cuts[i] >= T) return TW_ERR_SPLIT;
    if (T == 0) return TW_OK;

    hipStream_t sx = static_cast<hipStream_t>(stream_compute), sc = static_cast<hipStream_t>(stream_comm);
    hipStream_t sp = static_cast<hipStream_t>(parent);
    if (n_cuts == 0) {
        // nothing to weave: the chain runs on the compute stream, with no events. A
        // fused step that was to share the compute units has them to itself here and
        // takes whichever kernel the whole device runs fastest (same bits).
        if (parent_is_set && sx != sp) TW_TRY(stream_wait_stream(sx, sp));
        TW_TRY(launch_gemm(g1, sx));
        tw_fused_args alone = f;
        if (alone.cu_budget == TW_CU_SHARED) alone.cu_budget = 0;
        TW_TRY(launch_fused(alone, 0, T, nullptr, 0, sx));
        TW_TRY(launch_gemm(g2, sx));
        if (parent_is_set && join && sx != sp) TW_TRY(stream_wait_stream(sp, sx));
        return TW_OK;
    }
    if (parent_is_set) {
        hipEvent_t fork;
        TW_TRY(borrow_event(&fork));
        TW_HIP(hipEventRecord(fork, sp));
        if (sx != sp) TW_HIP(hipStreamWaitEvent(sx, fork, 0));
        if (sc != sp) TW_HIP(hipStreamWaitEvent(sc, fork, 0));
    }
    int cus = 0;
    TW_TRY(current_cu_count(&cus));
    const bool chains = takes_chains(*layer, cus);
    // The splits are woven two at a time, pair after pair on the same two streams:
    // stream order alone keeps a pair's first chain behind the previous pair's first
    // chain and its second behind the previous second, so no event links the pairs
    // and the tail of one pair overlaps the head of the next.
    const int n_splits = n_cuts + 1;
    auto row = [&](int i) { return i == 0 ? int64_t(0) : i == n_splits ? T : cuts[i - 1]; };
    for (int s = 0; s < n_splits; s += 2) {
        const int64_t lo = row(s), mid = row(s + 1), hi = s + 2 <= n_splits ? row(s + 2) : mid;
        TW_TRY(weave_pair(f, g1, g2, chains, parent_is_set && s == 0, lo, mid, hi, sx, sc));
    }
    if (parent_is_set && join) {
        if (sx != sp) TW_TRY(stream_wait_stream(sp, sx));
        if (sc != sp) TW_TRY(stream_wait_stream(sp, sc));
    }
    return TW_OK;
}

tw_status tw_weave_train(const tw_layer_args *layers, int n_layers, int64_t split_row, void *stream_compute,
                         void *stream_comm, void *parent, int parent_is_set, int join)
{
    if (n_layers < 0 || n_layers > TW_MAX_TRAIN) return TW_ERR_SHAPE;
    if (n_layers == 0) return TW_OK;
    if (!layers) return TW_ERR_NULL;
    // everything is checked before anything is launched
    const int64_t T = layers[0].fused.N;
    for (int i = 0; i < n_layers; ++i) {
        tw_gemm_args g1, g2;
        TW_TRY(validate_layer(&layers[i], stream_compute, stream_comm, &g1, &g2));
        if (layers[i].fused.N != T) return TW_ERR_SHAPE;
    }
    if (split_row < 0 || split_row > T) return TW_ERR_SPLIT;
    const bool whole = split_row == 0 || split_row == T;
    for (int i = 0; i < n_layers; ++i)
        TW_TRY(tw_weave_layer_cuts(&layers[i], &split_row, whole ? 0 : 1, stream_compute, stream_comm, parent,
                                   (i == 0 && parent_is_set) ? 1 : 0, 0));
    if (parent_is_set && join && T > 0) {
        hipStream_t sx = static_cast<hipStream_t>(stream_compute), sc = static_cast<hipStream_t>(stream_comm);
        hipStream_t sp = static_cast<hipStream_t>(parent);
        if (sx != sp) TW_TRY(stream_wait_stream(sp, sx));
        if (!whole && sc != sp) TW_TRY(stream_wait_stream(sp, sc));
    }
    return TW_OK;
}

tw_status tw_weave_layer(const tw_layer_args *layer, int64_t split_row, void *stream_compute,
                         void *stream_comm, void *parent, int parent_is_set, int join)
{
    if (!layer) return TW_ERR_NULL;
    TW_TRY(validate_fused(layer->fused));
    const int64_t T = layer->fused.N;
    if (split_row < 0 || split_row > T) return TW_ERR_SPLIT;
    const bool whole = split_row == 0 || split_row == T;
    return tw_weave_layer_cuts(layer, &split_row, whole ? 0 : 1, stream_compute, stream_comm, parent, parent_is_set,
                               join);
}

int tw_should_split(int64_t num_tokens, int64_t threshold)
{
    if (threshold <= 0) threshold = TW_DEFAULT_SPLIT_THRESHOLD;
    return num_tokens >= threshold ? 1 : 0;
}

int64_t tw_split_threshold(int64_t K1, int64_t H, int P, int64_t N2, int cus)
{
    if (K1 < 1 || H < 1 || P < 1 || N2 < 1 || cus < 1) return -1;
    // (1) the GEMM after the fused step must outlast it, or the second split's
    // fused kernel has nothing to hide behind and the last GEMM waits for it:
    // per token 2 H N2 flop at 1 PFLOP/s against 2 H (P + 3) bytes at 5 TB/s
    if (N2 < 200 * int64_t(P + 3)) return TW_NEVER_SPLIT;
    // (2) the fused kernel of the whole batch must be worth hiding: the waits,
    // the contention of co-resident kernels and the smaller GEMM tiles of a split
    // schedule cost about what 290 us of fused work (at the whole device's
    // ~5 TB/s) gain when overlapped
    const double row_bytes = 2.0 * double(H) * double(P + 3);
    const int64_t t_gain = static_cast<int64_t>(290.0 * 5.0e6 / row_bytes) + 1;
    // (3) half a batch must still give the narrower GEMM tiles for half of the
    // compute units, or its workgroups leave most of the device idle
    const int64_t n_min = H < N2 ? H : N2;
    const int64_t col_tiles = (n_min + kGemmTileN - 1) / kGemmTileN;
    const int64_t row_tiles = ((cus + 1) / 2 + col_tiles - 1) / col_tiles;
    const int64_t t_fill = 2 * row_tiles * kGemmTileM;
    const int64_t t = t_gain > t_fill ? t_gain : t_fill;
    return (t + kGemmTileM - 1) / kGemmTileM * kGemmTileM;
}

int64_t tw_policy_split_row(int64_t T, int64_t K1, int64_t H, int P, int64_t N2, int cus, int64_t threshold,
                            int64_t multiple)
{
    if (T < 0 || K1 < 1 || H < 1 || P < 1 || N2 < 1 || cus < 1) return -1;
    if (multiple <= 0) multiple = 64;
    const int64_t widths[2] = {H, N2}, depths[2] = {K1, H};
    if (threshold > 0) {  // the caller's threshold and nothing else
        if (T < threshold) return T;
        const int64_t k = tw_smart_split_point(T, multiple, widths, depths, 2, cus, nullptr, nullptr);
        return k < 0 ? T : k;
    }
    const int64_t thr = tw_split_threshold(K1, H, P, N2, cus);
    if (thr < 0 || thr == TW_NEVER_SPLIT || T <= thr / 2) return T;
    int64_t cost_split = 0, cost_unsplit = 0;
    const int64_t k = tw_smart_split_point(T, multiple, widths, depths, 2, cus, &cost_split, &cost_unsplit);
    if (k < 0 || k >= T) return T;
    // Above half the threshold, a batch is split when that costs no GEMM waves
    // (Section 4.1.1): whether a split wins there is decided by how the row tiles of
    // the halves and of the whole batch fall on the compute units.
    if (T < thr && cost_split > cost_unsplit) return T;
    return k;
}

tw_status tw_weave_layer_auto(const tw_layer_args *layer, int64_t threshold, int64_t multiple, void *stream_compute,
                              void *stream_comm, void *parent, int parent_is_set, int join, int64_t *split_row)
{
    if (!layer) return TW_ERR_NULL;
    const tw_fused_args &f = layer->fused;
    TW_TRY(validate_fused(f));
    if (layer->K1 < 0 || layer->N2 < 0) return TW_ERR_SHAPE;
    const int64_t T = f.N;
    int64_t k = T;  // unsplit unless the policy says otherwise
    if (T > 0 && layer->K1 > 0 && layer->N2 > 0) {
        int cus = 0;
        TW_TRY(current_cu_count(&cus));
        k = tw_policy_split_row(T, layer->K1, f.H, f.P, layer->N2, resolve_budget(layer->gemm_cu_budget, cus),
                                threshold, multiple);
        if (k < 0) k = T;
    }
    if (split_row) *split_row = k;
    return tw_weave_layer(layer, k, stream_compute, stream_comm, parent, parent_is_set, join);
}

tw_status tw_weave_tune(const tw_layer_args *layer, int64_t multiple, const int64_t *offsets, int n_offsets, int reps,
                        void *stream_compute, void *stream_comm, int64_t *best_row, float *us)
{
    if (!layer || !best_row || !us || (n_offsets > 0 && !offsets)) return TW_ERR_NULL;
    if (reps < 1 || reps > 64 || n_offsets < 0 || n_offsets > 16) return TW_ERR_SHAPE;
    const tw_fused_args &f = layer->fused;
    TW_TRY(validate_fused(f));
    if (layer->K1 < 0 || layer->N2 < 0) return TW_ERR_SHAPE;
    if (multiple <= 0) multiple = 64;
    const int64_t T = f.N;
    const int n_cand = 2 + n_offsets;
    int64_t rows[18];
    rows[0] = T;  // unsplit
    for (int i = 1; i < n_cand; ++i) rows[i] = -1;
    if (T > 0 && layer->K1 > 0 && layer->N2 > 0) {
        int cus = 0;
        TW_TRY(current_cu_count(&cus));
        const int64_t widths[2] = {f.H, layer->N2}, depths[2] = {layer->K1, f.H};
        rows[1] = tw_smart_split_point(T, multiple, widths, depths, 2, resolve_budget(layer->gemm_cu_budget, cus),
                                       nullptr, nullptr);
        const int64_t base = tw_split_point(T, multiple);
        for (int i = 0; i < n_offsets; ++i) rows[2 + i] = base + offsets[i];
    }
    for (int i = 1; i < n_cand; ++i) {
        if (rows[i] <= 0 || rows[i] >= T) rows[i] = -1;
        for (int j = 0; j < i && rows[i] > 0; ++j)
            if (rows[j] == rows[i]) rows[i] = -1;
    }
    hipStream_t sx = static_cast<hipStream_t>(stream_compute), sc = static_cast<hipStream_t>(stream_comm);
    struct Events {  // destroyed on every way out
        hipEvent_t begin = nullptr, end = nullptr;
        ~Events()
        {
            if (begin) (void)hipEventDestroy(begin);
            if (end) (void)hipEventDestroy(end);
        }
    } ev;
    TW_HIP(hipEventCreate(&ev.begin));
    TW_HIP(hipEventCreate(&ev.end));
    float samples[18][64];
    for (int r = -1; r < reps; ++r) {  // round -1 is the warm-up
        for (int c0 = 0; c0 < n_cand; ++c0) {
            const int c = (c0 + (r < 0 ? 0 : r)) % n_cand;
            if (rows[c] < 0) continue;
            TW_HIP(hipStreamSynchronize(sx));
            TW_HIP(hipStreamSynchronize(sc));
            TW_HIP(hipEventRecord(ev.begin, sx));
            TW_TRY(tw_weave_layer(layer, rows[c] == T ? 0 : rows[c], stream_compute, stream_comm, stream_compute, 1, 1));
            TW_HIP(hipEventRecord(ev.end, sx));
            TW_HIP(hipEventSynchronize(ev.end));
            float ms = 0.0f;
            TW_HIP(hipEventElapsedTime(&ms, ev.begin, ev.end));
            if (r >= 0) samples[c][r] = ms * 1000.0f;
        }
    }
    TW_HIP(hipStreamSynchronize(sc));
    int best = 0;
    for (int c = 0; c < n_cand; ++c) {
        if (rows[c] < 0) {
            us[c] = -1.0f;
            continue;
        }
        std::sort(samples[c], samples[c] + reps);
        us[c] = reps % 2 ? samples[c][reps / 2] : 0.5f * (samples[c][reps / 2 - 1] + samples[c][reps / 2]);
        if (us[c] < us[best]) best = c;
    }
    *best_row = rows[best];
    return TW_OK;
}

void tw_gemm_tile_shape(int *tile_m, int *tile_n)
{
    if (tile_m) *tile_m = kGemmTileM;
    if (tile_n) *tile_n = kGemmTileN;
}

static int64_t gemm_waves(int64_t rows, int64_t n_out, int64_t cus)
{
    if (rows <= 0) return 0;
    const int64_t wgs = ((rows + kGemmTileM - 1) / kGemmTileM) * ((n_out + kGemmTileN - 1) / kGemmTileN);
    return (wgs + cus - 1) / cus;
}

int64_t tw_smart_split_point(int64_t T, int64_t multiple, const int64_t *gemm_n_out, const int64_t *gemm_k,
                             int n_gemms, int cus, int64_t *cost_split, int64_t *cost_unsplit)
{
    if (T < 0 || n_gemms < 1 || cus < 1 || !gemm_n_out) return -1;
    for (int i = 0; i < n_gemms; ++i)
        if (gemm_n_out[i] < 1 || (gemm_k && gemm_k[i] < 1)) return -1;
    if (multiple <= 0) multiple = 1;
    auto cost_of = [&](int64_t rows) {
        int64_t c = 0;
        for (int i = 0; i < n_gemms; ++i) c += gemm_waves(rows, gemm_n_out[i], cus) * (gemm_k ? gemm_k[i] : 1);
        return c;
    };
    const int64_t unsplit = cost_of(T);
    if (cost_unsplit) *cost_unsplit = unsplit;
    if (cost_split) *cost_split = unsplit;
    const int64_t base = tw_split_point(T, multiple);
    if (base >= T) return T;
    // among cuts of equal cost, the one whose splits pad the fewest GEMM row tiles
    // (a cut inside a tile makes both splits work on that tile's rows)
    auto row_tiles = [](int64_t rows) { return (rows + kGemmTileM - 1) / kGemmTileM; };
    int64_t best_k = T, best_cost = INT64_MAX, best_tiles = INT64_MAX;
    for (int64_t k = base; k < T && k - base <= 512; k += multiple) {
        const int64_t cost = cost_of(k) + cost_of(T - k);
        const int64_t tiles = row_tiles(k) + row_tiles(T - k);
        if (cost < best_cost || (cost == best_cost && tiles < best_tiles)) {
            best_cost = cost;
            best_tiles = tiles;
            best_k = k;
        }
    }
    if (cost_split) *cost_split = best_cost;
    return best_k;
}

}  // extern "C"
