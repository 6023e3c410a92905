// Host side of the CTC library: argument validation, workspace layout, the per-call plan
// (which utterances run, in which order, how wide the lattice workgroups are) and the
// enqueueing of the kernels (upload, softmax, lattice, then gradient or backtrace).  No device memory is allocated here or anywhere else in
// the library (Section 4.3: allocation is kept off the training step; the caller hands in
// one workspace and this file carves it).

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

#include "ctc_internal.h"

// Workspace of ctc_loss_and_grad_device_static: device memory that belongs to the library's code
// object, one copy per GPU, so that the entry point needs no allocation by anybody.  In host code
// this name is only a handle for hipGetSymbolAddress; the kernels get the address it returns.
static __device__ __align__(256) unsigned char scratch[CTC_STATIC_WORKSPACE_BYTES];

namespace ctc {

namespace {

thread_local int g_last_hip_error = 0;
std::atomic<int> g_poll_budget{kDefaultPollBudget};
// Gradient rows inside the lattice launch where it has idle compute units: 0 = never; otherwise the
// percentage of the launch's expected duration up to which an utterance's chains must end for its rows
// to be written by the launch's workers (the rest are written by the gradient launch that follows).
std::atomic<int> g_overlap{kWorkerSharePercent};
std::atomic<int> g_sequential_chains{0};

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

inline bool record(int err)
{
    if (err != 0) g_last_hip_error = err;
    return err == 0;
}

}  // namespace

namespace {
// Compute units of the current device (asked once per device).
int compute_units()
{
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Region offsets from the batch totals (label symbols, label emissions, frames, lattice pairs).
void carve(int T, int B, int64_t sumL, int64_t emit, int64_t frames, int64_t ab, Layout* lay)
{
    Layout l;
    l.sumL = sumL;
    l.emit_floats = emit;
    l.frames = frames;
    l.ab_doubles = ab;
    size_t off = 0;
    l.meta = off;   off += static_cast<size_t>(B) * sizeof(Utt);            // 64 B each: stays 8-byte aligned
    l.order = off;  off += static_cast<size_t>(B) * 2 * sizeof(int32_t);
    l.labels = off; off += static_cast<size_t>(sumL) * sizeof(int32_t);
    l.tasks = off;  off += (static_cast<size_t>(B) * 6 + 1 + kXcds + 1) * sizeof(int32_t);
    l.labels8 = off; off += (static_cast<size_t>(sumL) + 3) / 4 * 4;
    l.upload_bytes = off;
    off = align_up(off);
    l.links = off;  off = align_up(off + static_cast<size_t>(sumL) * sizeof(int32_t));
    l.logp = off;   off = align_up(off + static_cast<size_t>(B) * sizeof(double));
    l.sink = off;   off = align_up(off + static_cast<size_t>(B) * 2 * kSinkWaves * kSinkBytes);
    l.chain_err = off; off = align_up(off + static_cast<size_t>(B) * sizeof(int32_t));
    l.done = off;   off = align_up(off + static_cast<size_t>(B) * kDoneStride * sizeof(int32_t));
    l.domain = off; off = align_up(off + static_cast<size_t>(B) * 2 * sizeof(int32_t));
    l.row_flags = off;
    off = align_up(off + static_cast<size_t>(B) * ((T + kFlagFrames - 1) / kFlagFrames) * sizeof(int32_t));
    l.status = off; off = align_up(off + static_cast<size_t>(B) * sizeof(int32_t));
    l.where = off;  off = align_up(off + static_cast<size_t>(B) * 2 * sizeof(int32_t));
    l.leftover = off; off = align_up(off + static_cast<size_t>(B) * sizeof(int32_t));
    l.lse = off;    off = align_up(off + static_cast<size_t>(B) * T * sizeof(float));
    l.emit_blank = off;
    off = align_up(off + (static_cast<size_t>(frames) + 2 * kBlankSlack) * sizeof(float));
    l.emit_blank64 = off;
    off = align_up(off + (static_cast<size_t>(frames) + 2 * kBlankSlack) * sizeof(double));
    l.emit_label = off;
    off = align_up(off + (static_cast<size_t>(emit) + 2 * kLabelSlack) * sizeof(float));
    l.alpha = off;  off = align_up(off + static_cast<size_t>(ab) * sizeof(double));
    l.beta = off;   off = align_up(off + static_cast<size_t>(ab) * sizeof(double));
    l.total = off;
    *lay = l;
}
}  // namespace

const PlanTable& plan_table(int max_label, bool crowded, bool symbol_major)
{
    struct Entry { int max_label; bool crowded, symbol_major; PlanTable table; };
    static std::mutex mutex;
    static std::vector<Entry*> entries;
    std::lock_guard<std::mutex> lock(mutex);
    for (const Entry* e : entries)
        if (e->max_label >= max_label && e->crowded == crowded && e->symbol_major == symbol_major) return e->table;
    Entry* e = new Entry{max_label, crowded, symbol_major, {}};
    for (int L = 0; L <= max_label; ++L) {
        const WavePlan one = plan_waves(L, crowded), two = plan_waves2(L, crowded);
        e->table.one[L] = static_cast<uint8_t>((one.waves - 1) | ((one.halo / 8) << 4) |
                                               (two_pairs_per_lane(L, crowded, symbol_major) ? 128 : 0));
        e->table.two[L] = static_cast<uint8_t>((two.waves - 1) | ((two.halo / 4) << 4));
    }
    entries.push_back(e);
    return e->table;
}

ctc_status_t make_layout(int T, int B, int A, const int32_t* label_lengths,
                         const int32_t* input_lengths, ctc_dtype_t dtype, Layout* lay)
{
    if (!label_lengths || !input_lengths || !lay) return CTC_STATUS_INVALID_VALUE;
    if (T < 1 || B < 1 || A < 1) return CTC_STATUS_INVALID_VALUE;
    if (dtype != CTC_DTYPE_F32 && dtype != CTC_DTYPE_BF16) return CTC_STATUS_INVALID_VALUE;
    int64_t sumL = 0, emit = 0, ab = 0, frames = 0;
    bool too_long = false;
    for (int b = 0; b < B; ++b) {
        const int64_t L = label_lengths[b], Tb = input_lengths[b];
        if (L < 0 || Tb < 0 || Tb > T) return CTC_STATUS_INVALID_VALUE;
        if (L > CTC_MAX_LABEL_LENGTH) too_long = true;
        sumL += L;
        emit += Tb * (A <= kDirectMaxA ? A : L);
        frames += Tb;
        // per-utterance byte offsets inside the kernels are 32-bit
        if (Tb * lattice_pitch(L) * 8 > INT32_MAX) too_long = true;
        ab += Tb * lattice_pitch(L);
    }
    if (too_long) return CTC_STATUS_UNSUPPORTED;
    if (sumL > INT32_MAX || frames > INT32_MAX) return CTC_STATUS_UNSUPPORTED;
    if (B > kMaxBatch) return CTC_STATUS_UNSUPPORTED;
    carve(T, B, sumL, emit, frames, ab, lay);
    return CTC_STATUS_SUCCESS;
}

// Layout for the device-metadata entry point: every utterance gets the room of the largest one
// the caller allows (T frames, max_label symbols), so that offsets need no lengths.
ctc_status_t make_layout_bounds(int T, int B, int A, int max_label, ctc_dtype_t dtype, Layout* lay)
{
    if (!lay || T < 1 || B < 1 || A < 1 || max_label < 0) return CTC_STATUS_INVALID_VALUE;
    if (dtype != CTC_DTYPE_F32 && dtype != CTC_DTYPE_BF16) return CTC_STATUS_INVALID_VALUE;
    if (max_label > CTC_MAX_LABEL_LENGTH || B > kMaxDeviceMetaB) return CTC_STATUS_UNSUPPORTED;
    const int64_t Tl = T, Bl = B, Ll = max_label;
    if (Tl * lattice_pitch(Ll) * 8 > INT32_MAX || Bl * Ll > INT32_MAX || Bl * Tl > INT32_MAX) return CTC_STATUS_UNSUPPORTED;
    carve(T, B, Bl * Ll, Bl * Tl * (A <= kDirectMaxA ? A : Ll), Bl * Tl, Bl * Tl * lattice_pitch(Ll), lay);
    return CTC_STATUS_SUCCESS;
}

namespace {

// Pinned host buffers for the per-call metadata image.  The upload kernel reads the image
// straight from host memory, so a slot may be rewritten only after that kernel has run: the
// launch that follows it on the stream stores the slot's generation number into a pinned flag
// word in front of the image, which the host checks before it reuses the slot (no event, so no
// marker packet sits between two kernels of a call).
//
// All slots of a device come from one allocation, made at the first call on that device
// (kInitialSlots slots of at least kMinSlotBytes each), so that no later call allocates -- the
// point of Section 4.3.  The host never waits for a slot: when every slot is still in flight
// (the caller has enqueued that many calls ahead of the GPU), or when a batch's image outgrows
// the slots, a further pool with twice the slots, or larger ones, is allocated and used from
// then on (earlier pools are left to drain and are kept, so their total is below the last
// pool's size); pools of one device stop growing at kMaxStagingBytes, and a call that finds
// every slot in flight then returns CTC_STATUS_NOT_READY at once.
constexpr int kInitialSlots = 8;
constexpr size_t kMinSlotBytes = size_t(256) << 10;
constexpr size_t kMaxStagingBytes = size_t(256) << 20;
constexpr size_t kFlagBytes = 64;            // the flag word sits in front of the image

struct StagingSlot {
    char* host = nullptr;                    // kFlagBytes of flag, then the image
    int generation = 0;                      // value the device stores once the image is free
    bool in_flight = false;
    int* flag() const { return reinterpret_cast<int*>(host); }
    char* image() const { return host + kFlagBytes; }
    // Has the device released the image?  (A plain read of pinned memory; never waits.)
    bool released() const { return *static_cast<volatile int*>(flag()) == generation; }
};

struct StagingPool {
    char* base = nullptr;
    size_t slot_bytes = 0;                   // of the image part of each slot
    std::vector<StagingSlot> slots;
    int next = 0;
};

struct DeviceStaging {
    int device = -1;
    size_t total_bytes = 0;
    std::vector<StagingPool*> pools;         // the last one serves new calls
    std::atomic<long> allocations{0};
};

std::mutex g_staging_mutex;
std::vector<DeviceStaging*> g_staging;

DeviceStaging* staging_of(int dev)
{
    for (DeviceStaging* d : g_staging)
        if (d->device == dev) return d;
    DeviceStaging* d = new DeviceStaging();
    d->device = dev;
    g_staging.push_back(d);
    return d;
}

// A new pool of `slots` slots of `slot_bytes` each.  nullptr: past the cap (status_out =
// NOT_READY) or the allocation failed (HIP_ERROR).
StagingPool* add_pool(DeviceStaging* d, int slots, size_t slot_bytes, ctc_status_t* status_out)
{
    const size_t stride = kFlagBytes + slot_bytes;
    const size_t bytes = stride * static_cast<size_t>(slots);
    if (d->total_bytes + bytes > kMaxStagingBytes) {
        *status_out = CTC_STATUS_NOT_READY;
        return nullptr;
    }
    void* mem = nullptr;
    if (!record(hipHostMalloc(&mem, bytes, hipHostMallocDefault))) {
        *status_out = CTC_STATUS_HIP_ERROR;
        return nullptr;
    }
    StagingPool* pool = new StagingPool();
    pool->base = static_cast<char*>(mem);
    pool->slot_bytes = slot_bytes;
    pool->slots.resize(static_cast<size_t>(slots));
    for (int i = 0; i < slots; ++i) {
        pool->slots[static_cast<size_t>(i)].host = pool->base + stride * static_cast<size_t>(i);
        *pool->slots[static_cast<size_t>(i)].flag() = 0;
    }
    d->pools.push_back(pool);
    d->total_bytes += bytes;
    d->allocations.fetch_add(1, std::memory_order_relaxed);
    return pool;
}

// Returns a free slot of at least `bytes`, or nullptr with the status to return.  Never waits.
// Caller holds g_staging_mutex.
StagingSlot* acquire_slot(size_t bytes, ctc_status_t* status_out)
{
    int dev = 0;
    if (!record(hipGetDevice(&dev))) {
        *status_out = CTC_STATUS_HIP_ERROR;
        return nullptr;
    }
    DeviceStaging* d = staging_of(dev);
    const size_t want = std::max(kMinSlotBytes, (2 * bytes + 65535) / 65536 * 65536 - kFlagBytes);
    StagingPool* pool = d->pools.empty() ? nullptr : d->pools.back();
    if (pool && bytes <= pool->slot_bytes) {
        const int n = static_cast<int>(pool->slots.size());
        for (int k = 0; k < n; ++k) {
            StagingSlot& slot = pool->slots[static_cast<size_t>((pool->next + k) % n)];
            if (slot.in_flight && slot.released()) slot.in_flight = false;
            if (!slot.in_flight) {
                pool->next = (pool->next + k + 1) % n;
                return &slot;
            }
        }
        // every slot is in flight: the caller runs that far ahead of the GPU
        pool = add_pool(d, 2 * n, pool->slot_bytes, status_out);
    } else if (pool) {
        pool = add_pool(d, static_cast<int>(pool->slots.size()), want, status_out);     // a larger image than any before
    } else {
        pool = add_pool(d, kInitialSlots, want, status_out);
    }
    if (!pool) return nullptr;
    pool->next = 1;
    return &pool->slots[0];
}

struct Call {
    Mode mode;
    const void* x;
    const int32_t* flat_labels;
    const int32_t* label_lengths;
    const int32_t* input_lengths;
    int T, B, A, blank;
    ctc_dtype_t dtype;
    float* costs;
    void* grads;             // kGrad only
    int32_t* alignment;      // kBest only
    void* ws;
    size_t ws_bytes;
    void* stream;
};

// Validates everything that can be validated on the host, builds the upload image
// (Utt records, run order, labels) and the launch parameters.
ctc_status_t prepare(const Call& c, const Layout& lay, Launch* out, char* image)
{
    if (lay.sumL > 0 && !c.flat_labels) return CTC_STATUS_INVALID_VALUE;
    if (reinterpret_cast<uintptr_t>(c.ws) % kAlign != 0) return CTC_STATUS_INVALID_VALUE;

    const size_t elem = (c.dtype == CTC_DTYPE_F32) ? 4 : 2;
    const size_t tensor_bytes = static_cast<size_t>(c.T) * c.B * c.A * elem;
    if (c.mode == Mode::kGrad) {
        const char* xa = static_cast<const char*>(c.x);
        const char* ga = static_cast<const char*>(c.grads);
        if (xa < ga + tensor_bytes && ga < xa + tensor_bytes) return CTC_STATUS_INVALID_VALUE;
        if (reinterpret_cast<uintptr_t>(c.grads) % elem) return CTC_STATUS_INVALID_VALUE;
    }
    if (reinterpret_cast<uintptr_t>(c.x) % elem) return CTC_STATUS_INVALID_VALUE;
    if (c.mode == Mode::kBest && reinterpret_cast<uintptr_t>(c.alignment) % sizeof(int32_t))
        return CTC_STATUS_INVALID_VALUE;

    Utt* meta = reinterpret_cast<Utt*>(image + lay.meta);
    int32_t* order = reinterpret_cast<int32_t*>(image + lay.order);
    int32_t* labels = reinterpret_cast<int32_t*>(image + lay.labels);
    uint8_t* labels8 = reinterpret_cast<uint8_t*>(image + lay.labels8);

    const bool symbol_major = emission_layout(c.A) == kEmitSymbolMajor;
    // Would the launch, planned for latency, put more than two wavefronts on every SIMD?
    int64_t latency_waves = 0;
    for (int b = 0; b < c.B; ++b) {
        const int L = c.label_lengths[b];
        latency_waves += two_pairs_per_lane(L, false, symbol_major) ? plan_waves2(L).waves : plan_waves(L).waves;
    }
    const bool crowded = latency_waves * (c.mode == Mode::kGrad ? 2 : 1) > kCrowdedWaves;

    int64_t lab_off = 0, e_off = 0, ab_off = 0, f_off = 0;
    int n_run = 0, max_waves = 1, max_frames = 0, max_label = 0;
    bool needs_barrier = false;
    for (int b = 0; b < c.B; ++b) {
        const int L = c.label_lengths[b], Tb = c.input_lengths[b];
        const int32_t* lab = c.flat_labels + lab_off;
        int repeats = 0;
        max_label = std::max(max_label, L);
        for (int i = 0; i < L; ++i) {
            const int32_t s = lab[i];
            if (s < 0 || s >= c.A || s == c.blank) return CTC_STATUS_INVALID_VALUE;
            if (i > 0 && s == lab[i - 1]) ++repeats;
            labels[lab_off + i] = s;
            labels8[lab_off + i] = static_cast<uint8_t>(s);          // (meaningful for alphabets up to 256 symbols)
        }
        // An alignment exists iff every symbol gets a frame and equal neighbours a blank between them.
        const bool runs = Tb > 0 && Tb >= L + repeats;
        Utt& m = meta[b];
        m.Tb = Tb;
        m.L = L;
        m.lab_off = static_cast<int32_t>(lab_off);
        m.flags = (runs ? kUttRuns : 0) | (two_pairs_per_lane(L, crowded, symbol_major) ? kUttTwoPairs : 0) |
                  ((Tb > kLinearMaxFrames || tight_fit(Tb, L, repeats)) ? kUttLogDomain : 0);
        m.f_off = static_cast<int32_t>(f_off);
        const WavePlan wp = plan_waves(L, crowded);
        m.waves = wp.waves;
        m.halo = wp.halo;
        const WavePlan wp2 = plan_waves2(L, crowded);
        m.waves2 = wp2.waves;
        m.halo2 = wp2.halo;
        m.poll_budget = g_poll_budget.load(std::memory_order_relaxed);
        m.e_off = e_off;
        m.ab_off = ab_off;
        m.e_direct = emission_layout(c.A);
        m.e_pitch = m.e_direct == kEmitSymbolMajor ? Tb : L;
        lab_off += L;
        e_off += static_cast<int64_t>(Tb) * (c.A <= kDirectMaxA ? c.A : L);
        f_off += Tb;
        ab_off += static_cast<int64_t>(Tb) * lattice_pitch(L);
        if (runs) {
            order[n_run++] = b;
            max_waves = std::max(max_waves, std::max(wp.waves, wp2.waves));
            needs_barrier = needs_barrier || wp.barrier;
            max_frames = std::max(max_frames, Tb);
        }
    }
    // The one-barrier-per-step kernel only has the log-domain recursion.
    if (needs_barrier)
        for (int b = 0; b < c.B; ++b) meta[b].flags |= kUttLogDomain;
    // Heaviest chains first, so the longest recursion does not start last; launches of more
    // chains than compute units are ordered for the SIMDs' loads (order_chains).
    auto chain_waves = [&](int b) {
        const bool two = (meta[b].flags & (kUttTwoPairs | kUttLogDomain)) == kUttTwoPairs && c.mode != Mode::kBest;
        return two ? meta[b].waves2 : meta[b].waves;
    };
    std::vector<int32_t> running(order, order + n_run);
    std::stable_sort(running.begin(), running.end(), [&](int a, int b) {
        return static_cast<int64_t>(meta[a].Tb) * chain_waves(a) > static_cast<int64_t>(meta[b].Tb) * chain_waves(b);
    });
    std::vector<int32_t> run_frames(static_cast<size_t>(n_run)), run_waves(static_cast<size_t>(n_run));
    for (int i = 0; i < n_run; ++i) {
        run_frames[i] = meta[running[i]].Tb;
        run_waves[i] = chain_waves(running[i]);
    }
    const int dirs = c.mode == Mode::kGrad ? 2 : 1;
    order_chains(running.data(), run_frames.data(), run_waves.data(), n_run, dirs, compute_units(), order);
    for (int i = n_run * dirs; i < 2 * c.B; ++i) order[i] = -1;

    // Gradient rows inside the lattice launch (kTaskRows), where the launch leaves at least a quarter
    // of the compute units without a chain.  (Narrow alphabets only: the workers run the gradient
    // of ctc_gradient_narrow_kernel.)
    const int n_cu = compute_units();
    int32_t* const task_die = reinterpret_cast<int32_t*>(image + lay.tasks);     // [kXcds + 1]
    int32_t* const task_prefix = task_die + kXcds + 1;                           // [2B + 1]
    int32_t* const task_info = task_prefix + 2 * c.B + 1;                        // [2B]
    int32_t* const task_first = task_info + 2 * c.B;                             // [2B]
    int n_entries = 0, n_tasks = 0;
    const bool sequential_chains = c.mode == Mode::kGrad && g_sequential_chains.load(std::memory_order_relaxed) != 0;
    const int share_percent = sequential_chains ? 0 : g_overlap.load(std::memory_order_relaxed);
    if (share_percent > 0 && c.mode == Mode::kGrad && c.A <= kDirectMaxA && !needs_barrier &&
        n_run > 0 && 2 * c.B <= kMaxTaskEntries && n_cu % kXcds == 0 && n_run * dirs + n_cu / 4 <= n_cu) {
        // The die of an utterance's chains: workgroup i runs on die i mod kXcds (order_chains puts an
        // utterance's two chains a multiple of kXcds entries apart).
        std::vector<int> die_of(static_cast<size_t>(c.B), 0);
        for (int i = 0; i < n_run * dirs; ++i)
            if ((order[i] & 1) == 0) die_of[static_cast<size_t>(order[i] >> 1)] = i % kXcds;
        // Chains end in the order of their frames, those that exchange between wavefronts a little later.
        auto ends_at = [&](int b) { return meta[b].Tb * (chain_waves(b) > 1 ? 5 : 4); };
        std::vector<int32_t> ending(running);
        std::stable_sort(ending.begin(), ending.end(), [&](int a, int b) { return ends_at(a) < ends_at(b); });
        const int last_end = ends_at(ending.back());
        const int blocks = (c.T + kTaskRows - 1) / kTaskRows;
        auto data_blocks = [&](int b) { return (meta[b].flags & kUttRuns) ? (meta[b].Tb + kTaskRows - 1) / kTaskRows : 0; };
        auto add = [&](int info, int first, int count) {
            if (count <= 0) return;
            task_prefix[n_entries] = n_tasks;
            task_info[n_entries] = info;
            task_first[n_entries] = first;
            ++n_entries;
            n_tasks += count;
        };
        for (int die = 0; die < kXcds; ++die) {
            task_die[die] = n_entries;
            // what needs no lattice first (shared out over the dies by utterance number) ...
            for (int b = die; b < c.B; b += kXcds) add(b | (kTaskRowsLog2 << kTaskRowsShift), data_blocks(b), blocks - data_blocks(b));
            // ... then the die's utterances as their chains end.  Those that end last are not worth waiting
            // for inside the launch: only the workers of the chains' own die can take them, a sixteenth of the
            // chip, and with every utterance given to the workers the launch was measured to end 15 us after
            // its last chain, against a gradient launch of 7 us for the last fifth: that launch takes them.
            for (int b : ending) {
                if (die_of[static_cast<size_t>(b)] != die) continue;
                if (static_cast<int64_t>(ends_at(b)) * 100 > static_cast<int64_t>(last_end) * share_percent) {
                    meta[b].flags |= kUttGradientLater;
                    continue;
                }
                add(b | kTaskWaits | (kTaskRowsLog2 << kTaskRowsShift), 0, data_blocks(b));
            }
        }
        task_die[kXcds] = n_entries;
        task_prefix[n_entries] = n_tasks;
    }

    if (c.ws_bytes < lay.total) return CTC_STATUS_WORKSPACE_TOO_SMALL;

    out->mode = c.mode;
    out->T = c.T; out->B = c.B; out->A = c.A; out->blank = c.blank;
    out->dtype = c.dtype;
    out->n_run = n_run;
    out->n_chains = n_run * dirs;
    out->max_waves = max_waves;
    out->max_frames = max_frames;
    out->max_label = max_label;
    out->needs_barrier = needs_barrier;
    out->x = c.x;
    out->grads = (c.mode == Mode::kGrad) ? c.grads : nullptr;
    out->alignment = (c.mode == Mode::kBest) ? c.alignment : nullptr;
    out->costs = c.costs;
    out->ws = static_cast<char*>(c.ws);
    out->labels = reinterpret_cast<const int32_t*>(static_cast<char*>(c.ws) + lay.labels);
    out->host_image = image;
    out->dev_label_lengths = nullptr;
    out->dev_input_lengths = nullptr;
    out->dev_status = nullptr;
    out->poll_budget = g_poll_budget.load(std::memory_order_relaxed);
    out->crowded = crowded;
    out->sequential_chains = sequential_chains;
    out->n_tasks = n_tasks;
    out->n_task_entries = n_entries;
    out->n_cu = n_cu;
    out->folded = c.A <= kDirectMaxA && c.B <= kNarrowMaxB && c.T < (1 << 29);
    out->lay = lay;
    return CTC_STATUS_SUCCESS;
}

// Cheap checks that need neither the layout nor a staging slot.
ctc_status_t precheck(const Call& c)
{
    if (!c.x || !c.label_lengths || !c.input_lengths || !c.costs || !c.ws) return CTC_STATUS_INVALID_VALUE;
    if (c.mode == Mode::kGrad && !c.grads) return CTC_STATUS_INVALID_VALUE;
    if (c.mode == Mode::kBest && !c.alignment) return CTC_STATUS_INVALID_VALUE;
    if (c.T < 1 || c.B < 1 || c.A < 1 || c.blank < 0 || c.blank >= c.A) return CTC_STATUS_INVALID_VALUE;
    return CTC_STATUS_SUCCESS;
}

// HIP events of a profiled call, destroyed however the call ends.
struct Events {
    hipEvent_t ev[CTC_NUM_KERNELS + 3] = {};
    bool create()
    {
        for (auto& e : ev)
            if (!record(hipEventCreate(&e))) return false;
        return true;
    }
    ~Events()
    {
        for (auto& e : ev)
            if (e) (void)hipEventDestroy(e);
    }
};

ctc_status_t run(const Call& c, float* kernel_ms)
{
    ctc_status_t st = precheck(c);
    if (st != CTC_STATUS_SUCCESS) return st;
    Layout lay;
    st = make_layout(c.T, c.B, c.A, c.label_lengths, c.input_lengths, c.dtype, &lay);
    if (st != CTC_STATUS_SUCCESS) return st;

    hipStream_t s = static_cast<hipStream_t>(c.stream);
    // Events 0..CTC_NUM_KERNELS bracket the launches; the last two are recorded back to back
    // and give what an interval with nothing in it reads, which is taken off every interval.
    Events events;
    hipEvent_t* const ev = events.ev;
    Launch p;
    {
        // The image is validated while it is written; on an error nothing has been enqueued and
        // the slot simply stays free.
        std::lock_guard<std::mutex> lock(g_staging_mutex);
        thread_local std::vector<char> scratch;          // validation without a device: see below
        static const bool have_device = [] {
            int ndev = 0;
            const bool ok = hipGetDeviceCount(&ndev) == hipSuccess && ndev > 0;
            if (!ok) (void)hipGetLastError();
            return ok;
        }();
        if (!have_device) {
            // No GPU (host-only checks of the argument validation): build the image in ordinary
            // memory so that every validation error is still reported, then stop.
            scratch.resize(lay.upload_bytes);
            st = prepare(c, lay, &p, scratch.data());
            return st != CTC_STATUS_SUCCESS ? st : CTC_STATUS_HIP_ERROR;
        }
        StagingSlot* const slot = acquire_slot(lay.upload_bytes, &st);
        if (!slot) return st;
        st = prepare(c, lay, &p, slot->image());
        if (st != CTC_STATUS_SUCCESS) return st;
        if (kernel_ms && !events.create()) return CTC_STATUS_HIP_ERROR;
        slot->generation += 1;
        p.host_flag = slot->flag();
        p.host_flag_value = slot->generation;
        // The upload launch's own time is not reported separately: it is a few microseconds and
        // overlaps the tail of whatever ran before on the stream.  (Narrow alphabets have none: their
        // softmax launch reads the image itself, and the lattice launch releases it.)
        if (!p.folded && !record(launch_setup(p, c.stream))) return CTC_STATUS_HIP_ERROR;
        // The image is released by the softmax launch, or by the lattice launch after it (narrow
        // alphabets).  Should the releasing launch fail to go out, nothing would ever release the slot
        // while a kernel may still be reading it: wait for the stream (an error path) and leave the
        // slot free.
        bool out = (!kernel_ms || record(hipEventRecord(ev[0], s))) && record(launch_softmax(p, c.stream)) &&
                   (!kernel_ms || record(hipEventRecord(ev[1], s)));
        if (out && p.folded)
            out = record(launch_lattice(p, c.stream)) && (!kernel_ms || record(hipEventRecord(ev[2], s)));
        if (!out) {
            (void)hipStreamSynchronize(s);
            return CTC_STATUS_HIP_ERROR;
        }
        slot->in_flight = true;
    }

    // Cost-only calls end with the lattice launch.
    // (Where the lattice launch carries the gradient rows itself, Launch::n_tasks, the gradient launch only
    // looks for utterances that the workers had to leave to it.)
    int (*const stages[CTC_NUM_KERNELS])(const Launch&, void*) = {
        launch_softmax, launch_lattice,
        c.mode == Mode::kGrad ? launch_gradient : (c.mode == Mode::kLoss ? nullptr : launch_backtrace)};
    for (int i = p.folded ? 2 : 1; i < CTC_NUM_KERNELS; ++i) {
        if (stages[i] && !record(stages[i](p, c.stream))) return CTC_STATUS_HIP_ERROR;
        if (kernel_ms && !record(hipEventRecord(ev[i + 1], s))) return CTC_STATUS_HIP_ERROR;
    }
    if (kernel_ms) {
        if (!record(hipEventRecord(ev[CTC_NUM_KERNELS + 1], s))) return CTC_STATUS_HIP_ERROR;
        if (!record(hipEventRecord(ev[CTC_NUM_KERNELS + 2], s))) return CTC_STATUS_HIP_ERROR;
        if (!record(hipStreamSynchronize(s))) return CTC_STATUS_HIP_ERROR;
        float empty = 0.0f;
        if (!record(hipEventElapsedTime(&empty, ev[CTC_NUM_KERNELS + 1], ev[CTC_NUM_KERNELS + 2])))
            return CTC_STATUS_HIP_ERROR;
        for (int i = 0; i < CTC_NUM_KERNELS; ++i) {
            if (!record(hipEventElapsedTime(&kernel_ms[i], ev[i], ev[i + 1]))) return CTC_STATUS_HIP_ERROR;
            kernel_ms[i] = stages[i] ? std::max(kernel_ms[i] - empty, 0.0f) : 0.0f;
        }
    }
    return CTC_STATUS_SUCCESS;
}

// Device-metadata call: nothing about the batch is known on the host beyond its bounds, so
// the launch shapes come from the bounds and a planning kernel fills in the rest.  Only kernel
// launches are enqueued (no copies, no host memory, no waiting), so the call may be recorded
// into a HIP graph.
ctc_status_t run_device(const void* x, const int32_t* labels, const int32_t* label_lengths,
                        const int32_t* input_lengths, int max_label, int T, int B, int A, int blank,
                        ctc_dtype_t dtype, float* costs, void* grads, int32_t* status, void* ws,
                        size_t ws_bytes, void* stream, float* kernel_ms = nullptr)
{
    if (!x || !label_lengths || !input_lengths || !costs || !status || !ws) return CTC_STATUS_INVALID_VALUE;
    if (max_label > 0 && !labels) return CTC_STATUS_INVALID_VALUE;
    if (T < 1 || B < 1 || A < 1 || blank < 0 || blank >= A) return CTC_STATUS_INVALID_VALUE;
    Layout lay;
    ctc_status_t st = make_layout_bounds(T, B, A, max_label, dtype, &lay);
    if (st != CTC_STATUS_SUCCESS) return st;
    if (reinterpret_cast<uintptr_t>(ws) % kAlign != 0) return CTC_STATUS_INVALID_VALUE;
    const size_t elem = (dtype == CTC_DTYPE_F32) ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(x) % elem || reinterpret_cast<uintptr_t>(grads) % elem)
        return CTC_STATUS_INVALID_VALUE;
    if (grads) {
        const size_t tensor_bytes = static_cast<size_t>(T) * B * A * elem;
        const char* xa = static_cast<const char*>(x);
        const char* ga = static_cast<const char*>(grads);
        if (xa < ga + tensor_bytes && ga < xa + tensor_bytes) return CTC_STATUS_INVALID_VALUE;
    }
    if (ws_bytes < lay.total) return CTC_STATUS_WORKSPACE_TOO_SMALL;

    Launch p;
    p.mode = grads ? Mode::kGrad : Mode::kLoss;
    p.T = T; p.B = B; p.A = A; p.blank = blank;
    p.dtype = dtype;
    p.n_run = B;                       // a lattice workgroup per utterance and direction; those that do not run leave at once
    p.n_chains = B * (grads ? 2 : 1);
    p.max_waves = 1;
    const bool symbol_major = emission_layout(A) == kEmitSymbolMajor;
    // Would the launch, planned for latency, put more than two wavefronts on every SIMD (prepare's question)?  The
    // labels' lengths are on the GPU; the answer here is for lengths spread evenly up to the bound.
    int64_t waves_up_to_bound = 0;
    for (int L = 0; L <= max_label; ++L)
        waves_up_to_bound += two_pairs_per_lane(L, false, symbol_major) ? plan_waves2(L).waves : plan_waves(L).waves;
    p.crowded = static_cast<int64_t>(B) * (grads ? 2 : 1) * waves_up_to_bound > static_cast<int64_t>(kCrowdedWaves) * (max_label + 1);
    for (int L = 0; L <= max_label; ++L)
        p.max_waves = std::max(p.max_waves, std::max(plan_waves(L, p.crowded).waves, plan_waves2(L, p.crowded).waves));
    p.max_frames = T;
    p.max_label = max_label;
    p.needs_barrier = plan_waves(max_label).barrier;
    p.x = x;
    p.grads = grads;
    p.alignment = nullptr;
    p.costs = costs;
    p.ws = static_cast<char*>(ws);
    p.labels = labels;
    p.host_image = nullptr;
    p.host_flag = nullptr;
    p.host_flag_value = 0;
    p.dev_label_lengths = label_lengths;
    p.dev_input_lengths = input_lengths;
    p.dev_status = status;
    p.poll_budget = g_poll_budget.load(std::memory_order_relaxed);
    p.n_tasks = 0;
    p.n_task_entries = 0;
    p.n_cu = 0;
    // Narrow alphabets: the softmax launch builds the records itself (no planning launch before it); every
    // utterance's setup workgroup weighs all B utterances for the run order, which is worth it up to here.
    p.folded = A <= kDirectMaxA && B <= kDeviceFoldMaxB && max_label > 0;
    // Gradient rows inside the lattice launch, under the conditions of prepare(); the task list is built on the GPU.
    const int n_cu = compute_units(), share_percent = g_overlap.load(std::memory_order_relaxed);
    p.n_cu = n_cu;
    if (p.folded && grads && share_percent > 0 && !p.needs_barrier && 2 * B <= kMaxTaskEntries && n_cu % kXcds == 0 &&
        p.n_chains + n_cu / 4 <= n_cu) {
        p.device_tasks = true;
        p.share_percent = share_percent;
        p.n_tasks = B * ((T + kTaskRows - 1) / kTaskRows);
        p.n_task_entries = 2 * B;
    }
    p.lay = lay;
    // Per-launch device times for measurements (ctc_profile_kernels_device): events around the launches as in run().
    Events events;
    hipEvent_t* const ev = events.ev;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (kernel_ms && !events.create()) return CTC_STATUS_HIP_ERROR;
    if (!p.folded && !record(launch_plan(p, stream))) return CTC_STATUS_HIP_ERROR;
    int (*const stages[CTC_NUM_KERNELS])(const Launch&, void*) = {launch_softmax, launch_lattice,
                                                                   grads ? launch_gradient : nullptr};
    if (kernel_ms && !record(hipEventRecord(ev[0], s))) return CTC_STATUS_HIP_ERROR;
    for (int i = 0; i < CTC_NUM_KERNELS; ++i) {
        if (stages[i] && !record(stages[i](p, stream))) return CTC_STATUS_HIP_ERROR;
        if (kernel_ms && !record(hipEventRecord(ev[i + 1], s))) return CTC_STATUS_HIP_ERROR;
    }
    if (kernel_ms) {
        if (!record(hipEventRecord(ev[CTC_NUM_KERNELS + 1], s))) return CTC_STATUS_HIP_ERROR;
        if (!record(hipEventRecord(ev[CTC_NUM_KERNELS + 2], s))) return CTC_STATUS_HIP_ERROR;
        if (!record(hipStreamSynchronize(s))) return CTC_STATUS_HIP_ERROR;
        float empty = 0.0f;
        if (!record(hipEventElapsedTime(&empty, ev[CTC_NUM_KERNELS + 1], ev[CTC_NUM_KERNELS + 2])))
            return CTC_STATUS_HIP_ERROR;
        for (int i = 0; i < CTC_NUM_KERNELS; ++i) {
            if (!record(hipEventElapsedTime(&kernel_ms[i], ev[i], ev[i + 1]))) return CTC_STATUS_HIP_ERROR;
            kernel_ms[i] = stages[i] ? std::max(kernel_ms[i] - empty, 0.0f) : 0.0f;
        }
    }
    return CTC_STATUS_SUCCESS;
}

// Address of `scratch` on the current device (each GPU holds its own copy at its own address):
// asked once per device, with that device current, and kept.
void* static_workspace()
{
    constexpr int kMaxDevices = 64;
    static std::mutex mutex;
    static void* address[kMaxDevices] = {};
    int dev = 0;
    if (!record(hipGetDevice(&dev))) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        g_last_hip_error = static_cast<int>(hipErrorInvalidDevice);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(mutex);
    if (!address[dev]) {
        void* ptr = nullptr;
        if (!record(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)))) return nullptr;
        address[dev] = ptr;
    }
    return address[dev];
}

}  // namespace
}  // namespace ctc

extern "C" {

ctc_status_t ctc_profile_kernels_device(const void* activations, const int32_t* labels,
                                        const int32_t* label_lengths, const int32_t* input_lengths,
                                        int max_label_length, int T, int B, int A, int blank,
                                        ctc_dtype_t dtype, float* costs, void* grads, int32_t* status_out,
                                        void* workspace, size_t workspace_bytes, hipStream_t stream,
                                        float* kernel_ms)
{
    if (!kernel_ms) return CTC_STATUS_INVALID_VALUE;
    return ctc::run_device(activations, labels, label_lengths, input_lengths, max_label_length, T, B, A,
                           blank, dtype, costs, grads, status_out, workspace, workspace_bytes, stream, kernel_ms);
}

ctc_status_t ctc_loss_and_grad_device_static(const void* activations, const int32_t* labels,
                                             const int32_t* label_lengths, const int32_t* input_lengths,
                                             int max_label_length, int T, int B, int A, int blank,
                                             ctc_dtype_t dtype, float* costs, void* grads,
                                             int32_t* status_out, hipStream_t stream)
{
    // Sizes first: a batch shape beyond the static workspace is refused before anything else happens.
    ctc::Layout lay;
    const ctc_status_t st = ctc::make_layout_bounds(T, B, A, max_label_length, dtype, &lay);
    if (st != CTC_STATUS_SUCCESS) return st;
    if (lay.total > CTC_STATIC_WORKSPACE_BYTES) return CTC_STATUS_WORKSPACE_TOO_SMALL;
    void* const ws = ctc::static_workspace();
    if (!ws) return CTC_STATUS_HIP_ERROR;
    return ctc::run_device(activations, labels, label_lengths, input_lengths, max_label_length, T, B, A,
                           blank, dtype, costs, grads, status_out, ws, CTC_STATIC_WORKSPACE_BYTES, stream);
}

ctc_status_t ctc_workspace_size_device(int T, int B, int A, int max_label_length, ctc_dtype_t dtype,
                                       size_t* bytes_out)
{
    if (!bytes_out) return CTC_STATUS_INVALID_VALUE;
    ctc::Layout lay;
    ctc_status_t st = ctc::make_layout_bounds(T, B, A, max_label_length, dtype, &lay);
    if (st == CTC_STATUS_SUCCESS) *bytes_out = lay.total;
    return st;
}

ctc_status_t ctc_loss_and_grad_device(const void* activations, const int32_t* labels,
                                      const int32_t* label_lengths, const int32_t* input_lengths,
                                      int max_label_length, int T, int B, int A, int blank,
                                      ctc_dtype_t dtype, float* costs, void* grads, int32_t* status_out,
                                      void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    return ctc::run_device(activations, labels, label_lengths, input_lengths, max_label_length, T, B, A,
                           blank, dtype, costs, grads, status_out, workspace, workspace_bytes, stream);
}


ctc_status_t ctc_workspace_size(int T, int B, int A, const int32_t* label_lengths,
                                const int32_t* input_lengths, ctc_dtype_t dtype, size_t* bytes_out)
{
    if (!bytes_out) return CTC_STATUS_INVALID_VALUE;
    ctc::Layout lay;
    ctc_status_t st = ctc::make_layout(T, B, A, label_lengths, input_lengths, dtype, &lay);
    if (st == CTC_STATUS_SUCCESS) *bytes_out = lay.total;
    return st;
}

ctc_status_t ctc_loss_and_grad(const void* activations, const int32_t* flat_labels,
                               const int32_t* label_lengths, const int32_t* input_lengths,
                               int T, int B, int A, int blank, ctc_dtype_t dtype, float* costs,
                               void* grads, void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    ctc::Call c{grads ? ctc::Mode::kGrad : ctc::Mode::kLoss, activations, flat_labels, label_lengths,
                input_lengths, T, B, A, blank, dtype, costs, grads, nullptr, workspace, workspace_bytes, stream};
    return ctc::run(c, nullptr);
}

ctc_status_t ctc_profile_kernels(const void* activations, const int32_t* flat_labels,
                                 const int32_t* label_lengths, const int32_t* input_lengths,
                                 int T, int B, int A, int blank, ctc_dtype_t dtype, float* costs,
                                 void* grads, void* workspace, size_t workspace_bytes, hipStream_t stream,
                                 float* kernel_ms)
{
    if (!kernel_ms) return CTC_STATUS_INVALID_VALUE;
    ctc::Call c{grads ? ctc::Mode::kGrad : ctc::Mode::kLoss, activations, flat_labels, label_lengths,
                input_lengths, T, B, A, blank, dtype, costs, grads, nullptr, workspace, workspace_bytes, stream};
    return ctc::run(c, kernel_ms);
}

ctc_status_t ctc_best_path(const void* activations, const int32_t* flat_labels,
                           const int32_t* label_lengths, const int32_t* input_lengths,
                           int T, int B, int A, int blank, ctc_dtype_t dtype, float* scores,
                           int32_t* alignment, void* workspace, size_t workspace_bytes, hipStream_t stream)
{
    ctc::Call c{ctc::Mode::kBest, activations, flat_labels, label_lengths, input_lengths, T, B, A, blank,
                dtype, scores, nullptr, alignment, workspace, workspace_bytes, stream};
    return ctc::run(c, nullptr);
}

ctc_status_t ctc_profile_best_path(const void* activations, const int32_t* flat_labels,
                                   const int32_t* label_lengths, const int32_t* input_lengths,
                                   int T, int B, int A, int blank, ctc_dtype_t dtype, float* scores,
                                   int32_t* alignment, void* workspace, size_t workspace_bytes,
                                   hipStream_t stream, float* kernel_ms)
{
    if (!kernel_ms) return CTC_STATUS_INVALID_VALUE;
    ctc::Call c{ctc::Mode::kBest, activations, flat_labels, label_lengths, input_lengths, T, B, A, blank,
                dtype, scores, nullptr, alignment, workspace, workspace_bytes, stream};
    return ctc::run(c, kernel_ms);
}

const char* ctc_kernel_name(int index)
{
    switch (index) {
        case CTC_KERNEL_SOFTMAX: return "ctc_softmax";
        case CTC_KERNEL_LATTICE: return "ctc_lattice";
        case CTC_KERNEL_GRADIENT: return "ctc_gradient";
        case CTC_KERNEL_BACKTRACE: return "ctc_backtrace";
        default: return nullptr;
    }
}

const char* ctc_status_string(ctc_status_t status)
{
    switch (status) {
        case CTC_STATUS_SUCCESS: return "success";
        case CTC_STATUS_INVALID_VALUE: return "invalid value";
        case CTC_STATUS_WORKSPACE_TOO_SMALL: return "workspace too small";
        case CTC_STATUS_HIP_ERROR: return "HIP runtime error";
        case CTC_STATUS_UNSUPPORTED: return "unsupported size";
        case CTC_STATUS_NOT_READY: return "too many calls in flight";
        default: return "unknown status";
    }
}

int ctc_last_hip_error(void) { return ctc::g_last_hip_error; }

long ctc_debug_staging_allocations(void)
{
    std::lock_guard<std::mutex> lock(ctc::g_staging_mutex);
    long n = 0;
    for (const ctc::DeviceStaging* d : ctc::g_staging) n += d->allocations.load(std::memory_order_relaxed);
    return n;
}

long ctc_debug_replay_emission_fetches(int T, int B, int A, const int32_t* label_lengths, const int32_t* input_lengths,
                                       int max_label_length, long* margin_floats)
{
    using namespace ctc;
    if (!label_lengths || !input_lengths) return -1;
    const bool bounds = max_label_length >= 0;
    Layout lay;
    const ctc_status_t st = bounds ? make_layout_bounds(T, B, A, max_label_length, CTC_DTYPE_F32, &lay)
                                   : make_layout(T, B, A, label_lengths, input_lengths, CTC_DTYPE_F32, &lay);
    if (st != CTC_STATUS_SUCCESS) return -1;
    const bool symbol_major = emission_layout(A) == kEmitSymbolMajor;
    // the regions as carved: slack, blocks, slack
    const int64_t label_floats = lay.emit_floats + 2 * static_cast<int64_t>(kLabelSlack);
    const int64_t blank_floats = lay.frames + 2 * static_cast<int64_t>(kBlankSlack);
    long violations = 0;
    int64_t margin = INT64_MAX;
    auto touch = [&](int64_t off, int64_t size) {
        if (off < 0 || off >= size) ++violations;
        margin = std::min(margin, std::min(off, size - 1 - off));
    };
    int64_t e_off = 0, f_off = 0;
    for (int b = 0; b < B; ++b) {
        const int L = label_lengths[b], Tb = input_lengths[b];
        // block offsets as the launcher (prepare) and the device-side planner (ctc_plan_kernel) set them
        Utt m{};
        m.Tb = Tb;
        m.L = L;
        m.e_direct = emission_layout(A);
        if (bounds) {
            m.f_off = b * T;
            m.e_off = static_cast<int64_t>(b) * T * (symbol_major ? A : max_label_length);
            m.e_pitch = symbol_major ? T : L;
        } else {
            m.f_off = static_cast<int32_t>(f_off);
            m.e_off = e_off;
            m.e_pitch = symbol_major ? Tb : L;
            e_off += static_cast<int64_t>(Tb) * (symbol_major ? A : L);
            f_off += Tb;
        }
        if (Tb < 1) continue;                       // its chains do not run
        for (int backward = 0; backward < 2; ++backward) {
            const int f0 = backward ? Tb - 1 : 0, fdir = backward ? -1 : 1;
            // Lanes at the ends of every range a pointer depends on: first and last label position, first
            // and last symbol; a lane without a label state, for either constant.
            struct LaneKind { bool has_label; int symbol, li, constant; };
            const LaneKind kinds[] = {{L > 0, 0, 0, 0}, {L > 0, A - 1, L - 1, 0}, {L > 0, 0, L - 1, 0}, {L > 0, A - 1, 0, 0},
                                      {false, 0, 0, kZeroEmission}, {false, 0, 0, kLogZeroEmission}};
            for (const LaneKind& k : kinds) {
                if (!k.has_label && k.constant == 0) continue;          // (L == 0: no label lanes)
                int64_t p = label_emission_offset(m, k.has_label, symbol_major, k.symbol, k.li, f0, k.constant);
                const int64_t step = label_emission_step(m, k.has_label, symbol_major, fdir);
                touch(p, label_floats);                                  // step 0
                auto fetch = [&](int) {
                    if (symbol_major) {
                        touch(p + fetch_window_first(backward != 0), label_floats);
                        touch(p + fetch_window_first(backward != 0) + kChunk - 1, label_floats);
                        p += step * kChunk;
                    } else {
                        for (int i = 0; i < kChunk; ++i) {
                            p += step;
                            touch(p, label_floats);
                        }
                    }
                };
                auto nothing = [](int, bool) {};
                chain_schedule(Tb, fetch, fetch, nothing, nothing, [] {});
                // the same pointer walk on the schedule with three register sets (run_chain_linear)
                p = label_emission_offset(m, k.has_label, symbol_major, k.symbol, k.li, f0, k.constant);
                chain_schedule3(Tb, fetch, fetch, fetch, nothing, nothing, nothing, [] {});
            }
            for (int lane = 0; lane < kChunk; ++lane) {
                const int64_t bp = blank_emission_offset(m, f0, fdir, lane);
                touch(bp, blank_floats);                                  // step 0 (lane 0's is the one used)
                auto fetch = [&](int s0) { touch(bp + static_cast<int64_t>(fdir) * s0, blank_floats); };
                auto nothing = [](int, bool) {};
                chain_schedule(Tb, fetch, fetch, nothing, nothing, [] {});
            }
            {
                // the scalar windows of the linear-domain chains (the block of doubles has the same extent)
                touch(blank64_window(m, f0, fdir, 0) + (fdir > 0 ? 0 : kChunk - 1), blank_floats);     // step 0
                auto fetch = [&](int s0) {
                    touch(blank64_window(m, f0, fdir, s0), blank_floats);
                    touch(blank64_window(m, f0, fdir, s0) + kChunk - 1, blank_floats);
                };
                auto nothing = [](int, bool) {};
                chain_schedule(Tb, fetch, fetch, nothing, nothing, [] {});
                auto fetch3 = [&](int s0) { fetch(blank64_chunk_with(s0)); };
                chain_schedule3(Tb, fetch3, fetch3, fetch3, nothing, nothing, nothing, [] {});
            }
        }
    }
    if (margin_floats) *margin_floats = margin == INT64_MAX ? -1 : static_cast<long>(margin);
    return violations;
}

void ctc_debug_set_overlap(int percent)
{
    ctc::g_overlap.store(percent < 0 ? ctc::kWorkerSharePercent : std::min(percent, 100), std::memory_order_relaxed);
}

extern "C" void ctc_debug_set_sequential_chains(int on)
{
    ctc::g_sequential_chains.store(on ? 1 : 0, std::memory_order_relaxed);
}

void ctc_debug_set_poll_budget(int polls)
{
    ctc::g_poll_budget.store(polls < 0 ? ctc::kDefaultPollBudget : polls, std::memory_order_relaxed);
}

}  // extern "C"
