// C-ABI layer of libstar: argument checks, planning, workspace, launches.
// Every step of the update itself runs in the kernels of star_kernels.hip.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "star.h"
#include "star_kernels.h"
#include "star_plan.h"

namespace {

thread_local std::string g_err;

star_status set_err(star_status s, const std::string& msg) {
    g_err = msg;
    return s;
}

star_status hip_fail(hipError_t e, const char* what) {
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    return STAR_ERR_DEVICE;
}

#define STAR_HIP(call)                                         \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return hip_fail(e_, #call);      \
    } while (0)

int initial_kernel_choice() {
    const char* e = std::getenv("STAR_KERNEL");
    if (!e) return STAR_KERNEL_AUTO;
    if (!std::strcmp(e, "seq")) return STAR_KERNEL_SEQ;
    if (!std::strcmp(e, "affine")) return STAR_KERNEL_AFFINE;
    if (!std::strcmp(e, "affine_mfma")) return STAR_KERNEL_AFFINE_MFMA;
    return STAR_KERNEL_AUTO;
}

const int g_env_kernel = initial_kernel_choice();   // what STAR_KERNEL_AUTO means for calls that do not choose

// The options of one call, resolved: never a process-wide state.
struct Opts {
    int kernel = STAR_KERNEL_AUTO;
    int64_t queue_min = 0;   // 0: the library's default for the call's shape (queue_min_for)
    bool direct_norms = false;   // STAR_OPT_DIRECT_NORMS
};

// Shards of at least this many elements take their tiles from the queue.  The queue's order pays once a call is
// long enough for its start-up (the first claims) and its few claims per workgroup not to show: measured on
// 2-96 Mi elements, 16 updates, that is from about 16 Mi elements on with 8 and more fp32 rows (16 Mi: 0.76
// against 0.66 of the HBM peak with 8 rows, equal with 16), from about 32 Mi with up to 4 fp32 rows, and from
// about 48 Mi with bf16 rows, whose tiles are half as heavy (16-32 Mi: the fixed assignment is 0-14 % ahead,
// 64 Mi and more: the queue 2-8 % -- with 16 rows; see below for the other row counts).  Norms and Gram matrix alone keep 16 Mi (few rows, vector registers: at 8 Mi
// the fixed assignment is 5-25 % ahead, from 24 Mi on the queue, whose tiles hold several chunks per thread, by
// 10 % to 4x).  The aggregation, a read of W rows with one row written, is faster with the fixed assignment far
// longer: 4-48 Mi elements 2-25 % ahead for every row count and dtype, equal from about 96 Mi on with 16 and more
// rows (the queue 2-3 % ahead from 96-144 Mi), and with light tiles -- up to 8 bf16 or 4 fp32 rows -- ahead at
// every length tried (256 Mi elements, 4 / 8 bf16 rows: 480 / 808 against 622 / 876 us).
int64_t queue_min_for(const Opts& opt, int grad_dtype, int rows, bool update, bool aggregation = false,
                      bool norms = false, bool literal = false, int groups = 1) {
    if (opt.queue_min > 0) return opt.queue_min;
    if (aggregation) {
        const int row_bytes = rows * (grad_dtype == STAR_F32 ? 16 : 8);   // per thread and tile
        // several groups per call with bf16 rows (as many output rows, written 8 bytes a thread): the fixed
        // assignment at every length, 8-128 Mi elements, 4 to 16 groups of 12 to 32 rows: level to 40 % ahead
        // (16 groups of 32 rows, 128 Mi: 2.77 against 3.64 ms); with fp32 rows the queue is 3-19 % ahead from 80 Mi
        if (grad_dtype == STAR_BF16 && groups > 1) return (int64_t)1 << 62;
        return row_bytes <= 64 ? (int64_t)1 << 62 : 4 * star::kQueueMinElements;
    }
    if (!update) return star::kQueueMinElements;
    // (A second A/B of the two tile orders, 8-320 Mi elements, 1-32 rows, moved the limits of the light updates up:
    // bf16 rows, 48-96 Mi elements: the fixed assignment 5-12 % ahead with up to 4 rows, 3-7 % with 8, level or ahead
    // with 32, behind with 16 from 64 Mi on; up to 4 fp32 rows: ahead or level up to 64 Mi; from 128 Mi on the two
    // orders are within 3 % of each other for every light update and the queue is kept.)
    // With norms on up to 6 rows (the few-rows form of the vector-register Gram matrix, whose queue tiles fold
    // their sums per chunk) the picture is another one again: bf16 rows gain 8-16 % from the queue from 16-32 Mi
    // elements on (6 rows, 16 / 48 Mi: 96 / 246 against 106 / 290 us), one fp32 row from 32 Mi, while 3 to 6 fp32
    // rows are 3-10 % faster with the fixed assignment up to 96 Mi (6 rows, 32 Mi: 220 against 245 us).
    // (The literal kernel with its direct norm sums, one or two updates: the queue from 32 Mi elements, 4 fp32 rows,
    // 48 / 64 Mi: 272 / 356 against 300 / 400 us.)
    if (norms && rows <= star::kFewRows) {
        if (literal) return 2 * star::kQueueMinElements;
        if (grad_dtype == STAR_BF16) return star::kQueueMinElements;
        return (rows <= 1 ? 2 : (rows <= 2 ? 4 : 8)) * star::kQueueMinElements;
    }
    if (grad_dtype == STAR_BF16) return (rows <= 4 ? 8 : (rows <= 12 ? 6 : 4)) * star::kQueueMinElements;
    return rows <= 4 ? 4 * star::kQueueMinElements : star::kQueueMinElements;
}

star_status resolve_options(const star_options* o, Opts* out) {
    out->kernel = g_env_kernel;
    out->queue_min = 0;
    out->direct_norms = false;
    if (!o) return STAR_OK;
    if (o->kernel != STAR_KERNEL_AUTO && o->kernel != STAR_KERNEL_SEQ && o->kernel != STAR_KERNEL_AFFINE &&
        o->kernel != STAR_KERNEL_AFFINE_MFMA)
        return set_err(STAR_ERR_KERNEL, "unknown kernel choice in star_options");
    if (o->flags & ~STAR_OPT_DIRECT_NORMS) return set_err(STAR_ERR_SHAPE, "unknown bit in star_options.flags");
    out->direct_norms = (o->flags & STAR_OPT_DIRECT_NORMS) != 0;
    if (o->queue_threshold < 0) return set_err(STAR_ERR_SHAPE, "star_options.queue_threshold is negative");
    if (o->kernel != STAR_KERNEL_AUTO) out->kernel = o->kernel;
    if (o->queue_threshold > 0) out->queue_min = o->queue_threshold;
    return STAR_OK;
}

// ---------------------------------------------------------------- workspace
// A ring of slots.  One call uses one slot: a pinned host staging buffer and a
// device buffer for the tables, a device buffer for the per-block partial sums
// and the reduced Gram matrix, and the 16-byte tile queue.  A slot's event is recorded after the last
// kernel that touches it; the slot is handed out again only once that event
// has completed, so calls on different streams never share live memory.
struct Slot {
    int device = -1;
    void* host = nullptr;     // pinned
    void* host_dev = nullptr; // the same memory as the device addresses it
    void* dev = nullptr;      // tables
    size_t table_cap = 0;
    double* partials = nullptr;
    size_t partial_cap = 0;   // doubles
    star::TileQueue* queue = nullptr;   // work queue of the slot's launches, zero whenever no kernel is running
    hipEvent_t done = nullptr;
    bool pending = false;     // `done` has been recorded after work that uses this slot
};

constexpr int kSlots = 8;
Slot g_slots[kSlots];
int g_next_slot = 0;
std::mutex g_mu;

struct DeviceInfo {
    int device = -1;
    int num_cu = 0;
};
DeviceInfo g_dev[16];

star_status device_info(int* device, int* num_cu) {
    STAR_HIP(hipGetDevice(device));
    if (*device < 0 || *device >= 16) return set_err(STAR_ERR_DEVICE, "device index out of range");
    DeviceInfo& d = g_dev[*device];
    if (d.device != *device) {
        int n = 0;
        STAR_HIP(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, *device));
        d.num_cu = n > 0 ? n : 1;
        d.device = *device;
    }
    *num_cu = d.num_cu;
    return STAR_OK;
}

void free_slot(Slot& s) {
    if (s.done) {
        if (s.pending) (void)hipEventSynchronize(s.done);
        (void)hipEventDestroy(s.done);
    }
    if (s.host) (void)hipHostFree(s.host);
    if (s.dev) (void)hipFree(s.dev);
    if (s.partials) (void)hipFree(s.partials);
    if (s.queue) (void)hipFree(s.queue);
    s = Slot();
}

// Grows one slot to the asked capacities (its previous work has completed).
star_status grow_slot(Slot& s, size_t table_bytes, size_t partial_doubles) {
    if (!s.queue) {
        STAR_HIP(hipMalloc(reinterpret_cast<void**>(&s.queue), 256));
        STAR_HIP(hipMemset(s.queue, 0, 256));
    }
    if (table_bytes > s.table_cap) {
        if (s.host) STAR_HIP(hipHostFree(s.host));
        if (s.dev) STAR_HIP(hipFree(s.dev));
        s.host = s.host_dev = s.dev = nullptr;
        s.table_cap = 0;
        const size_t cap = std::max<size_t>(table_bytes, 64 * 1024);
        STAR_HIP(hipHostMalloc(&s.host, cap, hipHostMallocDefault));
        STAR_HIP(hipHostGetDevicePointer(&s.host_dev, s.host, 0));
        STAR_HIP(hipMalloc(&s.dev, cap));
        s.table_cap = cap;
    }
    if (partial_doubles > s.partial_cap) {
        if (s.partials) STAR_HIP(hipFree(s.partials));
        s.partials = nullptr;
        s.partial_cap = 0;
        STAR_HIP(hipMalloc(reinterpret_cast<void**>(&s.partials), partial_doubles * sizeof(double)));
        s.partial_cap = partial_doubles;
    }
    return STAR_OK;
}

// Hands out the next slot with at least the asked capacities (g_mu held).
// Whenever a slot has to grow, the idle ones are grown with it, so that the
// allocations (which synchronise the device) happen in one call and not
// spread over the next seven.
star_status acquire_slot(int device, size_t table_bytes, size_t partial_doubles, Slot** out) {
    Slot& s = g_slots[g_next_slot];
    g_next_slot = (g_next_slot + 1) % kSlots;
    if (s.device != -1 && s.device != device) free_slot(s);   // its memory lives on another device
    if (s.pending) STAR_HIP(hipEventSynchronize(s.done));
    s.pending = false;
    if (!s.done) STAR_HIP(hipEventCreateWithFlags(&s.done, hipEventDisableTiming));
    const bool grows = table_bytes > s.table_cap || partial_doubles > s.partial_cap || !s.queue;
    s.device = device;
    star_status st = grow_slot(s, table_bytes, partial_doubles);
    if (st != STAR_OK) return st;
    if (grows) {
        for (Slot& o : g_slots) {
            if (&o == &s || (o.device != -1 && o.device != device)) continue;
            if (o.pending && hipEventQuery(o.done) != hipSuccess) continue;   // busy: it grows when its turn comes
            o.pending = false;
            o.device = device;
            st = grow_slot(o, table_bytes, partial_doubles);
            if (st != STAR_OK) return st;
        }
    }
    *out = &s;
    return STAR_OK;
}

// On every way out of a call, marks its slot busy until everything enqueued on
// the stream so far has run (also after a failed launch: earlier launches of
// the same call may still be using the slot).
struct SlotRelease {
    Slot* slot = nullptr;
    hipStream_t stream = nullptr;
    ~SlotRelease() {
        if (slot && hipEventRecord(slot->done, stream) == hipSuccess) slot->pending = true;
    }
};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Table layout in a slot (all offsets 256-byte aligned):
//   coef_f32 [U][Wp] | lr_f32 [U] | mask_u32 [U] | coef_f64 [U][Wp] | out pointers [U]
struct TableLayout {
    size_t coef32, lr32, mask, coef64, outptr, total;
};

TableLayout table_layout(int U, int Wp) {
    TableLayout t;
    size_t o = 0;
    t.coef32 = o; o = align_up(o + sizeof(float) * (size_t)U * Wp, 256);
    t.lr32 = o;   o = align_up(o + sizeof(float) * (size_t)U, 256);
    t.mask = o;   o = align_up(o + sizeof(uint32_t) * (size_t)U, 256);
    t.coef64 = o; o = align_up(o + sizeof(double) * (size_t)U * Wp, 256);
    t.outptr = o; o = align_up(o + sizeof(void*) * (size_t)U, 256);
    t.total = o;
    return t;
}

size_t partial_doubles_needed(int Wp, int U, int grid_cap) {
    const size_t ng = (size_t)Wp * (Wp + 1) / 2;
    const size_t useq = (size_t)std::min(U, std::max(star::seq_max_updates(Wp, true), star::reduce_max_updates(Wp, true)));
    // per-block partials of the larger of the two routes, plus the reduced Gram matrix
    return std::max(ng, useq) * (size_t)grid_cap + ng;
}

// Where the Gram matrix behind the norms is formed: on the matrix cores (aff_mfma_kernel) or in vector
// registers (aff_kernel, up to kMaxValuGramW rows).  The matrix instructions cost the same for 1 row as for 16
// (fp32: 64 per wave and tile, about 0.85 us), which a tile of few rows does not hide; the vector-register form
// needs W(W+1)/2 accumulators, 21 for 6 rows, 136 for 16.  Every limit below is a measured crossover of the two
// forms on MI355X (256 compute units), both forced through star_options.kernel on the same inputs;
// tests/test_host_logic.py pins the table.
bool gram_on_matrix_cores(int Wp, int grad_dtype, int choice, bool update, int64_t P) {
    if (Wp > star::kMaxValuGramW) return true;
    if (choice == STAR_KERNEL_AFFINE) return false;
    if (choice == STAR_KERNEL_AFFINE_MFMA) return true;
    const bool f32 = grad_dtype == STAR_F32;
    constexpr int64_t Mi = 1 << 20;
    if (!update) {
        // Norms or Gram matrix alone: a pure read.
        // fp32 rows: up to 8 on the vector ALUs, whose long-lived workgroups with a fixed assignment reach 0.80-0.88
        // of the HBM peak there (96 Mi elements, 7 / 8 rows: 400 / 458 against 497 / 545 us; 12 rows equal).
        if (f32) return Wp > 8;
        // bf16 rows: from 7 rows on the matrix cores at every length.  The light tiles of 3 to 6 rows are faster
        // there while that kernel splits its tiles evenly (12 Mi elements, 3 / 4 / 6 rows: 30 / 31 / 34 against
        // 39 / 44 / 54 us) and slower on long shards, where the vector-register form loads several chunks per
        // thread (96 Mi elements, 4 / 5 / 6 rows: 141 / 167 / 201 against 182 / 197 / 211 us).
        if (Wp >= 7) return true;
        if (Wp >= 5) return P <= 48 * Mi;
        if (Wp >= 3) return P <= 16 * Mi;
        return false;
    }
    // Update with norms.
    // Up to 6 rows the vector-register form, which with so few accumulators takes its tiles from the queue as well
    // (8 updates: 1 fp32 row 0.34 against 0.49 ms on 100 M elements, 4 rows 0.53 against 0.64; 1 bf16 row 0.59
    // against 0.66 ms on 200 M elements; 6 rows equal); from 7 rows on the matrix cores (7 and 8 rows: 2-6 % ahead
    // on long shards, 16 rows ahead at every length).  Two refinements on shorter shards:
    //  - fp32 rows, 7 or 8 of them, below 16 Mi elements: the vector-register form with its fixed assignment
    //    (1 Mi elements 21 against 28 us, 8 Mi 80 against 89 us, equal at 16 Mi);
    //  - bf16 rows, 3 to 8 of them: the matrix-core kernel up to 8 Mi elements, where it splits its tiles evenly over
    //    the workgroups (queue_geometry) and with tiles that light is 5-16 % ahead (6 rows, 2 / 4 / 8 Mi elements:
    //    20 / 30 / 50 against 24 / 36 / 60 us).  5 and 6 rows keep that lead until the vector-register form takes the
    //    queue at 48 Mi elements (6 rows, 16 / 32 / 40 Mi: 95 / 172 / 211 against 106 / 197 / 244 us; equal from 48 Mi
    //    on); 4 rows have it from 16 Mi on (32 Mi: 153 against 160 us; at 12 Mi the vector-register form is 4 % ahead);
    //    7 and 8 rows are level or 3 % behind between 8 and 16 Mi.
    if (f32) {
        if (Wp <= 8 && P < star::kQueueMinElements) return false;
        return Wp > star::kFewRows;
    }
    if (Wp >= 3 && Wp <= 8 && P <= 8 * Mi) return true;
    if (Wp >= 5 && Wp <= 6 && P < 48 * Mi) return true;
    if (Wp == 4 && P >= 16 * Mi && P < 48 * Mi) return true;
    if (Wp <= 8 && P < star::kQueueMinElements) return false;
    return Wp > star::kFewRows;
}

// What a call launches: decided here, once, for run() and for star_plan_choice.
struct Launch {
    star::Route route = star::Route::Affine;
    bool mfma = false;        // collapsed route: Gram matrix on the matrix cores
    int Wp = 1;               // row count of the kernel instantiation
    bool want_queue = false;  // the shard is long enough for queue order
    bool queue_order = false; // the main kernel really takes its tiles from the queue (aligned buffers assumed)
    bool seq_inline = false;  // step-by-step route: tables in the kernel arguments
    int umax = 1;             // step-by-step route: updates per launch
    int launches = 1;
    int finishing = 0;
    bool split_norms = false; // update by the collapsed map, norms by a separate direct pass (see decide)
    bool collapsed_in_seq = false;   // step-by-step kernel walks the updates for the norms, applies the update as one map
};

Launch decide(const star::Plan& plan, int grad_dtype, bool update, bool want_norms, int64_t P, const Opts& opt) {
    Launch l;
    l.route = star::choose_route(plan, grad_dtype == STAR_F32 ? 4 : 2, opt.kernel);
    // Norms from the Gram matrix, n^2 = c^T Gamma c, lose digits when the terms of that sum cancel.  With
    // the weightings of the paper (c >= 0) they cancel only if the rows themselves are anti-correlated;
    // with caller-given coefficients of both signs they cancel as a rule (a difference of two similar
    // rows).  Unless the caller forces an evaluation, such streams get their norms from the direct sums
    // of gbar^2 (step-by-step kernel, norms only), in a pass of its own beside the collapsed update; so
    // does any stream whose caller asks for it (STAR_OPT_DIRECT_NORMS).
    // So does a shard of a few thousand elements: the sum of a handful of elements' signed values cancels as a
    // matter of course (one element, 16 rows: kappa of 1000 is ordinary), the concentration that keeps kappa
    // near y_u needs dimension, and at that length the cost is a launch, not bandwidth.
    const bool tiny = P < star::kTinyShardElements;
    if (want_norms && (plan.negative_coef || opt.direct_norms || tiny) && opt.kernel == STAR_KERNEL_AUTO &&
        l.route == star::Route::Affine) {
        if (update) l.split_norms = true;
        else l.route = star::Route::Seq;
    }
    l.Wp = star::padded_rows(plan.Wc);
    // Update with norms, a stream so short that walking it costs next to nothing (fma_seq, the sum of y_u + 4 over
    // the updates): the literal kernel forms its norms directly, in the same pass, and needs one finishing launch
    // where the Gram route needs two.  On a short shard that launch is most of the difference (1 Mi elements:
    // 2 updates of 8 fp32 rows 14.5 against 20.1 us, one update of 32 bf16 rows 23 against 33 us; 4 Mi: 41 against
    // 46, 69 against 80 us; from 16 Mi on the collapsed kernel is level or ahead, at 64 Mi by up to 40 %).  With 17
    // to 32 fp32 rows the alternative is dearer -- the matrix cores' fp32 Gram matrix, or the collapsed update
    // with the norm walk -- and the literal kernel stays ahead at every length up to about 110 multiply-adds
    // (3 updates of 32 rows, 16 / 64 Mi elements: 438 / 1752 against 446 / 1953 us; 4 updates: 515 against 441).
    // (Its norms are direct sums, so streams that were given a direct norm pass above are served as well.)
    if (update && want_norms && l.route == star::Route::Affine && opt.kernel == STAR_KERNEL_AUTO &&
        plan.U <= star::seq_max_updates(l.Wp, true)) {
        const bool wide_f32 = grad_dtype == STAR_F32 && l.Wp > 16;
        // (bf16 rows: up to 16 Mi elements -- there the literal kernel is still 4-12 % ahead with 2, 8 and 32 rows
        // and level with 16; fp32 rows are level or 4 % behind at 16 Mi)
        const int64_t short_shard = grad_dtype == STAR_BF16 ? (16 << 20) : (4 << 20);
        if ((P <= short_shard && plan.fma_seq <= 48.0) || (wide_f32 && plan.fma_seq <= 112.0)) {
            l.route = star::Route::Seq;
            l.split_norms = false;
        }
    }
    // 17 to 32 fp32 rows, update with norms: the Gram matrix needs the fp32 matrix instructions (1536 flops per
    // element, only partly hidden: 0.60-0.64 of the HBM peak).  A short stream gets its norms cheaper from the
    // direct sums, y_u + 1 multiply-adds per update, in the same pass as the collapsed update.
    if (update && want_norms && l.route == star::Route::Affine && !l.split_norms && opt.kernel == STAR_KERNEL_AUTO &&
        grad_dtype == STAR_F32 && l.Wp > 16 && plan.U <= star::seq_max_updates(l.Wp, true) &&
        plan.fma_seq - 3.0 * plan.U <= star::direct_norm_fma_limit(l.Wp)) {
        l.route = star::Route::Seq;
        l.collapsed_in_seq = true;
    }
    l.want_queue = P >= queue_min_for(opt, grad_dtype, plan.Wc, update, false, update && want_norms,
                                      l.route == star::Route::Seq);
    if (l.route == star::Route::Affine) {
        const bool gram = want_norms;
        l.mfma = gram && gram_on_matrix_cores(l.Wp, grad_dtype, opt.kernel, update, P);
        l.queue_order = l.mfma || (l.want_queue && star::aff_takes_queue(gram, l.Wp, grad_dtype == STAR_F32, update));
        l.launches = (update || gram) ? 1 : 0;
        l.finishing = gram ? 2 : 0;
    } else {
        l.umax = star::seq_max_updates(l.Wp, want_norms);
        l.seq_inline = star::tables_fit_inline(plan.U, l.Wp) && plan.U <= l.umax;
        l.launches = (plan.U + l.umax - 1) / l.umax;
        l.queue_order = l.want_queue && (l.collapsed_in_seq || star::seq_takes_queue(std::min(plan.U, l.umax)));
        l.finishing = want_norms ? l.launches : 0;
    }
    return l;
}

// The shared body of star_group_update (update = true) and star_group_norms.  With `no_alloc` the
// call works in the fixed device array of star_scratch.hip instead of a workspace slot and allocates
// no device memory, pinned memory or event.
star_status run(bool update, float* params, float* momentum, const void* const* grad_rows, int grad_dtype,
                int64_t P, int32_t W, const star_updates* upd, const star_hparams* hp, int32_t wmode,
                float* norms_out, void* publish, int publish_dtype, const star_options* options, void* hip_stream,
                bool no_alloc = false) {
    g_err.clear();
    Opts opt;
    star_status st = resolve_options(options, &opt);
    if (st != STAR_OK) return st;
    if (!upd) return set_err(STAR_ERR_NULL, "updates struct is NULL");
    if (no_alloc && upd->U > star::kScratchMaxUpdates)
        return set_err(STAR_ERR_SHAPE, "U=" + std::to_string(upd->U) + " is more than the " +
                                           std::to_string(star::kScratchMaxUpdates) +
                                           " updates a call of star_group_update_noalloc accepts");
    if (update && !hp) return set_err(STAR_ERR_NULL, "hyper-parameter struct is NULL");
    if (!update && !norms_out) return set_err(STAR_ERR_NULL, "norms_out is NULL");
    if (!grad_rows) return set_err(STAR_ERR_NULL, "grad_rows is NULL");
    if (P < 0) return set_err(STAR_ERR_SHAPE, "P is negative");
    if (update && P > 0 && (!params || !momentum)) return set_err(STAR_ERR_NULL, "params or momentum is NULL");
    if (grad_dtype != STAR_F32 && grad_dtype != STAR_BF16) return set_err(STAR_ERR_DTYPE, "unknown gradient dtype");
    if (publish && publish_dtype != STAR_F32 && publish_dtype != STAR_BF16)
        return set_err(STAR_ERR_DTYPE, "unknown publish dtype");

    const bool want_norms = norms_out != nullptr;
    star::Plan plan;
    std::string msg;
    st = star::build_plan(W, upd, update ? hp : nullptr, wmode, want_norms, &plan, &msg);
    if (st != STAR_OK) return set_err(st, msg);
    const int U = plan.U, Wc = plan.Wc;
    if (P > 0)
        for (int k = 0; k < Wc; ++k)
            if (!grad_rows[plan.row_of[k]]) return set_err(STAR_ERR_NULL, "a gradient row used by a group is NULL");
    if (U == 0) return STAR_OK;

    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    if (P == 0) {
        if (want_norms) STAR_HIP(star::launch_fill(norms_out, U, 0.0f, stream));
        return STAR_OK;
    }

    int device = 0, num_cu = 1;
    st = device_info(&device, &num_cu);
    if (st != STAR_OK) return st;
    const int grid_cap = star::kGridCap;

    const Launch how = decide(plan, grad_dtype, update, want_norms, P, opt);
    if (how.split_norms) {
        // the rows do not change during the call, so the norms may come first
        const star_options direct = {STAR_KERNEL_SEQ, 0, opt.queue_min};   // the step-by-step kernel's sums are direct
        st = run(false, nullptr, nullptr, grad_rows, grad_dtype, P, W, upd, nullptr, hp->wmode, norms_out, nullptr, 0,
                 &direct, hip_stream, no_alloc);
        if (st != STAR_OK) return st;
        return run(true, params, momentum, grad_rows, grad_dtype, P, W, upd, hp, 0, nullptr, publish, publish_dtype,
                   options, hip_stream, no_alloc);
    }
    const star::Route route = how.route;
    const int Wp = how.Wp;

    // rows in compact order; padding rows repeat the last row with zero coefficients
    star::RowPtrs rows;
    bool vec_ok = !update || (aligned16(params) && aligned16(momentum) && aligned16(publish));
    for (int k = 0; k < STAR_MAX_WORKERS; ++k) {
        rows.p[k] = grad_rows[plan.row_of[std::min(k, Wc - 1)]];
        if (k < Wc && !aligned16(rows.p[k])) vec_ok = false;
    }

    // tables of the step-by-step kernel: in the kernel arguments when small and the whole stream fits in
    // one launch (a launch reads the inline tables from entry 0), else staged through the slot
    const bool seq_inline = route != star::Route::Affine && how.seq_inline;
    star::InlineTables inl;
    if (seq_inline) {
        for (int u = 0; u < U; ++u) {
            for (int k = 0; k < Wp; ++k) inl.coef[u * Wp + k] = k < Wc ? (float)plan.coef[(size_t)u * Wc + k] : 0.0f;
            inl.lr[u] = (float)plan.lr[u];
            inl.mask[u] = plan.mask[u];
        }
    }
    const bool need_seq_tables = route != star::Route::Affine && !seq_inline;
    const bool need_gram_coef = want_norms && route == star::Route::Affine;

    // a workspace slot only when something has to live in it (tables, norm partials)
    const TableLayout lay = table_layout(U, Wp);
    const bool want_queue = how.want_queue;
    const bool need_slot = need_seq_tables || need_gram_coef || want_norms || want_queue;
    std::unique_lock<std::mutex> lock(g_mu, std::defer_lock);
    Slot* slot = nullptr;
    std::vector<char> host_tables;   // no_alloc: the tables are built here and travel in kernel arguments
    char *h = nullptr, *d = nullptr;
    double* partials = nullptr;
    star::TileQueue* queue = nullptr;
    if (need_slot && no_alloc) {
        const size_t need_partials = want_norms ? partial_doubles_needed(Wp, U, grid_cap) : 0;
        if (lay.total > star::kScratchTableBytes || need_partials > star::kScratchPartialDoubles)
            return set_err(STAR_ERR_SHAPE, "the call needs more workspace than the fixed array of "
                                           "star_group_update_noalloc holds");
        void* base = nullptr;
        STAR_HIP(star::scratch_address(&base));
        queue = static_cast<star::TileQueue*>(base);
        d = static_cast<char*>(base) + 256;
        partials = reinterpret_cast<double*>(d + star::kScratchTableBytes);
        host_tables.assign(lay.total, 0);
        h = host_tables.data();
        // the array keeps what the last call left: the queue must start at zero (a call that failed
        // half-way may not have put it back); tables and partials are written before they are read
        STAR_HIP(star::launch_queue_clear(queue, stream));
    } else if (need_slot) {
        lock.lock();
        st = acquire_slot(device, (need_seq_tables || need_gram_coef) ? lay.total : 0,
                          want_norms ? partial_doubles_needed(Wp, U, grid_cap) : 0, &slot);
        if (st != STAR_OK) return st;
        h = static_cast<char*>(slot->host);
        d = static_cast<char*>(slot->dev);
        partials = slot->partials;
        queue = slot->queue;
    }
    SlotRelease release{slot, stream};
    if (need_seq_tables) {
        float* c32 = reinterpret_cast<float*>(h + lay.coef32);
        float* l32 = reinterpret_cast<float*>(h + lay.lr32);
        uint32_t* mk = reinterpret_cast<uint32_t*>(h + lay.mask);
        for (int u = 0; u < U; ++u) {
            for (int k = 0; k < Wp; ++k) c32[(size_t)u * Wp + k] = k < Wc ? (float)plan.coef[(size_t)u * Wc + k] : 0.0f;
            l32[u] = (float)plan.lr[u];
            mk[u] = plan.mask[u];
        }
    }
    if (need_gram_coef) {
        double* c64 = reinterpret_cast<double*>(h + lay.coef64);
        for (int u = 0; u < U; ++u)
            for (int k = 0; k < Wp; ++k) c64[(size_t)u * Wp + k] = k < Wc ? plan.coef[(size_t)u * Wc + k] : 0.0;
    }
    // The step-by-step tables are read by every workgroup and are copied to the device.  The Gram
    // coefficients (a few KB, read once, by the one small kernel that ends the call) are read where they
    // are, in the slot's pinned host buffer: no copy engine in the stream.
    const double* gram_coef = nullptr;
    if (no_alloc) {
        if (need_seq_tables) STAR_HIP(star::launch_upload(d, h, lay.coef64, stream));
        if (need_gram_coef) {
            STAR_HIP(star::launch_upload(d + lay.coef64, h + lay.coef64, sizeof(double) * (size_t)U * Wp, stream));
            gram_coef = reinterpret_cast<const double*>(d + lay.coef64);
        }
    } else {
        if (need_seq_tables) STAR_HIP(hipMemcpyAsync(d, h, lay.coef64, hipMemcpyHostToDevice, stream));
        if (slot && slot->host_dev)
            gram_coef = reinterpret_cast<const double*>(static_cast<char*>(slot->host_dev) + lay.coef64);
    }

    hipError_t e = hipSuccess;
    int grid = 0;
    // collapsed update (with or without the Gram matrix)
    if (route == star::Route::Affine) {
        const bool gram = want_norms;
        if (update || gram) {
            star::AffArgs a;
            a.params = params;
            a.momentum = momentum;
            a.rows = rows;
            std::memset(&a.cf, 0, sizeof a.cf);
            if (update) {
                a.cf.dp = (float)(plan.M[0] - 1.0);
                a.cf.m01 = (float)plan.M[1];
                a.cf.m10 = (float)plan.M[2];
                a.cf.m11 = (float)plan.M[3];
                for (int k = 0; k < Wc; ++k) {
                    a.cf.b0[k] = (float)plan.B[k];
                    a.cf.b1[k] = (float)plan.B[Wc + k];
                }
            }
            a.P = P;
            a.vec_ok = vec_ok ? 1 : 0;
            a.publish = update ? publish : nullptr;
            a.publish_dtype = publish_dtype;
            a.partials = partials;
            a.queue = want_queue ? queue : nullptr;
            // (fp32 buffers that are not 16-byte aligned go one element per lane, and a matrix-core tile of 256
            // elements costs what one of 1024 does: up to 16 rows the vector-register form is faster there,
            // 32 Mi elements, 16 rows: 0.66 against 1.10 ms; with bf16 rows it is the other way round)
            const bool mfma = how.mfma && !(!vec_ok && grad_dtype == STAR_F32 && Wp <= star::kMaxValuGramW);
            if (mfma) a.queue = queue;   // that kernel always takes its tiles from the queue
            e = mfma ? star::launch_affine_mfma(Wp, grad_dtype, update, a, num_cu, grid_cap, &grid, stream)
                     : star::launch_affine(Wp, grad_dtype, update, gram, a, num_cu, grid_cap, &grid, stream);
            if (e != hipSuccess) return hip_fail(e, "launch of the collapsed update kernel");
            if (gram) {
                const int ng = Wp * (Wp + 1) / 2;
                double* gamma = partials + (size_t)ng * grid;
                e = star::launch_reduce(partials, ng, grid, gamma, nullptr, stream);
                if (e != hipSuccess) return hip_fail(e, "launch of the Gram reduction");
                e = star::launch_gram_norms(gamma, gram_coef, U, Wp, norms_out, stream);
                if (e != hipSuccess) return hip_fail(e, "launch of the norm kernel");
            }
        }
    }
    // step-by-step evaluation
    if (route == star::Route::Seq) {
        const bool seq_update = update;
        const int umax = how.umax;
        star::AffCoef cf;
        std::memset(&cf, 0, sizeof cf);
        if (how.collapsed_in_seq) {
            cf.dp = (float)(plan.M[0] - 1.0);
            cf.m01 = (float)plan.M[1];
            cf.m10 = (float)plan.M[2];
            cf.m11 = (float)plan.M[3];
            for (int k = 0; k < Wc; ++k) {
                cf.b0[k] = (float)plan.B[k];
                cf.b1[k] = (float)plan.B[Wc + k];
            }
        }
        for (int u0 = 0; u0 < U; u0 += umax) {
            const int n = std::min(umax, U - u0);
            star::SeqArgs a;
            a.params = params;
            a.momentum = momentum;
            a.rows = rows;
            a.coef = seq_inline ? nullptr : reinterpret_cast<const float*>(d + lay.coef32) + (size_t)u0 * Wp;
            a.lr = seq_inline ? nullptr : reinterpret_cast<const float*>(d + lay.lr32) + u0;
            a.mask = seq_inline ? nullptr : reinterpret_cast<const uint32_t*>(d + lay.mask) + u0;
            a.inl = &inl;
            a.cf = how.collapsed_in_seq ? &cf : nullptr;
            a.U = n;
            a.mu = (float)plan.mu;
            a.wd = (float)plan.wd;
            a.P = P;
            a.vec_ok = vec_ok ? 1 : 0;
            a.publish = (seq_update && u0 + n == U) ? publish : nullptr;   // the last launch holds the final params
            a.publish_dtype = publish_dtype;
            a.partials = partials;
            a.queue = want_queue ? queue : nullptr;
            e = star::launch_seq(Wp, grad_dtype, seq_update, want_norms, a, num_cu, grid_cap, &grid, stream);
            if (e != hipSuccess) return hip_fail(e, "launch of the step-by-step kernel");
            if (want_norms) {
                e = star::launch_reduce(partials, n, grid, nullptr, norms_out + u0, stream);
                if (e != hipSuccess) return hip_fail(e, "launch of the norm reduction");
            }
        }
    }
    return STAR_OK;
}

// Body of star_group_reduce.
star_status run_reduce(void* const* out_rows, int out_dtype, const void* const* grad_rows, int grad_dtype, int64_t P,
                       int32_t W, const star_updates* upd, int32_t wmode, float* norms_out,
                       const star_options* options, void* hip_stream) {
    g_err.clear();
    Opts opt;
    star_status st = resolve_options(options, &opt);
    if (st != STAR_OK) return st;
    if (!upd) return set_err(STAR_ERR_NULL, "updates struct is NULL");
    if (!grad_rows) return set_err(STAR_ERR_NULL, "grad_rows is NULL");
    if (!out_rows && upd->U > 0) return set_err(STAR_ERR_NULL, "out_rows is NULL");
    if (P < 0) return set_err(STAR_ERR_SHAPE, "P is negative");
    if (grad_dtype != STAR_F32 && grad_dtype != STAR_BF16) return set_err(STAR_ERR_DTYPE, "unknown gradient dtype");
    if (out_dtype != STAR_F32 && out_dtype != STAR_BF16) return set_err(STAR_ERR_DTYPE, "unknown output dtype");
    const bool want_norms = norms_out != nullptr;
    star::Plan plan;
    std::string msg;
    st = star::build_plan(W, upd, nullptr, wmode, want_norms, &plan, &msg);
    if (st != STAR_OK) return set_err(st, msg);
    const int U = plan.U, Wc = plan.Wc;
    if (P > 0) {
        for (int k = 0; k < Wc; ++k)
            if (!grad_rows[plan.row_of[k]]) return set_err(STAR_ERR_NULL, "a gradient row used by a group is NULL");
        for (int u = 0; u < U; ++u)
            if (!out_rows[u]) return set_err(STAR_ERR_NULL, "an output row is NULL");
    }
    if (U == 0) return STAR_OK;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    if (P == 0) {
        if (want_norms) STAR_HIP(star::launch_fill(norms_out, U, 0.0f, stream));
        return STAR_OK;
    }
    int device = 0, num_cu = 1;
    st = device_info(&device, &num_cu);
    if (st != STAR_OK) return st;
    const int grid_cap = star::kGridCap;
    const int Wp = star::padded_rows(Wc);
    star::RowPtrs rows;
    bool vec_ok = true;
    for (int k = 0; k < STAR_MAX_WORKERS; ++k) {
        rows.p[k] = grad_rows[plan.row_of[std::min(k, Wc - 1)]];
        if (k < Wc && !aligned16(rows.p[k])) vec_ok = false;
    }
    for (int u = 0; u < U; ++u)
        if (!aligned16(out_rows[u])) vec_ok = false;

    std::lock_guard<std::mutex> lock(g_mu);
    const TableLayout lay = table_layout(U, Wp);
    Slot* slot = nullptr;
    st = acquire_slot(device, lay.total, want_norms ? partial_doubles_needed(Wp, U, grid_cap) : 0, &slot);
    if (st != STAR_OK) return st;
    SlotRelease release{slot, stream};
    char* h = static_cast<char*>(slot->host);
    char* d = static_cast<char*>(slot->dev);
    // inline tables only when one launch takes the whole stream: a launch reads them from entry 0
    const bool use_inline = star::tables_fit_inline(U, Wp) && U <= star::reduce_max_updates(Wp, want_norms);
    star::InlineTables inl;
    if (use_inline) {
        for (int u = 0; u < U; ++u) {
            for (int k = 0; k < Wp; ++k) inl.coef[u * Wp + k] = k < Wc ? (float)plan.coef[(size_t)u * Wc + k] : 0.0f;
            inl.mask[u] = plan.mask[u];
            inl.out[u] = out_rows[u];
        }
    } else {
        float* c32 = reinterpret_cast<float*>(h + lay.coef32);
        uint32_t* mk = reinterpret_cast<uint32_t*>(h + lay.mask);
        void** op = reinterpret_cast<void**>(h + lay.outptr);
        for (int u = 0; u < U; ++u) {
            for (int k = 0; k < Wp; ++k) c32[(size_t)u * Wp + k] = k < Wc ? (float)plan.coef[(size_t)u * Wc + k] : 0.0f;
            mk[u] = plan.mask[u];
            op[u] = out_rows[u];
        }
        STAR_HIP(hipMemcpyAsync(d, h, lay.total, hipMemcpyHostToDevice, stream));
    }
    const int umax = star::reduce_max_updates(Wp, want_norms);
    for (int u0 = 0; u0 < U; u0 += umax) {
        const int n = std::min(umax, U - u0);
        star::ReduceArgs a;
        a.rows = rows;
        a.coef = use_inline ? nullptr : reinterpret_cast<const float*>(d + lay.coef32) + (size_t)u0 * Wp;
        a.mask = use_inline ? nullptr : reinterpret_cast<const uint32_t*>(d + lay.mask) + u0;
        a.out = use_inline ? nullptr : reinterpret_cast<void* const*>(d + lay.outptr) + u0;
        a.inl = &inl;
        a.U = n;
        a.out_dtype = out_dtype;
        a.P = P;
        a.vec_ok = vec_ok ? 1 : 0;
        a.norms = want_norms ? 1 : 0;
        a.partials = slot->partials;
        a.queue = P >= queue_min_for(opt, grad_dtype, Wc, false, true, false, false, n) ? slot->queue : nullptr;
        int grid = 0;
        hipError_t e = star::launch_group_reduce(Wp, grad_dtype, a, num_cu, grid_cap, &grid, stream);
        if (e != hipSuccess) return hip_fail(e, "launch of the aggregation kernel");
        if (want_norms) {
            e = star::launch_reduce(slot->partials, n, grid, nullptr, norms_out + u0, stream);
            if (e != hipSuccess) return hip_fail(e, "launch of the norm reduction");
        }
    }
    return STAR_OK;
}

// Body of star_group_gram.
star_status run_gram(const void* const* grad_rows, int grad_dtype, int64_t P, int32_t W, double* gram_out,
                     const star_options* options, void* hip_stream) {
    g_err.clear();
    Opts opt;
    star_status st = resolve_options(options, &opt);
    if (st != STAR_OK) return st;
    if (!grad_rows || !gram_out) return set_err(STAR_ERR_NULL, "grad_rows or gram_out is NULL");
    if (P < 0) return set_err(STAR_ERR_SHAPE, "P is negative");
    if (W < 1 || W > star::kMaxGramW) return set_err(STAR_ERR_SHAPE, "the Gram matrix is built for 1 to 32 rows");
    if (grad_dtype != STAR_F32 && grad_dtype != STAR_BF16) return set_err(STAR_ERR_DTYPE, "unknown gradient dtype");
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    if (P == 0) {
        hipError_t e0 = star::launch_gram_unpack(nullptr, W, W, gram_out, stream);
        return e0 == hipSuccess ? STAR_OK : hip_fail(e0, "launch of the Gram unpack kernel");
    }
    star::AffArgs a;
    std::memset(&a, 0, sizeof a);
    bool vec_ok = true;
    for (int k = 0; k < STAR_MAX_WORKERS; ++k) {
        a.rows.p[k] = grad_rows[std::min(k, W - 1)];
        if (k < W && !a.rows.p[k]) return set_err(STAR_ERR_NULL, "a gradient row is NULL");
        if (k < W && !aligned16(a.rows.p[k])) vec_ok = false;
    }
    int device = 0, num_cu = 1;
    st = device_info(&device, &num_cu);
    if (st != STAR_OK) return st;
    std::lock_guard<std::mutex> lock(g_mu);
    Slot* slot = nullptr;
    st = acquire_slot(device, 0, partial_doubles_needed(star::padded_rows(W), 1, star::kGridCap), &slot);
    if (st != STAR_OK) return st;
    SlotRelease release{slot, stream};
    a.P = P;
    a.vec_ok = vec_ok ? 1 : 0;
    a.partials = slot->partials;
    int grid = 0;
    const int Wp = star::padded_rows(W);   // rows beyond W repeat the last one; their entries are not copied out
    const bool mfma = gram_on_matrix_cores(Wp, grad_dtype, opt.kernel, false, P);
    a.queue = (mfma || P >= queue_min_for(opt, grad_dtype, W, false)) ? slot->queue : nullptr;
    hipError_t e = mfma ? star::launch_affine_mfma(Wp, grad_dtype, false, a, num_cu, star::kGridCap, &grid, stream)
                        : star::launch_affine(Wp, grad_dtype, false, true, a, num_cu, star::kGridCap, &grid, stream);
    if (e != hipSuccess) return hip_fail(e, "launch of the Gram kernel");
    const int ng = Wp * (Wp + 1) / 2;
    double* gamma = slot->partials + (size_t)ng * grid;
    e = star::launch_reduce(slot->partials, ng, grid, gamma, nullptr, stream);
    if (e != hipSuccess) return hip_fail(e, "launch of the Gram reduction");
    e = star::launch_gram_unpack(gamma, Wp, W, gram_out, stream);
    if (e != hipSuccess) return hip_fail(e, "launch of the Gram unpack kernel");
    return STAR_OK;
}

}  // namespace

extern "C" {

star_status star_group_update(float* params, float* momentum, const void* const* grad_rows, star_dtype grad_dtype,
                              int64_t P, int32_t W, const star_updates* upd, const star_hparams* hp,
                              float* norms_out, void* hip_stream) {
    return run(true, params, momentum, grad_rows, (int)grad_dtype, P, W, upd, hp, 0, norms_out, nullptr, 0, nullptr,
               hip_stream);
}

star_status star_group_update_noalloc(float* params, float* momentum, const void* const* grad_rows,
                                      star_dtype grad_dtype, int64_t P, int32_t W, const star_updates* upd,
                                      const star_hparams* hp, float* norms_out, void* hip_stream) {
    return run(true, params, momentum, grad_rows, (int)grad_dtype, P, W, upd, hp, 0, norms_out, nullptr, 0, nullptr,
               hip_stream, true);
}

star_status star_group_update_publish(float* params, float* momentum, const void* const* grad_rows,
                                      star_dtype grad_dtype, int64_t P, int32_t W, const star_updates* upd,
                                      const star_hparams* hp, float* norms_out, void* publish,
                                      star_dtype publish_dtype, void* hip_stream) {
    if (!publish && P > 0) return set_err(STAR_ERR_NULL, "publish buffer is NULL");
    return run(true, params, momentum, grad_rows, (int)grad_dtype, P, W, upd, hp, 0, norms_out, publish,
               (int)publish_dtype, nullptr, hip_stream);
}

star_status star_group_update_opt(float* params, float* momentum, const void* const* grad_rows, star_dtype grad_dtype,
                                  int64_t P, int32_t W, const star_updates* upd, const star_hparams* hp,
                                  float* norms_out, void* publish, star_dtype publish_dtype, const star_options* opt,
                                  void* hip_stream) {
    return run(true, params, momentum, grad_rows, (int)grad_dtype, P, W, upd, hp, 0, norms_out, publish,
               (int)publish_dtype, opt, hip_stream);
}

star_status star_group_norms(const void* const* grad_rows, star_dtype grad_dtype, int64_t P, int32_t W,
                             const star_updates* upd, int32_t wmode, float* norms_out, void* hip_stream) {
    return run(false, nullptr, nullptr, grad_rows, (int)grad_dtype, P, W, upd, nullptr, wmode, norms_out, nullptr, 0,
               nullptr, hip_stream);
}

star_status star_group_norms_opt(const void* const* grad_rows, star_dtype grad_dtype, int64_t P, int32_t W,
                                 const star_updates* upd, int32_t wmode, float* norms_out, const star_options* opt,
                                 void* hip_stream) {
    return run(false, nullptr, nullptr, grad_rows, (int)grad_dtype, P, W, upd, nullptr, wmode, norms_out, nullptr, 0,
               opt, hip_stream);
}

star_status star_group_reduce(void* const* out_rows, star_dtype out_dtype, const void* const* grad_rows,
                              star_dtype grad_dtype, int64_t P, int32_t W, const star_updates* upd, int32_t wmode,
                              float* norms_out, void* hip_stream) {
    return run_reduce(out_rows, (int)out_dtype, grad_rows, (int)grad_dtype, P, W, upd, wmode, norms_out, nullptr,
                      hip_stream);
}

star_status star_group_reduce_opt(void* const* out_rows, star_dtype out_dtype, const void* const* grad_rows,
                                  star_dtype grad_dtype, int64_t P, int32_t W, const star_updates* upd, int32_t wmode,
                                  float* norms_out, const star_options* opt, void* hip_stream) {
    return run_reduce(out_rows, (int)out_dtype, grad_rows, (int)grad_dtype, P, W, upd, wmode, norms_out, opt,
                      hip_stream);
}

star_status star_group_gram(const void* const* grad_rows, star_dtype grad_dtype, int64_t P, int32_t W,
                            double* gram_out, void* hip_stream) {
    return run_gram(grad_rows, (int)grad_dtype, P, W, gram_out, nullptr, hip_stream);
}

star_status star_group_gram_opt(const void* const* grad_rows, star_dtype grad_dtype, int64_t P, int32_t W,
                                double* gram_out, const star_options* opt, void* hip_stream) {
    return run_gram(grad_rows, (int)grad_dtype, P, W, gram_out, opt, hip_stream);
}

star_status star_noise_scale(int32_t W, const double* gram, double batch_per_worker, double* grad_sq,
                             double* trace_cov, double* noise_scale) {
    g_err.clear();
    if (!gram) return set_err(STAR_ERR_NULL, "gram is NULL");
    if (W < 2 || W > STAR_MAX_WORKERS) return set_err(STAR_ERR_SHAPE, "needs between 2 and 32 workers");
    if (!(batch_per_worker > 0.0) || !std::isfinite(batch_per_worker))
        return set_err(STAR_ERR_HPARAM, "batch size per worker must be positive");
    // S = mean_w |g_w|^2 ;  n2 = |mean_w g_w|^2 = (1/W^2) sum_ab Gamma_ab
    double S = 0.0, total = 0.0;
    for (int a = 0; a < W; ++a) {
        S += gram[(size_t)a * W + a];
        for (int b = 0; b < W; ++b) total += gram[(size_t)a * W + b];
    }
    S /= W;
    const double n2 = total / ((double)W * W);
    // E S = |G|^2 + tr/b,  E n2 = |G|^2 + tr/(W b)   ->   two unbiased estimates
    const double tr = batch_per_worker * (S - n2) * W / (W - 1.0);
    const double g2 = (W * n2 - S) / (W - 1.0);
    if (grad_sq) *grad_sq = g2;
    if (trace_cov) *trace_cov = tr;
    if (noise_scale) *noise_scale = tr / g2;
    return STAR_OK;
}

star_status star_plan_affine(int32_t W, const star_updates* upd, const star_hparams* hp, double M[4], double* B) {
    g_err.clear();
    if (!hp || !M || !B) return set_err(STAR_ERR_NULL, "hp, M or B is NULL");
    star::Plan plan;
    std::string msg;
    star_status st = star::build_plan(W, upd, hp, 0, false, &plan, &msg);
    if (st != STAR_OK) return set_err(st, msg);
    for (int i = 0; i < 4; ++i) M[i] = plan.M[i];
    for (int w = 0; w < 2 * W; ++w) B[w] = 0.0;
    for (int k = 0; k < plan.Wc; ++k) {
        B[plan.row_of[k]] = plan.B[k];
        B[W + plan.row_of[k]] = plan.B[plan.Wc + k];
    }
    return STAR_OK;
}

star_status star_plan_choice(int64_t P, int32_t W, star_dtype grad_dtype, const star_updates* upd,
                             const star_hparams* hp, int32_t update, int32_t want_norms, const star_options* options,
                             star_plan_info* info) {
    g_err.clear();
    Opts opt;
    star_status st = resolve_options(options, &opt);
    if (st != STAR_OK) return st;
    if (!info) return set_err(STAR_ERR_NULL, "info is NULL");
    if (update && !hp) return set_err(STAR_ERR_NULL, "hp is NULL");
    if (P < 0) return set_err(STAR_ERR_SHAPE, "P is negative");
    if (grad_dtype != STAR_F32 && grad_dtype != STAR_BF16) return set_err(STAR_ERR_DTYPE, "unknown gradient dtype");
    if (!update && !want_norms) return set_err(STAR_ERR_NULL, "neither the update nor the norms are asked for");
    star::Plan plan;
    std::string msg;
    st = star::build_plan(W, upd, update ? hp : nullptr, hp ? hp->wmode : 0, want_norms != 0, &plan, &msg);
    if (st != STAR_OK) return set_err(st, msg);
    Launch how = decide(plan, (int)grad_dtype, update != 0, want_norms != 0, P, opt);
    if (how.split_norms) {   // the update as if without norms, plus the launches of the direct norm pass
        Opts direct = opt;
        direct.kernel = STAR_KERNEL_SEQ;
        const Launch norms = decide(plan, (int)grad_dtype, false, true, P, direct);
        how = decide(plan, (int)grad_dtype, true, false, P, opt);
        how.launches += norms.launches;
        how.finishing += norms.finishing;
    }
    std::memset(info, 0, sizeof *info);
    info->kernel = how.route == star::Route::Seq ? STAR_KERNEL_SEQ : (how.mfma ? STAR_KERNEL_AFFINE_MFMA : STAR_KERNEL_AFFINE);
    info->grad_dtype = (int32_t)grad_dtype;
    info->rows_used = plan.Wc;
    info->rows_padded = how.Wp;
    info->queue_order = how.queue_order ? 1 : 0;
    info->launches = how.launches;
    info->finishing_launches = how.finishing;
    info->tables_inline = how.route == star::Route::Seq ? (how.seq_inline ? 1 : 0) : (want_norms ? 0 : 1);
    info->collapsed_update = (update && (how.route == star::Route::Affine || how.collapsed_in_seq)) ? 1 : 0;
    info->fma_seq = plan.fma_seq;
    info->fma_affine = plan.fma_affine;
    return STAR_OK;
}

star_status star_plan_claims(int32_t workgroups, int32_t tiles_per_claim, int64_t* first_tile, int32_t* count,
                             int64_t* base) {
    g_err.clear();
    if (workgroups < 1) return set_err(STAR_ERR_SHAPE, "workgroups must be positive");
    if (tiles_per_claim < 1) return set_err(STAR_ERR_SHAPE, "tiles_per_claim must be positive");
    if (!first_tile || !count || !base) return set_err(STAR_ERR_NULL, "an output pointer is NULL");
    for (int32_t b = 0; b < workgroups; ++b) {
        const star::FirstClaim f = star::first_claim_of(b, workgroups, tiles_per_claim);
        first_tile[b] = f.t0;
        count[b] = f.n;
        *base = (int64_t)f.base;
    }
    return STAR_OK;
}

star_status star_plan_even_split(int32_t workgroups, int64_t tiles, int64_t* first_tile, int32_t* count) {
    g_err.clear();
    if (workgroups < 1) return set_err(STAR_ERR_SHAPE, "workgroups must be positive");
    if (tiles < 0) return set_err(STAR_ERR_SHAPE, "tiles is negative");
    if (!first_tile || !count) return set_err(STAR_ERR_NULL, "an output pointer is NULL");
    for (int32_t b = 0; b < workgroups; ++b) {
        const star::FirstClaim f = star::first_claim_of(b, workgroups, -1, tiles);
        first_tile[b] = f.t0;
        count[b] = f.n;
    }
    return STAR_OK;
}

size_t star_workspace_bytes(int64_t P, int32_t W, int32_t U) {
    if (P <= 0 || W < 1 || W > STAR_MAX_WORKERS || U <= 0) return 0;
    const int Wp = star::padded_rows(W);
    const int grid_cap = star::kGridCap;
    return std::max<size_t>(table_layout(U, Wp).total, 64 * 1024) +
           sizeof(double) * partial_doubles_needed(Wp, U, grid_cap) + 256 /* tile queue */;
}

const char* star_last_error(void) { return g_err.c_str(); }

const char* star_version(void) { return "libstar 0.1 (gfx950)"; }

void star_shutdown(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    for (Slot& s : g_slots) free_slot(s);
    g_next_slot = 0;
}

}  // extern "C"
