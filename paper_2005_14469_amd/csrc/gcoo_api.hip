// Host side of the C ABI declared in include/gcoo.h: argument checks, device-buffer layout,
// kernel selection and launches.  No compute happens on the host.
#include "gcoo.h"

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>

#include <atomic>
#include <mutex>

#include "gcoo_build_kernels.hpp"
#include "gcoo_sched.hpp"
#include "gcoo_sched_build.hpp"
#include "gcoo_share.hpp"
#include "gcoo_share_build.hpp"
#include "gcoo_spdm_launch.hpp"
#include "gcoo_spdm_lds_kernel.hpp"

namespace {

thread_local std::string g_hip_error;

int hip_fail(hipError_t e, const char* what)
{
    g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return GCOO_EHIP;
}

#define HIP_TRY(expr)                                  \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) return hip_fail(e_, #expr); \
    } while (0)

constexpr size_t kAlign = 256;
size_t al(size_t bytes) { return (bytes + kAlign - 1) / kAlign * kAlign; }

// Device memory for gcoo_dense_nnz(), which is handed no device buffer: kDenseSlots counters per
// device, addressed through hipGetSymbolAddress.  Every call takes the next slot (round robin), so
// calls that overlap on one device - other streams, other host threads - count into different
// words as long as fewer than kDenseSlots of them are in flight at once.
constexpr unsigned kDenseSlots = 256;
__device__ unsigned long long g_dense_total[kDenseSlots];
std::atomic<unsigned> g_dense_next{0};

// Scratch of gcoo_from_csr_device_static(), the conversion for callers that may not allocate device
// memory: the second buffer of the per-group radix sort (3 arrays of nnz words) and the counter from
// which the share schedule's streams take their place.  One copy per device, held until the process
// ends.  Host code never uses the array's name as an address: static_scratch() asks the runtime for
// the address on the current device, once per device, and everything goes through that pointer.
constexpr int64_t kStaticMaxNnz = 2 * 1024 * 1024;
constexpr size_t kStaticSortBytes = (size_t)kStaticMaxNnz * 4;        // each of the three arrays, a multiple of 256
constexpr size_t kStaticScratchBytes = 3 * kStaticSortBytes + 256;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
unsigned char* g_static_ptr[kMaxDevices] = {};

int static_scratch(unsigned char** out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return GCOO_EINVAL;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        unsigned char* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(g_static_scratch)));
        if (!ptr) return GCOO_EHIP;
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return GCOO_OK;
}

// Carve-up of the caller's device buffer.  Offsets depend on (m, nnz, g) only.
struct Layout {
    size_t values, rows, cols, gIdxes, nnzPerGroup;        // the five arrays of the format
    size_t sched_hdr, sched;                               // run schedule of the register kernel
    size_t order;                                          // groups by falling size, then those sizes (matrices of few groups)
    size_t share_ucols, share_ucount, share_hdr, share_blocks, share_sbase, share_alloc;   // share schedule (may be empty)
    size_t tmp_cols, tmp_rows, tmp_vals;                   // conversion scratch (second sort buffer)
    size_t in_row_ptr, in_cols, in_vals;                   // staging of a host CSR input
    size_t counter;                                        // device words: nnz (8 bytes), largest group (8), column-out-of-range flag (4)
    size_t persistent;                                     // bytes up to here stay in use after the conversion
    // offsets from here on are relative to the scratch area: the caller's buffer from `persistent` on, or the
    // library's static scratch
    size_t blk;                                            // dense input: entries per (group, column block)
    size_t total;
};

// Column windows of the run schedule: bands of kWindowCols columns (a band of B of that many
// rows by one column tile stays in the L2 of the XCD working on the tile), at most kMaxWindows,
// and fewer when the matrix has so many groups that the per-window headers would dominate.
constexpr int64_t kWindowCols = 2048;

void pick_windows(int64_t k, int64_t g, int32_t* nw, int32_t* window_cols)
{
    const int64_t wc = kWindowCols;
    int64_t n = (k + wc - 1) / wc;
    const int64_t cap_groups = g > 0 ? (int64_t(1) << 22) / g : gcoo::kMaxWindows;
    int64_t cap = gcoo::kMaxWindows;
    if (cap_groups < cap) cap = cap_groups;
    if (cap < 1) cap = 1;
    if (n > cap) n = cap;
    if (n < 1) n = 1;
    *nw = (int32_t)n;
    *window_cols = (int32_t)((k + n - 1) / n > 0 ? (k + n - 1) / n : 1);
}

// Column blocks of the dense-input kernels: kDenseThreads*vw columns each.  The block table in the
// layout is sized for vw = 1 (the most blocks).
int64_t dense_blocks(int64_t k, int vw = 1) { return (k + gcoo::kDenseThreads * vw - 1) / (gcoo::kDenseThreads * vw); }

// 4 when rows of A can be read with 16-byte loads, else 1.
int dense_vec_width(const float* A, int64_t lda, int64_t k)
{
    return (k % 4 == 0 && lda % 4 == 0 && reinterpret_cast<uintptr_t>(A) % 16 == 0) ? 4 : 1;
}

// The share schedule costs conversion time (0.04 ms at 320 000 entries) and memory, so it is built only where
// the workgroup-shared kernel is the one gcoo_spdm() will pick.  Measured on MI355X with uniform random square
// matrices (n = 4000 .. 14000, density 0.1 % .. 10 %, N = n), against the register kernel at its best group height:
// the workgroup-shared kernel wins from 3500 columns on at 0.8 % density or more (n = 8000: by 10 .. 30 % between
// 1 % and 5 %; n = 4000, 2 %: 12 %) and from 9000 columns on already at 0.4 % (n = 10000, 0.5 %: 1.0 against 1.23 ms; n = 14000: 1.7 .. 2.3x between 0.5 %
// and 2 %); at n = 8000 and 0.5 % the two kernels are level and the schedule's cost decides for the register
// kernel.  The B tile of a column tile then no longer stays in L2 between the groups that need it, and what
// the register kernel pays per run (a 1 KB segment through the vector cache) costs more than the per-band steps
// of the workgroup-shared kernel.  Above 6 % the register kernel, which reuses a fetched segment along runs of
// up to eight entries, is ahead (10 %: 2.9 against 3.2 ms at n = 8000); at 0.1 % and at n <= 3000 too.
// gcoo_set_share_policy() overrides the choice.
std::atomic<int> g_share_policy{GCOO_SHARE_AUTO};
// A conversion lays its buffer out more than once (size check, handle, inner handle): it reads the policy once, when
// it starts, and every layout of that call uses that value, whatever another thread sets meanwhile.
thread_local int t_policy_of_call = -1;
struct PolicyOfCall {
    bool outermost;
    PolicyOfCall() : outermost(t_policy_of_call < 0) { if (outermost) t_policy_of_call = g_share_policy.load(std::memory_order_relaxed); }
    ~PolicyOfCall() { if (outermost) t_policy_of_call = -1; }
};
int share_policy_now() { return t_policy_of_call >= 0 ? t_policy_of_call : g_share_policy.load(std::memory_order_relaxed); }

bool share_schedule_possible(int64_t m, int64_t k, int64_t nnz, int32_t p)
{
    return p <= gcoo::kShareMaxP && k <= gcoo::kShareMaxK && nnz > 0 && m > 0 && k > 0;
}

// (density and shape only: also the rule by which gcoo_default_p() picks a height for that kernel)
bool share_shape_preferred(int64_t m, int64_t k, int64_t nnz)
{
    if (m <= 0 || k <= 0 || nnz <= 0 || k > gcoo::kShareMaxK) return false;
    const double density = (double)nnz / ((double)m * (double)k);
    if (density > 0.06) return false;
    // Whole steps (conversion + product) measured on uniform random square matrices, n = 2000 .. 14000: the wider A, the
    // less of a column tile of B stays in an XCD's L2 between the groups that read it, and the sooner fetching each
    // row once per 8 groups pays for the second schedule that the conversion then builds.
    // (From 9000 columns on it is ahead down to 0.05 % - 8 to 16 % of the step at n = 10000 .. 14000 - but a conversion
    // sees neither the width of B nor how even the rows are, and a second schedule built for nothing costs a matrix
    // with few long rows a third of its step: the limit stays where the gain is large.)
    if (k >= 7000) return density >= 0.0035;
    if (k >= 5500) return density >= 0.008;
    return k >= 3500 && density >= 0.015;
}

bool share_kernel_preferred(int64_t m, int64_t k, int64_t nnz, int32_t p)
{
    return share_schedule_possible(m, k, nnz, p) && share_shape_preferred(m, k, nnz);
}

bool share_schedule_wanted(int64_t m, int64_t k, int64_t nnz, int32_t p)
{
    const int policy = share_policy_now();
    if (policy == GCOO_SHARE_NEVER || !share_schedule_possible(m, k, nnz, p)) return false;
    return policy == GCOO_SHARE_ALWAYS || share_kernel_preferred(m, k, nnz, p);
}

// A workgroup of that kernel runs for a whole (super-group, column tile): how well `items` of them fill
// the 256 compute units, as the fraction of the rounds they need that is work.
double fill_of_rounds(int64_t items)
{
    if (items <= 0) return 0.0;
    const int64_t rounds = (items + 255) / 256;
    return (double)items / (double)(rounds * 256);
}

int64_t share_items(int64_t m, int32_t p, int64_t N)
{
    const int64_t g = (m + p - 1) / p;
    return gcoo::share_super_groups(g) * ((N + 255) / 256);
}

// Group height for the workgroup-shared kernel: taller groups mean fewer rows of B fetched per
// multiply-add, but the workgroups must fill their rounds over the compute units.  The time of a launch goes
// like rounds x (time of a workgroup), and the time of a workgroup like p plus a part that does not depend
// on p (the per-band steps); measured best heights: 42 at 8000 x 8000 (768 workgroups = 3 rounds), 48 at
// 14000 x 14000, 32 at 4000 x 4000 (256 workgroups), which this rule reproduces.
int32_t share_best_p(int64_t m, int64_t N)
{
    int32_t best = 32;
    int64_t best_cost = INT64_MAX;
    for (int32_t p = gcoo::kShareMaxP; p >= 24; --p) {
        const int64_t rounds = (share_items(m, p, N) + 255) / 256;
        const int64_t cost = rounds * (p + 24);
        if (cost < best_cost) { best_cost = cost; best = p; }
    }
    return best;
}

Layout make_layout(int64_t m, int64_t k, int64_t nnz, int64_t g, int32_t p, bool scratch_inside = true)
{
    int32_t nw, wc;
    pick_windows(k, g, &nw, &wc);
    Layout L{};
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at += al(bytes ? bytes : 1); return o; };
    const size_t n4 = (size_t)nnz * 4;
    // the arrays whose size does not depend on nnz come first, so that a dense input can be
    // counted into them before nnz is known
    L.gIdxes = take((size_t)(g + 1) * 4);
    L.nnzPerGroup = take((size_t)g * 4);
    L.counter = take(32);
    L.blk = take((size_t)g * (size_t)dense_blocks(k) * 4);
    L.values = take(n4);
    L.rows = take(n4);
    L.cols = take(n4);
    L.sched_hdr = take((size_t)g * nw * gcoo::kMaxRun * sizeof(gcoo::SchedClass));
    L.sched = take((size_t)gcoo::sched_words(nnz, g, nw) * 4);
    L.order = take(g <= gcoo::kOrderMaxGroups && p <= gcoo::kSchedMaxP ? (size_t)g * 8 : 0);
    const bool share = share_schedule_wanted(m, k, nnz, p);
    const int64_t nQ = gcoo::share_super_groups(g);
    L.share_ucols = take(share ? n4 : 0);
    L.share_ucount = take(share ? (size_t)nQ * 4 : 0);
    L.share_hdr = take(share ? (size_t)gcoo::share_hdr_words(nnz, g) * 4 : 0);
    L.share_blocks = take(share ? (size_t)gcoo::share_stream_blocks(nnz, g, k) * gcoo::kShareBlockWords * 4 : 0);
    L.share_sbase = take(share ? (size_t)nQ * gcoo::kShareW * 4 : 0);
    L.persistent = at;
    if (!scratch_inside) {
        // the fixed carve-up of the static scratch (no staging of a host input there)
        L.tmp_cols = 0;
        L.tmp_rows = kStaticSortBytes;
        L.tmp_vals = 2 * kStaticSortBytes;
        L.share_alloc = 3 * kStaticSortBytes;
        L.in_row_ptr = L.in_cols = L.in_vals = 0;
        L.total = L.persistent;
        return L;
    }
    at = 0;
    L.share_alloc = take(share ? 4 : 0);
    L.tmp_cols = take(n4);
    L.tmp_rows = take(n4);
    L.tmp_vals = take(n4);
    L.in_row_ptr = take((size_t)(m + 1) * 4);
    L.in_cols = take(n4);
    L.in_vals = take(n4);
    L.total = L.persistent + at;
    return L;
}

// Groups taller than the fast kernels serve (p > 64) get a second, kernel-private copy of the matrix regrouped at
// kInnerP rows: the buffer of such a handle is its own layout followed by that of the inner handle.
constexpr int32_t kInnerP = 32;
bool wants_inner(int32_t p) { return p > gcoo::kSchedMaxP; }
size_t total_bytes(int64_t m, int64_t k, int64_t nnz, int32_t p, bool scratch_inside)
{
    const size_t own = make_layout(m, k, nnz, (m + p - 1) / p, p, scratch_inside).total;
    if (!wants_inner(p)) return own;
    return al(own) + make_layout(m, k, nnz, (m + kInnerP - 1) / kInnerP, kInnerP, scratch_inside).total;
}

bool dims_ok(int64_t m, int64_t k, int64_t nnz, int32_t p)
{
    return m >= 0 && k >= 0 && nnz >= 0 && p >= 1 && p <= GCOO_MAX_P && m <= INT32_MAX && k <= INT32_MAX &&
           nnz <= INT32_MAX;
}

int radix_passes(int64_t k)
{
    int bits = 0;
    while (bits < 31 && ((int64_t)1 << bits) < k) ++bits;   // column indices fit in `bits` bits
    int passes = (bits + 7) / 8;
    return passes < 1 ? 1 : passes;
}

}  // namespace

struct gcoo_matrix {
    // Everything below is set by the conversion and only read afterwards.
    int64_t m, k, nnz, g;
    int32_t p;
    int32_t nw, window_cols;
    bool has_sched;            // the run schedule of the register kernel was built (p <= 64)
    bool has_share;            // the share schedule was built
    bool share_preferred;      // and the kernel that reads it is the automatic choice
    int device;
    char* base;
    Layout L;
    // p > 64: the same matrix regrouped at kInnerP rows per group, with the schedules of the fast kernels, in the
    // part of the caller's buffer behind this handle's own; gcoo_spdm() multiplies with it.  Owned.
    gcoo_matrix* inner = nullptr;
    ~gcoo_matrix() { delete inner; }
    float* values() const { return reinterpret_cast<float*>(base + L.values); }
    int32_t* rows() const { return reinterpret_cast<int32_t*>(base + L.rows); }
    int32_t* cols() const { return reinterpret_cast<int32_t*>(base + L.cols); }
    int32_t* gIdxes() const { return reinterpret_cast<int32_t*>(base + L.gIdxes); }
    int32_t* nnzPerGroup() const { return reinterpret_cast<int32_t*>(base + L.nnzPerGroup); }
    gcoo::SchedClass* sched_hdr() const { return reinterpret_cast<gcoo::SchedClass*>(base + L.sched_hdr); }
    uint32_t* sched() const { return reinterpret_cast<uint32_t*>(base + L.sched); }
    bool has_order() const { return has_sched && g > 0 && g <= gcoo::kOrderMaxGroups; }
    int32_t* order() const { return reinterpret_cast<int32_t*>(base + L.order); }
    unsigned long long* stats() const { return reinterpret_cast<unsigned long long*>(base + L.counter); }
    uint32_t* bad_col() const { return reinterpret_cast<uint32_t*>(base + L.counter + 16); }
    int32_t* share_ucols() const { return reinterpret_cast<int32_t*>(base + L.share_ucols); }
    int32_t* share_ucount() const { return reinterpret_cast<int32_t*>(base + L.share_ucount); }
    uint32_t* share_hdr() const { return reinterpret_cast<uint32_t*>(base + L.share_hdr); }
    uint32_t* share_blocks() const { return reinterpret_cast<uint32_t*>(base + L.share_blocks); }
    int32_t* share_sbase() const { return reinterpret_cast<int32_t*>(base + L.share_sbase); }
    int64_t share_nq() const { return gcoo::share_super_groups(g); }
};

namespace {

int new_handle(int64_t m, int64_t k, int64_t nnz, int32_t p, void* dev_buf, gcoo_matrix** out, bool scratch_inside = true)
{
    gcoo_matrix* h = new (std::nothrow) gcoo_matrix;
    if (!h) return GCOO_ENOMEM;
    h->m = m; h->k = k; h->nnz = nnz; h->p = p;
    h->g = (m + p - 1) / p;
    h->base = static_cast<char*>(dev_buf);
    h->L = make_layout(m, k, nnz, h->g, p, scratch_inside);
    h->has_share = share_schedule_wanted(m, k, nnz, p);
    h->share_preferred = h->has_share && share_kernel_preferred(m, k, nnz, p);
    h->has_sched = h->p <= gcoo::kSchedMaxP;
    pick_windows(k, h->g, &h->nw, &h->window_cols);
    if (hipGetDevice(&h->device) != hipSuccess) h->device = -1;
    *out = h;
    return GCOO_OK;
}

// The kernel-private schedules that a conversion ends with: the run schedule of the register kernel
// (every matrix of at most 64 rows per group) and, where wanted, the share schedule.  Both are built
// here, on the conversion's stream, so that the handle is never written again.
// share_fill may ask for more dynamic LDS than a kernel gets by default: raised once per device (a compute unit
// has 160 KB; the kernel's static variables take a little of it).
constexpr int kShareFillMaxLds = 156 * 1024;
hipError_t share_fill_lds_limit()
{
    static std::atomic<unsigned> done[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gcoo::share_fill), hipFuncAttributeMaxDynamicSharedMemorySize, kShareFillMaxLds);
    if (e == hipSuccess) done[dev].store(1u, std::memory_order_release);
    return e;
}

// `scratch`: the conversion's scratch area (the counter of share_fill sits in it).
int launch_build_schedule(const gcoo_matrix* h, char* scratch, hipStream_t s)
{
    uint32_t* share_alloc = reinterpret_cast<uint32_t*>(scratch + h->L.share_alloc);
    if (h->g > 0 && h->has_sched) {
        // the groups by falling size, where the matrix has few of them: a workgroup more of the small-workgroup
        // instance, a launch of its own beside the large-workgroup instance
        int32_t* order = h->has_order() ? h->order() : nullptr;
        if (h->nnz / (h->g * h->nw) <= 1024) {
            const dim3 grid((unsigned)(h->g * h->nw + (order ? (h->g + 255) / 256 : 0)));
            gcoo::build_schedule<256><<<grid, dim3(256), 0, s>>>(h->gIdxes(), h->rows(), h->cols(), h->values(), h->p, h->g, h->nw,
                                                                 h->window_cols, h->sched_hdr(), h->sched(), order, order ? order + h->g : nullptr);
        } else {
            const dim3 grid((unsigned)(h->g * h->nw));
            gcoo::build_schedule<1024><<<grid, dim3(1024), 0, s>>>(h->gIdxes(), h->rows(), h->cols(), h->values(), h->p, h->g, h->nw,
                                                                   h->window_cols, h->sched_hdr(), h->sched(), nullptr, nullptr);
            HIP_TRY(hipGetLastError());
            if (order) gcoo::group_order_by_size<<<dim3((unsigned)((h->g + 1023) / 1024)), dim3(1024), 0, s>>>(h->gIdxes(), (int32_t)h->g, order, order + h->g);
        }
        HIP_TRY(hipGetLastError());
    }
    if (h->g > 0 && h->has_share) {
        const size_t bitmap_bytes = (size_t)((h->k + 31) / 32) * 4;
        // the bitmaps of the groups, one workgroup each, where they fit the second sort buffer (free by now: 12 bytes
        // per entry); otherwise one workgroup per super-group marks all its entries itself
        uint32_t* parts = nullptr;
        if ((uint64_t)h->g * bitmap_bytes <= (uint64_t)h->nnz * 12u) {
            parts = reinterpret_cast<uint32_t*>(scratch + h->L.tmp_cols);
            gcoo::share_mark_groups<<<dim3((unsigned)h->g), dim3(gcoo::kShareBuildThreads), bitmap_bytes, s>>>(h->gIdxes(), h->cols(), h->k, parts);
            HIP_TRY(hipGetLastError());
        }
        gcoo::share_union<<<dim3((unsigned)h->share_nq()), dim3(gcoo::kShareBuildThreads), bitmap_bytes, s>>>(
            h->gIdxes(), h->cols(), h->g, h->k, gcoo::kShareW, h->share_ucols(), h->share_ucount(), share_alloc, parts);
        HIP_TRY(hipGetLastError());
        // LDS of share_fill: its per-band tables and room for the columns of a group of up to twice the mean size
        // (between 8 K and 28 K entries: two workgroups share a compute unit up to 80 KB each)
        const size_t table_bytes = 4 * (size_t)((h->k + gcoo::kShareBandRows - 1) / gcoo::kShareBandRows + 1) * 4;
        int64_t stage_cap = 2 * (h->nnz / h->g + 1);
        stage_cap = stage_cap < 8192 ? 8192 : (stage_cap > 28672 ? 28672 : stage_cap);
        if (table_bytes + (size_t)stage_cap * 4 > (size_t)kShareFillMaxLds) stage_cap = 0;
        const size_t fill_lds = table_bytes + (size_t)stage_cap * 4;
        HIP_TRY(share_fill_lds_limit());
        gcoo::share_fill<<<dim3((unsigned)(h->share_nq() * gcoo::kShareW)), dim3(gcoo::kShareBuildThreads), fill_lds, s>>>(
            h->gIdxes(), h->rows(), h->cols(), h->values(), h->p, h->g, h->k, h->share_ucols(), h->share_ucount(), h->share_hdr(),
            h->share_blocks(), h->share_sbase(), share_alloc, (int32_t)stage_cap);
        HIP_TRY(hipGetLastError());
    }
    return GCOO_OK;
}

}  // namespace

extern "C" {

int gcoo_set_share_policy(int policy)
{
    if (policy < GCOO_SHARE_AUTO || policy > GCOO_SHARE_NEVER) return GCOO_EINVAL;
    g_share_policy.store(policy, std::memory_order_relaxed);
    return GCOO_OK;
}

int32_t gcoo_default_p(int64_t m, int64_t k, int64_t nnz, int64_t N)
{
    if (m < 0 || k < 0 || nnz < 0 || N < 0) return 0;
    if (N > 0 && N % 4 == 0 && share_policy_now() != GCOO_SHARE_NEVER && share_shape_preferred(m, k, nnz)) {
        const int32_t p = share_best_p(m, N);
        const int64_t items = share_items(m, p, N);
        if (items >= 192 && (k >= 9000 || fill_of_rounds(items) >= 0.8)) return p;
    }
    // Between 6 % and 12 % density most groups touch most columns, and what the register kernel
    // fetches falls with the number of groups: 38 rows (the tall accumulator file) beat 32 by
    // 8 .. 28 % from 6000 columns on (whole steps, n = 6000 .. 14000, s = 0.9 and 0.93); at 20 % and
    // more, and at n = 4000, the two are within a few per cent either way.
    if (m > 0 && k >= 5000 && N % 4 == 0) {
        const double density = (double)nnz / ((double)m * (double)k);
        if (density > 0.06 && density <= 0.12) return 38;
    }
    return 32;
}

size_t gcoo_device_bytes(int64_t m, int64_t k, int64_t nnz, int32_t p)
{
    if (!dims_ok(m, k, nnz, p)) return 0;
    return total_bytes(m, k, nnz, p, true);
}

}  // extern "C"

namespace {

// gcoo_from_csr() and gcoo_from_csr_device().  nnz_known < 0: learn nnz from the input.
// static_scratch_ptr != nullptr: the conversion's scratch is that area instead of the tail of dev_buf (device input with
// nnz given only).
int from_csr(int64_t m, int64_t k, const int32_t* row_ptr, const int32_t* col_idx, const float* vals, int src_on_device,
             int64_t nnz_known, int32_t p, void* dev_buf, size_t dev_buf_bytes, void* stream, gcoo_matrix** out,
             unsigned char* static_scratch_ptr = nullptr)
{
    const PolicyOfCall policy_of_call;
    const bool inside = static_scratch_ptr == nullptr;
    if (!out) return GCOO_EINVAL;
    *out = nullptr;
    if (!row_ptr || !dev_buf || !dims_ok(m, k, 0, p)) return GCOO_EINVAL;
    if (reinterpret_cast<uintptr_t>(dev_buf) % kAlign) return GCOO_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);

    const int64_t g = (m + p - 1) / p;
    int64_t nnz;
    if (src_on_device && nnz_known >= 0) {          // everything the host can check, before the first launch
        if (nnz_known > 0 && (!col_idx || !vals)) return GCOO_EINVAL;
        if (dev_buf_bytes < total_bytes(m, k, nnz_known, p, inside)) return GCOO_ENOMEM;
    }
    // nnz and the size of the largest group are computed on the device and stay there (the counters
    // sit at an offset of the buffer that does not depend on nnz); the launches that need the
    // latter read it there.
    const Layout L0 = make_layout(m, k, 0, g, p, inside);
    if (dev_buf_bytes < L0.total) return GCOO_ENOMEM;
    unsigned long long* stats = reinterpret_cast<unsigned long long*>(static_cast<char*>(dev_buf) + L0.counter);
    if (src_on_device) {
        // With nnz given nothing is read back here; otherwise nnz comes back in one small copy.
        if (nnz_known >= 0) {
            nnz = nnz_known;
        } else {
            gcoo::group_stats_from_row_ptr<<<dim3(1), dim3(256), 0, s>>>(row_ptr, m, p, g, stats);
            HIP_TRY(hipGetLastError());
            unsigned long long got[2] = {0, 0};
            HIP_TRY(hipMemcpyAsync(got, stats, sizeof(got), hipMemcpyDeviceToHost, s));
            HIP_TRY(hipStreamSynchronize(s));
            if (got[0] > (unsigned long long)INT32_MAX) return GCOO_EBOUNDS;
            nnz = (int64_t)got[0];
        }
    } else {
        if (row_ptr[0] != 0) return GCOO_EBOUNDS;
        for (int64_t i = 0; i < m; ++i)
            if (row_ptr[i + 1] < row_ptr[i]) return GCOO_EBOUNDS;
        nnz = row_ptr[m];
        if (nnz > 0 && (!col_idx || !vals)) return GCOO_EINVAL;
        for (int64_t e = 0; e < nnz; ++e)
            if (col_idx[e] < 0 || col_idx[e] >= k) return GCOO_EBOUNDS;
    }
    if (nnz > 0 && (!col_idx || !vals)) return GCOO_EINVAL;
    const Layout L = make_layout(m, k, nnz, g, p, inside);
    if (dev_buf_bytes < total_bytes(m, k, nnz, p, inside)) return GCOO_ENOMEM;

    gcoo_matrix* h = nullptr;
    int rc = new_handle(m, k, nnz, p, dev_buf, &h, inside);
    if (rc != GCOO_OK) return rc;
    char* base = h->base;
    char* scratch = inside ? base + L.persistent : reinterpret_cast<char*>(static_scratch_ptr);

    const int32_t* d_row_ptr = row_ptr;
    const int32_t* d_cols = col_idx;
    const float* d_vals = vals;
    if (!src_on_device) {
        int32_t* sp = reinterpret_cast<int32_t*>(scratch + L.in_row_ptr);
        int32_t* sc = reinterpret_cast<int32_t*>(scratch + L.in_cols);
        float* sv = reinterpret_cast<float*>(scratch + L.in_vals);
        hipError_t e = hipMemcpyAsync(sp, row_ptr, (size_t)(m + 1) * 4, hipMemcpyHostToDevice, s);
        if (e == hipSuccess && nnz > 0) e = hipMemcpyAsync(sc, col_idx, (size_t)nnz * 4, hipMemcpyHostToDevice, s);
        if (e == hipSuccess && nnz > 0) e = hipMemcpyAsync(sv, vals, (size_t)nnz * 4, hipMemcpyHostToDevice, s);
        // the caller may release its host arrays as soon as this call returns
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) { delete h; return hip_fail(e, "copy of the CSR input to the device"); }
        d_row_ptr = sp; d_cols = sc; d_vals = sv;
    }

    // Algorithm 1, step 1: group index and counts straight from row_ptr (also writes the sentinel).
    {
        const unsigned blocks = (unsigned)((g + 1 + 255) / 256) + 1u;     // the last one computes the statistics
        gcoo::group_index_from_row_ptr<<<dim3(blocks), dim3(256), 0, s>>>(d_row_ptr, m, p, g, (int32_t)nnz, h->gIdxes(), h->nnzPerGroup(),
                                                                         stats, h->bad_col());
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) { delete h; return hip_fail(e, "group_index_from_row_ptr"); }
    }
    // Algorithm 1, step 2: stable per-group radix sort on the column, 8 bits per pass, ping-pong
    // between the scratch triple and the final arrays so that the last pass lands in the latter.
    if (g > 0 && nnz > 0) {
        const int passes = radix_passes(k);
        int32_t* fin_c = h->cols(); int32_t* fin_r = h->rows(); float* fin_v = h->values();
        int32_t* tmp_c = reinterpret_cast<int32_t*>(scratch + L.tmp_cols);
        int32_t* tmp_r = reinterpret_cast<int32_t*>(scratch + L.tmp_rows);
        float* tmp_v = reinterpret_cast<float*>(scratch + L.tmp_vals);
        const int32_t* src_c = d_cols; const int32_t* src_r = nullptr; const float* src_v = d_vals;
        // Two passes and large groups: high digit first, then the low digit bucket by bucket (see the
        // kernel); otherwise low digit first, whole groups.
        const int64_t buckets = (k + 255) / 256;
        const bool high_first = passes == 2 && nnz / g >= 6000 && g * buckets <= 0x7fffffffLL;
        for (int pass = 0; pass < passes; ++pass) {
            const bool to_final = ((passes - 1 - pass) % 2) == 0;
            int32_t* dc = to_final ? fin_c : tmp_c;
            int32_t* dr = to_final ? fin_r : tmp_r;
            float* dv = to_final ? fin_v : tmp_v;
            const int shift = high_first ? 8 * (1 - pass) : 8 * pass;
            if (pass == 0)
                gcoo::sort_groups_by_col_digit<true, gcoo::kSortWaves><<<dim3((unsigned)g), dim3(gcoo::kSortWaves * gcoo::kWave), 0, s>>>(
                    h->gIdxes(), d_row_ptr, m, p, src_c, src_r, src_v, dc, dr, dv, shift, 0, (int32_t)k, h->bad_col());
            else if (high_first)
                gcoo::sort_groups_by_col_digit<false, gcoo::kSortBucketWaves><<<dim3((unsigned)(g * buckets)), dim3(gcoo::kSortBucketWaves * gcoo::kWave), 0, s>>>(
                    h->gIdxes(), d_row_ptr, m, p, src_c, src_r, src_v, dc, dr, dv, shift, (int32_t)buckets, (int32_t)k, h->bad_col());
            else
                gcoo::sort_groups_by_col_digit<false, gcoo::kSortWaves><<<dim3((unsigned)g), dim3(gcoo::kSortWaves * gcoo::kWave), 0, s>>>(
                    h->gIdxes(), d_row_ptr, m, p, src_c, src_r, src_v, dc, dr, dv, shift, 0, (int32_t)k, h->bad_col());
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) { delete h; return hip_fail(e, "sort_groups_by_col_digit"); }
            src_c = dc; src_r = dr; src_v = dv;
        }
    }
    rc = launch_build_schedule(h, scratch, s);
    if (rc != GCOO_OK) { delete h; return rc; }
    if (wants_inner(p)) {
        // the same entries once more, regrouped at kInnerP rows, from the CSR arrays on the device (a host input's
        // staged copy is still in this handle's scratch area, which the inner conversion does not touch)
        const size_t own = al(L.total);
        rc = from_csr(m, k, d_row_ptr, d_cols, d_vals, 1, nnz, kInnerP, base + own, dev_buf_bytes - own, stream, &h->inner,
                      static_scratch_ptr);
        if (rc != GCOO_OK) { delete h; return rc; }
    }
    *out = h;
    return GCOO_OK;
}

}  // namespace

extern "C" {

size_t gcoo_static_handle_bytes(int64_t m, int64_t k, int64_t nnz, int32_t p)
{
    if (!dims_ok(m, k, nnz, p) || nnz > kStaticMaxNnz) return 0;
    return total_bytes(m, k, nnz, p, false);
}

int gcoo_from_csr_device_static(int64_t m, int64_t k, int64_t nnz, const int32_t* row_ptr_dev, const int32_t* col_idx_dev,
                                const float* vals_dev, int32_t p, void* out_buf, size_t out_buf_bytes, void* stream,
                                gcoo_matrix** out)
{
    if (out) *out = nullptr;
    if (nnz < 0 || nnz > INT32_MAX) return GCOO_EINVAL;
    if (nnz > kStaticMaxNnz) return GCOO_ELIMIT;
    unsigned char* scratch = nullptr;
    int rc = static_scratch(&scratch);
    if (rc != GCOO_OK) return rc;
    return from_csr(m, k, row_ptr_dev, col_idx_dev, vals_dev, 1, nnz, p, out_buf, out_buf_bytes, stream, out, scratch);
}

int gcoo_from_csr(int64_t m, int64_t k, const int32_t* row_ptr, const int32_t* col_idx, const float* vals,
                  int src_on_device, int32_t p, void* dev_buf, size_t dev_buf_bytes, void* stream, gcoo_matrix** out)
{
    return from_csr(m, k, row_ptr, col_idx, vals, src_on_device, -1, p, dev_buf, dev_buf_bytes, stream, out);
}

int gcoo_from_csr_device(int64_t m, int64_t k, int64_t nnz, const int32_t* row_ptr_dev, const int32_t* col_idx_dev,
                         const float* vals_dev, int32_t p, void* dev_buf, size_t dev_buf_bytes, void* stream, gcoo_matrix** out)
{
    if (nnz < 0 || nnz > INT32_MAX) { if (out) *out = nullptr; return GCOO_EINVAL; }
    return from_csr(m, k, row_ptr_dev, col_idx_dev, vals_dev, 1, nnz, p, dev_buf, dev_buf_bytes, stream, out);
}

int gcoo_dense_nnz(int64_t m, int64_t k, const float* A_dev, int64_t lda, void* stream, int64_t* nnz)
{
    if (!nnz || m < 0 || k < 0 || lda < k || (m > 0 && k > 0 && !A_dev)) return GCOO_EINVAL;
    *nnz = 0;
    if (m == 0 || k == 0) return GCOO_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    unsigned long long* dptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&dptr), HIP_SYMBOL(g_dense_total)));
    dptr += g_dense_next.fetch_add(1u, std::memory_order_relaxed) % kDenseSlots;
    unsigned long long got = 0;
    HIP_TRY(hipMemsetAsync(dptr, 0, 8, s));
    const unsigned blocks = (unsigned)(m < 2048 ? m : 2048);
    if (dense_vec_width(A_dev, lda, k) == 4)
        gcoo::count_dense_total<4><<<dim3(blocks), dim3(256), 0, s>>>(A_dev, lda, m, k, dptr);
    else
        gcoo::count_dense_total<1><<<dim3(blocks), dim3(256), 0, s>>>(A_dev, lda, m, k, dptr);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemcpyAsync(&got, dptr, 8, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    *nnz = (int64_t)got;
    return GCOO_OK;
}

int gcoo_from_dense(int64_t m, int64_t k, const float* A_dev, int64_t lda, int32_t p, void* dev_buf, size_t dev_buf_bytes,
                    void* stream, gcoo_matrix** out)
{
    const PolicyOfCall policy_of_call;
    if (!out) return GCOO_EINVAL;
    *out = nullptr;
    if (!dev_buf || !dims_ok(m, k, 0, p) || lda < k || (m > 0 && k > 0 && !A_dev)) return GCOO_EINVAL;
    if (reinterpret_cast<uintptr_t>(dev_buf) % kAlign) return GCOO_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t g = (m + p - 1) / p;
    // gIdxes / nnzPerGroup / counter sit at the front of the buffer at offsets that do not
    // depend on nnz, so step 1 can run before the buffer size for this nnz is checked.
    const Layout L0 = make_layout(m, k, 0, g, p);
    if (dev_buf_bytes < L0.total) return GCOO_ENOMEM;
    char* base = static_cast<char*>(dev_buf);
    int32_t* cnt = reinterpret_cast<int32_t*>(base + L0.nnzPerGroup);
    int32_t* idx = reinterpret_cast<int32_t*>(base + L0.gIdxes);
    int32_t* blk = reinterpret_cast<int32_t*>(base + L0.blk);
    unsigned long long* tot = reinterpret_cast<unsigned long long*>(base + L0.counter);
    unsigned long long total = 0;
    const int vw = dense_vec_width(A_dev, lda, k);
    const int64_t nblk = dense_blocks(k, vw);
    // one workgroup per (group, column block); a band holds fewer than 2^31 elements so that
    // 32-bit counts cannot wrap before the total is checked
    if (nblk > 0 && g > 0x7fffffffLL / nblk) return GCOO_EINVAL;
    if ((int64_t)p * k > INT32_MAX) return GCOO_EINVAL;
    if (g > 0) {
        if (nblk > 0) {
            const dim3 grid((unsigned)(nblk * g)), block(gcoo::kDenseThreads);
            if (vw == 4) gcoo::count_dense_blocks<4><<<grid, block, 0, s>>>(A_dev, lda, m, k, p, nblk, blk);
            else gcoo::count_dense_blocks<1><<<grid, block, 0, s>>>(A_dev, lda, m, k, p, nblk, blk);
            HIP_TRY(hipGetLastError());
        }
        gcoo::scan_dense_blocks<<<dim3((unsigned)g), dim3(256), 0, s>>>(blk, nblk, cnt);
        HIP_TRY(hipGetLastError());
        gcoo::scan_group_counts<<<dim3(1), dim3(256), 0, s>>>(cnt, g, idx, tot);
        HIP_TRY(hipGetLastError());
        unsigned long long got[2] = {0, 0};
        HIP_TRY(hipMemcpyAsync(got, tot, sizeof(got), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        total = got[0];
    } else {
        HIP_TRY(hipMemsetAsync(idx, 0, 4, s));          // only the sentinel exists
        HIP_TRY(hipMemsetAsync(tot, 0, 16, s));
    }
    HIP_TRY(hipMemsetAsync(base + L0.counter + 16, 0, 4, s));   // no column can be out of range here
    if (total > (unsigned long long)INT32_MAX) return GCOO_EINVAL;
    const int64_t nnz = (int64_t)total;
    const Layout L = make_layout(m, k, nnz, g, p);
    if (dev_buf_bytes < total_bytes(m, k, nnz, p, true)) return GCOO_ENOMEM;
    gcoo_matrix* h = nullptr;
    int rc = new_handle(m, k, nnz, p, dev_buf, &h);
    if (rc != GCOO_OK) return rc;
    if (g > 0 && nnz > 0) {
        const dim3 grid((unsigned)(nblk * g)), block(gcoo::kDenseThreads);
        if (vw == 4)
            gcoo::fill_dense_blocks<4><<<grid, block, 0, s>>>(A_dev, lda, m, k, p, nblk, h->gIdxes(), blk, h->values(), h->rows(), h->cols());
        else
            gcoo::fill_dense_blocks<1><<<grid, block, 0, s>>>(A_dev, lda, m, k, p, nblk, h->gIdxes(), blk, h->values(), h->rows(), h->cols());
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) { delete h; return hip_fail(e, "fill_dense_blocks"); }
    }
    rc = launch_build_schedule(h, h->base + h->L.persistent, s);
    if (rc != GCOO_OK) { delete h; return rc; }
    if (wants_inner(p)) {
        const size_t own = al(L.total);
        rc = gcoo_from_dense(m, k, A_dev, lda, kInnerP, base + own, dev_buf_bytes - own, stream, &h->inner);
        if (rc != GCOO_OK) { delete h; return rc; }
    }
    *out = h;
    return GCOO_OK;
}

}  // extern "C"

namespace {

struct Shape {
    bool al4;          // N, both leading dimensions and both base addresses fit 16-byte accesses: what the
                       // workgroup-shared kernel's loads straight to LDS need
    bool wide_pitch;   // row pitch of B in bytes does not fit 32 bits: LDS variant only
    int64_t N;
};

Shape shape_of(const float* B, int64_t ldb, int64_t N, const float* C, int64_t ldc)
{
    const uintptr_t pb = reinterpret_cast<uintptr_t>(B), pc = reinterpret_cast<uintptr_t>(C);
    Shape s;
    s.al4 = (N % 4 == 0) && (ldb % 4 == 0) && (ldc % 4 == 0) && (pb % 16 == 0) && (pc % 16 == 0);
    s.wide_pitch = ldb > 0x3fffffffLL;
    s.N = N;
    return s;
}

// Instance of the register kernel that serves this p and N: its columns per lane, 0 if none does;
// kTallInstance for four columns per lane with the tall accumulator file (33 <= p <= 38).  The instances
// take any N of at least their columns per lane and any leading dimensions and base addresses: the one lane that
// would reach beyond N computes the last columns of the row instead (lane_cols() in gcoo_spdm_kernels.hpp), and
// rows that are aligned to 4 bytes only are read and written with unaligned 16-byte accesses.
constexpr int kTallInstance = 38;
int sched_width(int32_t p, const Shape& sh)
{
    if (sh.wide_pitch) return 0;
    if (p <= 32 && sh.N >= 4) return 4;
    if (p <= 38 && sh.N >= 4) return kTallInstance;
    if (p <= 64 && sh.N >= 2) return 2;
    // There is no one-column-per-lane instance (65 <= p <= 128, or N = 1): a run of one on an 8000 x 8000
    // matrix with p = 128 ended in a GPU memory fault whose cause was never found, and it was taken out of
    // the build.  Such calls get the LDS kernel (automatic choice) or GCOO_EINVAL (explicit GCOO_VARIANT_REG).
    return 0;
}

}  // namespace

namespace gcoo {
hipError_t launch_spdm_sched(int V, const SpdmArgs& a, hipStream_t s)
{
    if (V == 4) return launch_spdm_sched_v4(a, s);
    if (V == 38) return launch_spdm_sched_v4_tall(a, s);
    if (V == 2) return launch_spdm_sched_v2(a, s);
    return hipErrorInvalidValue;
}
}  // namespace gcoo

namespace {

bool share_operands_ok(const gcoo_matrix* A, const Shape& sh, int64_t ldb)
{
    // (the kernel keeps byte offsets into B in 32 bits, each up to 3072 above the place it stands for)
    return sh.al4 && (uint64_t)A->k * (uint64_t)ldb * 4u <= 0xffffffffull - 4096u;
}

int check_spdm_args(const gcoo_matrix* A, const float* B, int64_t ldb, int64_t N, const float* C, int64_t ldc)
{
    if (!A || N < 0 || ldb < N || ldc < N || N > INT32_MAX) return GCOO_EINVAL;
    if (N > 0 && A->m > 0 && !C) return GCOO_EINVAL;
    if (N > 0 && A->nnz > 0 && !B) return GCOO_EINVAL;
    return GCOO_OK;
}

}  // namespace

extern "C" {

int gcoo_spdm_pick(const gcoo_matrix* A, const float* B_dev, int64_t ldb, int64_t N, const float* C_dev, int64_t ldc)
{
    int rc = check_spdm_args(A, B_dev, ldb, N, C_dev, ldc);
    if (rc != GCOO_OK) return rc;
    if (A->inner) A = A->inner;        // groups taller than 64 rows: the fast kernels run on the regrouped copy
    const Shape sh = shape_of(B_dev, ldb, N, C_dev, ldc);
    // the workgroup-shared kernel wants enough workgroups to occupy the chip (one per 8p rows and 256 columns),
    // and below 9000 columns its margin does not survive a last round that is mostly idle
    const int64_t items = A->share_nq() * ((N + 255) / 256);
    if (A->share_preferred && share_operands_ok(A, sh, ldb) && items >= 192 && (A->k >= 9000 || fill_of_rounds(items) >= 0.8))
        return GCOO_VARIANT_SHARE;
    return (A->has_sched && sched_width(A->p, sh)) ? GCOO_VARIANT_REG : GCOO_VARIANT_LDS;
}

int gcoo_spdm_variant(const gcoo_matrix* A, const float* B_dev, int64_t ldb, int64_t N, float* C_dev, int64_t ldc,
                      void* stream, int variant)
{
    int rc = check_spdm_args(A, B_dev, ldb, N, C_dev, ldc);
    if (rc != GCOO_OK) return rc;
    if (variant < GCOO_VARIANT_AUTO || variant > GCOO_VARIANT_SHARE) return GCOO_EINVAL;
    if (variant == GCOO_VARIANT_AUTO) variant = gcoo_spdm_pick(A, B_dev, ldb, N, C_dev, ldc);
    if (A->m == 0 || N == 0) return GCOO_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);

    if (variant == GCOO_VARIANT_LDS) {
        const int64_t tiles = (N + 63) / 64;
        const int64_t total = A->g * tiles;
        if (total > 0x7fffffffLL) return GCOO_EINVAL;
        const size_t smem = (size_t)A->p * 64 * sizeof(float);
        gcoo::spdm_lds<<<dim3((unsigned)total), dim3(64), smem, s>>>(A->values(), A->rows(), A->cols(), A->gIdxes(), A->m,
                                                                     A->p, B_dev, ldb, N, C_dev, ldc, A->g);
        HIP_TRY(hipGetLastError());
        return GCOO_OK;
    }
    if (A->inner) A = A->inner;        // the schedules of the kernels below belong to the regrouped copy
    if (variant == GCOO_VARIANT_SHARE) {
        const Shape sh = shape_of(B_dev, ldb, N, C_dev, ldc);
        if (!A->has_share || !share_operands_ok(A, sh, ldb)) return GCOO_EINVAL;
        gcoo::ShareArgs a{A->share_hdr(), A->share_blocks(), A->share_sbase(), A->share_ucols(), A->share_ucount(), A->gIdxes(),
                          A->m, A->p, A->g, A->share_nq(), B_dev, ldb, N, C_dev, ldc};
        hipError_t e = gcoo::launch_spdm_share(a, s);
        if (e != hipSuccess) return hip_fail(e, "spdm_share launch");
        return GCOO_OK;
    }
    const int V = sched_width(A->p, shape_of(B_dev, ldb, N, C_dev, ldc));
    if (V == 0 || !A->has_sched) return GCOO_EINVAL;
    const int cols_per_lane = V == kTallInstance ? 4 : V;
    // Heavy groups are shared by a workgroup in the standard instances only, and only a launch of few
    // items can have any: then the kernels decide group by group, from the statistics on the device.
    const bool heavy = V != kTallInstance && gcoo::sched_heavy_possible(A->nnz, A->g, (N + 64 * cols_per_lane - 1) / (64 * cols_per_lane));
    gcoo::SpdmArgs a{A->sched_hdr(), A->sched(), A->gIdxes(), A->m, A->p, A->g, A->nw, B_dev, ldb, N, C_dev, ldc,
                     A->nnz, heavy ? A->stats() : nullptr, (heavy && A->has_order()) ? A->order() : nullptr};
    hipError_t e = gcoo::launch_spdm_sched(V, a, s);
    if (e != hipSuccess) return hip_fail(e, "spdm_sched launch");
    return GCOO_OK;
}

int gcoo_spdm(const gcoo_matrix* A, const float* B_dev, int64_t ldb, int64_t N, float* C_dev, int64_t ldc, void* stream)
{
    return gcoo_spdm_variant(A, B_dev, ldb, N, C_dev, ldc, stream, GCOO_VARIANT_AUTO);
}

int gcoo_free(gcoo_matrix* A)
{
    delete A;
    return GCOO_OK;
}

int gcoo_info(const gcoo_matrix* A, int64_t* m, int64_t* k, int64_t* nnz, int32_t* p, int64_t* g)
{
    if (!A) return GCOO_EINVAL;
    if (m) *m = A->m;
    if (k) *k = A->k;
    if (nnz) *nnz = A->nnz;
    if (p) *p = A->p;
    if (g) *g = A->g;
    return GCOO_OK;
}

int gcoo_export(const gcoo_matrix* A, float* values, int32_t* rows, int32_t* cols, int64_t* gIdxes, int32_t* nnzPerGroup,
                void* stream)
{
    if (!A) return GCOO_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t n4 = (size_t)A->nnz * 4;
    if (values && n4) HIP_TRY(hipMemcpyAsync(values, A->values(), n4, hipMemcpyDeviceToHost, s));
    if (rows && n4) HIP_TRY(hipMemcpyAsync(rows, A->rows(), n4, hipMemcpyDeviceToHost, s));
    if (cols && n4) HIP_TRY(hipMemcpyAsync(cols, A->cols(), n4, hipMemcpyDeviceToHost, s));
    if (nnzPerGroup && A->g) HIP_TRY(hipMemcpyAsync(nnzPerGroup, A->nnzPerGroup(), (size_t)A->g * 4, hipMemcpyDeviceToHost, s));
    int32_t* narrow = nullptr;
    if (gIdxes) {
        narrow = new (std::nothrow) int32_t[(size_t)A->g + 1];
        if (!narrow) return GCOO_ENOMEM;
        hipError_t e = hipMemcpyAsync(narrow, A->gIdxes(), (size_t)(A->g + 1) * 4, hipMemcpyDeviceToHost, s);
        if (e != hipSuccess) { delete[] narrow; return hip_fail(e, "hipMemcpyAsync(gIdxes)"); }
    }
    uint32_t bad = 0;
    hipError_t e = hipMemcpyAsync(&bad, A->bad_col(), 4, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (gIdxes && e == hipSuccess)
        for (int64_t i = 0; i <= A->g; ++i) gIdxes[i] = narrow[i];
    delete[] narrow;
    if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
    return bad ? GCOO_EBOUNDS : GCOO_OK;
}

int gcoo_export_share(const gcoo_matrix* A, uint32_t* hdr, uint32_t* blocks, int32_t* sbase, int32_t* ucount, int32_t* ucols,
                      int64_t* hdr_words, int64_t* block_count, void* stream)
{
    if (!A || !A->has_share) return GCOO_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t hw = gcoo::share_hdr_words(A->nnz, A->g), nb = gcoo::share_stream_blocks(A->nnz, A->g, A->k);
    if (hdr_words) *hdr_words = hw;
    if (block_count) *block_count = nb;
    if (hdr) HIP_TRY(hipMemcpyAsync(hdr, A->share_hdr(), (size_t)hw * 4, hipMemcpyDeviceToHost, s));
    if (blocks) HIP_TRY(hipMemcpyAsync(blocks, A->share_blocks(), (size_t)nb * gcoo::kShareBlockWords * 4, hipMemcpyDeviceToHost, s));
    if (sbase) HIP_TRY(hipMemcpyAsync(sbase, A->share_sbase(), (size_t)A->share_nq() * gcoo::kShareW * 4, hipMemcpyDeviceToHost, s));
    if (ucount) HIP_TRY(hipMemcpyAsync(ucount, A->share_ucount(), (size_t)A->share_nq() * 4, hipMemcpyDeviceToHost, s));
    if (ucols && A->nnz) HIP_TRY(hipMemcpyAsync(ucols, A->share_ucols(), (size_t)A->nnz * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    return GCOO_OK;
}

const char* gcoo_strerror(int status)
{
    switch (status) {
        case GCOO_OK: return "ok";
        case GCOO_EINVAL: return "invalid argument";
        case GCOO_EBOUNDS: return "malformed CSR input (row_ptr not non-decreasing from 0, or column out of range)";
        case GCOO_ENOMEM: return "device buffer too small (see gcoo_device_bytes) or host allocation failed";
        case GCOO_EHIP: return "HIP runtime error (see gcoo_last_hip_error)";
        case GCOO_ELIMIT: return "input larger than the fixed scratch of gcoo_from_csr_device_static (at most 2097152 stored entries)";
        default: return "unknown status";
    }
}

const char* gcoo_last_hip_error(void) { return g_hip_error.c_str(); }

}  // extern "C"
