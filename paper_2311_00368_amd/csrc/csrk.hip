// C-ABI of the csrk library (declared in include/csrk.h): argument checks, kernel
// selection by dense width and alignment, per-device scratch for partial rows, launches.
#include "../../include/csrk.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "kernels_ktile.hpp"
#include "kernels_ktile_fused.hpp"
#include "kernels_ktile_narrow.hpp"
#include "kernels_nnzsplit.hpp"

// What csrk_plan_create found out about a pattern (see include/csrk.h).
struct csrk_plan_s {
    int dev;                  // device the plan was made on
    int M, K;
    long long nnz;
    const int32_t *rowptr, *colidx;   // the caller's arrays (not copied)
    bool sorted;              // columns non-decreasing inside every row
    bool even;                // longest row <= 2 * mean + 64 (what the per-call row analysis asks)
    int32_t *dflags;          // 8 device words laid out like the per-call flags: {0, 1, 0, even, ...}
    void *ws;                 // scratch owned by the plan (csrk_plan_reserve), or NULL
    size_t ws_bytes;
    // Schedule for uneven rows (patterns that are sorted but not `even`): rows sorted by length and cut into blocks
    // of 64 (4 per wavefront of a tiled kernel), every block's K cut into as many ranges as its share of the work
    // asks for.  All arrays live in one device allocation (`sched_mem`).
    struct Sched {
        int n_items = 0;          // workgroups: (block, range) pairs, heaviest first
        int n_comb = 0;           // blocks whose K is cut (their partial rows are added up afterwards)
        int n_slots = 0;          // partial-row slots (one per item of a cut block), kSchedRows rows each
        const int32_t *perm = nullptr;    // rows in schedule order, padded with M to whole blocks
        const int4 *items = nullptr;      // block, range, ranges, first slot of the range
        const int4 *comb = nullptr;       // block, first slot, ranges
    } sched;
    void *sched_mem = nullptr;
    bool has_sched = false;
};

namespace {

using namespace csrk;

thread_local char g_err[512] = "";

csrk_status fail(csrk_status code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define CSRK_HIP(call)                                                                          \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess)                                                                   \
            return fail(CSRK_HIP_ERROR, "%s failed: %s", #call, hipGetErrorString(e_));         \
    } while (0)

constexpr int kMaxDevices = 64;
constexpr int kMaxKSplit = 8;

// What the library knows about a device: filled in once, read-only afterwards.
struct DeviceInfo {
    std::atomic<bool> init{false};
    int cus = 0;
    int workers = 0;        // wavefronts the equal-nonzero split is cut into
};

// The scratch area the library allocates by itself for the plain entry points (one per device, grown on demand,
// kept until csrk_release_workspace).  Only touched under g_mu.
struct LazyScratch {
    float *head = nullptr;
    int32_t *head_row = nullptr;
    size_t head_floats = 0;
    int flag_set = 0;       // which of the two sets of per-call flag words the next tiled attempt uses (see tile_go)
};

// Everything ONE call works with.  It lives on the calling thread's stack, so calls that bring their own scratch
// (a caller's workspace, a plan's, the static array) share no state with each other and take no lock.  The plain
// entry points fill it from the device's LazyScratch under g_mu and write the changes back when they return.
struct DeviceState {
    int cus = 0;
    int workers = 0;
    float *head = nullptr;  // workers x width floats: partial sums of rows entered mid-way (or partial outputs of a K-split call)
    int32_t *head_row = nullptr;  // workers ints, 8 spare words, two sets of 8 flag words
    size_t head_floats = 0;
    bool fixed = false;     // scratch of a given size that this call may neither grow nor replace
    LazyScratch *lazy = nullptr;    // where head / head_row / flag_set go back to (plain entry points)
    int pending_ksplit = 0; // > 1: the tiled kernel of this call left that many partial outputs in `head`
    int32_t *plan_flags = nullptr;  // flag words of the plan this call runs under (instead of the per-call ones)
    int flag_set = 0;
    float inline_density = __builtin_nanf("");   // not NaN: the tiled kernel of this call analyses the rows itself
    bool attempted = false; // this call has made an unplanned tiled attempt (its set of flag words is used up)
};

DeviceInfo g_info[kMaxDevices];
LazyScratch g_lazy[kMaxDevices];
std::mutex g_mu;

// optional per-call event pairs around the main kernels (csrk_profile_enable)
struct Recorder {
    std::vector<hipEvent_t> start, stop;
    std::vector<int> kind;
    std::atomic<int> used{0};   // calls without a lock (own scratch) may record from several threads
};
Recorder g_rec;

// One event pair per call, around all of its kernels: the row analysis, the tiled kernel with its reduction (if
// one is tried), the general kernel (which stands down if the tiled one did the call) and the combine step.
struct CallRecord {
    int slot = -1;
    int kind;
    hipStream_t st;
    CallRecord(int k, hipStream_t s) : kind(k), st(s) {}
    void begin() {
        if (slot < 0 && g_rec.used.load() < (int)g_rec.start.size()) {
            const int mine = g_rec.used.fetch_add(1);
            if (mine < (int)g_rec.start.size()) {
                slot = mine;
                g_rec.kind[slot] = kind;
                (void)hipEventRecord(g_rec.start[slot], st);
            } else {
                g_rec.used.fetch_sub(1);
            }
        }
    }
    void end() {
        if (slot >= 0) (void)hipEventRecord(g_rec.stop[slot], st);
        slot = -2;
    }
    ~CallRecord() { end(); }    // a call that fails half-way still closes its pair
};

int env_int(const char *name, int dflt) {
    const char *s = getenv(name);
    if (!s || !*s) return dflt;
    const long v = strtol(s, nullptr, 10);
    return v > 0 ? (int)v : dflt;
}

csrk_status device_info(const DeviceInfo **out, int *ordinal = nullptr) {
    int dev = 0;
    CSRK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(CSRK_UNSUPPORTED, "device ordinal %d not supported", dev);
    DeviceInfo &d = g_info[dev];
    if (!d.init.load(std::memory_order_acquire)) {
        std::lock_guard<std::mutex> lock(g_mu);
        if (!d.init.load(std::memory_order_relaxed)) {
            int cus = 0;
            CSRK_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
            // 8 wavefronts per SIMD, 4 SIMDs per CU: every CU gets a full complement of shares
            int workers = env_int("CSRK_WORKERS", cus * 32);
            workers = (workers + kWavesPerBlock - 1) / kWavesPerBlock * kWavesPerBlock;
            d.workers = workers;
            d.cus = cus;
            d.init.store(true, std::memory_order_release);
        }
    }
    *out = &d;
    if (ordinal) *ordinal = dev;
    return CSRK_OK;
}

// ints at the head of a scratch area: worker table, 8 spare words, two sets of 8 flag words; padded to 256 bytes
size_t scratch_int_bytes(int workers) { return ((sizeof(int32_t) * ((size_t)workers + 8 + 2 * 8)) + 255) / 256 * 256; }

// Where a call's scratch comes from.
struct ScratchSource {
    void *mem = nullptr;    // a caller's workspace, a plan's, or the static array; NULL: the device's lazily grown one
    size_t bytes = 0;
};

// Holds g_mu for calls on the lazily grown scratch (they share it, and its flag words take turns between calls);
// calls with scratch of their own take no lock.
struct CallLock {
    bool held = false;
    void take() {
        g_mu.lock();
        held = true;
    }
    ~CallLock() {
        if (held) g_mu.unlock();
    }
};

// Fills the per-call state.  With a ScratchSource the area is cut into its int part and its float part here and no
// allocation ever happens; `lock` is taken only for the lazily grown scratch.
csrk_status begin_call(DeviceState &d, const ScratchSource &src, CallLock &lock) {
    const DeviceInfo *info = nullptr;
    int dev = 0;
    if (csrk_status s = device_info(&info, &dev)) return s;
    d.cus = info->cus;
    d.workers = info->workers;
    if (src.mem) {
        if (reinterpret_cast<uintptr_t>(src.mem) & 255u)
            return fail(CSRK_INVALID_ARG, "workspace must be 256-byte aligned");
        const size_t ints = scratch_int_bytes(d.workers);
        if (src.bytes < ints + 256)
            return fail(CSRK_WORKSPACE, "workspace of %zu bytes is too small (at least %zu are needed)", src.bytes, ints + 256);
        d.head_row = static_cast<int32_t *>(src.mem);
        d.head = reinterpret_cast<float *>(static_cast<char *>(src.mem) + ints);
        d.head_floats = (src.bytes - ints) / sizeof(float);
        d.fixed = true;
        return CSRK_OK;
    }
    lock.take();
    LazyScratch &g = g_lazy[dev];
    d.lazy = &g;
    d.head = g.head;
    d.head_row = g.head_row;
    d.head_floats = g.head_floats;
    d.flag_set = g.flag_set;
    return CSRK_OK;
}

// scratch for `width` columns of partial rows of the equal-nonzero split, or `min_floats` floats if that is
// more (partial outputs of a K-split launch).  The lazily grown scratch grows (hipMalloc, and a device
// synchronisation before the old area is freed), never shrinks; scratch that was handed in is only checked.
csrk_status ensure_scratch(DeviceState &d, int width, size_t min_floats = 0) {
    size_t need = (size_t)d.workers * (size_t)width;
    if (min_floats > need) need = min_floats;
    if (d.fixed) {
        if (need > d.head_floats)
            return fail(CSRK_WORKSPACE, "workspace too small: this call needs %zu bytes", scratch_int_bytes(d.workers) + need * sizeof(float));
        return CSRK_OK;
    }
    LazyScratch &g = *d.lazy;
    if (!g.head_row) {
        const size_t bytes = scratch_int_bytes(d.workers);
        if (hipMalloc((void **)&g.head_row, bytes) != hipSuccess) {
            g.head_row = nullptr;
            return fail(CSRK_WORKSPACE, "cannot allocate %zu bytes of scratch", bytes);
        }
        // both sets start with a clear ordering flag; from then on each tiled attempt clears the other set's
        if (hipMemset(g.head_row, 0, bytes) != hipSuccess) {
            (void)hipFree(g.head_row);
            g.head_row = nullptr;
            return fail(CSRK_HIP_ERROR, "cannot clear the flag words of the scratch area");
        }
        g.flag_set = 0;
        d.flag_set = 0;
        d.head_row = g.head_row;
    }
    if (need > g.head_floats) {
        if (g.head) {
            CSRK_HIP(hipDeviceSynchronize());
            CSRK_HIP(hipFree(g.head));
            g.head = nullptr;
            g.head_floats = 0;
            d.head = nullptr;
            d.head_floats = 0;
        }
        if (hipMalloc((void **)&g.head, need * sizeof(float)) != hipSuccess) {
            g.head = nullptr;
            return fail(CSRK_WORKSPACE, "cannot allocate %zu bytes of scratch", need * sizeof(float));
        }
        g.head_floats = need;
        d.head = g.head;
        d.head_floats = need;
    }
    return CSRK_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

csrk_status check_dims(const char *fn, int M, int K, long long w1, long long w2) {
    if (M < 0 || K < 0 || w1 < 0 || w2 < 0) return fail(CSRK_INVALID_ARG, "%s: negative dimension", fn);
    // element offsets into dense operands are formed in 64 bits, row/column numbers in 32
    if ((long long)M >= (1ll << 31) - 1 || (long long)K >= (1ll << 31) - 1 || w1 >= (1ll << 24) || w2 >= (1ll << 24))
        return fail(CSRK_UNSUPPORTED, "%s: dimension too large", fn);
    return CSRK_OK;
}

// --- kernel selection ---------------------------------------------------------------
// A dense width W is covered by groups of LG lanes holding VEC floats each (T tiles per
// lane).  Fast path: W % 4 == 0 and 16-byte aligned operands -> 128-bit accesses.
struct WidthCfg {
    int vec, lg, t;
};

WidthCfg out_width_cfg(int N, bool vec4) {
    if (vec4) {
        if (N <= 32) return {4, 8, 1};
        if (N <= 64) return {4, 16, 1};
        if (N <= 128) return {4, 32, 1};
        if (N <= 256) return {4, 64, 1};
        return {4, 64, 2};
    }
    return {1, 64, 1};
}

WidthCfg dot_width_cfg(int D, bool vec4) {
    if (vec4) {
        if (D <= 32) return {4, 8, 1};
        if (D <= 64) return {4, 16, 1};
        if (D <= 128) return {4, 32, 1};
        if (D <= 256) return {4, 64, 1};
        return {4, 64, 0};
    }
    return {1, 64, 0};
}

template <int VEC, int LG, int T>
void launch_spmm(dim3 grid, hipStream_t st, int M, int N, const int32_t *rp, const int32_t *ci, const float *v,
                 const float *B, float *O, float *head, int32_t *head_row, const int32_t *gate, const int32_t *even) {
    hipLaunchKernelGGL((spmm_nnzsplit_kernel<VEC, LG, T>), grid, dim3(kBlockThreads), 0, st, M, N, rp, ci, v, B, O,
                       head, head_row, gate, even);
}

template <int VEC, int LG, int T>
void launch_sddmm(dim3 grid, hipStream_t st, int M, int D, const int32_t *rp, const int32_t *ci, const float *v,
                  const float *A, const float *B, float *P, const int32_t *gate, const int32_t *even) {
    hipLaunchKernelGGL((sddmm_nnzsplit_kernel<VEC, LG, T>), grid, dim3(kBlockThreads), 0, st, M, D, rp, ci, v, A, B,
                       P, gate, even);
}

template <int VD, int LD, int TD, int VN, int LN, int TN>
void launch_fused(dim3 grid, hipStream_t st, int M, int D, int N, const int32_t *rp, const int32_t *ci,
                  const float *v, const float *A, const float *B, const float *C, float *O, float *head,
                  int32_t *head_row, const int32_t *gate, const int32_t *even) {
    hipLaunchKernelGGL((fusedmm_nnzsplit_kernel<VD, LD, TD, VN, LN, TN>), grid, dim3(kBlockThreads), 0, st, M, D, N,
                       rp, ci, v, A, B, C, O, head, head_row, gate, even);
}

template <int VD, int LD, int TD>
bool launch_fused_n(const WidthCfg &nc, dim3 grid, hipStream_t st, int M, int D, int N, const int32_t *rp,
                    const int32_t *ci, const float *v, const float *A, const float *B, const float *C, float *O,
                    float *head, int32_t *head_row, const int32_t *gate, const int32_t *even) {
#define CSRK_FUSED_CASE(VN, LN, TN)                                                                           \
    if (nc.vec == VN && nc.lg == LN && nc.t == TN) {                                                          \
        launch_fused<VD, LD, TD, VN, LN, TN>(grid, st, M, D, N, rp, ci, v, A, B, C, O, head, head_row, gate, even); \
        return true;                                                                                          \
    }
    CSRK_FUSED_CASE(4, 8, 1)
    CSRK_FUSED_CASE(4, 16, 1)
    CSRK_FUSED_CASE(4, 32, 1)
    CSRK_FUSED_CASE(4, 64, 1)
    CSRK_FUSED_CASE(4, 64, 2)
    CSRK_FUSED_CASE(1, 64, 1)
#undef CSRK_FUSED_CASE
    return false;
}

// last kernel of an SPMM / FusedMM call: heads of the equal-nonzero split, or the partial outputs of a K-split
// tiled launch (see combine_heads_kernel)
void launch_combine(DeviceState &d, hipStream_t st, int M, int N, float *O, const int32_t *gate, const int32_t *even,
                    bool even_any_m, bool vec4) {
    const size_t count4 = (size_t)M * (size_t)N / 4;     // K-split launches run only with N % 4 == 0
    hipLaunchKernelGGL(combine_heads_kernel, dim3((d.workers + kWavesPerBlock - 1) / kWavesPerBlock),
                       dim3(kBlockThreads), 0, st, M, N, d.workers, O, d.head, d.head_row, gate, vec4 ? 1 : 0, count4,
                       d.pending_ksplit, reinterpret_cast<const float4 *>(d.head), even, even_any_m ? 1 : 0);
    d.pending_ksplit = 0;
}

// --- one wavefront per row -----------------------------------------------------------------
// For sparse matrices so small that a call is latency, not throughput: below 8 M cells of S (where no tiled
// kernel is tried either) and with at most 2048 columns, so that even a full row is at most 32 chunks for its
// wavefront.  One launch instead of the equal-nonzero split's two (kernel + combine step), and a shorter chain of
// dependent loads inside it.  A wavefront walks its row alone, 64 / (lanes per entry) entries at a time, so wide
// outputs (few entries side by side) pay only with enough rows to keep every CU busy meanwhile; measured on the
// small shapes of the paper's grid: SPMM +14..+89 % except N = 128 with 1-2 k rows (-20 %), FusedMM +5..+60 % at
// N = 32 and -46..+12 % at N = 128.  CSRK_ROWS=2 forces it for every shape it can run (tests), =3 switches it off.
bool rows_mode_ok(int M, int K, int N, bool wider_for_narrow = true) {
    const int mode = env_int("CSRK_ROWS", 1);
    if (mode == 3) return false;
    if (mode == 2) return true;
    if (K > 2048) return false;
    // outputs of 32 columns or fewer: up to 16 M cells (measured at 6k/2k on the paper's grid against what ran
    // before, the narrow tiled kernel at 20-30 % density and the failed attempt at 10 %: +7..+42 % in all three
    // operations; at 16 M cells, 8k/2k, the tiled kernel is ahead again at 30 %)
    // (not for planned SDDMM calls: with the attempt's extra launches gone the tiled kernel stays 12 % ahead there)
    return (long long)M * K < ((N <= 32 && wider_for_narrow ? 16ll : 8ll) << 20);
}

// Larger matrices that get no tiled attempt (or whose attempt the device turns down) still gain from whole rows
// where the rows are even, which only the row analysis can tell: worth its launch (3-6 us) from 8 M cells, if the
// kernel can act on the answer (FusedMM's whole-row branch needs more than half as many rows as wavefronts);
// not beyond 256 K rows, where that single-workgroup kernel itself takes tens of microseconds.
bool even_rows_worth_asking(const DeviceState &d, int M, int K, bool fused) {
    if (env_int("CSRK_ROWS", 1) == 3) return false;
    if (fused && 2ll * M <= d.workers) return false;
    return (long long)M * K >= (8ll << 20) && M <= (1 << 18);
}

// wavefronts per row: enough wavefronts in flight for every CU whatever M is, and more of them where few entries
// go side by side (wide outputs: a wavefront then walks its part of the row in more steps)
int rows_wpr(int M, int N) {
    const int want = N > 64 ? 8192 : 3072;
    return M >= want ? 1 : (2 * M >= want ? 2 : 4);
}

dim3 rows_grid(int M, int wpr, int ytiles) {
    const long long blocks = ((long long)M * wpr + kWavesPerBlock - 1) / kWavesPerBlock;
    return dim3((unsigned)(blocks < 8192 ? blocks : 8192), ytiles);
}

template <int VD, int LD, int TD>
bool launch_fused_rows_n(const WidthCfg &nc, hipStream_t st, int M, int D, int N, const int32_t *rp, const int32_t *ci,
                         const float *v, const float *A, const float *B, const float *C, float *O) {
#define CSRK_FUSED_ROWS_CASE(VN, LN, TN)                                                                       \
    if (nc.vec == VN && nc.lg == LN && nc.t == TN) {                                                           \
        const int wpr = rows_wpr(M, N);                                                                        \
        hipLaunchKernelGGL((fusedmm_rows_kernel<VD, LD, TD, VN, LN, TN>), rows_grid(M, wpr, 1), dim3(kBlockThreads), \
                           0, st, M, D, N, rp, ci, v, A, B, C, O, wpr);                                        \
        return true;                                                                                           \
    }
    CSRK_FUSED_ROWS_CASE(4, 8, 1)
    CSRK_FUSED_ROWS_CASE(4, 16, 1)
    CSRK_FUSED_ROWS_CASE(4, 32, 1)
    CSRK_FUSED_ROWS_CASE(4, 64, 1)
    CSRK_FUSED_ROWS_CASE(4, 64, 2)
#undef CSRK_FUSED_ROWS_CASE
    return false;
}

// --- LDS-tiled path ---------------------------------------------------------------------
// Host-side eligibility (shapes only); the device-side analysis has the last word.
// Rows of S per wavefront in the LDS-tiled SPMM/FusedMM kernels (one workgroup of 16 wavefronts per CU at a
// time): 4, 2 or 1.  More rows spread the per-tile work (staging, barriers) over more entries, but the grid
// runs in rounds of `CUs` workgroups and a last round that is mostly empty costs as much as a full one:
// pick the count with the least rounds x (rows + one half row's worth of per-tile work); ties go to more rows.
// `three`: the kernel also comes with 3 rows per wavefront (for FusedMM, whose score stage maps its four groups of
// 16 lanes onto 1, 2 or 4 rows, it is the 4-row layout with one row left empty): 12 k rows are 256 workgroups of
// 48 rows, one full round, where 64 rows leave a quarter of the CUs without work and 32 rows take two rounds.
int tile_rows_for(const DeviceState &d, int M, int max_rows = 4, bool three = false) {
    int best = max_rows;
    long long best_cost = -1;
    for (int rows = max_rows; rows >= 1; rows = (rows == 4 && three) ? 3 : (rows == 3 ? 2 : rows >> 1)) {
        const long long blocks = ((long long)M + kTileWaves * rows - 1) / (kTileWaves * rows);
        const long long rounds = (blocks + d.cus - 1) / d.cus;
        const long long cost = rounds * (2 * rows + 1);
        if (best_cost < 0 || cost < best_cost) {
            best_cost = cost;
            best = rows;
        }
    }
    return best;
}
// K-split (the small-M regime): when 64-row workgroups leave CUs without work, keep 4 rows per wavefront and cut K
// into S ranges instead, one workgroup per (row block, range) - the counterpart, for the reduction dimension, of
// the paper's NT work-items per row (section "SDDMM", the NT heuristic).  Returns S (1 = no split).  Every range
// keeps at least four tiles (with fewer the split measured slower than one row per wavefront over the whole of K).
// The choice is by the cost model of tile_rows_for, rounds of `CUs` workgroups x per-workgroup work: without a
// split rounds x (2 rows + 1) for 4, 3, 2 or 1 rows per wavefront, with S ranges rounds x 9 / S, marked up by 3 %
// per range for the partial outputs that are written and added up; the cheapest wins.  Measured over S = 1..8 at
// 3072 / 5000 / 6144 / 7168 / 10000 / 12288 rows (four shapes each, SPMM and FusedMM) the best S was
// 5 / 3 / 5 / 2 / 3 / 4; "as many ranges as it takes to reach the CU count" (6 / 4 / 3 / 3 / 2 / 2) put a nearly
// empty second round behind the first and cost 25-40 %.
struct TileGrid {
    int ksplit;      // ranges of K (1 = no split)
    double fill;     // work of the grid / capacity of the rounds it takes, by the cost model (1 = no CU ever idle)
};
TileGrid tile_grid_for(const DeviceState &d, int M, int K, int tile_height, int rows_per_block, bool three = true) {
    const long long tiles = ((long long)K + tile_height - 1) / tile_height;
    const long long blocks = ((long long)M + rows_per_block - 1) / rows_per_block;
    auto rounds_of = [&](long long groups) { return (double)((groups + d.cus - 1) / d.cus); };
    double best_cost = 1e30;
    for (int rows = 4; rows >= 1; --rows)                          // no split (`three`: the kernel has a 3-row version here)
        if (rows != 3 || three)
            best_cost = fmin(best_cost, rounds_of(((long long)M + kTileWaves * rows - 1) / (kTileWaves * rows)) * (2 * rows + 1));
    int best = 1;
    const int mode = env_int("CSRK_KSPLIT", 1);                    // 2 = off (tests and measurements)
    const int forced = env_int("CSRK_KSPLIT_S", 0);                // measurements: this many ranges if K allows
    if (forced) {
        if (forced <= tiles && forced <= kMaxKSplit) best = forced;
    } else if (mode != 2 && blocks < d.cus) {
        long long smax = tiles / 4;
        if (smax > kMaxKSplit) smax = kMaxKSplit;
        for (long long s = 2; s <= smax; ++s) {
            const double cost = rounds_of(blocks * s) * 9.0 / (double)s / (1.0 - 0.03 * (double)s);
            if (cost < best_cost) {
                best_cost = cost;
                best = (int)s;
            }
        }
    }
    const double ideal = (double)M / 64.0 * 9.0 / (double)d.cus;   // 4 rows per wavefront on every CU all the time
    return {best, ideal / best_cost};
}
int ksplit_for(const DeviceState &d, int M, int K, int tile_height, int rows_per_block, bool three = true) {
    return tile_grid_for(d, M, K, tile_height, rows_per_block, three).ksplit;
}
constexpr float kTileMinDensity = 0.02f;      // wide tiled kernels and tiled SDDMM
constexpr double kWellFilled = 0.87;          // TileGrid::fill from which a grid counts as filling the CUs
constexpr float kNarrowMinDensity = 0.25f;    // FusedMM with outputs of 32 columns or fewer (measured cross-over with whole rows)

int32_t *tile_flags(DeviceState &d) { return d.plan_flags ? d.plan_flags : d.head_row + d.workers + 8 + 8 * d.flag_set; }
// the set of flag words the next unplanned tiled attempt will use (nothing to look after under a plan, nor with
// scratch that was handed in: such calls keep no state from one call to the next and always analyse by a launch
// of reset_flags_kernel, which clears the ordering flag of the set it fills)
int32_t *other_flags(DeviceState &d) { return (d.plan_flags || d.fixed) ? nullptr : d.head_row + d.workers + 8 + 8 * (1 - d.flag_set); }

// CSRK_KTILE=2 (tests) takes the tiled kernels wherever they can run, whatever the density and row lengths
// (a negative threshold tells the analysis kernel so)
// Density from which the wide tiled kernels beat what runs otherwise (whole rows; equal shares for FusedMM with few
// rows), by the size of the gathered dense operand (columns: 2, 4, 8, 16 MB and more) and by M (rows of the table:
// below 2048, 4096, 8192 rows, and above); 1 = never.  Read off a grid of 100 (M, K, N, density) points with
// whole calls timed.
float wide_min_density(int M, int K, int N, bool fused, bool well_filled = false) {
    if (env_int("CSRK_KTILE", 1) == 2) return -1.f;
    const long long dense_bytes = (long long)K * N * 4;
    const int size = dense_bytes >= (16ll << 20) ? 3 : dense_bytes >= (8ll << 20) ? 2 : dense_bytes >= (4ll << 20) ? 1 : 0;
    const int rows = M < 2048 ? 0 : M < 4096 ? 1 : M < 8192 ? 2 : 3;
    static const float spmm[4][4] = {{1.f, 1.f, 0.20f, 0.05f}, {1.f, 0.08f, 0.05f, 0.015f}, {0.10f, 0.08f, 0.06f, kTileMinDensity},
                                     {0.07f, 0.06f, 0.035f, kTileMinDensity}};
    static const float fusedmm[4][4] = {{1.f, 1.f, 0.08f, 0.04f}, {1.f, 0.08f, 0.035f, kTileMinDensity},
                                        {0.10f, 0.06f, 0.06f, kTileMinDensity}, {0.075f, 0.07f, 0.04f, kTileMinDensity}};
    // (re-measured at 2048 ... 20000 rows with the K ranges chosen as they are now.  From 4096 rows: at 8 MB whole rows
    // keep up to 5 % - level at 4096 rows, 11-20 % ahead at 6144 - and at 16 MB to 2 %, by 13-34 % from 10000 rows; from
    // 32 MB the tiled kernel is 6-38 % ahead at 2 %.  2048 to 4095 rows: tiled 16 % ahead at 10 % and 4 MB, 25-36 % at
    // 2 % and 16 MB and more.  FusedMM from 8192 rows at 4 MB: whole rows 28 % ahead at 5 %.)
    // 4096 to 8191 rows whose grid fills the CUs (`well_filled`: 4096 rows split into ranges of K do, 6144 rows leave a
    // quarter of the last round empty): tiled 20-60 % ahead at 5 % and 8 MB and at 2 % from 16 MB, 8 % at 5 % and 4 MB
    if (rows == 2 && well_filled) {
        static const float filled[4] = {0.09f, 0.06f, 0.04f, 0.015f};
        return size == 1 && !fused ? 0.045f : filled[size];      // (FusedMM at 4 MB and 5 %: whole rows 5-7 % ahead)
    }
    if (rows >= 2 && size == 3 && dense_bytes < (32ll << 20)) return 0.03f;
    return fused ? fusedmm[rows][size] : spmm[rows][size];
}
// Density from which the narrow tiled kernels beat what runs otherwise (whole rows for even matrices, which
// is all the tiled kernels take), read off grids of (M, K, N, density) measured on MI355X with whole calls timed.  It falls with the size of the gathered dense operand (the general
// path gathers at L2 speed while K x N floats fit an XCD's 4 MB L2 and collapses beyond, the tiled kernels do not
// care) and with M (every workgroup stages the whole operand through LDS whatever its rows hold: fewer rows per
// CU, less to spread that over).
float narrow_min_density(int M, int K, int N, bool fused, bool well_filled = false) {
    if (env_int("CSRK_KTILE", 1) == 2) return -1.f;
    const long long dense_bytes = (long long)K * N * 4;
    // (FusedMM at 32 columns: the tiled kernel passes whole rows at 20 % only on the largest shapes, 24k/8k and 32k/8k)
    if (N <= 32)
        return fused ? ((M >= 24576 && K >= 8192) ? 0.18f : kNarrowMinDensity) : (dense_bytes >= (2ll << 20) ? 0.12f : 0.15f);
    const int size = dense_bytes >= (8ll << 20) ? 3 : dense_bytes >= (4ll << 20) ? 2 : dense_bytes >= (2ll << 20) ? 1 : 0;
    const int rows = M < 8192 ? 0 : M < 12288 ? 1 : 2;
    static const float spmm[3][4] = {{0.17f, 0.17f, 0.15f, 0.06f}, {0.15f, 0.09f, 0.08f, 0.05f}, {0.08f, 0.07f, 0.07f, 0.045f}};
    static const float fusedmm[3][4] = {{0.17f, 0.15f, 0.09f, 0.05f}, {0.15f, 0.09f, 0.09f, 0.05f}, {0.13f, 0.09f, 0.085f, 0.045f}};
    // Below 8192 rows the attempt got cheap enough, once the row analysis had moved into the tiled kernel, for 10 % at
    // 2 MB and more - where the grid fills the CUs (`well_filled`: 4096 rows in 4 ranges of K do exactly; 4k/4k/128 is
    // 9-13 % faster tiled there).  Not at 3072 or between 5000 and 7168 rows, whose grids leave 15-20 % of the rounds
    // empty and where whole rows stay 5-25 % ahead at 10 %.
    if (rows == 0 && size >= 1 && well_filled) return fminf(fused ? fusedmm[0][size] : spmm[0][size], 0.095f);
    // FusedMM at 12288 rows (no 3-row kernel at that width) needs 11 % at 2 MB, where 16384 rows win from 9 %
    if (fused && rows == 2 && size == 1 && M < 16384) return 0.11f;
    if (fused && rows == 2 && size == 0 && N > 64) return 0.08f;
    return fused ? fusedmm[rows][size] : spmm[rows][size];
}
// ... and the tiled SDDMM kernel (64 lanes = 64 entries of one row: short segments waste lanes)
float sddmm_min_density(int M, int K, int D) {
    if (env_int("CSRK_KTILE", 1) == 2) return -1.f;
    const bool big = (long long)K * D * 4 >= (8ll << 20);
    // rows of B of more than 64 floats: whole rows keep up to 10 % with an operand below 4 MB (12k/4k/128: +37 %) and,
    // below 16384 rows, below 8 MB (10000 and 12288 rows by 8192 columns: +25..+37 %; level at 8192 rows; from 24k
    // rows the tiled kernel is 2-18 % ahead there)
    if (M >= 8192 && D > 64 && ((long long)K * D * 4 < (4ll << 20) || (!big && M < 16384))) return 0.12f;
    if (M < 8192) return big ? 0.08f : 0.15f;
    if (M < 12288) return big ? 0.05f : (D > 64 ? 0.09f : 0.08f);
    return big ? 0.05f : (D > 64 ? 0.09f : 0.05f);
}

constexpr int kWideSlab = 512;      // columns one wide tiled kernel holds in registers
constexpr int kWideMaxN = 2048;     // widest output the wide tiled kernels take, in slabs (wide_slab_width)
bool ktile_shape_ok(const DeviceState &d, int M, int K, int N) {
    const int mode = env_int("CSRK_KTILE", 1);       // 1 auto, 2 force where the kernel can run, 3 off
    if (mode == 3) return false;
    // the wide tiled kernels read the dense operand through a buffer descriptor, whose extent is a 32-bit byte count
    if ((long long)K * N * 4 >= (1ll << 32)) return false;
    if (N % 4 != 0 || N > kWideMaxN || N <= 128) return mode == 2 && N % 4 == 0 && N <= kWideMaxN;
    if (mode == 2) return true;
    // Measured cross-over with the general path (whose gathers run at L2 speed while the dense operand fits an
    // XCD's L2 and collapse beyond): a dense operand of 8 MB or more with at least 1024 rows, 4 MB with 2048,
    // 2 MB with 4096.  Small M is handled by cutting K into ranges (ksplit_for).  CSRK_KTILE_MIN_MB overrides
    // the 4 (tests).
    const long long dense_bytes = (long long)K * N * 4;
    const long long min_bytes = (long long)env_int("CSRK_KTILE_MIN_MB", 4) << 20;
    return (M >= 1024 && dense_bytes >= 2 * min_bytes) || (M >= 2048 && dense_bytes >= min_bytes) ||
           (M >= 4096 && dense_bytes >= min_bytes / 2);
}

constexpr int kSddmmMaxD = 1024;    // longest dot product the tiled SDDMM kernel takes, 128 floats per launch
bool sddmm_tile_shape_ok(const DeviceState &d, int M, int K, int D) {
    const int mode = env_int("CSRK_KTILE", 1);
    if (mode == 3 || D % 4 != 0 || D > 128 || D < 4) return false;
    if (mode == 2) return true;
    // below 8 M cells of S a call takes 10-30 us whichever kernel does it, and a failed attempt (row analysis plus
    // a tiled launch that stands down, about 5 us) costs more than a successful one gains
    return (long long)M >= 16ll * d.cus && (long long)M * K >= (8ll << 20);
}

template <int DMAX, int ROWS>
csrk_status launch_sddmm_ktile(DeviceState &d, hipStream_t st, int M, int K, int D, const int32_t *rp,
                               const int32_t *ci, const float *v, const float *A, const float *B, float *P, int ld,
                               int col0, int accumulate) {
    using L = SddmmTileLds<DMAX, ROWS>;
    static_assert(L::kBytes <= 160 * 1024, "tile does not fit the 160 KB of LDS of a gfx950 CU");
    auto kern = sddmm_ktile_kernel<DMAX, ROWS>;
    static bool attr_set[kMaxDevices] = {};
    int dev = 0;
    CSRK_HIP(hipGetDevice(&dev));
    if (!attr_set[dev]) {
        CSRK_HIP(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, L::kBytes));
        attr_set[dev] = true;
    }
    const int rb = kTileWaves * ROWS;
    hipLaunchKernelGGL(kern, dim3((M + rb - 1) / rb), dim3(kTileThreads), L::kBytes, st, M, K, D, ld, accumulate, rp,
                       ci, v, A + col0, B + col0, P, tile_flags(d), d.inline_density, other_flags(d));
    CSRK_HIP(hipGetLastError());
    return CSRK_OK;
}

template <int DMAX>
csrk_status launch_sddmm_ktile_rows(DeviceState &d, hipStream_t st, int M, int K, int D, const int32_t *rp,
                                    const int32_t *ci, const float *v, const float *A, const float *B, float *P,
                                    int ld = 0, int col0 = 0, int accumulate = 0) {
    // ld != 0: columns [col0, col0 + D) of rows of A and B that are `ld` floats long, one piece of a longer dot
    // product; accumulate: add this piece to what P holds
    if (ld == 0) ld = D;
    // (cutting K into ranges for small M, as SPMM and FusedMM do, measured no gain here: the tile is 288-1152
    // rows high, so a K of a few thousand leaves too few tiles per range)
    // rows per wavefront by the same rule as SPMM / FusedMM (the 128-wide kernel takes at most two: its score loop
    // is twice as long and four rows would spill)
    constexpr int kMaxRows = DMAX <= 64 ? 4 : 2;
    switch (tile_rows_for(d, M, kMaxRows, true)) {
        case 4:
            if constexpr (kMaxRows >= 4) return launch_sddmm_ktile<DMAX, 4>(d, st, M, K, D, rp, ci, v, A, B, P, ld, col0, accumulate);
            [[fallthrough]];
        case 3:
            if constexpr (kMaxRows >= 4) return launch_sddmm_ktile<DMAX, 3>(d, st, M, K, D, rp, ci, v, A, B, P, ld, col0, accumulate);
            [[fallthrough]];
        case 2: return launch_sddmm_ktile<DMAX, 2>(d, st, M, K, D, rp, ci, v, A, B, P, ld, col0, accumulate);
        default: return launch_sddmm_ktile<DMAX, 1>(d, st, M, K, D, rp, ci, v, A, B, P, ld, col0, accumulate);
    }
}

// a density threshold of the wide tiled kernels (outputs of more than 128 columns), marked for the row analysis as
// one that goes with moderately uneven rows (row_analysis); "never" (1) and "always" (negative) stay what they are
float uneven_ok(float min_density) { return min_density >= 0.f && min_density < 1.f ? min_density + kUnevenOk : min_density; }

csrk_status launch_analysis(DeviceState &d, hipStream_t st, int M, int K, const int32_t *rp, float min_density) {
    int32_t *flags = tile_flags(d);
    // column order is verified inside the tiled kernels themselves
    hipLaunchKernelGGL(reset_flags_kernel, dim3(1), dim3(1024), 0, st, M, K, rp, min_density, flags, other_flags(d));
    CSRK_HIP(hipGetLastError());
    return CSRK_OK;
}

// Up to this many rows the tiled kernels do the row analysis themselves: every workgroup reads rowptr (32 KB at
// the limit, from L2) for a microsecond or two, against 3-6 us and a kernel boundary for the analysis launch.
constexpr int kInlineAnalysisMaxRows = 8192;

// Row analysis for a tiled attempt.  Without a plan: the analysis kernel, and the attempt always goes ahead (the
// device has the last word).  With a plan the answer is known on the host: what the analysis kernel and the
// kernels' own order check would find was found when the plan was made.
csrk_status tiled_attempt(DeviceState &d, const csrk_plan_s *plan, hipStream_t st, int M, int K, const int32_t *rp,
                          float min_density, bool *go) {
    if (!plan) {
        *go = true;
        d.attempted = true;
        if (!d.fixed && M <= kInlineAnalysisMaxRows) {      // the tiled kernel's workgroups read rowptr themselves (tile_go)
            d.inline_density = min_density;
            return CSRK_OK;
        }
        return launch_analysis(d, st, M, K, rp, min_density);
    }
    // (a plan knows `even` only; uneven patterns have their schedule, see sched_usable)
    const float threshold = min_density >= kUnevenOk ? min_density - kUnevenOk : min_density;
    const bool dense = (double)plan->nnz >= (double)threshold * (double)M * (double)K;
    *go = plan->sorted && (min_density < 0.f || (dense && plan->even));
    return CSRK_OK;
}

// Planned calls on a small S (below 8 M cells, where unplanned calls take the whole-row kernels because a tiled
// attempt costs three more launches than it gains): with a plan either way is ONE launch, and the narrow LDS-tiled
// kernels then win from about 12 rows per CU on dense enough patterns.  Measured with planned calls on the small
// shapes of the paper's grid, tiled against whole rows: at 3-4 k rows and K = 1024, SDDMM 1.09-1.45x at 20-30 %
// (0.86-1.06 at 10 %), SPMM 1.12-1.55x at width 128 and 20-30 % (width 32: 1.04-1.12 at 30 % only), FusedMM
// 1.08-1.49x at width 128 and 30 %, and at 20 % with 4 k rows (1.14; 0.86 with 3 k); with 1-2 k rows the tiled
// kernels lose throughout (0.3-0.9).  `kind`: 0 SPMM, 1 SDDMM, 2 FusedMM; W: output width (dot length for SDDMM).
bool plan_small_tiled(const DeviceState &d, const csrk_plan_s *plan, int M, int K, int W, int kind) {
    if (!plan || !plan->sorted || !plan->even || env_int("CSRK_KTILE", 1) != 1 || env_int("CSRK_ROWS", 1) != 1)
        return false;
    if (W % 4 != 0 || W < 4 || W > 128) return false;
    if ((long long)M * K >= (8ll << 20) || K > 2048 || M < 12 * d.cus) return false;
    const double density = (double)plan->nnz / ((double)M * (double)K);
    if (kind == 1) return density >= 0.15;
    if (kind == 0) return W > 64 ? density >= 0.15 : density >= 0.25;
    return W > 64 && (density >= 0.25 || (M >= 16 * d.cus && density >= 0.15));
}

// per-call state of the flag words: a plan's own words for the duration of a planned call; after an unplanned tiled
// attempt the two per-call sets change places
struct PlanScope {
    DeviceState &d;
    PlanScope(DeviceState &dev, const csrk_plan_s *plan) : d(dev) {
        d.plan_flags = plan ? plan->dflags : nullptr;
        d.inline_density = __builtin_nanf("");
        d.attempted = false;
    }
    ~PlanScope() {
        // the next attempt on the lazily grown scratch takes the set of flag words this one has cleared
        if (d.lazy && d.attempted) d.lazy->flag_set = d.flag_set ^ 1;
    }
};

// narrow outputs (N <= 128): G entries side by side per wavefront.  Thresholds below were read off a
// sweep of the paper's 72 benchmark shapes on MI355X (tiled against general kernel, per shape).
bool narrow_shape_ok(const DeviceState &d, int M, int K, int N, bool fused) {
    const int mode = env_int("CSRK_KTILE", 1);
    if (mode == 3 || N % 4 != 0 || N > 128 || N < 4) return false;
    if (mode == 2) return true;
    const long long rows_per_cu = (long long)M / d.cus;
    if (N <= 32) return rows_per_cu >= (fused ? 96 : 32);   // tiny dense operand: the general path's gathers stay in cache
    // at least 12 rows per CU (3072 rows: with K cut into ranges the tiled kernels are 10-45 % ahead of whole rows
    // at 20 % density there), and enough cells of S (see sddmm_tile_shape_ok)
    return rows_per_cu >= 12 && (long long)M * K >= (8ll << 20);
}

// A plan's schedule as a launch sees it (see csrk_plan_s::Sched): the tiled kernels then take their rows and K
// ranges from the schedule instead of from the grid.
struct SchedPart {
    const int32_t *perm;
    const int4 *items;
    int n_items;
    size_t partial_offset;      // floats into the scratch area where the partial rows start
};

// tile height of the narrow SPMM kernel: as high as LDS allows with the 128-entry look-ahead in mind (256 rows
// of 128 columns, 384 of 64 or 32)
template <int G>
constexpr int narrow_kt() {
    return G == 2 ? 256 : 384;
}

template <int G, int ROWS>
csrk_status launch_narrow_rows(DeviceState &d, hipStream_t st, int M, int K, int N, const int32_t *rp,
                               const int32_t *ci, const float *v, const float *C, float *O, int ksplit = 1,
                               const SchedPart *sp = nullptr) {
    constexpr int KT = narrow_kt<G>();
    using L = NarrowLds<G, KT>;
    static_assert(L::kBytes <= 160 * 1024, "tile does not fit the 160 KB of LDS of a gfx950 CU");
    // register prefetch of the next tile: all of a thread's loads
    constexpr int kPer = KT / (kTileThreads / (64 / G));
    auto kern = ktile_narrow_kernel<G, KT, ROWS, kPer>;
    static bool attr_set[kMaxDevices] = {};
    int dev = 0;
    CSRK_HIP(hipGetDevice(&dev));
    if (!attr_set[dev]) {
        CSRK_HIP(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, L::kBytes));
        attr_set[dev] = true;
    }
    const int rb = kTileWaves * ROWS;
    hipLaunchKernelGGL(kern, sp ? dim3(sp->n_items) : dim3((M + rb - 1) / rb, ksplit), dim3(kTileThreads), L::kBytes, st,
                       M, K, N, rp, ci, v, C, O, tile_flags(d), d.head + (sp ? sp->partial_offset : 0), d.inline_density,
                       other_flags(d), sp ? sp->perm : (const int32_t *)nullptr, sp ? sp->items : (const int4 *)nullptr);
    CSRK_HIP(hipGetLastError());
    if (ksplit > 1) d.pending_ksplit = ksplit;     // the call's last kernel adds the partial outputs (launch_combine)
    return CSRK_OK;
}

template <int G>
csrk_status launch_narrow_g(DeviceState &d, hipStream_t st, int M, int K, int N, const int32_t *rp,
                            const int32_t *ci, const float *v, const float *C, float *O) {
    // small M: keep 4 rows per wavefront and cut K into ranges instead
    // (not for outputs of 32 columns or fewer, G = 8: there the split never measured faster)
    const int ksplit = G == 8 ? 1 : ksplit_for(d, M, K, narrow_kt<G>(), kTileWaves * 4);
    if (ksplit > 1) {
        if (csrk_status s = ensure_scratch(d, N, (size_t)ksplit * (size_t)M * (size_t)N)) return s;
        return launch_narrow_rows<G, 4>(d, st, M, K, N, rp, ci, v, C, O, ksplit);
    }
    switch (tile_rows_for(d, M, 4, true)) {
        case 4: return launch_narrow_rows<G, 4>(d, st, M, K, N, rp, ci, v, C, O);
        case 3: return launch_narrow_rows<G, 3>(d, st, M, K, N, rp, ci, v, C, O);
        case 2: return launch_narrow_rows<G, 2>(d, st, M, K, N, rp, ci, v, C, O);
        default: return launch_narrow_rows<G, 1>(d, st, M, K, N, rp, ci, v, C, O);
    }
}

// narrow SPMM: G entries side by side, G chosen by the output width
csrk_status launch_narrow(DeviceState &d, hipStream_t st, int M, int K, int N, const int32_t *rp, const int32_t *ci,
                          const float *v, const float *C, float *O) {
    if (N > 64) return launch_narrow_g<2>(d, st, M, K, N, rp, ci, v, C, O);
    if (N > 32) return launch_narrow_g<4>(d, st, M, K, N, rp, ci, v, C, O);
    return launch_narrow_g<8>(d, st, M, K, N, rp, ci, v, C, O);
}

template <int T, int KT, int ROWS>
csrk_status launch_ktile_rows(DeviceState &d, hipStream_t st, int M, int K, int N, int ld, int col0, const int32_t *rp,
                              const int32_t *ci, const float *v, const float *B, float *O, int ksplit = 1,
                              const SchedPart *sp = nullptr) {
    using L = KTileLds<T, KT>;
    static_assert(L::kBytes <= 160 * 1024, "tile does not fit the 160 KB of LDS of a gfx950 CU");
    static_assert((KT * T * 64) % kTileThreads == 0, "the staging loop copies whole rounds of 1024 float4");
    auto kern = ktile_kernel<T, KT, ROWS>;
    static bool attr_set[kMaxDevices] = {};
    int dev = 0;
    CSRK_HIP(hipGetDevice(&dev));
    if (!attr_set[dev]) {
        CSRK_HIP(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, L::kBytes));
        attr_set[dev] = true;
    }
    const int rb = kTileWaves * ROWS;
    hipLaunchKernelGGL(kern, sp ? dim3(sp->n_items) : dim3((M + rb - 1) / rb, ksplit), dim3(kTileThreads), L::kBytes, st,
                       M, K, N, ld, rp, ci, v, B + col0, O + col0, tile_flags(d),
                       d.head + col0 + (sp ? sp->partial_offset : 0), d.inline_density, other_flags(d), (long long *)nullptr,
                       sp ? sp->perm : (const int32_t *)nullptr, sp ? sp->items : (const int4 *)nullptr);
    CSRK_HIP(hipGetLastError());
    if (ksplit > 1) d.pending_ksplit = ksplit;     // the call's last kernel adds the partial outputs (launch_combine)
    return CSRK_OK;
}

// One launch of the wide SPMM kernel over columns [col0, col0 + N) of operands whose rows are `ld` floats long
// (ld = N, col0 = 0: the whole operand).  Partial outputs of a K-split launch keep the full row length, so one
// combine step serves all the slabs of a call.
template <int T, int KT>
csrk_status launch_ktile(DeviceState &d, hipStream_t st, int M, int K, int N, int ld, int col0, const int32_t *rp,
                         const int32_t *ci, const float *v, const float *B, float *O, int fixed_ksplit = 0) {
    const int ksplit = fixed_ksplit ? fixed_ksplit : ksplit_for(d, M, K, KT, kTileWaves * 4);
    if (ksplit > 1) {
        if (csrk_status s = ensure_scratch(d, ld, (size_t)ksplit * (size_t)M * (size_t)ld)) return s;
        return launch_ktile_rows<T, KT, 4>(d, st, M, K, N, ld, col0, rp, ci, v, B, O, ksplit);
    }
    switch (tile_rows_for(d, M, 4, true)) {
        case 4: return launch_ktile_rows<T, KT, 4>(d, st, M, K, N, ld, col0, rp, ci, v, B, O);
        case 3: return launch_ktile_rows<T, KT, 3>(d, st, M, K, N, ld, col0, rp, ci, v, B, O);
        case 2: return launch_ktile_rows<T, KT, 2>(d, st, M, K, N, ld, col0, rp, ci, v, B, O);
        default: return launch_ktile_rows<T, KT, 1>(d, st, M, K, N, ld, col0, rp, ci, v, B, O);
    }
}

// Outputs wider than the 512 columns one wide tiled kernel holds in registers go in slabs of 512 columns and a
// remainder, one launch per slab (the 256-wide kernel for a remainder of up to 256 columns).  Every slab walks S
// again: 8 bytes per entry against 2 KB of dense row per entry and slab.  All slabs of a call are cut into the same
// number of K ranges - one combine step adds their partial outputs - chosen for the tallest tile among their kernels.
bool wide_remainder_is_small(int N) { return N % kWideSlab != 0 && N % kWideSlab <= 256; }

// FusedMM's 3-row version carries the score-stage work and registers of four rows, so it pays only where 48-row
// workgroups save a whole round of the grid against 32-row ones and the accumulate stage is long: measured at
// 24 k rows +10 % at width 128 and -3 % at width 32; at 12 k rows (one round either way) -1..-2 %.
bool fused_three_rows(const DeviceState &d, int M, int N) {
    return N > 64 && (long long)M > 64ll * d.cus;
}

template <int T, int KT, int ROWS, int SL, int LIVE = ROWS>
csrk_status launch_fused_ktile_rows(DeviceState &d, hipStream_t st, int M, int K, int D, int N, int ld, int col0,
                                    const int32_t *rp, const int32_t *ci, const float *v, const float *A, const float *B,
                                    const float *C, float *O, int ksplit = 1, const SchedPart *sp = nullptr) {
    using L = FusedTileLds<T, KT, ROWS, SL>;
    static_assert(L::kBytes <= 160 * 1024, "tile does not fit the 160 KB of LDS of a gfx950 CU");
    static_assert((KT * T * 64) % kTileThreads == 0, "the staging loop copies whole rounds of 1024 float4");
    // how much of the next tile is prefetched into registers: as many of a thread's loads as still fit in 128
    // registers beside the accumulators (5 of 6 for one 256-wide piece of output, 5 of 8 for two)
    constexpr int kPer = KT * T * 64 / kTileThreads;
    constexpr int kPrefetch = T == 2 ? 5 : kPer - 1;
    auto kern = fused_ktile_kernel<T, KT, ROWS, SL, kPrefetch, LIVE>;
    static bool attr_set[kMaxDevices] = {};
    int dev = 0;
    CSRK_HIP(hipGetDevice(&dev));
    if (!attr_set[dev]) {
        CSRK_HIP(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, L::kBytes));
        attr_set[dev] = true;
    }
    const int rb = kTileWaves * LIVE;
    hipLaunchKernelGGL(kern, sp ? dim3(sp->n_items) : dim3((M + rb - 1) / rb, ksplit), dim3(kTileThreads), L::kBytes, st,
                       M, K, D, N, ld, rp, ci, v, A, B, C + col0, O + col0, tile_flags(d),
                       d.head + col0 + (sp ? sp->partial_offset : 0), d.inline_density, other_flags(d), (long long *)nullptr,
                       sp ? sp->perm : (const int32_t *)nullptr, sp ? sp->items : (const int4 *)nullptr);
    CSRK_HIP(hipGetLastError());
    if (ksplit > 1) d.pending_ksplit = ksplit;     // the call's last kernel adds the partial outputs (launch_combine)
    return CSRK_OK;
}

template <int T, int KT, int SL>
csrk_status launch_fused_ktile(DeviceState &d, hipStream_t st, int M, int K, int D, int N, int ld, int col0,
                               const int32_t *rp, const int32_t *ci, const float *v, const float *A, const float *B,
                               const float *C, float *O, int fixed_ksplit = 0) {
    // columns [col0, col0 + N) of C and O, whose rows are `ld` floats long (see launch_ktile); every slab of a wider
    // output computes the scores again, a sixth of its work at 512 columns
    const int ksplit = fixed_ksplit ? fixed_ksplit : ksplit_for(d, M, K, KT, kTileWaves * 4, fused_three_rows(d, M, N));
    if (ksplit > 1) {
        if (csrk_status s = ensure_scratch(d, ld, (size_t)ksplit * (size_t)M * (size_t)ld)) return s;
        return launch_fused_ktile_rows<T, KT, 4, SL>(d, st, M, K, D, N, ld, col0, rp, ci, v, A, B, C, O, ksplit);
    }
    // 3 rows per wavefront: the kernel laid out for 4, the fourth row of every wavefront empty (see fused_three_rows)
    switch (tile_rows_for(d, M, 4, fused_three_rows(d, M, N))) {
        case 4: return launch_fused_ktile_rows<T, KT, 4, SL>(d, st, M, K, D, N, ld, col0, rp, ci, v, A, B, C, O);
        case 3: return launch_fused_ktile_rows<T, KT, 4, SL, 3>(d, st, M, K, D, N, ld, col0, rp, ci, v, A, B, C, O);
        case 2: return launch_fused_ktile_rows<T, KT, 2, SL>(d, st, M, K, D, N, ld, col0, rp, ci, v, A, B, C, O);
        default: return launch_fused_ktile_rows<T, KT, 1, SL>(d, st, M, K, D, N, ld, col0, rp, ci, v, A, B, C, O);
    }
}

// --- narrow FusedMM (N <= 128, D <= 128): fused_narrow_kernel -------------------------------------------
// tile height: as many rows as the C and B tiles plus the 64-entry slots (32 KB) leave room for in 160 KB, in whole
// rounds of the staging loop: 160 / 192 / 256 rows for outputs up to 128 / 64 / 32 columns with dot lengths up to 64
// (measured against 128 rows: 32k/8k and 8k/8k at width 64 +10..+13 %, 24k/8k at width 32 +23 %, the rest level);
// 128 rows with 128-float rows of B
template <int G, int DMAX>
constexpr int fused_narrow_kt() {
    if (DMAX == 64) return G == 2 ? 160 : (G == 4 ? 192 : 256);
    return 128;
}

template <int G, int ROWS, int DMAX, int LIVE = ROWS>
csrk_status launch_fused_narrow_rows(DeviceState &d, hipStream_t st, int M, int K, int D, int N, const int32_t *rp,
                                     const int32_t *ci, const float *v, const float *A, const float *B,
                                     const float *C, float *O, int ksplit = 1, int ld = 0, int col0 = 0,
                                     const SchedPart *sp = nullptr) {
    if (ld == 0) ld = N;        // otherwise: columns [col0, col0 + N) of C and O, whose rows are `ld` floats long
    constexpr int KT = fused_narrow_kt<G, DMAX>();
    constexpr int SL = 64;
    using L = FusedNarrowLds<G, KT, ROWS, SL, DMAX>;
    static_assert(L::kBytes <= 160 * 1024, "tile does not fit the 160 KB of LDS of a gfx950 CU");
    // register prefetch of the next tile: as many of a thread's loads as fit in 128 registers beside the score
    // stage (which is twice as long for 128-float rows of B)
    constexpr int kPer = KT / (kTileThreads / (64 / G));
    constexpr int kPrefetch = DMAX == 128 ? (kPer - 1 < 2 ? kPer - 1 : 2) : (kPer <= 2 ? kPer : kPer - 1);
    auto kern = fused_narrow_kernel<G, KT, ROWS, SL, DMAX, kPrefetch, LIVE>;
    static bool attr_set[kMaxDevices] = {};
    int dev = 0;
    CSRK_HIP(hipGetDevice(&dev));
    if (!attr_set[dev]) {
        CSRK_HIP(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, L::kBytes));
        attr_set[dev] = true;
    }
    const int rb = kTileWaves * LIVE;
    hipLaunchKernelGGL(kern, sp ? dim3(sp->n_items) : dim3((M + rb - 1) / rb, ksplit), dim3(kTileThreads), L::kBytes, st,
                       M, K, D, N, ld, rp, ci, v, A, B, C + col0, O + col0, tile_flags(d),
                       d.head + col0 + (sp ? sp->partial_offset : 0), d.inline_density, other_flags(d),
                       sp ? sp->perm : (const int32_t *)nullptr, sp ? sp->items : (const int4 *)nullptr);
    CSRK_HIP(hipGetLastError());
    if (ksplit > 1) d.pending_ksplit = ksplit;     // the call's last kernel adds the partial outputs (launch_combine)
    return CSRK_OK;
}

template <int G, int DMAX>
csrk_status launch_fused_narrow_g(DeviceState &d, hipStream_t st, int M, int K, int D, int N, const int32_t *rp,
                                  const int32_t *ci, const float *v, const float *A, const float *B, const float *C,
                                  float *O, int ld = 0, int col0 = 0, int fixed_ksplit = 0) {
    if (ld == 0) ld = N;        // otherwise a slab of a wider output (see launch_ktile), all slabs with one K-split
    // small M: keep 4 rows per wavefront and cut K into ranges (not for outputs of 32 columns or fewer)
    const int ksplit = fixed_ksplit ? fixed_ksplit
                       : G == 8     ? 1
                                    : ksplit_for(d, M, K, fused_narrow_kt<G, DMAX>(), kTileWaves * 4, fused_three_rows(d, M, N));
    if (ksplit > 1) {
        if (csrk_status s = ensure_scratch(d, ld, (size_t)ksplit * (size_t)M * (size_t)ld)) return s;
        return launch_fused_narrow_rows<G, 4, DMAX>(d, st, M, K, D, N, rp, ci, v, A, B, C, O, ksplit, ld, col0);
    }
    switch (tile_rows_for(d, M, 4, fused_three_rows(d, M, N))) {
        case 4: return launch_fused_narrow_rows<G, 4, DMAX>(d, st, M, K, D, N, rp, ci, v, A, B, C, O, 1, ld, col0);
        case 3: return launch_fused_narrow_rows<G, 4, DMAX, 3>(d, st, M, K, D, N, rp, ci, v, A, B, C, O, 1, ld, col0);
        case 2: return launch_fused_narrow_rows<G, 2, DMAX>(d, st, M, K, D, N, rp, ci, v, A, B, C, O, 1, ld, col0);
        default: return launch_fused_narrow_rows<G, 1, DMAX>(d, st, M, K, D, N, rp, ci, v, A, B, C, O, 1, ld, col0);
    }
}

template <int DMAX>
csrk_status launch_fused_narrow_d(DeviceState &d, hipStream_t st, int M, int K, int D, int N, const int32_t *rp,
                                  const int32_t *ci, const float *v, const float *A, const float *B, const float *C,
                                  float *O) {
    if (N > 64) return launch_fused_narrow_g<2, DMAX>(d, st, M, K, D, N, rp, ci, v, A, B, C, O);
    if (N > 32) return launch_fused_narrow_g<4, DMAX>(d, st, M, K, D, N, rp, ci, v, A, B, C, O);
    return launch_fused_narrow_g<8, DMAX>(d, st, M, K, D, N, rp, ci, v, A, B, C, O);
}

csrk_status launch_fused_narrow(DeviceState &d, hipStream_t st, int M, int K, int D, int N, const int32_t *rp,
                                const int32_t *ci, const float *v, const float *A, const float *B, const float *C,
                                float *O) {
    if (D > 64) return launch_fused_narrow_d<128>(d, st, M, K, D, N, rp, ci, v, A, B, C, O);
    return launch_fused_narrow_d<64>(d, st, M, K, D, N, rp, ci, v, A, B, C, O);
}

// --- planned calls on uneven rows: the schedule made by csrk_plan_create (csrk_plan_s::Sched) --------------------
// Cost of a workgroup in units of one stored entry's work: it stages every dense row of its K range whatever the
// rows of S hold, which costs about as much as kSchedRowCost entries per dense row, plus its entries.  The aim is
// kSchedPerCu workgroups per CU, the heaviest first, none cut finer than kSchedMinSegment columns of K.
// Measured on 8192 x 8192, log-normal row lengths (mean 10 % of K, sigma 1), FusedMM D = 64 N = 512 / SPMM N = 512,
// in us: row cost 16 with 2 per CU 536 / 428; 8 with 3: 576 / 492; 16 with 3: 590 / 467; 8 with 2: 637 / 502;
// 32 with 3: 616 / 505; 4 with 3: 610 / 495; ranges down to 256 columns: 609-775 / 488-673.  A second class of
// blocks of 16 rows (one per wavefront) for the longest rows, so that they could be cut finer, only cost time
// (677 / 550 with 8 and 3): the one-row kernels pay the per-tile barriers for a quarter of the work.
constexpr int kSchedRows = 64;
constexpr double kSchedRowCost = 16.0;
constexpr int kSchedMinSegment = 512;
constexpr int kSchedPerCu = 2;

struct SchedHost {
    std::vector<int32_t> perm;
    std::vector<int4> items, comb;
    int n_slots = 0;
};

// rows (by length, longest first) -> blocks of kSchedRows -> (block, range) items
void build_schedule(int M, int K, const std::vector<int32_t> &rp, int cus, SchedHost &out) {
    std::vector<int32_t> order(M);
    for (int i = 0; i < M; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return rp[a + 1] - rp[a] > rp[b + 1] - rp[b]; });
    const int blocks = (M + kSchedRows - 1) / kSchedRows;
    const int max_seg = K / kSchedMinSegment > 1 ? K / kSchedMinSegment : 1;
    const double total = (double)rp[M] + kSchedRowCost * (double)K * (double)blocks;
    const double target = total / ((double)cus * kSchedPerCu);
    struct Item {
        int4 it;
        double cost;
    };
    std::vector<Item> items;
    out.perm.assign((size_t)blocks * kSchedRows, M);
    for (int i = 0; i < M; ++i) out.perm[i] = order[i];
    for (int b = 0; b < blocks; ++b) {
        double work = 0;
        for (int i = 0; i < kSchedRows; ++i) {
            const int32_t row = out.perm[(size_t)b * kSchedRows + i];
            if (row < M) work += (double)(rp[row + 1] - rp[row]);
        }
        const double cost = kSchedRowCost * (double)K + work;
        int nseg = (int)(cost / target + 0.5);
        nseg = nseg < 1 ? 1 : (nseg > max_seg ? max_seg : nseg);
        int slot0 = 0;
        if (nseg > 1) {
            slot0 = out.n_slots;
            out.n_slots += nseg;
            out.comb.push_back(make_int4(b, slot0, nseg, 0));
        }
        for (int sgm = 0; sgm < nseg; ++sgm) items.push_back(Item{make_int4(b, sgm, nseg, slot0 + sgm), cost / nseg});
    }
    std::stable_sort(items.begin(), items.end(), [](const Item &x, const Item &y) { return x.cost > y.cost; });
    for (const Item &i : items) out.items.push_back(i.it);
}

// the plan's device copy of the schedule: one allocation, the int4 tables first
csrk_status upload_schedule(csrk_plan_s *plan, const SchedHost &h, hipStream_t stream) {
    const size_t off_comb = h.items.size() * sizeof(int4);
    const size_t off_perm = off_comb + h.comb.size() * sizeof(int4);
    const size_t bytes = off_perm + h.perm.size() * sizeof(int32_t);
    std::vector<char> image(bytes, 0);
    memcpy(image.data(), h.items.data(), h.items.size() * sizeof(int4));
    if (!h.comb.empty()) memcpy(image.data() + off_comb, h.comb.data(), h.comb.size() * sizeof(int4));
    memcpy(image.data() + off_perm, h.perm.data(), h.perm.size() * sizeof(int32_t));
    void *mem = nullptr;
    if (hipMalloc(&mem, bytes) != hipSuccess) return fail(CSRK_WORKSPACE, "csrk_plan_create: cannot allocate %zu bytes for the schedule", bytes);
    if (hipMemcpyAsync(mem, image.data(), bytes, hipMemcpyHostToDevice, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess) {
        (void)hipFree(mem);
        return fail(CSRK_HIP_ERROR, "csrk_plan_create: copying the schedule failed");
    }
    plan->sched_mem = mem;
    char *base = static_cast<char *>(mem);
    plan->sched.n_items = (int)h.items.size();
    plan->sched.n_comb = (int)h.comb.size();
    plan->sched.n_slots = h.n_slots;
    plan->sched.items = reinterpret_cast<const int4 *>(base);
    plan->sched.comb = reinterpret_cast<const int4 *>(base + off_comb);
    plan->sched.perm = reinterpret_cast<const int32_t *>(base + off_perm);
    plan->has_sched = true;
    return CSRK_OK;
}

// floats of scratch the partial rows of a scheduled call take, for rows of `ld` floats
size_t sched_partial_floats(const csrk_plan_s *plan, int ld) {
    return (size_t)plan->sched.n_slots * (size_t)kSchedRows * (size_t)ld;
}

// A planned call takes the schedule if the plan has one, the shape is one the tiled kernels serve in one launch,
// the pattern is dense enough for them, and the scratch at hand holds the partial rows.
// Measured on the pattern above, planned FusedMM D = 64 / SPMM, schedule against equal shares of the stored
// entries: N = 512 536 / 428 us against 1601 / 1370, N = 256 347 / 256 against 703 / 492; N = 128 311 / 218 against
// 312 / 171, N = 64 237 / 147 against 168 / 91: with 128 columns or fewer the staging of whole tiles for rows that
// hold few entries costs more than the gathers it replaces, so such outputs take the schedule only where the tiled
// kernels are forced (CSRK_KTILE=2, tests).
bool sched_usable(const DeviceState &d, const csrk_plan_s *plan, int K, int N, int D, bool fused) {
    const int mode = env_int("CSRK_KTILE", 1);
    if (!plan || !plan->has_sched || env_int("CSRK_SCHED", 1) != 1 || mode == 3) return false;
    if (N % 4 != 0 || N < 4 || N > kWideSlab || D % 4 != 0 || D > 64) return false;
    if (N <= 128 && mode != 2) return false;
    if (N > 128 && (long long)K * N * 4 >= (1ll << 32)) return false;
    const double density = (double)plan->nnz / ((double)plan->M * (double)plan->K);
    if (density < (double)wide_min_density(plan->M, K, N, fused, true)) return false;
    if (d.fixed && sched_partial_floats(plan, N) > d.head_floats) return false;
    return true;
}

csrk_status launch_sched_combine(DeviceState &d, const csrk_plan_s *plan, hipStream_t st, int N, float *O) {
    const csrk_plan_s::Sched &k = plan->sched;
    if (k.n_comb > 0)
        hipLaunchKernelGGL(sched_combine_kernel, dim3(k.n_comb), dim3(256), 0, st, plan->M, N, N, kSchedRows, k.perm, k.comb,
                           (const float *)d.head, O);
    CSRK_HIP(hipGetLastError());
    return CSRK_OK;
}

csrk_status sched_spmm(DeviceState &d, const csrk_plan_s *plan, hipStream_t st, int N, const float *v, const float *B,
                       float *O) {
    if (csrk_status s = ensure_scratch(d, N, sched_partial_floats(plan, N))) return s;
    const int M = plan->M, K = plan->K;
    const int32_t *rp = plan->rowptr, *ci = plan->colidx;
    const SchedPart sp{plan->sched.perm, plan->sched.items, plan->sched.n_items, 0};
    csrk_status s = N <= 32    ? launch_narrow_rows<8, 4>(d, st, M, K, N, rp, ci, v, B, O, 1, &sp)
                    : N <= 64  ? launch_narrow_rows<4, 4>(d, st, M, K, N, rp, ci, v, B, O, 1, &sp)
                    : N <= 128 ? launch_narrow_rows<2, 4>(d, st, M, K, N, rp, ci, v, B, O, 1, &sp)
                    : N <= 256 ? launch_ktile_rows<1, 128, 4>(d, st, M, K, N, N, 0, rp, ci, v, B, O, 1, &sp)
                               : launch_ktile_rows<2, 64, 4>(d, st, M, K, N, N, 0, rp, ci, v, B, O, 1, &sp);
    if (s) return s;
    return launch_sched_combine(d, plan, st, N, O);
}

csrk_status sched_fused(DeviceState &d, const csrk_plan_s *plan, hipStream_t st, int D, int N, const float *v,
                        const float *A, const float *B, const float *C, float *O) {
    if (csrk_status s = ensure_scratch(d, N, sched_partial_floats(plan, N))) return s;
    const int M = plan->M, K = plan->K;
    const int32_t *rp = plan->rowptr, *ci = plan->colidx;
    const SchedPart sp{plan->sched.perm, plan->sched.items, plan->sched.n_items, 0};
    csrk_status s =
        N <= 32    ? launch_fused_narrow_rows<8, 4, 64>(d, st, M, K, D, N, rp, ci, v, A, B, C, O, 1, 0, 0, &sp)
        : N <= 64  ? launch_fused_narrow_rows<4, 4, 64>(d, st, M, K, D, N, rp, ci, v, A, B, C, O, 1, 0, 0, &sp)
        : N <= 128 ? launch_fused_narrow_rows<2, 4, 64>(d, st, M, K, D, N, rp, ci, v, A, B, C, O, 1, 0, 0, &sp)
        : N <= 256 ? launch_fused_ktile_rows<1, 96, 4, 64>(d, st, M, K, D, N, N, 0, rp, ci, v, A, B, C, O, 1, &sp)
                   : launch_fused_ktile_rows<2, 64, 4, 32>(d, st, M, K, D, N, N, 0, rp, ci, v, A, B, C, O, 1, &sp);
    if (s) return s;
    return launch_sched_combine(d, plan, st, N, O);
}

// --- validation kernels -------------------------------------------------------------
__global__ void validate_rowptr_kernel(int M, const int32_t *rowptr, int32_t *flags) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0 && rowptr[0] != 0) atomicOr(flags, 1);
    if (i < M && rowptr[i + 1] < rowptr[i]) atomicOr(flags, 2);
}

__global__ void validate_colidx_kernel(int M, int K, const int32_t *rowptr, const int32_t *colidx, int32_t *flags) {
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    for (int r = wave; r < M; r += nwaves) {
        const int rs = rowptr[r], re = rowptr[r + 1];
        for (int j = rs + lane; j < re; j += 64) {
            const int k = colidx[j];
            if (k < 0 || k >= K) atomicOr(flags, 4);
            if (j > rs && colidx[j - 1] >= k) atomicOr(flags + 1, 1);
        }
    }
}

// ---- bfloat16 dense operands (stored values and outputs stay FP32, arithmetic is FP32) -------------------
// The general kernels only (equal shares, or whole rows where the row analysis finds the rows even): a group of
// LG lanes covers the width with 8 bfloat16 (one 128-bit load) per lane.

WidthCfg out_width_cfg_bf16(int N, bool vec8) {
    if (vec8) {
        if (N <= 64) return {8, 8, 1};
        if (N <= 128) return {8, 16, 1};
        if (N <= 256) return {8, 32, 1};
        if (N <= 512) return {8, 64, 1};
        return {8, 64, 2};
    }
    return {1, 64, 1};
}

WidthCfg dot_width_cfg_bf16(int D, bool vec8) {
    if (vec8) {
        if (D <= 64) return {8, 8, 1};
        if (D <= 128) return {8, 16, 1};
        return {8, 64, 0};
    }
    return {1, 64, 0};
}

template <int VD, int LD, int TD>
bool launch_fused_rows_bf16_n(const WidthCfg &nc, hipStream_t st, int M, int D, int N, const int32_t *rp,
                              const int32_t *ci, const float *v, const bf16_t *A, const bf16_t *B, const bf16_t *C,
                              float *O) {
#define CSRK_FUSED_ROWS_BF16_CASE(VN, LN, TN)                                                                     \
    if (nc.vec == VN && nc.lg == LN && nc.t == TN) {                                                              \
        const int wpr = rows_wpr(M, N);                                                                           \
        hipLaunchKernelGGL((fusedmm_rows_kernel<VD, LD, TD, VN, LN, TN, bf16_t>), rows_grid(M, wpr, 1),            \
                           dim3(kBlockThreads), 0, st, M, D, N, rp, ci, v, A, B, C, O, wpr);                      \
        return true;                                                                                              \
    }
    CSRK_FUSED_ROWS_BF16_CASE(8, 8, 1)
    CSRK_FUSED_ROWS_BF16_CASE(8, 16, 1)
    CSRK_FUSED_ROWS_BF16_CASE(8, 32, 1)
    CSRK_FUSED_ROWS_BF16_CASE(8, 64, 1)
#undef CSRK_FUSED_ROWS_BF16_CASE
    return false;
}

template <int VD, int LD, int TD>
bool launch_fused_bf16_n(const WidthCfg &nc, dim3 grid, hipStream_t st, int M, int D, int N, const int32_t *rp,
                         const int32_t *ci, const float *v, const bf16_t *A, const bf16_t *B, const bf16_t *C, float *O,
                         float *head, int32_t *head_row, const int32_t *even) {
#define CSRK_FUSED_BF16_CASE(VN, LN, TN)                                                                          \
    if (nc.vec == VN && nc.lg == LN && nc.t == TN) {                                                              \
        hipLaunchKernelGGL((fusedmm_nnzsplit_kernel<VD, LD, TD, VN, LN, TN, bf16_t>), grid, dim3(kBlockThreads), 0, st, \
                           M, D, N, rp, ci, v, A, B, C, O, head, head_row, nullptr, even);                        \
        return true;                                                                                              \
    }
    CSRK_FUSED_BF16_CASE(8, 8, 1)
    CSRK_FUSED_BF16_CASE(8, 16, 1)
    CSRK_FUSED_BF16_CASE(8, 32, 1)
    CSRK_FUSED_BF16_CASE(8, 64, 1)
    CSRK_FUSED_BF16_CASE(8, 64, 2)
    CSRK_FUSED_BF16_CASE(1, 64, 1)
#undef CSRK_FUSED_BF16_CASE
    return false;
}

// --- scratch for the entry point that may not allocate --------------------------------------------------------
// A fixed area in the library's own device image: 64 KB for the worker table and flag words plus 16 MB of partial
// rows (8192 workers x 512 columns) or partial outputs.  Every device the library runs on holds its own copy, at
// its own address, until the process ends.
constexpr size_t kStaticScratchBytes = (size_t(16) << 20) + (size_t(64) << 10);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// The array's name is only a host-side stand-in for the symbol: the device address is asked for once per device,
// with that device current, and host code passes that pointer - never the name - to kernels.
void *g_static_scratch[kMaxDevices] = {};

csrk_status static_scratch_ptr(void **out) {
    int dev = 0;
    CSRK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(CSRK_UNSUPPORTED, "device ordinal %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_static_scratch[dev]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(CSRK_HIP_ERROR, "hipGetSymbolAddress of the static scratch failed: %s", hipGetErrorString(e));
        g_static_scratch[dev] = ptr;
    }
    *out = g_static_scratch[dev];
    return CSRK_OK;
}

// --- which kernel family takes a call -------------------------------------------------------------------------
// The host's part of the choice, from sizes, alignment and (planned calls) what the plan knows: one chain of
// questions per operation, asked here and nowhere else.  A family with `gated` set is an ATTEMPT: the device's row
// analysis (or the plan's facts) still has to find S dense enough (`min_density`) and its rows even enough.
enum Family : int {
    kFamGeneral = 0,    // equal shares of the stored entries, or whole rows where the rows are found even
    kFamRows,           // whole-row kernels, chosen by the host alone (small S)
    kFamNarrow,         // LDS-tiled, outputs of up to 128 columns
    kFamWide,           // LDS-tiled, 132 to 2048 columns (beyond 512 in slabs)
    kFamNarrowSlabs,    // FusedMM with dot products of 65-128 floats and a wide output: the narrow kernel per 128 columns
    kFamSddmmTile,      // LDS-tiled SDDMM, dot products of up to 128 floats
    kFamSddmmPieces,    // ... longer dot products, 128 floats at a time
    kFamSchedule,       // a plan's schedule for uneven rows
};
struct Choice {
    Family family = kFamGeneral;
    float min_density = 0.f;
    bool gated = false;
};

Choice choose_spmm(const DeviceState &d, const csrk_plan_s *plan, int M, int K, int N, bool vec4) {
    if (!vec4) return Choice{};
    if (sched_usable(d, plan, K, N, 0, false)) return Choice{kFamSchedule};
    if (plan_small_tiled(d, plan, M, K, N, 0)) return Choice{kFamNarrow};
    if (rows_mode_ok(M, K, N)) return Choice{kFamRows};
    if (narrow_shape_ok(d, M, K, N, false)) {
        const bool filled = tile_grid_for(d, M, K, N > 64 ? narrow_kt<2>() : narrow_kt<4>(), kTileWaves * 4).fill >= kWellFilled;
        return Choice{kFamNarrow, narrow_min_density(M, K, N, false, filled), true};
    }
    if (ktile_shape_ok(d, M, K, N)) {
        // (row analysis, then the LDS-tiled kernel; the general kernels behind it stand down unless S turns out
        // unsuitable: unsorted columns, too sparse, rows too uneven)
        const bool filled = tile_grid_for(d, M, K, N <= 256 ? 128 : 64, kTileWaves * 4).fill >= kWellFilled;
        return Choice{kFamWide, uneven_ok(wide_min_density(M, K, N, false, filled)), true};
    }
    return Choice{};
}

Choice choose_sddmm(const DeviceState &d, const csrk_plan_s *plan, int M, int K, int D, bool vec4, bool in_place) {
    if (!vec4) return Choice{};
    if (plan_small_tiled(d, plan, M, K, D, 1)) return Choice{kFamSddmmTile};
    if (dot_width_cfg(D, vec4).t == 1 && rows_mode_ok(M, K, D, plan == nullptr)) return Choice{kFamRows};
    // In place (P aliases vals) a tiled kernel that meets unsorted columns has already overwritten values which the
    // general kernel would need to redo the call: without a plan to vouch for the order, such calls skip the attempt.
    const bool may_attempt = plan != nullptr || !in_place;
    if (may_attempt && sddmm_tile_shape_ok(d, M, K, D)) return Choice{kFamSddmmTile, sddmm_min_density(M, K, D), true};
    // Dot products longer than the 128 floats a row of the tile holds: 128 floats at a time, one launch of the
    // tiled kernel per piece, the second and later pieces adding to P (each reads vals again, so not when P
    // aliases vals).  16384^2 / 20 %, D = 256: 5.6 ms in the general kernel, whose gathers outgrow L2.
    if (D > 128 && D <= kSddmmMaxD && !in_place && sddmm_tile_shape_ok(d, M, K, 128))
        return Choice{kFamSddmmPieces, sddmm_min_density(M, K, 128), true};
    return Choice{};
}

Choice choose_fused(const DeviceState &d, const csrk_plan_s *plan, int M, int K, int D, int N, bool nvec4, bool dvec4) {
    if (!nvec4 || !dvec4) return Choice{};
    if (D >= 4 && sched_usable(d, plan, K, N, D, true)) return Choice{kFamSchedule};
    if (D > 128) return Choice{};
    if (plan_small_tiled(d, plan, M, K, N, 2)) return Choice{kFamNarrow};
    if (N <= 512 && rows_mode_ok(M, K, N)) return Choice{kFamRows};
    if (narrow_shape_ok(d, M, K, N, true)) {
        const int kt = D > 64 ? 128 : (N > 64 ? fused_narrow_kt<2, 64>() : fused_narrow_kt<4, 64>());
        const bool filled = tile_grid_for(d, M, K, kt, kTileWaves * 4, fused_three_rows(d, M, N)).fill >= kWellFilled;
        return Choice{kFamNarrow, narrow_min_density(M, K, N, true, filled), true};
    }
    if (D <= 64 && ktile_shape_ok(d, M, K, N)) {
        const bool filled =
            tile_grid_for(d, M, K, N <= 256 ? 96 : 64, kTileWaves * 4, fused_three_rows(d, M, N)).fill >= kWellFilled;
        return Choice{kFamWide, uneven_ok(wide_min_density(M, K, N, true, filled)), true};
    }
    if (D > 64 && ktile_shape_ok(d, M, K, N)) {
        // Dot products of 65 to 128 floats with a wide output: the wide kernel has no room for such rows of B beside
        // its tile of C, so the narrow kernel takes the output 128 columns at a time, one launch per slab, each
        // computing the scores again (half of a slab's work).  Measured on 16384^2 / 20 %, D = 128: N = 512
        // 11.4 -> 4.9 ms, N = 256 5.6 -> 2.5 ms; level with the general kernels at 5 % (8192^2).
        const float min_density =
            env_int("CSRK_KTILE", 1) == 2 ? -1.f : ((long long)K * N * 4 >= (16ll << 20) ? 0.06f : 0.10f);
        return Choice{kFamNarrowSlabs, min_density, true};
    }
    return Choice{};
}

}  // namespace

extern "C" {

const char *csrk_last_error(void) { return g_err; }

csrk_status csrk_explain_choice(int op, int cus, int M, int K, int N, int D, long long nnz, int longest_row,
                                int planned, int *family) {
    if (!family) return fail(CSRK_INVALID_ARG, "csrk_explain_choice: family must not be NULL");
    if (cus <= 0 || M <= 0 || K <= 0 || nnz < 0 || longest_row < 0)
        return fail(CSRK_INVALID_ARG, "csrk_explain_choice: sizes must be positive");
    DeviceState d;
    d.cus = cus;
    d.workers = (cus * 32 + kWavesPerBlock - 1) / kWavesPerBlock * kWavesPerBlock;
    const double mean = (double)nnz / (double)M;
    const bool even = (double)longest_row <= 2.0 * mean + 64.0;
    csrk_plan_s facts{0, M, K, nnz, nullptr, nullptr, true, even, nullptr, nullptr, 0};
    facts.has_sched = !even && M >= 256 && K >= 2 * kSchedMinSegment && nnz > 0;     // as csrk_plan_create decides
    const csrk_plan_s *plan = planned ? &facts : nullptr;
    Choice ch;
    bool fused = false;
    switch (op) {
        case CSRK_OP_SPMM: ch = choose_spmm(d, plan, M, K, N, N % 4 == 0); break;
        case CSRK_OP_SDDMM: ch = choose_sddmm(d, plan, M, K, D, D % 4 == 0 && D > 0, false); break;
        case CSRK_OP_FUSEDMM:
            ch = choose_fused(d, plan, M, K, D, N, N % 4 == 0, D % 4 == 0 && D > 0);
            fused = true;
            break;
        default: return fail(CSRK_INVALID_ARG, "csrk_explain_choice: unknown operation %d", op);
    }
    bool attempted = false;
    if (ch.gated) {     // what the row analysis (row_analysis in kernels_ktile.hpp) or the plan's facts would say
        attempted = true;
        const bool wide = ch.min_density >= kUnevenOk;
        const double threshold = wide ? (double)(ch.min_density - kUnevenOk) : (double)ch.min_density;
        const bool dense = (double)nnz >= threshold * (double)M * (double)K;
        const bool suits = planned ? even : (even || (wide && (double)longest_row <= 16.0 * mean + 64.0));
        if (!(ch.min_density < 0.f || (dense && suits))) ch.family = kFamGeneral;
    }
    switch (ch.family) {
        case kFamRows: *family = CSRK_FAMILY_ROWS; break;
        case kFamNarrow:
        case kFamNarrowSlabs: *family = CSRK_FAMILY_TILED_NARROW; break;
        case kFamWide: *family = CSRK_FAMILY_TILED_WIDE; break;
        case kFamSddmmTile:
        case kFamSddmmPieces: *family = CSRK_FAMILY_TILED_SDDMM; break;
        case kFamSchedule: *family = CSRK_FAMILY_SCHEDULE; break;
        default: {
            // the general kernels deal out whole rows where they know the rows to be even
            const bool asked = planned || attempted || (op != CSRK_OP_SDDMM && even_rows_worth_asking(d, M, K, fused));
            *family = asked && even ? CSRK_FAMILY_GENERAL_ROWS : CSRK_FAMILY_GENERAL_SHARES;
        }
    }
    return CSRK_OK;
}

const char *csrk_version(void) { return "csrk 0.1 gfx950"; }

static csrk_status spmm_run(const csrk_plan_s *plan, const ScratchSource &scratch, int M, int K, int N,
                            const int32_t *rowptr, const int32_t *colidx, const float *vals, const float *B, float *O,
                            hipStream_t stream) {
    if (csrk_status s = check_dims("spmm_csr", M, K, N, 0)) return s;
    if (M == 0 || N == 0) return CSRK_OK;
    if (!rowptr || !O) return fail(CSRK_INVALID_ARG, "spmm_csr: rowptr and O must not be NULL");
    if (K > 0 && !B) return fail(CSRK_INVALID_ARG, "spmm_csr: B must not be NULL");
    CallLock lock;
    DeviceState state;
    DeviceState *d = &state;
    if (csrk_status s = begin_call(state, scratch, lock)) return s;
    d->pending_ksplit = 0;
    if (csrk_status s = ensure_scratch(*d, N)) return s;
    PlanScope scope(*d, plan);
    const bool vec4 = (N % 4 == 0) && aligned16(B) && aligned16(O) && aligned16(d->head);
    const WidthCfg c = out_width_cfg(N, vec4);
    const int tile = c.vec * c.lg * c.t;
    const dim3 grid(d->workers / kWavesPerBlock, (N + tile - 1) / tile);
    const int32_t *gate = nullptr;
    CallRecord rec(1, stream);
    rec.begin();
    const Choice ch = choose_spmm(*d, plan, M, K, N, vec4);
    if (ch.family == kFamSchedule) {
        const csrk_status s = sched_spmm(*d, plan, stream, N, vals, B, O);
        rec.end();
        return s;
    }
    if (ch.family == kFamRows) {
        const int wpr = rows_wpr(M, N);
        const dim3 rgrid = rows_grid(M, wpr, (N + tile - 1) / tile);
#define CSRK_SPMM_ROWS_CASE(V, L, T)                                                                              \
    if (c.vec == V && c.lg == L && c.t == T)                                                                      \
        hipLaunchKernelGGL((spmm_rows_kernel<V, L, T>), rgrid, dim3(kBlockThreads), 0, stream, M, N, rowptr, colidx, \
                           vals, B, O, wpr);
        CSRK_SPMM_ROWS_CASE(4, 8, 1)
        CSRK_SPMM_ROWS_CASE(4, 16, 1)
        CSRK_SPMM_ROWS_CASE(4, 32, 1)
        CSRK_SPMM_ROWS_CASE(4, 64, 1)
        CSRK_SPMM_ROWS_CASE(4, 64, 2)
#undef CSRK_SPMM_ROWS_CASE
        rec.end();
        CSRK_HIP(hipGetLastError());
        return CSRK_OK;
    }
    if (ch.family == kFamNarrow || ch.family == kFamWide) {
        bool go = !ch.gated;
        if (ch.gated)
            if (csrk_status s = tiled_attempt(*d, plan, stream, M, K, rowptr, ch.min_density, &go)) return s;
        if (go && ch.family == kFamNarrow) {
            gate = tile_flags(*d);
            if (csrk_status s = launch_narrow(*d, stream, M, K, N, rowptr, colidx, vals, B, O)) return s;
        } else if (go) {
            gate = tile_flags(*d);
            if (N <= kWideSlab) {
                csrk_status s = N <= 256 ? launch_ktile<1, 128>(*d, stream, M, K, N, N, 0, rowptr, colidx, vals, B, O)
                                         : launch_ktile<2, 64>(*d, stream, M, K, N, N, 0, rowptr, colidx, vals, B, O);
                if (s) return s;
            } else {
                const int S = ksplit_for(*d, M, K, wide_remainder_is_small(N) ? 128 : 64, kTileWaves * 4);
                for (int c0 = 0; c0 < N; c0 += kWideSlab) {
                    const int w = N - c0 < kWideSlab ? N - c0 : kWideSlab;
                    csrk_status s = w <= 256 ? launch_ktile<1, 128>(*d, stream, M, K, w, N, c0, rowptr, colidx, vals, B, O, S)
                                             : launch_ktile<2, 64>(*d, stream, M, K, w, N, c0, rowptr, colidx, vals, B, O, S);
                    if (s) return s;
                }
            }
        }
    }
    const int32_t *even = nullptr;          // device flag: rows even enough to be dealt out whole
    if (plan) {
        if (gate) {     // the plan vouches for the pattern: the tiled kernel has done the call
            if (d->pending_ksplit > 1) launch_combine(*d, stream, M, N, O, gate, gate + 3, c.vec >= 4 && c.t == 1, vec4);
            rec.end();
            CSRK_HIP(hipGetLastError());
            return CSRK_OK;
        }
        even = plan->even ? plan->dflags + 3 : nullptr;
    } else if (gate) {
        even = tile_flags(*d) + 3;
    } else if (even_rows_worth_asking(*d, M, K, false)) {
        if (csrk_status s = launch_analysis(*d, stream, M, K, rowptr, 2.f)) return s;
        even = tile_flags(*d) + 3;
    }
#define CSRK_SPMM_CASE(V, L, T)                                                                           \
    if (c.vec == V && c.lg == L && c.t == T)                                                              \
        launch_spmm<V, L, T>(grid, stream, M, N, rowptr, colidx, vals, B, O, d->head, d->head_row, gate, even);
    CSRK_SPMM_CASE(4, 8, 1)
    CSRK_SPMM_CASE(4, 16, 1)
    CSRK_SPMM_CASE(4, 32, 1)
    CSRK_SPMM_CASE(4, 64, 1)
    CSRK_SPMM_CASE(4, 64, 2)
    CSRK_SPMM_CASE(1, 64, 1)
#undef CSRK_SPMM_CASE
    CSRK_HIP(hipGetLastError());
    // a planned call knows on the host what the combine step would find on the device: whole rows were dealt out
    // (same condition as in the kernels), there are no partial rows to add, and the launch is left out
    const bool any_m = c.vec >= 4 && c.t == 1;
    if (!(plan && even && (any_m || 2ll * M > d->workers)))
        launch_combine(*d, stream, M, N, O, gate, even, any_m, vec4);
    rec.end();
    CSRK_HIP(hipGetLastError());
    return CSRK_OK;
}

static csrk_status sddmm_run(const csrk_plan_s *plan, const ScratchSource &scratch, int M, int K, int D,
                             const int32_t *rowptr, const int32_t *colidx, const float *vals, const float *A,
                             const float *B, float *P, hipStream_t stream) {
    if (csrk_status s = check_dims("sddmm_csr", M, K, D, 0)) return s;
    if (M == 0 || K == 0) return CSRK_OK;
    if (!rowptr) return fail(CSRK_INVALID_ARG, "sddmm_csr: rowptr must not be NULL");
    if (D > 0 && (!A || !B)) return fail(CSRK_INVALID_ARG, "sddmm_csr: A and B must not be NULL");
    CallLock lock;
    DeviceState state;
    DeviceState *d = &state;
    if (csrk_status s = begin_call(state, scratch, lock)) return s;
    PlanScope scope(*d, plan);
    const bool vec4 = (D % 4 == 0) && D > 0 && aligned16(A) && aligned16(B);
    const WidthCfg c = dot_width_cfg(D, vec4);
    const dim3 grid(d->workers / kWavesPerBlock);
    const int32_t *gate = nullptr;
    CallRecord rec(2, stream);
    rec.begin();
    const Choice ch = choose_sddmm(*d, plan, M, K, D, vec4, P == vals);
    if (ch.family == kFamRows) {
        const int wpr = rows_wpr(M, D);
        const dim3 rgrid = rows_grid(M, wpr, 1);
#define CSRK_SDDMM_ROWS_CASE(V, L, T)                                                                               \
    if (c.vec == V && c.lg == L && c.t == T)                                                                        \
        hipLaunchKernelGGL((sddmm_rows_kernel<V, L, T>), rgrid, dim3(kBlockThreads), 0, stream, M, D, rowptr, colidx, \
                           vals, A, B, P, wpr);
        CSRK_SDDMM_ROWS_CASE(4, 8, 1)
        CSRK_SDDMM_ROWS_CASE(4, 16, 1)
        CSRK_SDDMM_ROWS_CASE(4, 32, 1)
        CSRK_SDDMM_ROWS_CASE(4, 64, 1)
#undef CSRK_SDDMM_ROWS_CASE
        rec.end();
        CSRK_HIP(hipGetLastError());
        return CSRK_OK;
    }
    if (ch.family == kFamSddmmTile || ch.family == kFamSddmmPieces) {
        if (csrk_status s = ensure_scratch(*d, 1)) return s;
        bool go = !ch.gated;
        if (ch.gated)
            if (csrk_status s = tiled_attempt(*d, plan, stream, M, K, rowptr, ch.min_density, &go)) return s;
        if (go && ch.family == kFamSddmmTile) {
            gate = tile_flags(*d);
            csrk_status s = D <= 32   ? launch_sddmm_ktile_rows<32>(*d, stream, M, K, D, rowptr, colidx, vals, A, B, P)
                            : D <= 64 ? launch_sddmm_ktile_rows<64>(*d, stream, M, K, D, rowptr, colidx, vals, A, B, P)
                                      : launch_sddmm_ktile_rows<128>(*d, stream, M, K, D, rowptr, colidx, vals, A, B, P);
            if (s) return s;
        } else if (go) {
            gate = tile_flags(*d);
            for (int c0 = 0; c0 < D; c0 += 128)
                if (csrk_status s = launch_sddmm_ktile_rows<128>(*d, stream, M, K, D - c0 < 128 ? D - c0 : 128, rowptr, colidx,
                                                                 vals, A, B, P, D, c0, c0 > 0))
                    return s;
        }
    }
    if (plan && gate) {     // the plan vouches for the pattern: the tiled kernel has done the call
        rec.end();
        CSRK_HIP(hipGetLastError());
        return CSRK_OK;
    }
    // device flag: rows even enough to be dealt out whole
    const int32_t *even = plan ? (plan->even ? plan->dflags + 3 : nullptr) : gate ? tile_flags(*d) + 3 : nullptr;
#define CSRK_SDDMM_CASE(V, L, T)                                                        \
    if (c.vec == V && c.lg == L && c.t == T)                                            \
        launch_sddmm<V, L, T>(grid, stream, M, D, rowptr, colidx, vals, A, B, P, gate, even);
    CSRK_SDDMM_CASE(4, 8, 1)
    CSRK_SDDMM_CASE(4, 16, 1)
    CSRK_SDDMM_CASE(4, 32, 1)
    CSRK_SDDMM_CASE(4, 64, 1)
    CSRK_SDDMM_CASE(4, 64, 0)
    CSRK_SDDMM_CASE(1, 64, 0)
#undef CSRK_SDDMM_CASE
    rec.end();
    CSRK_HIP(hipGetLastError());
    return CSRK_OK;
}

static csrk_status fusedmm_run(const csrk_plan_s *plan, const ScratchSource &scratch, int M, int K, int D, int N,
                               const int32_t *rowptr, const int32_t *colidx, const float *vals, const float *A,
                               const float *B, const float *C, float *O, hipStream_t stream) {
    if (csrk_status s = check_dims("fusedmm_csr", M, K, D, N)) return s;
    if (M == 0 || N == 0) return CSRK_OK;
    if (!rowptr || !O) return fail(CSRK_INVALID_ARG, "fusedmm_csr: rowptr and O must not be NULL");
    if (K > 0 && !C) return fail(CSRK_INVALID_ARG, "fusedmm_csr: C must not be NULL");
    if (K > 0 && D > 0 && (!A || !B)) return fail(CSRK_INVALID_ARG, "fusedmm_csr: A and B must not be NULL");
    CallLock lock;
    DeviceState state;
    DeviceState *d = &state;
    if (csrk_status s = begin_call(state, scratch, lock)) return s;
    d->pending_ksplit = 0;
    if (csrk_status s = ensure_scratch(*d, N)) return s;
    PlanScope scope(*d, plan);
    const bool dvec4 = (D % 4 == 0) && D > 0 && aligned16(A) && aligned16(B);
    const bool nvec4 = (N % 4 == 0) && aligned16(C) && aligned16(O) && aligned16(d->head);
    const WidthCfg dc = dot_width_cfg(D, dvec4);
    const WidthCfg nc = out_width_cfg(N, nvec4);
    const int tile = nc.vec * nc.lg * nc.t;
    const dim3 grid(d->workers / kWavesPerBlock, (N + tile - 1) / tile);
    bool done = false;
    const int32_t *gate = nullptr;
    CallRecord rec(3, stream);
    rec.begin();
    const Choice ch = choose_fused(*d, plan, M, K, D, N, nvec4, dvec4);
    if (ch.family == kFamSchedule) {
        const csrk_status s = sched_fused(*d, plan, stream, D, N, vals, A, B, C, O);
        rec.end();
        return s;
    }
    if (ch.family == kFamRows) {
        bool launched = false;
        if (dc.lg == 8) launched = launch_fused_rows_n<4, 8, 1>(nc, stream, M, D, N, rowptr, colidx, vals, A, B, C, O);
        if (dc.lg == 16) launched = launch_fused_rows_n<4, 16, 1>(nc, stream, M, D, N, rowptr, colidx, vals, A, B, C, O);
        if (dc.lg == 32) launched = launch_fused_rows_n<4, 32, 1>(nc, stream, M, D, N, rowptr, colidx, vals, A, B, C, O);
        if (launched) {
            rec.end();
            CSRK_HIP(hipGetLastError());
            return CSRK_OK;
        }
    } else if (ch.family != kFamGeneral) {
        bool go = !ch.gated;
        if (ch.gated)
            if (csrk_status s = tiled_attempt(*d, plan, stream, M, K, rowptr, ch.min_density, &go)) return s;
        if (go) gate = tile_flags(*d);
        if (go && ch.family == kFamNarrow) {
            if (csrk_status s = launch_fused_narrow(*d, stream, M, K, D, N, rowptr, colidx, vals, A, B, C, O)) return s;
        } else if (go && ch.family == kFamWide) {
            if (N <= kWideSlab) {
                csrk_status s =
                    N <= 256 ? launch_fused_ktile<1, 96, 64>(*d, stream, M, K, D, N, N, 0, rowptr, colidx, vals, A, B, C, O)
                             : launch_fused_ktile<2, 64, 32>(*d, stream, M, K, D, N, N, 0, rowptr, colidx, vals, A, B, C, O);
                if (s) return s;
            } else {
                const int S = ksplit_for(*d, M, K, wide_remainder_is_small(N) ? 96 : 64, kTileWaves * 4,
                                         fused_three_rows(*d, M, N));
                for (int c0 = 0; c0 < N; c0 += kWideSlab) {
                    const int w = N - c0 < kWideSlab ? N - c0 : kWideSlab;
                    csrk_status s =
                        w <= 256 ? launch_fused_ktile<1, 96, 64>(*d, stream, M, K, D, w, N, c0, rowptr, colidx, vals, A, B, C, O, S)
                                 : launch_fused_ktile<2, 64, 32>(*d, stream, M, K, D, w, N, c0, rowptr, colidx, vals, A, B, C, O, S);
                    if (s) return s;
                }
            }
        } else if (go) {        // kFamNarrowSlabs
            constexpr int kSlab = 128;
            const int S = ksplit_for(*d, M, K, fused_narrow_kt<2, 128>(), kTileWaves * 4, fused_three_rows(*d, M, kSlab));
            for (int c0 = 0; c0 < N; c0 += kSlab) {
                const int w = N - c0 < kSlab ? N - c0 : kSlab;
                if (csrk_status s = launch_fused_narrow_g<2, 128>(*d, stream, M, K, D, w, rowptr, colidx, vals, A, B, C, O,
                                                                  N, c0, S))
                    return s;
            }
        }
    }
    const int32_t *even = nullptr;          // device flag: rows even enough to be dealt out whole
    if (plan) {
        if (gate) {     // the plan vouches for the pattern: the tiled kernel has done the call
            if (d->pending_ksplit > 1) launch_combine(*d, stream, M, N, O, gate, gate + 3, false, nvec4);
            rec.end();
            CSRK_HIP(hipGetLastError());
            return CSRK_OK;
        }
        even = plan->even ? plan->dflags + 3 : nullptr;
    } else if (gate) {
        even = tile_flags(*d) + 3;
    } else if (even_rows_worth_asking(*d, M, K, true)) {
        if (csrk_status s = launch_analysis(*d, stream, M, K, rowptr, 2.f)) return s;
        even = tile_flags(*d) + 3;
    }
#define CSRK_DOT_CASE(V, L, T)                                                                            \
    if (!done && dc.vec == V && dc.lg == L && dc.t == T)                                                  \
        done = launch_fused_n<V, L, T>(nc, grid, stream, M, D, N, rowptr, colidx, vals, A, B, C, O, d->head, \
                                       d->head_row, gate, even);
    CSRK_DOT_CASE(4, 8, 1)
    CSRK_DOT_CASE(4, 16, 1)
    CSRK_DOT_CASE(4, 32, 1)
    CSRK_DOT_CASE(4, 64, 1)
    CSRK_DOT_CASE(4, 64, 0)
    CSRK_DOT_CASE(1, 64, 0)
#undef CSRK_DOT_CASE
    if (!done) return fail(CSRK_UNSUPPORTED, "fusedmm_csr: no kernel for D=%d N=%d", D, N);
    CSRK_HIP(hipGetLastError());
    if (!(plan && even && 2ll * M > d->workers))     // planned call, whole rows: no partial rows to add
        launch_combine(*d, stream, M, N, O, gate, even, false, nvec4);
    rec.end();
    CSRK_HIP(hipGetLastError());
    return CSRK_OK;
}

csrk_status spmm_csr(int M, int K, int N, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                     const float *B, float *O, hipStream_t stream) {
    return spmm_run(nullptr, ScratchSource{}, M, K, N, rowptr, colidx, vals, B, O, stream);
}

csrk_status sddmm_csr(int M, int K, int D, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                      const float *A, const float *B, float *P, hipStream_t stream) {
    return sddmm_run(nullptr, ScratchSource{}, M, K, D, rowptr, colidx, vals, A, B, P, stream);
}

csrk_status fusedmm_csr(int M, int K, int D, int N, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                        const float *A, const float *B, const float *C, float *O, hipStream_t stream) {
    return fusedmm_run(nullptr, ScratchSource{}, M, K, D, N, rowptr, colidx, vals, A, B, C, O, stream);
}

// --- the same calls on a workspace of the caller's: nothing allocated, nothing shared ------------------------

// floats of scratch behind the int part that a call of this shape can need, whichever kernels it takes: partial
// rows of the equal-nonzero split (one per worker), or the partial outputs of a K-split launch of a tiled kernel
static size_t workspace_floats(const DeviceInfo &info, int op, int M, int K, int N) {
    if (op == CSRK_OP_SDDMM) return (size_t)info.workers;
    size_t floats = (size_t)info.workers * (size_t)(N > 0 ? N : 1);
    DeviceState probe;
    probe.cus = info.cus;
    probe.workers = info.workers;
    int smax = 1;
    for (int kt : {64, 96, 128, 160, 192, 256, 384})      // tile heights of the tiled SPMM / FusedMM kernels
        for (int three = 0; three < 2; ++three) {
            const int s = ksplit_for(probe, M, K, kt, kTileWaves * 4, three != 0);
            smax = s > smax ? s : smax;
        }
    if (smax > 1 && (size_t)smax * (size_t)M * (size_t)N > floats) floats = (size_t)smax * (size_t)M * (size_t)N;
    return floats;
}

csrk_status csrk_workspace_bytes(int op, int M, int K, int N, int D, size_t *bytes) {
    (void)D;        // part of the shape for symmetry with the calls; no kernel's scratch depends on it
    if (!bytes) return fail(CSRK_INVALID_ARG, "csrk_workspace_bytes: bytes must not be NULL");
    if (op != CSRK_OP_SPMM && op != CSRK_OP_SDDMM && op != CSRK_OP_FUSEDMM)
        return fail(CSRK_INVALID_ARG, "csrk_workspace_bytes: unknown operation %d", op);
    if (M < 0 || K < 0 || N < 0) return fail(CSRK_INVALID_ARG, "csrk_workspace_bytes: negative dimension");
    const DeviceInfo *info = nullptr;
    if (csrk_status s = device_info(&info)) return s;
    *bytes = scratch_int_bytes(info->workers) + (workspace_floats(*info, op, M, K, N) * sizeof(float) + 255) / 256 * 256;
    return CSRK_OK;
}

csrk_status spmm_csr_ws(int M, int K, int N, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                        const float *B, float *O, void *workspace, size_t workspace_bytes, hipStream_t stream) {
    if (!workspace) return fail(CSRK_INVALID_ARG, "spmm_csr_ws: workspace must not be NULL");
    return spmm_run(nullptr, ScratchSource{workspace, workspace_bytes}, M, K, N, rowptr, colidx, vals, B, O, stream);
}

csrk_status sddmm_csr_ws(int M, int K, int D, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                         const float *A, const float *B, float *P, void *workspace, size_t workspace_bytes,
                         hipStream_t stream) {
    if (!workspace) return fail(CSRK_INVALID_ARG, "sddmm_csr_ws: workspace must not be NULL");
    return sddmm_run(nullptr, ScratchSource{workspace, workspace_bytes}, M, K, D, rowptr, colidx, vals, A, B, P, stream);
}

csrk_status fusedmm_csr_ws(int M, int K, int D, int N, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                           const float *A, const float *B, const float *C, float *O, void *workspace,
                           size_t workspace_bytes, hipStream_t stream) {
    if (!workspace) return fail(CSRK_INVALID_ARG, "fusedmm_csr_ws: workspace must not be NULL");
    return fusedmm_run(nullptr, ScratchSource{workspace, workspace_bytes}, M, K, D, N, rowptr, colidx, vals, A, B, C, O,
                       stream);
}

// --- plans: the pattern analysed once, calls without per-call analysis or stand-by launches ---------------

static csrk_status plan_usable(const char *who, const csrk_plan_s *plan) {
    if (!plan) return fail(CSRK_INVALID_ARG, "%s: plan must not be NULL", who);
    int dev = 0;
    CSRK_HIP(hipGetDevice(&dev));
    if (dev != plan->dev) return fail(CSRK_INVALID_ARG, "%s: plan was made on device %d, current device is %d", who, plan->dev, dev);
    return CSRK_OK;
}

csrk_status fusedmm_csr_static(int M, int K, int D, int N, const int32_t *rowptr, const int32_t *colidx,
                               const float *vals, const float *A, const float *B, const float *C, float *O,
                               hipStream_t stream) {
    if (csrk_status s = check_dims("fusedmm_csr_static", M, K, D, N)) return s;
    // refuse up front what cannot fit, with the sizes in the message (the call itself would also notice)
    const DeviceInfo *info = nullptr;
    if (csrk_status s = device_info(&info)) return s;
    const size_t need = scratch_int_bytes(info->workers) + workspace_floats(*info, CSRK_OP_FUSEDMM, M, K, N) * sizeof(float);
    if (need > kStaticScratchBytes)
        return fail(CSRK_WORKSPACE,
                    "fusedmm_csr_static: this shape needs %zu bytes of scratch, the static area holds %zu (outputs of up to "
                    "512 columns; up to 16 MB of partial outputs for short matrices): use fusedmm_csr_ws",
                    need, kStaticScratchBytes);
    void *ptr = nullptr;
    if (csrk_status s = static_scratch_ptr(&ptr)) return s;
    return fusedmm_run(nullptr, ScratchSource{ptr, kStaticScratchBytes}, M, K, D, N, rowptr, colidx, vals, A, B, C, O,
                       stream);
}

// the plan's own scratch if csrk_plan_reserve made it large enough for this call; otherwise the device's lazily
// grown one (and its lock)
static ScratchSource plan_scratch(const csrk_plan_s *plan, int op, int N) {
    if (!plan->ws) return ScratchSource{};
    const DeviceInfo *info = nullptr;
    if (device_info(&info) != CSRK_OK) return ScratchSource{};
    size_t floats = workspace_floats(*info, op, plan->M, plan->K, N);
    if (plan->has_sched && op != CSRK_OP_SDDMM && sched_partial_floats(plan, N) > floats) floats = sched_partial_floats(plan, N);
    const size_t need = scratch_int_bytes(info->workers) + floats * sizeof(float);
    return need <= plan->ws_bytes ? ScratchSource{plan->ws, plan->ws_bytes} : ScratchSource{};
}

csrk_status csrk_plan_reserve(csrk_plan *plan, int max_N) {
    if (csrk_status s = plan_usable("csrk_plan_reserve", plan)) return s;
    if (max_N < 0 || max_N >= (1 << 24)) return fail(CSRK_INVALID_ARG, "csrk_plan_reserve: width out of range");
    size_t bytes = 0;
    if (csrk_status s = csrk_workspace_bytes(CSRK_OP_FUSEDMM, plan->M, plan->K, max_N, 0, &bytes)) return s;
    if (plan->has_sched) {      // the partial rows of the plan's schedule for uneven rows
        const DeviceInfo *info = nullptr;
        if (csrk_status s = device_info(&info)) return s;
        const size_t with_sched = scratch_int_bytes(info->workers) + sched_partial_floats(plan, max_N) * sizeof(float);
        bytes = with_sched > bytes ? with_sched : bytes;
    }
    if (plan->ws && plan->ws_bytes >= bytes) return CSRK_OK;
    void *mem = nullptr;
    if (hipMalloc(&mem, bytes) != hipSuccess) return fail(CSRK_WORKSPACE, "csrk_plan_reserve: cannot allocate %zu bytes", bytes);
    if (plan->ws) {
        // calls enqueued earlier may still be using the old area
        if (hipDeviceSynchronize() != hipSuccess || hipFree(plan->ws) != hipSuccess) {
            (void)hipFree(mem);
            return fail(CSRK_HIP_ERROR, "csrk_plan_reserve: releasing the previous workspace failed");
        }
    }
    plan->ws = mem;
    plan->ws_bytes = bytes;
    return CSRK_OK;
}

// frees what a plan owns (the caller holds g_mu, or the plan has not been handed out yet)
static csrk_status csrk_plan_destroy_unlocked(csrk_plan_s *plan) {
    hipError_t e = hipFree(plan->dflags);
    for (void *mem : {plan->ws, plan->sched_mem})
        if (mem) {
            const hipError_t e2 = hipFree(mem);
            if (e == hipSuccess) e = e2;
        }
    delete plan;
    if (e != hipSuccess) return fail(CSRK_HIP_ERROR, "csrk_plan_destroy: hipFree: %s", hipGetErrorString(e));
    return CSRK_OK;
}

csrk_status csrk_plan_create(int M, int K, const int32_t *rowptr, const int32_t *colidx, hipStream_t stream,
                             csrk_plan **out) {
    if (!out) return fail(CSRK_INVALID_ARG, "csrk_plan_create: out must not be NULL");
    *out = nullptr;
    if (M < 0 || K < 0) return fail(CSRK_INVALID_ARG, "csrk_plan_create: negative dimension");
    if (!rowptr) return fail(CSRK_INVALID_ARG, "csrk_plan_create: rowptr must not be NULL");
    const ScratchSource scratch{};      // the device's lazily grown scratch
    CallLock lock;
    DeviceState state;
    DeviceState *d = &state;
    if (csrk_status s = begin_call(state, scratch, lock)) return s;
    if (csrk_status s = ensure_scratch(*d, 1)) return s;
    int dev = 0;
    CSRK_HIP(hipGetDevice(&dev));
    // structure first (the walk over colidx needs a sane rowptr), then column order, then row lengths
    int32_t *vflags = d->head_row + d->workers;   // two spare words behind the worker table
    int32_t host[2] = {0, 0};
    int32_t nnz = 0;
    CSRK_HIP(hipMemcpyAsync(vflags, host, sizeof(host), hipMemcpyHostToDevice, stream));
    hipLaunchKernelGGL(validate_rowptr_kernel, dim3(M / 256 + 1), dim3(256), 0, stream, M, rowptr, vflags);
    CSRK_HIP(hipGetLastError());
    CSRK_HIP(hipMemcpyAsync(host, vflags, sizeof(host), hipMemcpyDeviceToHost, stream));
    CSRK_HIP(hipMemcpyAsync(&nnz, rowptr + M, sizeof(nnz), hipMemcpyDeviceToHost, stream));
    CSRK_HIP(hipStreamSynchronize(stream));
    if (host[0] != 0) return fail(CSRK_INVALID_ARG, "csrk_plan_create: rowptr is not a valid row pointer array");
    if (nnz > 0 && !colidx) return fail(CSRK_INVALID_ARG, "csrk_plan_create: colidx must not be NULL");
    int32_t analysis[8] = {0, 0, 0, 1, 0, 0, 0, 0};
    if (M > 0 && nnz > 0) {
        hipLaunchKernelGGL(validate_colidx_kernel, dim3(1024), dim3(256), 0, stream, M, K, rowptr, colidx, vflags);
        CSRK_HIP(hipGetLastError());
        CSRK_HIP(hipMemcpyAsync(host, vflags, sizeof(host), hipMemcpyDeviceToHost, stream));
        hipLaunchKernelGGL(reset_flags_kernel, dim3(1), dim3(1024), 0, stream, M, K, rowptr, 0.f, tile_flags(*d),
                           (int32_t *)nullptr);
        CSRK_HIP(hipGetLastError());
        CSRK_HIP(hipMemcpyAsync(analysis, tile_flags(*d), 4 * sizeof(int32_t), hipMemcpyDeviceToHost, stream));
        CSRK_HIP(hipStreamSynchronize(stream));
        if (host[0] != 0) return fail(CSRK_INVALID_ARG, "csrk_plan_create: colidx holds columns outside [0, K)");
    }
    csrk_plan_s *plan = new csrk_plan_s{dev, M, K, (long long)nnz, rowptr, colidx, host[1] == 0, analysis[3] != 0, nullptr, nullptr, 0};
    if (hipMalloc(&plan->dflags, 8 * sizeof(int32_t)) != hipSuccess) {
        delete plan;
        return fail(CSRK_HIP_ERROR, "csrk_plan_create: hipMalloc of the plan's flag words failed");
    }
    const int32_t words[8] = {0, 1, 0, plan->even ? 1 : 0, 0, 0, 0, 0};
    if (hipMemcpyAsync(plan->dflags, words, sizeof(words), hipMemcpyHostToDevice, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess) {
        (void)hipFree(plan->dflags);
        delete plan;
        return fail(CSRK_HIP_ERROR, "csrk_plan_create: copying the plan's flag words failed");
    }
    // uneven rows with ordered columns: a schedule for the tiled kernels (see csrk_plan_s::Sched)
    if (plan->sorted && !plan->even && M >= 256 && K >= 2 * kSchedMinSegment && nnz > 0 && env_int("CSRK_SCHED", 1) == 1) {
        std::vector<int32_t> rp((size_t)M + 1);
        SchedHost host_sched;
        if (hipMemcpyAsync(rp.data(), rowptr, rp.size() * sizeof(int32_t), hipMemcpyDeviceToHost, stream) != hipSuccess ||
            hipStreamSynchronize(stream) != hipSuccess) {
            (void)csrk_plan_destroy_unlocked(plan);
            return fail(CSRK_HIP_ERROR, "csrk_plan_create: reading rowptr back failed");
        }
        build_schedule(M, K, rp, d->cus, host_sched);
        if (csrk_status s = upload_schedule(plan, host_sched, stream)) {
            (void)csrk_plan_destroy_unlocked(plan);
            return s;
        }
    }
    *out = plan;
    return CSRK_OK;
}

csrk_status csrk_plan_destroy(csrk_plan *plan) {
    if (!plan) return CSRK_OK;
    std::lock_guard<std::mutex> lock(g_mu);
    return csrk_plan_destroy_unlocked(plan);
}

csrk_status csrk_plan_info(const csrk_plan *plan, long long *nnz, int *sorted, int *even) {
    if (!plan) return fail(CSRK_INVALID_ARG, "csrk_plan_info: plan must not be NULL");
    if (nnz) *nnz = plan->nnz;
    if (sorted) *sorted = plan->sorted ? 1 : 0;
    if (even) *even = plan->even ? 1 : 0;
    return CSRK_OK;
}

csrk_status spmm_csr_plan(const csrk_plan *plan, int N, const float *vals, const float *B, float *O,
                          hipStream_t stream) {
    if (csrk_status s = plan_usable("spmm_csr_plan", plan)) return s;
    return spmm_run(plan, plan_scratch(plan, CSRK_OP_SPMM, N), plan->M, plan->K, N, plan->rowptr, plan->colidx, vals, B, O,
                    stream);
}

csrk_status sddmm_csr_plan(const csrk_plan *plan, int D, const float *vals, const float *A, const float *B, float *P,
                           hipStream_t stream) {
    if (csrk_status s = plan_usable("sddmm_csr_plan", plan)) return s;
    return sddmm_run(plan, plan_scratch(plan, CSRK_OP_SDDMM, 0), plan->M, plan->K, D, plan->rowptr, plan->colidx, vals, A,
                     B, P, stream);
}

csrk_status fusedmm_csr_plan(const csrk_plan *plan, int D, int N, const float *vals, const float *A, const float *B,
                             const float *C, float *O, hipStream_t stream) {
    if (csrk_status s = plan_usable("fusedmm_csr_plan", plan)) return s;
    return fusedmm_run(plan, plan_scratch(plan, CSRK_OP_FUSEDMM, N), plan->M, plan->K, D, N, plan->rowptr, plan->colidx,
                       vals, A, B, C, O, stream);
}

csrk_status spmm_csr_bf16(int M, int K, int N, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                          const uint16_t *B, float *O, hipStream_t stream) {
    if (csrk_status s = check_dims("spmm_csr_bf16", M, K, N, 0)) return s;
    if (M == 0 || N == 0) return CSRK_OK;
    if (!rowptr || !O) return fail(CSRK_INVALID_ARG, "spmm_csr_bf16: rowptr and O must not be NULL");
    if (K > 0 && !B) return fail(CSRK_INVALID_ARG, "spmm_csr_bf16: B must not be NULL");
    const ScratchSource scratch{};      // the device's lazily grown scratch
    CallLock lock;
    DeviceState state;
    DeviceState *d = &state;
    if (csrk_status s = begin_call(state, scratch, lock)) return s;
    d->pending_ksplit = 0;
    if (csrk_status s = ensure_scratch(*d, N)) return s;
    const bool vec8 = (N % 8 == 0) && aligned16(B) && aligned16(O) && aligned16(d->head);
    const WidthCfg c = out_width_cfg_bf16(N, vec8);
    const int tile = c.vec * c.lg * c.t;
    const dim3 grid(d->workers / kWavesPerBlock, (N + tile - 1) / tile);
    CallRecord rec(11, stream);
    rec.begin();
    if (vec8 && rows_mode_ok(M, K, N)) {     // small S: a row per 1, 2 or 4 wavefronts, one launch
        const int wpr = rows_wpr(M, N);
        const dim3 rgrid = rows_grid(M, wpr, (N + tile - 1) / tile);
#define CSRK_SPMM_ROWS_BF16_CASE(V, L, T)                                                                          \
    if (c.vec == V && c.lg == L && c.t == T)                                                                       \
        hipLaunchKernelGGL((spmm_rows_kernel<V, L, T, bf16_t>), rgrid, dim3(kBlockThreads), 0, stream, M, N, rowptr, \
                           colidx, vals, B, O, wpr);
        CSRK_SPMM_ROWS_BF16_CASE(8, 8, 1)
        CSRK_SPMM_ROWS_BF16_CASE(8, 16, 1)
        CSRK_SPMM_ROWS_BF16_CASE(8, 32, 1)
        CSRK_SPMM_ROWS_BF16_CASE(8, 64, 1)
        CSRK_SPMM_ROWS_BF16_CASE(8, 64, 2)
#undef CSRK_SPMM_ROWS_BF16_CASE
        rec.end();
        CSRK_HIP(hipGetLastError());
        return CSRK_OK;
    }
    const int32_t *even = nullptr;
    if (even_rows_worth_asking(*d, M, K, false)) {
        if (csrk_status s = launch_analysis(*d, stream, M, K, rowptr, 2.f)) return s;
        even = tile_flags(*d) + 3;
    }
#define CSRK_SPMM_BF16_CASE(V, L, T)                                                                               \
    if (c.vec == V && c.lg == L && c.t == T)                                                                       \
        hipLaunchKernelGGL((spmm_nnzsplit_kernel<V, L, T, bf16_t>), grid, dim3(kBlockThreads), 0, stream, M, N, rowptr, \
                           colidx, vals, B, O, d->head, d->head_row, nullptr, even);
    CSRK_SPMM_BF16_CASE(8, 8, 1)
    CSRK_SPMM_BF16_CASE(8, 16, 1)
    CSRK_SPMM_BF16_CASE(8, 32, 1)
    CSRK_SPMM_BF16_CASE(8, 64, 1)
    CSRK_SPMM_BF16_CASE(8, 64, 2)
    CSRK_SPMM_BF16_CASE(1, 64, 1)
#undef CSRK_SPMM_BF16_CASE
    CSRK_HIP(hipGetLastError());
    launch_combine(*d, stream, M, N, O, nullptr, even, c.vec >= 4 && c.t == 1, vec8);
    rec.end();
    CSRK_HIP(hipGetLastError());
    return CSRK_OK;
}

csrk_status sddmm_csr_bf16(int M, int K, int D, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                           const uint16_t *A, const uint16_t *B, float *P, hipStream_t stream) {
    if (csrk_status s = check_dims("sddmm_csr_bf16", M, K, D, 0)) return s;
    if (M == 0 || K == 0) return CSRK_OK;
    if (!rowptr) return fail(CSRK_INVALID_ARG, "sddmm_csr_bf16: rowptr must not be NULL");
    if (D > 0 && (!A || !B)) return fail(CSRK_INVALID_ARG, "sddmm_csr_bf16: A and B must not be NULL");
    const ScratchSource scratch{};      // the device's lazily grown scratch
    CallLock lock;
    DeviceState state;
    DeviceState *d = &state;
    if (csrk_status s = begin_call(state, scratch, lock)) return s;
    const bool vec8 = (D % 8 == 0) && D > 0 && aligned16(A) && aligned16(B);
    const WidthCfg c = dot_width_cfg_bf16(D, vec8);
    const dim3 grid(d->workers / kWavesPerBlock);
    CallRecord rec(12, stream);
    rec.begin();
    if (vec8 && c.t == 1 && rows_mode_ok(M, K, D)) {
        const int wpr = rows_wpr(M, D);
        const dim3 rgrid = rows_grid(M, wpr, 1);
        if (c.lg == 8)
            hipLaunchKernelGGL((sddmm_rows_kernel<8, 8, 1, bf16_t>), rgrid, dim3(kBlockThreads), 0, stream, M, D, rowptr,
                               colidx, vals, A, B, P, wpr);
        else
            hipLaunchKernelGGL((sddmm_rows_kernel<8, 16, 1, bf16_t>), rgrid, dim3(kBlockThreads), 0, stream, M, D, rowptr,
                               colidx, vals, A, B, P, wpr);
        rec.end();
        CSRK_HIP(hipGetLastError());
        return CSRK_OK;
    }
#define CSRK_SDDMM_BF16_CASE(V, L, T)                                                                              \
    if (c.vec == V && c.lg == L && c.t == T)                                                                       \
        hipLaunchKernelGGL((sddmm_nnzsplit_kernel<V, L, T, bf16_t>), grid, dim3(kBlockThreads), 0, stream, M, D, rowptr, \
                           colidx, vals, A, B, P, nullptr, nullptr);
    CSRK_SDDMM_BF16_CASE(8, 8, 1)
    CSRK_SDDMM_BF16_CASE(8, 16, 1)
    CSRK_SDDMM_BF16_CASE(8, 64, 0)
    CSRK_SDDMM_BF16_CASE(1, 64, 0)
#undef CSRK_SDDMM_BF16_CASE
    rec.end();
    CSRK_HIP(hipGetLastError());
    return CSRK_OK;
}

csrk_status fusedmm_csr_bf16(int M, int K, int D, int N, const int32_t *rowptr, const int32_t *colidx,
                             const float *vals, const uint16_t *A, const uint16_t *B, const uint16_t *C, float *O,
                             hipStream_t stream) {
    if (csrk_status s = check_dims("fusedmm_csr_bf16", M, K, D, N)) return s;
    if (M == 0 || N == 0) return CSRK_OK;
    if (!rowptr || !O) return fail(CSRK_INVALID_ARG, "fusedmm_csr_bf16: rowptr and O must not be NULL");
    if (K > 0 && !C) return fail(CSRK_INVALID_ARG, "fusedmm_csr_bf16: C must not be NULL");
    if (K > 0 && D > 0 && (!A || !B)) return fail(CSRK_INVALID_ARG, "fusedmm_csr_bf16: A and B must not be NULL");
    const ScratchSource scratch{};      // the device's lazily grown scratch
    CallLock lock;
    DeviceState state;
    DeviceState *d = &state;
    if (csrk_status s = begin_call(state, scratch, lock)) return s;
    d->pending_ksplit = 0;
    if (csrk_status s = ensure_scratch(*d, N)) return s;
    const bool dvec8 = (D % 8 == 0) && D > 0 && aligned16(A) && aligned16(B);
    const bool nvec8 = (N % 8 == 0) && aligned16(C) && aligned16(O) && aligned16(d->head);
    const WidthCfg dc = dot_width_cfg_bf16(D, dvec8);
    const WidthCfg nc = out_width_cfg_bf16(N, nvec8);
    const int tile = nc.vec * nc.lg * nc.t;
    const dim3 grid(d->workers / kWavesPerBlock, (N + tile - 1) / tile);
    CallRecord rec(13, stream);
    rec.begin();
    if (nvec8 && dvec8 && dc.t == 1 && N <= 512 && rows_mode_ok(M, K, N)) {
        const bool launched =
            dc.lg == 8 ? launch_fused_rows_bf16_n<8, 8, 1>(nc, stream, M, D, N, rowptr, colidx, vals, A, B, C, O)
                       : launch_fused_rows_bf16_n<8, 16, 1>(nc, stream, M, D, N, rowptr, colidx, vals, A, B, C, O);
        if (launched) {
            rec.end();
            CSRK_HIP(hipGetLastError());
            return CSRK_OK;
        }
    }
    const int32_t *even = nullptr;
    if (even_rows_worth_asking(*d, M, K, true)) {
        if (csrk_status s = launch_analysis(*d, stream, M, K, rowptr, 2.f)) return s;
        even = tile_flags(*d) + 3;
    }
    bool done = false;
#define CSRK_DOT_BF16_CASE(V, L, T)                                                                                \
    if (!done && dc.vec == V && dc.lg == L && dc.t == T)                                                           \
        done = launch_fused_bf16_n<V, L, T>(nc, grid, stream, M, D, N, rowptr, colidx, vals, A, B, C, O, d->head,  \
                                            d->head_row, even);
    CSRK_DOT_BF16_CASE(8, 8, 1)
    CSRK_DOT_BF16_CASE(8, 16, 1)
    CSRK_DOT_BF16_CASE(8, 64, 0)
    CSRK_DOT_BF16_CASE(1, 64, 0)
#undef CSRK_DOT_BF16_CASE
    if (!done) return fail(CSRK_UNSUPPORTED, "fusedmm_csr_bf16: no kernel for D=%d N=%d", D, N);
    CSRK_HIP(hipGetLastError());
    launch_combine(*d, stream, M, N, O, nullptr, even, false, nvec8);
    rec.end();
    CSRK_HIP(hipGetLastError());
    return CSRK_OK;
}

csrk_status csrk_validate_csr(int M, int K, const int32_t *rowptr, const int32_t *colidx, hipStream_t stream,
                              int *problems, int *sorted) {
    if (M < 0 || K < 0) return fail(CSRK_INVALID_ARG, "csrk_validate_csr: negative dimension");
    if (!rowptr) return fail(CSRK_INVALID_ARG, "csrk_validate_csr: rowptr must not be NULL");
    const ScratchSource scratch{};      // the device's lazily grown scratch
    CallLock lock;
    DeviceState state;
    DeviceState *d = &state;
    if (csrk_status s = begin_call(state, scratch, lock)) return s;
    if (csrk_status s = ensure_scratch(*d, 1)) return s;
    int32_t *flags = d->head_row + d->workers;    // two spare words behind the worker table
    int32_t host[2] = {0, 0};
    CSRK_HIP(hipMemcpyAsync(flags, host, sizeof(host), hipMemcpyHostToDevice, stream));
    hipLaunchKernelGGL(validate_rowptr_kernel, dim3(M / 256 + 1), dim3(256), 0, stream, M, rowptr, flags);
    CSRK_HIP(hipGetLastError());
    CSRK_HIP(hipMemcpyAsync(host, flags, sizeof(host), hipMemcpyDeviceToHost, stream));
    CSRK_HIP(hipStreamSynchronize(stream));
    if (host[0] == 0 && M > 0 && colidx) {       // only walk colidx under a sane rowptr
        hipLaunchKernelGGL(validate_colidx_kernel, dim3(1024), dim3(256), 0, stream, M, K, rowptr, colidx, flags);
        CSRK_HIP(hipGetLastError());
        CSRK_HIP(hipMemcpyAsync(host, flags, sizeof(host), hipMemcpyDeviceToHost, stream));
        CSRK_HIP(hipStreamSynchronize(stream));
    }
    if (problems) *problems = host[0];
    if (sorted) *sorted = host[1] == 0;
    return CSRK_OK;
}

// --- measuring aids ------------------------------------------------------------------------------------------

__global__ void row_rotation_kernel(float *out) {
    // lane l puts its own number into `a`; after fma_row_rotated<S>(acc = 0, a, b = 1) acc is the number of the lane
    // whose `a` the rotation handed over
    const int lane = threadIdx.x;
    const float a = (float)lane;
    static_for<0, 16>([&](auto sc) {
        constexpr int S = decltype(sc)::value;
        float acc = 0.f;
        fma_row_rotated<S>(acc, a, 1.f);
        out[S * kWave + lane] = acc;
    });
}

csrk_status csrk_debug_row_rotation(float *out, hipStream_t stream) {
    if (!out) return fail(CSRK_INVALID_ARG, "csrk_debug_row_rotation: out must not be NULL");
    hipLaunchKernelGGL(row_rotation_kernel, dim3(1), dim3(kWave), 0, stream, out);
    CSRK_HIP(hipGetLastError());
    return CSRK_OK;
}

csrk_status csrk_tile_phases(int op, int M, int K, int D, int N, const int32_t *rowptr, const int32_t *colidx,
                             const float *vals, const float *A, const float *B, const float *C, float *O,
                             hipStream_t stream, double *cycles, int *tiles) {
    if (op != CSRK_OP_SPMM && op != CSRK_OP_FUSEDMM) return fail(CSRK_INVALID_ARG, "csrk_tile_phases: SPMM or FusedMM");
    if (!cycles || !tiles || !rowptr || !O || !C) return fail(CSRK_INVALID_ARG, "csrk_tile_phases: NULL argument");
    if (N != 512 || M <= 0 || M % 64 != 0 || K <= 0 || (op == CSRK_OP_FUSEDMM && (D != 64 || !A || !B)))
        return fail(CSRK_UNSUPPORTED, "csrk_tile_phases: only the 512-column kernels with 4 rows per wavefront (M a multiple of 64, D = 64)");
    if (!aligned16(C) || !aligned16(O) || (op == CSRK_OP_FUSEDMM && (!aligned16(A) || !aligned16(B))))
        return fail(CSRK_INVALID_ARG, "csrk_tile_phases: operands must be 16-byte aligned");
    const int groups = M / 64;
    const size_t waves = (size_t)groups * kTileWaves;
    long long *dtim = nullptr;
    int32_t *dflags = nullptr;
    CSRK_HIP(hipMalloc((void **)&dtim, waves * kPhases * sizeof(long long)));
    if (hipMalloc((void **)&dflags, 8 * sizeof(int32_t)) != hipSuccess) {
        (void)hipFree(dtim);
        return fail(CSRK_HIP_ERROR, "csrk_tile_phases: hipMalloc failed");
    }
    const int32_t words[8] = {0, 1, 0, 1, 0, 0, 0, 0};      // nothing unsorted seen, tiled kernel allowed, rows even
    hipError_t e = hipMemcpyAsync(dflags, words, sizeof(words), hipMemcpyHostToDevice, stream);
    if (e == hipSuccess) e = hipMemsetAsync(dtim, 0, waves * kPhases * sizeof(long long), stream);
    const float no_inline = __builtin_nanf("");
    if (e == hipSuccess) {
        if (op == CSRK_OP_SPMM) {
            using L = KTileLds<2, 64>;
            auto kern = ktile_kernel<2, 64, 4, true>;
            e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, L::kBytes);
            if (e == hipSuccess) {
                hipLaunchKernelGGL(kern, dim3(groups), dim3(kTileThreads), L::kBytes, stream, M, K, N, N, rowptr, colidx, vals,
                                   C, O, dflags, (float *)nullptr, no_inline, (int32_t *)nullptr, dtim,
                                   (const int32_t *)nullptr, (const int4 *)nullptr);
                e = hipGetLastError();
            }
        } else {
            using L = FusedTileLds<2, 64, 4, 32>;
            auto kern = fused_ktile_kernel<2, 64, 4, 32, 5, 4, true>;
            e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, L::kBytes);
            if (e == hipSuccess) {
                hipLaunchKernelGGL(kern, dim3(groups), dim3(kTileThreads), L::kBytes, stream, M, K, D, N, N, rowptr, colidx,
                                   vals, A, B, C, O, dflags, (float *)nullptr, no_inline, (int32_t *)nullptr, dtim,
                                   (const int32_t *)nullptr, (const int4 *)nullptr);
                e = hipGetLastError();
            }
        }
    }
    std::vector<long long> host(waves * kPhases);
    int32_t seen[8] = {0};
    if (e == hipSuccess) e = hipMemcpyAsync(host.data(), dtim, host.size() * sizeof(long long), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipMemcpyAsync(seen, dflags, sizeof(seen), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    (void)hipFree(dtim);
    (void)hipFree(dflags);
    if (e != hipSuccess) return fail(CSRK_HIP_ERROR, "csrk_tile_phases: %s", hipGetErrorString(e));
    if (seen[0] != 0) return fail(CSRK_INVALID_ARG, "csrk_tile_phases: the pattern's columns are not ascending");
    for (int i = 0; i < kPhases; ++i) cycles[i] = 0.0;
    for (size_t w = 0; w < waves; ++w)
        for (int i = 0; i < kPhases; ++i) cycles[i] += (double)host[w * kPhases + i];
    for (int i = 0; i < kPhases; ++i) cycles[i] /= (double)waves;
    *tiles = (K + 63) / 64;
    return CSRK_OK;
}

csrk_status csrk_profile_enable(int max_records) {
    std::lock_guard<std::mutex> lock(g_mu);
    for (hipEvent_t e : g_rec.start) (void)hipEventDestroy(e);
    for (hipEvent_t e : g_rec.stop) (void)hipEventDestroy(e);
    g_rec.start.clear();
    g_rec.stop.clear();
    g_rec.kind.clear();
    g_rec.used = 0;
    if (max_records < 0) return fail(CSRK_INVALID_ARG, "csrk_profile_enable: negative count");
    for (int i = 0; i < max_records; ++i) {
        hipEvent_t a, b;
        CSRK_HIP(hipEventCreate(&a));
        CSRK_HIP(hipEventCreate(&b));
        g_rec.start.push_back(a);
        g_rec.stop.push_back(b);
        g_rec.kind.push_back(0);
    }
    return CSRK_OK;
}

csrk_status csrk_profile_collect(float *ms, int *kinds, int capacity, int *count) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (!count || capacity < 0 || (capacity > 0 && (!ms || !kinds)))
        return fail(CSRK_INVALID_ARG, "csrk_profile_collect: bad arguments");
    int n = 0;
    for (int i = 0; i < g_rec.used && n < capacity; ++i) {
        CSRK_HIP(hipEventSynchronize(g_rec.stop[i]));
        CSRK_HIP(hipEventElapsedTime(&ms[n], g_rec.start[i], g_rec.stop[i]));
        kinds[n] = g_rec.kind[i];
        ++n;
    }
    *count = n;
    g_rec.used = 0;
    return CSRK_OK;
}

csrk_status csrk_release_workspace(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    int dev = 0;
    CSRK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return CSRK_OK;
    LazyScratch &g = g_lazy[dev];
    CSRK_HIP(hipDeviceSynchronize());
    if (g.head) CSRK_HIP(hipFree(g.head));
    if (g.head_row) CSRK_HIP(hipFree(g.head_row));
    g.head = nullptr;
    g.head_row = nullptr;
    g.head_floats = 0;
    return CSRK_OK;
}

}  // extern "C"
