// LDS-tiled kernels for large, fairly dense S (the 16384 x 16384 / 20 % class).
//
// Why: every multiply-add of SPMM needs one fresh element of the gathered dense row.
// Gathering those rows with global loads is capped by the CU's vector-memory path
// (about 56 B/clk/CU measured on MI355X when the rows hit in L2, a quarter of that
// once the dense operand spills out of the 4 MB L2 of an XCD), while LDS delivers
// about 175 B/clk/CU to 128-bit reads.  So a workgroup stages a K-tile of the dense
// operand in LDS once and all of its rows gather from there.
//
// Shape: one workgroup of 16 wavefronts owns RB = 16*ROWS consecutive rows of S and the
// whole output width (T tiles of 256 columns: lane l holds columns 4l..4l+3 of each
// tile, so a gathered row is one conflict-free 128-bit LDS read per tile).  It sweeps K
// in tiles of KT columns: [barrier] all threads copy C[k0:k0+KT, :] into LDS [barrier],
// then every wavefront processes, for each of its ROWS rows, the stored entries whose
// column falls in the tile, accumulating in registers.  A row's entries for a tile are
// found without any precomputed pointers: the wavefront keeps a cursor per row and a
// 64-entry look-ahead chunk of (colidx, vals) in registers; because columns ascend
// within a row, the entries of the current tile are a prefix of the chunk, whose
// length is a ballot + popcount.
//
// Instruction budget (the kernel is bound by VALU issue and LDS delivery together, not by HBM):
//  - The chunk is parked in a small per-wavefront LDS slot as (column, value) pairs
//    and entries are fetched back two at a time with one 128-bit read whose address is
//    the same in every lane (an LDS broadcast).  That puts column and value in VGPRs of
//    all lanes with no VALU work; v_readlane_b32 would cost two 8-cycle VALU slots per
//    entry, a third of the kernel's time when measured.
//  - Per entry that leaves one address computation plus the 4*T multiply-adds.
//  - Entries go in batches of 4: pair reads, then all row reads, then the multiply-adds,
//    so LDS latency overlaps.
//  - The look-ahead chunks are reloaded in one place, after the tile's arithmetic, and
//    the next tile of the dense operand is requested into registers right after the
//    tile barrier: no vector-memory wait ever sits inside the arithmetic.
//
// Requirements: columns of every row non-decreasing; S dense enough for the LDS copy to
// pay.  Density and row-length spread are read off rowptr first (tile_go below).  Ordering is
// verified by the tiled kernels themselves at no extra memory traffic: every look-ahead
// chunk they load is compared lane against neighbouring lane (one DPP shift and a
// compare), and chunks overlap, so every adjacent pair of a row passes through the check.
// A kernel that meets a descending pair raises flags[0]; its output is then unspecified
// (never out of bounds: the cursors only move inside the row and LDS reads cannot fault)
// and the general kernels, which are launched right behind it, redo the whole call.
//
// Small M: a launch may cut K into ranges, one workgroup per (row block, range); see KSplit below.
//
// The FusedMM version of this kernel (same accumulate stage plus a score stage) is in
// kernels_ktile_fused.hpp; the tiled SDDMM kernel is at the end of this file.
#pragma once
#include <type_traits>

#include "device_util.hpp"

namespace csrk {

constexpr int kTileThreads = 1024;
constexpr int kTileWaves = kTileThreads / kWave;

// added to a density threshold handed to the row analysis: moderately uneven rows are acceptable (see row_analysis)
constexpr float kUnevenOk = 4.f;

// flags[0] != 0: some row has descending columns.  flags[1] != 0: dense enough.
__device__ __forceinline__ bool ktile_ok(const int32_t *flags) { return flags[0] == 0 && flags[1] != 0; }

// The per-call row analysis of the tiled kernels: decides from rowptr alone whether the tiled kernels suit S.
// nnz = rowptr[M] must reach `min_density` of M*K, and no row may be much longer than the mean row (the tiled
// kernels give every wavefront a fixed set of rows and synchronise per tile, so skewed row lengths are left to
// the equal-nonzero split of the general kernels).  A negative `min_density` switches both criteria off (used
// by tests to reach the tiled kernels with any pattern).  kUnevenOk + threshold: the caller's kernel is one of the
// wide ones (more than 128 output columns), for which moderately uneven rows - longest up to 16 mean rows - still
// beat the general kernels' gathers of long dense rows (8192^2, log-normal row lengths with mean 10 % of K and
// sigma 1, longest = 10 means, unplanned FusedMM D = 64 / SPMM: N = 512 680 / 452 us against 1570 / 1362, N = 256
// 545 / 332 against 703 / 496; N = 128 and 64 the other way round, 394 / 206 against 313 / 171 and 327 / 145
// against 182 / 101).
//
// Run by a whole workgroup of up to 1024 threads; `red` is room for 16 ints in LDS.  Returns, in every thread,
// bit 0: the tiled kernel may run, bit 1: rows even (for the general kernels: rows can be dealt out whole).
__device__ __forceinline__ int row_analysis(int M, int K, const int32_t *__restrict__ rowptr, float min_density,
                                            int *red) {
    int longest = 0;
    constexpr int U = 8;                     // row lengths requested together per thread
    for (long long r0 = threadIdx.x; r0 < M; r0 += blockDim.x * U) {
        int lo[U], hi[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // unconditional loads (a row past the end repeats the last row): conditional ones are waited for one by one
            long long r = r0 + u * (long long)blockDim.x;
            r = r < M ? r : M - 1;
            lo[u] = rowptr[r];
            hi[u] = rowptr[r + 1];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) longest = hi[u] - lo[u] > longest ? hi[u] - lo[u] : longest;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const int o = __shfl_xor(longest, off);
        longest = o > longest ? o : longest;
    }
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = longest;
    __syncthreads();
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) longest = red[w] > longest ? red[w] : longest;
    const double nnz = (double)rowptr[M];
    const double mean = M > 0 ? nnz / (double)M : 0.0;
    const bool wide = min_density >= kUnevenOk;
    const double threshold = wide ? (double)(min_density - kUnevenOk) : (double)min_density;
    const bool dense = nnz >= threshold * (double)M * (double)K;
    const bool even = (double)longest <= 2.0 * mean + 64.0;
    const bool suits = even || (wide && (double)longest <= 16.0 * mean + 64.0);
    __syncthreads();                         // `red` may be reused by the caller
    return (((dense && suits) || min_density < 0.f) ? 1 : 0) | (even ? 2 : 0);
}

// The analysis as a launch of its own (one workgroup), ahead of tiled kernels on matrices with so many rows that
// every workgroup of the tiled kernel reading all of rowptr itself would cost more than this launch, and for the
// general kernels where only they run.  Leaves flags[1] (tiled kernel may run) and flags[3] (rows even), clears
// the ordering flag of this set of flag words and of the other set (see tile_go).
__global__ __launch_bounds__(1024) void reset_flags_kernel(int M, int K, const int32_t *__restrict__ rowptr,
                                                          float min_density, int32_t *flags, int32_t *other) {
    __shared__ int red[16];
    const int verdict = row_analysis(M, K, rowptr, min_density, red);
    if (threadIdx.x == 0) {
        flags[0] = 0;
        flags[1] = verdict & 1;
        flags[3] = (verdict >> 1) & 1;
        if (other) other[0] = 0;
    }
}

// First thing in every tiled kernel: may it run?  Two ways of knowing.  `inline_density` is a number (not NaN): the
// kernel does the row analysis itself - every workgroup reads rowptr and reaches the same verdict, workgroup 0
// leaves it in flags[1] and flags[3] for the kernels launched behind this one - which saves the analysis launch
// (3-6 us and a kernel boundary) where M is small enough for that to be cheap.  Otherwise the verdict is already in
// `flags` (reset_flags_kernel ran, or a plan made them).
// The ordering flag flags[0] cannot be cleared here (a workgroup that starts late would wipe out another's report),
// so the library keeps two sets of flag words and alternates between them: whoever analyses for a call on one set
// clears flags[0] of the OTHER set, which the next call will use.
__device__ __forceinline__ bool tile_go(int M, int K, const int32_t *__restrict__ rowptr, float inline_density,
                                        int32_t *flags, int32_t *other, int *red) {
    if (inline_density != inline_density) return ktile_ok(flags);
    const int verdict = row_analysis(M, K, rowptr, inline_density, red);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        flags[1] = verdict & 1;
        flags[3] = (verdict >> 1) & 1;
        if (other) other[0] = 0;
    }
    return (verdict & 1) != 0;
}

// Lanes whose column is smaller than the column in the lane before them (lane 0 compares with itself).
__device__ __forceinline__ unsigned long long descending_lanes(int k) {
    const int prev = __builtin_amdgcn_update_dpp(k, k, 0x138 /* wave_shr:1 */, 0xf, 0xf, false);
    return __ballot(prev > k);
}

// Full check of the column order of the rows of one row block, done by the workgroups of a K-split launch
// themselves before they start: the S workgroups that share the block (blockIdx.y = 0 .. S-1) each take every
// S-th slice of 1024 neighbouring pairs of the block's entries.  A descending pair is harmless only if its second
// entry is the first of a row; the block's row starts (at most 64) sit one per lane, so that question is one
// compare and a ballot.  Returns true if this workgroup saw a descending pair inside a row.
// Needed because a K-split workgroup starts inside each row, at a position found by binary search, and the
// order check built into the tiled kernels sees only the entries it streams - which proves nothing about a
// row that is not sorted.  (A separate kernel for this check, one thread per stored entry with a binary search
// of rowptr per descending pair, cost 10 us at 1.7 M entries - a dozen dependent loads in a few thousand
// threads; counting descending pairs against row starts with atomics cost 25.)
template <int RB>
__device__ __forceinline__ bool ksplit_block_unsorted(int M, const int32_t *__restrict__ rowptr,
                                                      const int32_t *__restrict__ colidx) {
    static_assert(RB <= kWave, "one row start per lane");
    const int lane = lane_id();
    const int rb0 = blockIdx.x * RB;
    const int rows = M - rb0 < RB ? M - rb0 : RB;
    const int e0 = uniform(rowptr[rb0]), e1 = uniform(rowptr[rb0 + rows]);
    if (e1 - e0 < 2) return false;
    const int start = rowptr[rb0 + (lane < rows ? lane : 0)];     // row starts of the block (lane 0: e0, never asked for)
    constexpr int U = 4;                    // pairs requested together per thread (loads under no condition: an entry
                                            // past the end re-reads the last pair)
    const int slice = (int)blockDim.x, S = (int)gridDim.y;
    bool bad = false;
    for (long long j0 = (long long)e0 + 1 + (long long)blockIdx.y * slice + threadIdx.x; j0 - threadIdx.x < e1;
         j0 += (long long)S * slice * U) {
        int before[U], here[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            long long j = j0 + (long long)u * S * slice;
            j = j < e1 ? j : e1 - 1;
            before[u] = colidx[j - 1];
            here[u] = colidx[j];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long j = j0 + (long long)u * S * slice;
            unsigned long long desc = __ballot(j < e1 && before[u] > here[u]);
            while (desc) {                  // about one per row boundary that falls into this wavefront's 64 pairs
                const int l = __builtin_ctzll(desc);
                desc &= desc - 1;
                const int jj = __builtin_amdgcn_readlane((int)j, l);
                if (__ballot(lane < rows && start == jj) == 0) bad = true;
            }
        }
    }
    return bad;
}

// K-split bookkeeping shared by the tiled kernels.  A launch with gridDim.y = S > 1 gives workgroup (x, y) the
// rows of block x and the columns [kb, ke) of K; it leaves its result rows in `partial` (S x M x N floats) and
// ksplit_reduce adds the S partial rows in the order of y: no atomics on floats, same bits every run.
struct KSplit {
    int kb, ke;
};
// One workgroup's job: a block of RB rows and a range of K.  A regular launch reads it off the grid (row block
// blockIdx.x, range blockIdx.y of gridDim.y).  A launch over a plan's SCHEDULE for uneven rows (rows sorted by length
// when the plan was made, so that the rows of a block are about equally long, and every block's K cut into as many
// ranges as its share of the work asks for - the paper's NT work-items per row, section "SDDMM", with NT chosen per
// block of rows) reads entry blockIdx.x of the schedule: x = block, y = range, z = ranges of that block, w = where
// the block's partial rows of this range go in the scratch area (blocks whose K is cut).  The rows of block b are
// perm[b * RB ...]; padding entries of perm hold M ("no row").
struct TileJob {
    int block, seg, nseg, slot;
    bool sched;
};
__device__ __forceinline__ TileJob tile_job(const int4 *items) {
    TileJob j;
    j.sched = items != nullptr;
    if (j.sched) {
        const int4 it = items[blockIdx.x];
        j.block = uniform(it.x);
        j.seg = uniform(it.y);
        j.nseg = uniform(it.z);
        j.slot = uniform(it.w);
    } else {
        j.block = blockIdx.x;
        j.seg = blockIdx.y;
        j.nseg = gridDim.y;
        j.slot = 0;
    }
    return j;
}
template <int KT>
__device__ __forceinline__ KSplit job_range(const TileJob &j, int K) {
    const int tiles = (K + KT - 1) / KT;
    const int per = (tiles + j.nseg - 1) / j.nseg;
    KSplit r;
    r.kb = j.seg * per * KT;
    r.ke = r.kb + per * KT;
    r.ke = r.ke < K ? r.ke : K;
    r.kb = r.kb < K ? r.kb : K;
    return r;
}
// the row of S at position idx of the job's block (M or more: no row)
__device__ __forceinline__ int job_row(const TileJob &j, const int32_t *perm, int RB, int idx) {
    return j.sched ? uniform(perm[j.block * RB + idx]) : j.block * RB + idx;
}
// where that row's result goes: its row of O, or - if the block's K is cut - a partial row in the scratch area
__device__ __forceinline__ float *job_out(const TileJob &j, float *O, float *partial, int M, int ld, int RB, int idx,
                                          int row) {
    if (j.nseg <= 1) return O + (size_t)row * ld;
    return partial + (j.sched ? (size_t)j.slot * RB + idx : (size_t)j.seg * M + row) * ld;
}

// Adds up the partial rows of the blocks of a schedule whose K was cut: one workgroup per such block (table entry:
// x = block, y = first slot, z = ranges), in the order of the ranges - no float atomics, same bits every run.
__global__ __launch_bounds__(256) void sched_combine_kernel(int M, int N, int ld, int RB, const int32_t *__restrict__ perm,
                                                           const int4 *__restrict__ table, const float *__restrict__ partial,
                                                           float *__restrict__ O) {
    const int4 t = table[blockIdx.x];
    const int n4 = N >> 2, ld4 = ld >> 2;
    for (int e = threadIdx.x; e < RB * n4; e += blockDim.x) {
        const int idx = e / n4, c4 = e % n4;
        const int row = perm[t.x * RB + idx];
        if (row >= M) continue;
        f32x4 sum = reinterpret_cast<const f32x4 *>(partial)[((size_t)t.y * RB + idx) * ld4 + c4];
        for (int s = 1; s < t.z; ++s) sum += reinterpret_cast<const f32x4 *>(partial)[((size_t)(t.y + s) * RB + idx) * ld4 + c4];
        reinterpret_cast<f32x4 *>(O)[(size_t)row * ld4 + c4] = sum;
    }
}

// position of the first entry of [p0, p1) whose column is >= kb (columns ascending)
__device__ __forceinline__ int first_entry_at_or_after(const int32_t *colidx, int p0, int p1, int kb) {
    if (kb <= 0 || p1 <= p0) return p0;
    return p0 + wave_lower_bound(colidx + p0, p1 - p0, kb);
}

// O = sum over y of partial[y] (S x M x N floats), in the order of y: the second half of a K-split call, run by
// the whole grid of the call's last kernel (combine_heads_kernel, when the tiled kernel did the call).  A later
// launch rather than a "last workgroup adds" inside the tiled kernel: the device-wide fences that needs write
// back and invalidate an XCD's whole L2 each time, which cost three times what the split gained.
__device__ __forceinline__ void ksplit_reduce(size_t count4, int S, const float4 *__restrict__ partial,
                                              float4 *__restrict__ O) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count4; i += (size_t)gridDim.x * blockDim.x) {
        float4 sum = partial[i];
        for (int y = 1; y < S; ++y) {
            const float4 p = partial[(size_t)y * count4 + i];
            sum.x += p.x;
            sum.y += p.y;
            sum.z += p.z;
            sum.w += p.w;
        }
        O[i] = sum;
    }
}

// Where a wavefront's cycles go, phase by phase (a measuring build of a kernel; the production instantiations
// have ON = false and none of this exists in them).  lap(i) adds the cycles since the previous lap to counter i.
// Reading the clock waits for outstanding LDS / scalar-memory operations of the wavefront, so laps sit only where
// the kernel drains them anyway (around barriers) or where the perturbation is itself of interest.
constexpr int kPhases = 8;
template <bool ON>
struct PhaseClock {
    long long last = 0;
    long long acc[kPhases] = {};
    __device__ __forceinline__ void start() {
        if constexpr (ON) last = clock64();
    }
    __device__ __forceinline__ void lap(int i) {
        if constexpr (ON) {
            const long long now = clock64();
            acc[i] += now - last;
            last = now;
        }
    }
    // lane 0 of every wavefront leaves its counters at out[(workgroup * waves + wave) * kPhases ...]
    __device__ __forceinline__ void store(long long *out, int waves_per_group, int wave, int lane) const {
        if constexpr (ON) {
            if (out && lane == 0) {
                long long *o = out + ((size_t)(blockIdx.y * gridDim.x + blockIdx.x) * waves_per_group + wave) * kPhases;
#pragma unroll
                for (int i = 0; i < kPhases; ++i) o[i] = acc[i];
            }
        }
    }
};
// phases of the tiled SPMM / FusedMM kernels
enum : int { kPhBarrier1 = 0, kPhCommit = 1, kPhBarrier2 = 2, kPhIssue = 3, kPhCompute = 4, kPhReload = 5, kPhScore = 6 };

template <int T, int KT, int WAVES = kTileWaves>
struct KTileLds {
    static constexpr int kRowFloats = T * 256;
    static constexpr int kCFloats = KT * kRowFloats;
    // (column, value) pairs: two 64-entry slots per wavefront, so that the next row's chunk is
    // written while the current row is consumed
    static constexpr int kEntFloats = WAVES * 2 * kWave * 2;
    static constexpr int kBytes = (kCFloats + kEntFloats) * 4;
};

// SPMM: O[row, :] = sum over the row's entries of value * B[column, :] (Algorithm 2), B called Cmat here.
// TIMED: the measuring build (see PhaseClock); `tim` receives kPhases counters per wavefront.
// WAVES: wavefronts per workgroup (16: one workgroup per CU; 8: two, each with a tile half as high, so that one
// computes while the other sits at a barrier or stages its tile).
template <int T, int KT, int ROWS, bool TIMED = false, int WAVES = kTileWaves>
__global__ __launch_bounds__(WAVES *kWave, WAVES == 16 ? 4 : 2) void ktile_kernel(
    int M, int K, int N, int ld, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ vals, const float *__restrict__ Cmat, float *__restrict__ O, int32_t *flags,
    float *partial, float inline_density, int32_t *other_flags, long long *tim = nullptr,
    const int32_t *__restrict__ perm = nullptr, const int4 *__restrict__ items = nullptr) {
    using L = KTileLds<T, KT, WAVES>;
    constexpr int kThreads = WAVES * kWave;
    PhaseClock<TIMED> clk;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    if (!tile_go(M, K, rowptr, inline_density, flags, other_flags, reinterpret_cast<int *>(lds))) return;
    constexpr int kRowBytes = L::kRowFloats * 4;
    const int lane = lane_id();
    const int wave = uniform(threadIdx.x >> 6);
    float *ct = lds;                        // KT x (T*256) floats
    int2 *ent = reinterpret_cast<int2 *>(lds + L::kCFloats) + wave * (2 * kWave);

    const TileJob job = tile_job(items);
    constexpr int RB = WAVES * ROWS;
    const int n = lane * 4;                 // this lane's first column inside each 256-wide tile
    const unsigned lane_b = (unsigned)lane * 4u;    // ... and its byte offset in a lane-wide load of a chunk

    const KSplit ks = job_range<KT>(job, K);    // the whole of K unless the job is one range of several
    if (!job.sched && job.nseg > 1 && ksplit_block_unsorted<RB>(M, rowptr, colidx)) {
        if (lane == 0) flags[0] = 1;        // the reduction stands down, the general kernels redo the call
    }
    int rows[ROWS];
    int pos[ROWS], end[ROWS];
    int kc[ROWS];
    float vc[ROWS];
    float acc[ROWS][T][4];
    unsigned long long bad = 0;             // lanes that ever saw a descending pair of columns
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int row = job_row(job, perm, RB, wave * ROWS + r);
        rows[r] = row;
        pos[r] = row < M ? uniform(rowptr[row]) : 0;
        end[r] = row < M ? uniform(rowptr[row + 1]) : 0;
        if (job.nseg > 1) pos[r] = first_entry_at_or_after(colidx, pos[r], end[r], ks.kb);
        const bool ok = lane < end[r] - pos[r];
        kc[r] = ok ? lane_elem(colidx + pos[r], lane_b) : 0x7fffffff;
        vc[r] = ok ? (vals ? lane_elem(vals + pos[r], lane_b) : 1.f) : 0.f;
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[r][t][v] = 0.f;
    }

    // ---- staging of the dense tiles: global -> registers (`issue`), registers -> LDS (`commit`)
    const int n4 = N >> 2;                  // float4s of a dense row that this launch works on ...
    const int ld4 = ld >> 2;                // ... out of this many (a launch may take a slab of the columns)
    constexpr int kRow4 = T * 64;
    constexpr int kPer = KT * kRow4 / kThreads;
    static_assert((KT * kRow4) % kThreads == 0, "the staging loop copies whole rounds of float4s");
    f32x4 stage[kPer];
    // Thread t copies float4 number (t % kRow4) of tile rows t / kRow4, + kStep, + 2 kStep, ...: its
    // offset inside a tile never changes, so a tile costs this thread kPer loads off a uniform
    // scalar base with a 32-bit offset of its own.  Threads past the width of a narrower launch re-read the
    // row's last float4 (those LDS columns are only ever read by lanes whose accumulators are not stored), rows
    // past K in the last tile read as zeros (no entry points at them): every thread issues every load, under
    // no condition.
    constexpr int kStep = kThreads / kRow4;      // tile rows covered by one round of loads
    const int my_kk = threadIdx.x / kRow4, my_c4 = threadIdx.x % kRow4;
    const int col4 = my_c4 < n4 ? my_c4 : n4 - 1;
    const unsigned my_off = ((unsigned)my_kk * (unsigned)ld4 + (unsigned)col4) * 16u;
    const unsigned step_bytes = (unsigned)kStep * (unsigned)ld4 * 16u;
    // rows of the operand from this launch's first column on (rows past K read as zeros)
    const DenseView cview = dense_view(Cmat, (unsigned)(((size_t)K * ld - (ld - N)) * 4));
    // loads number [I0, I1) of this thread for the tile that starts at column k0
    auto issue = [&](int k0, auto i0c, auto i1c) {
        constexpr int I0 = decltype(i0c)::value, I1 = decltype(i1c)::value;
        const unsigned tile = (unsigned)k0 * (unsigned)ld4 * 16u;      // uniform
#pragma unroll
        for (int i = I0; i < I1; ++i) stage[i] = load_f32x4(cview, my_off, tile + i * step_bytes);
    };
    auto commit = [&]() {
        f32x4 *dst = reinterpret_cast<f32x4 *>(ct);
#pragma unroll
        for (int i = 0; i < kPer; ++i) dst[i * kThreads + threadIdx.x] = stage[i];
    };

    if (ks.kb < ks.ke) issue(ks.kb, std::integral_constant<int, 0>{}, std::integral_constant<int, kPer>{});
    clk.start();
    for (int k0 = ks.kb; k0 < ks.ke; k0 += KT) {
        __syncthreads();                    // previous tile fully consumed
        clk.lap(kPhBarrier1);
        commit();
        if constexpr (TIMED) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        clk.lap(kPhCommit);
        __syncthreads();
        clk.lap(kPhBarrier2);
        // The next tile is requested into registers while this one is worked on - but NOT by all wavefronts at once
        // here: 16 wavefronts issuing 8 loads of 1 KB each at the same moment fill the vector-memory queue, which
        // takes them at 64 bytes a clock, and every wavefront then sits in its load instructions for some 3000
        // cycles before its first multiply-add (measured: a fifth of the kernel's time, and as much again at the
        // next barrier, where the wavefronts that got through first wait for the last).  A wavefront issues its
        // loads at the start of one of its rows instead, a different row from wavefront to wavefront, so that at
        // any moment only a quarter of them are in the queue while the others keep the LDS and the VALUs busy.
        const bool more = k0 + KT < ks.ke;
        const int issue_row = wave % ROWS;
        const int kend = k0 + KT;
        // lane's byte offset in a tile row, minus the tile origin; unsigned so that the products with
        // large column numbers wrap instead of overflowing (the sum below is always a small offset)
        const unsigned lb = (unsigned)(n * 4) - (unsigned)k0 * (unsigned)kRowBytes;
        int cnts[ROWS];
        ent[lane] = make_int2(kc[0], __builtin_bit_cast(int, vc[0]));
        static_for<0, ROWS>([&](auto rc) {
            constexpr int r = decltype(rc)::value;
            if (more && issue_row == r) {
                clk.lap(kPhCompute);
                issue(k0 + KT, std::integral_constant<int, 0>{}, std::integral_constant<int, kPer>{});
                clk.lap(kPhIssue);
            }
            // entries of this tile = leading lanes of the chunk with column < kend
            const int cnt = __builtin_popcountll(__ballot(kc[r] < kend));
            cnts[r] = cnt;
            // order check on the chunk, here where it is first used (not where it was requested,
            // which would make the request a wait)
            bad |= descending_lanes(kc[r]);
            if constexpr (r + 1 < ROWS)
                ent[((r + 1) & 1) * kWave + lane] = make_int2(kc[r + 1], __builtin_bit_cast(int, vc[r + 1]));
            const int2 *e = ent + (r & 1) * kWave;     // this row's slot
            auto batch = [&](int t, auto count) {
                constexpr int CNT = decltype(count)::value;
                float c[CNT][T][4];
                int2 ks[CNT];
                // same address in all lanes (an LDS broadcast), two pairs per 128-bit read; t is a multiple of 4
#pragma unroll
                for (int u = 0; u + 1 < CNT; u += 2) {
                    const int4 two = *reinterpret_cast<const int4 *>(e + t + u);
                    ks[u] = make_int2(two.x, two.y);
                    ks[u + 1] = make_int2(two.z, two.w);
                }
                if constexpr (CNT % 2 == 1) ks[CNT - 1] = e[t + CNT - 1];
#pragma unroll
                for (int u = 0; u < CNT; ++u) {
                    const char *crow = reinterpret_cast<const char *>(ct) + ((unsigned)ks[u].x * (unsigned)kRowBytes + lb);
#pragma unroll
                    for (int tt = 0; tt < T; ++tt)
                        load_vec<4>(reinterpret_cast<const float *>(crow + tt * 1024), c[u][tt]);
                }
#pragma unroll
                for (int u = 0; u < CNT; ++u) {
                    const float sv = __builtin_bit_cast(float, ks[u].y);
#pragma unroll
                    for (int tt = 0; tt < T; ++tt)
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[r][tt][v] = fmaf(sv, c[u][tt][v], acc[r][tt][v]);
                }
            };
            // all entries [0, cnt) of the slot, in batches of 4
            auto run = [&](int cnt) {
                int t = 0;
                for (; t + 4 <= cnt; t += 4) batch(t, std::integral_constant<int, 4>{});
                // the last 1-3 entries as a pair and a single: two plain ifs keep the accumulators in place, where a
                // switch over the three cases made the compiler copy them in and out
                if (cnt - t >= 2) {
                    batch(t, std::integral_constant<int, 2>{});
                    t += 2;
                }
                if (cnt - t >= 1) batch(t, std::integral_constant<int, 1>{});
            };
            if constexpr (KT > kWave) {
                // A row whose whole chunk lies in the tile (64 or more entries of it in one tile: dense rows) gets its
                // next chunk with a blocking load and goes through the same slot again.
                for (int c = cnt;;) {
                    run(c);
                    pos[r] += c;
                    if (__builtin_expect(c < kWave || pos[r] >= end[r], 1)) break;
                    const int lastk = __builtin_amdgcn_readlane(kc[r], kWave - 1);
                    const bool okn = lane < end[r] - pos[r];
                    kc[r] = okn ? lane_elem(colidx + pos[r], lane_b) : 0x7fffffff;
                    vc[r] = okn ? (vals ? lane_elem(vals + pos[r], lane_b) : 1.f) : 0.f;
                    bad |= descending_lanes(kc[r]);
                    if (__builtin_amdgcn_readlane(kc[r], 0) < lastk) bad |= 1;     // descending across the chunk boundary
                    c = __builtin_popcountll(__ballot(kc[r] < kend));
                    if (c == 0) break;
                    ent[(r & 1) * kWave + lane] = make_int2(kc[r], __builtin_bit_cast(int, vc[r]));
                }
            } else {
                // A tile of at most 64 columns holds more than a chunk of one row only if columns repeat, and a
                // full chunk only for a dense row: the simple continuation, one entry at a time, is enough (and
                // keeps this, the 512-wide kernel, free of the loop above, which costs it 2 %).
                run(cnt);
                pos[r] += cnt;
                if (cnt == kWave) {
                    int lastk = __builtin_amdgcn_readlane(kc[r], kWave - 1);
                    while (pos[r] < end[r]) {
                        const int k = uniform(colidx[pos[r]]);
                        if (k < lastk) bad |= 1;     // descending across the chunk boundary or inside this run
                        lastk = k;
                        if (k >= kend) break;
                        const float s = vals ? __builtin_bit_cast(float, uniform(__builtin_bit_cast(int, vals[pos[r]]))) : 1.f;
                        const float *crow = ct + (k - k0) * L::kRowFloats + n;
#pragma unroll
                        for (int tt = 0; tt < T; ++tt) {
                            float c[4];
                            load_vec<4>(crow + tt * 256, c);
#pragma unroll
                            for (int v = 0; v < 4; ++v) acc[r][tt][v] = fmaf(s, c[v], acc[r][tt][v]);
                        }
                        ++pos[r];
                    }
                }
            }
        });
        clk.lap(kPhCompute);
        // look-ahead chunks for the next tile, all requested here, after the arithmetic (requested
        // earlier, inside the row loop, they measure slower)
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            if (cnts[r] > 0) {
                const bool okn = lane < end[r] - pos[r];
                kc[r] = okn ? lane_elem(colidx + pos[r], lane_b) : 0x7fffffff;          // uniform base + lane
                vc[r] = okn ? (vals ? lane_elem(vals + pos[r], lane_b) : 1.f) : 0.f;
            }
        }
        clk.lap(kPhReload);
    }
    clk.store(tim, WAVES, wave, lane);
    if (bad != 0 && lane == 0) flags[0] = 1;   // the general kernels behind this one redo the call
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int row = rows[r];
        if (row < M) {
            float *out = job_out(job, O, partial, M, ld, RB, wave * ROWS + r, row);
#pragma unroll
            for (int tt = 0; tt < T; ++tt)
                if (n + tt * 256 < N) store_vec<4>(out + n + tt * 256, acc[r][tt]);
        }
    }
}


// ---------------------------------------------------------------------------------------
// LDS-tiled SDDMM.  Lanes are ENTRIES here, not columns: a wavefront takes a chunk of 64
// stored entries of one row and lane j walks the dot length for its own entry, reading its
// row of B from the LDS tile 128 bits at a time.  No cross-lane reduction, results leave as
// one coalesced 256-byte store per chunk (Algorithm 1's loop nest with the two loops swapped
// between lanes and time).
//
// Sixty-four lanes that each read 16 bytes of a different, arbitrary row would collide in the
// LDS banks (rows start at the same bank), so every lane walks its row in a ROTATED order:
// at step s lane i (numbered inside its group of 16 lanes) reads the 16-byte piece number
// (i - s) mod 16 of its row.  The 16 lanes the LDS serves together then touch 16 different
// pieces, i.e. all banks once, whatever rows they are in; no padding is needed.  The row of
// A that multiplies these pieces is spread over the same 16 lanes, piece i in lane i, and
// the rotation `row_ror:s` of the DPP operand of the multiply-add hands lane i piece (i - s)
// at no extra instruction.  Nothing is carried from tile to tile except the per-row cursor
// and look-ahead chunk, found exactly as in ktile_kernel; the next tile of B is fetched into
// registers while the current one is worked on.  P may alias vals: each lane reads its value
// before writing its result.
// ---------------------------------------------------------------------------------------
template <int DMAX, int ROWS>
struct SddmmTileLds {
    static constexpr int kPieces = DMAX / 4;                    // 128-bit pieces per LDS row
    static constexpr int kKT = 147456 / (DMAX * 4);             // tile height: 144 KB of rows of B
    static constexpr int kTileFloats = kKT * DMAX;
    static constexpr int kAFloats = kTileWaves * ROWS * DMAX;   // the workgroup's rows of A, zero beyond D
    static constexpr int kBytes = (kTileFloats + kAFloats) * 4;
};

template <int DMAX, int ROWS>
__global__ __launch_bounds__(kTileThreads) void sddmm_ktile_kernel(
    int M, int K, int D, int ld, int accumulate, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *vals, const float *__restrict__ A, const float *__restrict__ Bmat, float *P, int32_t *flags,
    float inline_density, int32_t *other_flags) {
    // D: the piece of the dot product this launch computes, out of rows of A and B that are `ld` floats long (the
    // caller offsets A and B to the piece's first column); accumulate != 0: add to what P holds (a later piece)
    using L = SddmmTileLds<DMAX, ROWS>;
    constexpr int KT = L::kKT;
    constexpr int C = L::kPieces;
    constexpr int S = C < 16 ? C : 16;      // steps of the dot loop
    constexpr int H = C / S;                // 16-piece halves of a row (2 when DMAX = 128)
    constexpr int GL = 4;                   // LDS reads per group
    constexpr int NG = S * H / GL;
    static_assert(S * H % GL == 0, "whole groups of reads");
    extern __shared__ __attribute__((aligned(16))) float lds[];
    if (!tile_go(M, K, rowptr, inline_density, flags, other_flags, reinterpret_cast<int *>(lds))) return;
    const int lane = lane_id();
    const int wave = uniform(threadIdx.x >> 6);
    const int row0 = blockIdx.x * (kTileWaves * ROWS) + wave * ROWS;
    const int d4n = D >> 2;                 // float4s per row of A / B
    const int ld4 = ld >> 2;                // float4s from one row of A / B to the next
    float *arows = lds + L::kTileFloats + wave * (ROWS * DMAX);   // this wavefront's rows of A

    // row_ror:s hands lane i the value of lane (i - s) mod 16 (fixed by the instruction set; a GPU test checks
    // fma_row_rotated against a host loop), so at step s lane i holds piece (i - s) of A and reads that piece of B
    const int i16 = lane & 15;
    int off[S];                             // byte offset in an LDS row of the piece read at step s
#pragma unroll
    for (int s = 0; s < S; ++s) off[s] = ((i16 - s) & (S - 1)) * 16;

    // vals == NULL means all ones: the value loads then read colidx instead (any readable array of
    // the same length serves) and their results are not used
    const bool has_vals = vals != nullptr;
    const float *vsrc = has_vals ? vals : reinterpret_cast<const float *>(colidx);
    // Two look-ahead chunks per row: columns and values of the next 128 entries, requested at the end of a
    // tile for the next one.  A row's entries of a tile (115 on average at 20 % and D = 64) then need no load
    // inside the tile's arithmetic; only a row with more than 128 entries in one tile loads as it goes.
    int pos[ROWS], end[ROWS], kc[ROWS], kc2[ROWS];
    float vc[ROWS], vc2[ROWS];
    unsigned long long bad = 0;             // lanes that ever saw a descending pair of columns
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int row = row0 + r;
        pos[r] = row < M ? uniform(rowptr[row]) : 0;
        end[r] = row < M ? uniform(rowptr[row + 1]) : 0;
        const int j = pos[r] + lane;
        kc[r] = j < end[r] ? colidx[j] : 0x7fffffff;
        vc[r] = j < end[r] ? vsrc[j] : 1.f;
        kc2[r] = j + kWave < end[r] ? colidx[j + kWave] : 0x7fffffff;
        vc2[r] = j + kWave < end[r] ? vsrc[j + kWave] : 1.f;
        // the row of A into LDS, zero beyond D (piece `lane` of each row; read back per tile, 16 bytes per lane)
        if (lane < C) {
            float piece[4] = {0.f, 0.f, 0.f, 0.f};
            if (row < M && lane < d4n) load_vec<4>(A + (size_t)row * ld + lane * 4, piece);
            store_vec<4>(arows + r * DMAX + lane * 4, piece);
        }
    }

    // ---- staging of the tiles of B: global -> registers (`issue`), registers -> LDS (`commit`)
    constexpr int kRound = kTileThreads / C;            // tile rows covered by one round of loads
    constexpr int kPer = KT / kRound;
    static_assert(KT % kRound == 0, "tile height must be whole rounds of loads");
    float4 stage[kPer];
    const int my_kk = threadIdx.x / C, my_c = threadIdx.x % C;
    const bool my_col = my_c < d4n;
    // Every thread issues the same kPer loads for every tile, with no branch around them, so that
    // the compiler can count outstanding loads exactly and waits for a look-ahead chunk do not also
    // wait for the tile behind it.  Threads of the padding columns (D < DMAX) re-read the row's last
    // piece and write zeros; rows past K in the last tile re-read row K-1 and are never used.
    const size_t my_off = (size_t)my_kk * ld4 + (my_col ? my_c : d4n - 1);
    const size_t step_off = (size_t)kRound * ld4;
    // loads number [I0, I1) of this thread for the tile that starts at row k0
    auto issue = [&](int k0, auto i0c, auto i1c) {
        constexpr int I0 = decltype(i0c)::value, I1 = decltype(i1c)::value;
        const float4 *src = reinterpret_cast<const float4 *>(Bmat);
        if (k0 + KT <= K) {
            const float4 *tile = src + (size_t)k0 * ld4;   // uniform
#pragma unroll
            for (int i = I0; i < I1; ++i) stage[i] = tile[i * step_off + my_off];
        } else {                                           // last, partial tile: clamp the row
#pragma unroll
            for (int i = I0; i < I1; ++i) {
                const int k = k0 + i * kRound + my_kk;
                stage[i] = src[(size_t)(k < K ? k : K - 1) * ld4 + (my_col ? my_c : d4n - 1)];
            }
        }
    };
    auto commit = [&]() {
        float4 *dst = reinterpret_cast<float4 *>(lds);   // row kk, piece c sits at float4 number kk * C + c
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            float4 x = stage[i];
            if (!my_col) x = make_float4(0.f, 0.f, 0.f, 0.f);
            dst[i * kTileThreads + threadIdx.x] = x;
        }
    };

    issue(0, std::integral_constant<int, 0>{}, std::integral_constant<int, kPer>{});
    for (int k0 = 0; k0 < K; k0 += KT) {
        __syncthreads();                    // previous tile fully consumed
        commit();
        __syncthreads();
        // The next tile is requested while this one is worked on, a share of a thread's loads ahead of each of the
        // wavefront's rows rather than all of them behind the barrier: 16 wavefronts issuing 9 loads of 1 KB each at
        // the same moment fill the vector-memory queue (64 bytes a clock) and sit in their load instructions before
        // their first chunk; after the first row the wavefronts are no longer in step and the shares interleave.
        const bool more = k0 + KT < K;
        const int kend = k0 + KT;
        static_for<0, ROWS>([&](auto rc) {
            constexpr int r = decltype(rc)::value;
            if (more)
                issue(k0 + KT, std::integral_constant<int, r * kPer / ROWS>{}, std::integral_constant<int, (r + 1) * kPer / ROWS>{});
            float a[H][4];                  // this lane's pieces of the row of A
#pragma unroll
            for (int h = 0; h < H; ++h) load_vec<4>(arows + r * DMAX + (h * 16 + (i16 & (S - 1))) * 4, a[h]);
            // one chunk: lane j < cnt scores entry pos[r] + j, whose column is kcur and value vcur
            auto chunk = [&](int kcur, float vcur, int cnt) {
                const int j = pos[r] + lane;
                const bool in = lane < cnt;
                const char *brow = reinterpret_cast<const char *>(lds) + (unsigned)(in ? kcur - k0 : 0) * (DMAX * 4);
                // the row's S * H pieces in groups of GL reads, the next group requested before the
                // multiply-adds of the current one
                float dot = 0.f;
                float b[2][GL][4];
                auto read_group = [&](auto gc) {
                    constexpr int g = decltype(gc)::value;
                    static_for<0, GL>([&](auto uc) {
                        constexpr int q = g * GL + decltype(uc)::value;
                        load_vec<4>(reinterpret_cast<const float *>(brow + off[q / H] + (q % H) * 256),
                                    b[g & 1][decltype(uc)::value]);
                    });
                };
                read_group(std::integral_constant<int, 0>{});
                static_for<0, NG>([&](auto gc) {
                    constexpr int g = decltype(gc)::value;
                    if constexpr (g + 1 < NG) read_group(std::integral_constant<int, g + 1>{});
                    static_for<0, GL>([&](auto uc) {
                        constexpr int u = decltype(uc)::value;
                        constexpr int q = g * GL + u;
#pragma unroll
                        for (int c = 0; c < 4; ++c) fma_row_rotated<q / H>(dot, a[q % H][c], b[g & 1][u][c]);
                    });
                });
                if (in) {
                    const float scaled = (has_vals ? vcur : 1.f) * dot;
                    P[j] = accumulate ? P[j] + scaled : scaled;
                }
                pos[r] += cnt;
            };
            // the look-ahead registers hold what was loaded from clamped positions: mask the lanes past the row's end
            const int left = end[r] - pos[r];
            const int k1 = lane < left ? kc[r] : 0x7fffffff;
            const int k2 = lane + kWave < left ? kc2[r] : 0x7fffffff;
            const int cnt1 = __builtin_popcountll(__ballot(k1 < kend));
            bad |= descending_lanes(k1);        // checked where first used, not where requested
            if (cnt1 > 0) {
                chunk(k1, vc[r], cnt1);
                if (cnt1 == kWave) {
                    // the whole first chunk lay in the tile: on to the second, and check the pair that straddles the two
                    bad |= descending_lanes(k2);
                    if (__builtin_amdgcn_readlane(k1, kWave - 1) > __builtin_amdgcn_readlane(k2, 0)) bad |= 1;
                    int cnt = __builtin_popcountll(__ballot(k2 < kend));
                    if (cnt > 0) chunk(k2, vc2[r], cnt);
                    // rare: more than 128 entries of this row in the tile; go on chunk by chunk with blocking loads
                    int lastk = __builtin_amdgcn_readlane(k2, kWave - 1);
                    while (cnt == kWave && pos[r] < end[r]) {
                        const int jn = pos[r] + lane;
                        const int jl = jn < end[r] ? jn : end[r] - 1;
                        const int kl = colidx[jl];
                        const float vl = vsrc[jl];
                        const int k3 = jn < end[r] ? kl : 0x7fffffff;
                        bad |= descending_lanes(k3);
                        if (lastk > __builtin_amdgcn_readlane(k3, 0)) bad |= 1;
                        lastk = __builtin_amdgcn_readlane(k3, kWave - 1);
                        cnt = __builtin_popcountll(__ballot(k3 < kend));
                        if (cnt > 0) chunk(k3, vl, cnt);
                    }
                }
                // look-ahead chunks for the next tile (positions clamped into the row, which has entries here)
                const int j = pos[r] + lane;
                const int j1 = j < end[r] ? j : end[r] - 1;
                const int j2 = j + kWave < end[r] ? j + kWave : end[r] - 1;
                kc[r] = colidx[j1];
                vc[r] = vsrc[j1];
                kc2[r] = colidx[j2];
                vc2[r] = vsrc[j2];
            }
        });
    }
    if (bad != 0 && lane == 0) flags[0] = 1;   // the general kernel behind this one redoes the call
}

}  // namespace csrk
