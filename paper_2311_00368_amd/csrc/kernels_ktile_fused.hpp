// LDS-tiled FusedMM for wide outputs (128 < N <= 512 per launch, wider outputs in column slabs;
// D <= 64): O = (S .* (A B^T)) C with the scores kept on the CU (Algorithm 3's `arow`).
//
// The accumulate stage is the SPMM tile kernel's: a workgroup of 16 wavefronts owns 16*ROWS rows
// of S, sweeps K in tiles of KT columns of C staged in LDS, and every wavefront adds, for each of
// its rows, score * C[k, :] for the entries of the tile (lane l holds columns 4l..4l+3 of each
// 256-wide piece of the output; entries in batches of 4 fetched as (column, score) pairs by LDS
// broadcast reads).
//
// The score stage runs ONCE per tile for all rows of the wavefront, with lanes as ENTRIES: the
// 64 lanes are 4 groups of 16; a group belongs to one row (ROWS = 4: group g is row g; fewer rows:
// several groups per row) and its lane i scores the row's entry number base + i of the tile,
// walking the dot length in 16 pieces of 4 floats.  The tile's rows of B sit in LDS (64 floats
// each, zero beyond D); the row of A is spread over the group, piece i in lane i, and lane i walks
// its row of B in rotated order - piece (i - s) mod 16 at step s - taking the matching piece of A
// through the row_ror:s rotation of the multiply-add's DPP operand.  The 16 lanes the LDS serves
// together therefore read 16 different pieces (all banks once) whatever rows of B they are in, no
// cross-lane reduction is needed, and one chain of 16 reads scores up to 64 entries.  The finished
// score times the stored value overwrites the value half of the entry's pair in the wavefront's
// LDS slot, where the accumulate stage finds it.
#pragma once
#include "kernels_ktile.hpp"

namespace csrk {

// SL: entries per row that the wavefront's LDS slot holds (32 or 64); a row with more entries than that in
// one tile goes through the slot in parts.
template <int T, int KT, int ROWS, int SL>
struct FusedTileLds {
    static constexpr int kRowFloats = T * 256;
    static constexpr int kCFloats = KT * kRowFloats;            // tile of C
    static constexpr int kBFloats = KT * 64;                    // tile of B, rows zero-padded to 64 floats
    static constexpr int kEntFloats = kTileWaves * ROWS * SL * 2;      // one slot of SL (column, value) pairs per row
    static constexpr int kBytes = (kCFloats + kBFloats + kEntFloats) * 4;
};

// PF: how many of a thread's kPer loads of the next C tile are issued one tile ahead; the rest and the
// B tile are loaded at the start of their own tile (all of it ahead, B included, when PF == kPer).
// LIVE: rows a wavefront really owns.  LIVE = 3 with ROWS = 4 is the 48-rows-per-workgroup version (see
// tile_rows_for on the host): laid out for four rows, the fourth one of every wavefront empty.
// TIMED: the measuring build (see PhaseClock in kernels_ktile.hpp); `tim` receives kPhases counters per wavefront.
template <int T, int KT, int ROWS, int SL, int PF, int LIVE = ROWS, bool TIMED = false>
__global__ __launch_bounds__(kTileThreads) void fused_ktile_kernel(
    int M, int K, int D, int N, int ld, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ vals, const float *__restrict__ A, const float *__restrict__ Bmat,
    const float *__restrict__ Cmat, float *__restrict__ O, int32_t *flags, float *partial, float inline_density,
    int32_t *other_flags, long long *tim = nullptr, const int32_t *__restrict__ perm = nullptr,
    const int4 *__restrict__ items = nullptr) {
    using L = FusedTileLds<T, KT, ROWS, SL>;
    PhaseClock<TIMED> clk;
    static_assert(SL == 32 || SL == 64, "slot sizes");
    static_assert(ROWS == 1 || ROWS == 2 || ROWS == 4, "a row owns 4 / ROWS groups of 16 lanes");
    extern __shared__ __attribute__((aligned(16))) float lds[];
    if (!tile_go(M, K, rowptr, inline_density, flags, other_flags, reinterpret_cast<int *>(lds))) return;
    constexpr int kRowBytes = L::kRowFloats * 4;
    constexpr int kGroupsPerRow = 4 / ROWS;
    constexpr int kPass = 16 * kGroupsPerRow;      // entries of a row scored per pass
    constexpr int kExtra = 8;                      // entries beyond a pass that are scored one by one instead of by another pass
    const int lane = lane_id();
    const int wave = uniform(threadIdx.x >> 6);
    float *ct = lds;
    float *bt = lds + L::kCFloats;
    int2 *ent = reinterpret_cast<int2 *>(bt + L::kBFloats) + wave * (ROWS * SL);

    // (row_ror:s hands lane i the value of lane (i - s) mod 16 of its row of 16 lanes: fixed by the instruction set;
    // a GPU test checks fma_row_rotated against a host loop.)
    const int i16 = lane & 15;

    static_assert(LIVE >= 1 && LIVE <= ROWS, "rows owned within rows laid out");
    const TileJob job = tile_job(items);
    constexpr int RB = kTileWaves * LIVE;
    const int n = lane * 4;                 // this lane's first column inside each 256-wide piece of the output
    const unsigned lane_b = (unsigned)lane * 4u;    // ... and its byte offset in a lane-wide load of a chunk
    const int my_r = (lane >> 4) / kGroupsPerRow;       // the row this lane's group scores entries of
    const int my_first = ((lane >> 4) % kGroupsPerRow) * 16 + i16;   // ... and which entry of a pass

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
        const int row = r < LIVE ? job_row(job, perm, RB, wave * LIVE + r) : M;
        rows[r] = row;
        const bool live = row < M;
        pos[r] = live ? uniform(rowptr[row]) : 0;
        end[r] = live ? uniform(rowptr[row + 1]) : 0;
        if (job.nseg > 1) pos[r] = first_entry_at_or_after(colidx, pos[r], end[r], ks.kb);
        const bool ok = lane < end[r] - pos[r];
        kc[r] = ok ? lane_elem(colidx + pos[r], lane_b) : 0x7fffffff;
        vc[r] = ok ? (vals ? lane_elem(vals + pos[r], lane_b) : 1.f) : 0.f;
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[r][t][v] = 0.f;
    }
    float a[4] = {0.f, 0.f, 0.f, 0.f};      // piece i16 of this group's row of A, zero beyond D
    {
        int my_row = M;                     // the row of S this lane's group scores entries of
#pragma unroll
        for (int r = 0; r < ROWS; ++r) my_row = my_r == r ? rows[r] : my_row;
        if (my_row < M && i16 * 4 < D) load_vec<4>(A + (size_t)my_row * D + i16 * 4, a);
    }

    // ---- staging of the dense tiles: global -> registers (`issue`), registers -> LDS (`commit`)
    const int n4 = N >> 2;                  // float4s of a row of C that this launch works on ...
    const int ld4 = ld >> 2;                // ... out of this many (a launch may take a slab of the columns)
    constexpr int kRow4 = T * 64;
    constexpr int kPer = KT * kRow4 / kTileThreads;
    constexpr int kPerB = (KT * 16 + kTileThreads - 1) / kTileThreads;
    static_assert(PF >= -1 && PF <= kPer, "prefetch depth beyond the tile");
    f32x4 stage[kPer];
    f32x4 stageb[kPerB];
    constexpr int kStep = kTileThreads / kRow4;      // tile rows covered by one round of loads
    const int my_kk = threadIdx.x / kRow4, my_c4 = threadIdx.x % kRow4;
    // Every thread issues every load, under no condition: threads past the width of a narrower launch re-read the
    // row's last float4 (LDS columns only read by lanes whose accumulators are not stored), rows past K in the last
    // tile re-read row K-1 (no entry points at them).
    const int col4 = my_c4 < n4 ? my_c4 : n4 - 1;
    const unsigned my_off = ((unsigned)my_kk * (unsigned)ld4 + (unsigned)col4) * 16u;
    const unsigned step_bytes = (unsigned)kStep * (unsigned)ld4 * 16u;
    // the operands through buffer descriptors: scalar tile offset + one 32-bit offset per thread, rows past K read
    // as zeros (see DenseView)
    const DenseView cview = dense_view(Cmat, (unsigned)(((size_t)K * ld - (ld - N)) * 4));
    const DenseView bview = dense_view(Bmat, (unsigned)((size_t)K * D * 4));
    auto issue = [&](int k0, auto i0c, auto i1c) {
        constexpr int I0 = decltype(i0c)::value, I1 = decltype(i1c)::value;
        const unsigned tile = (unsigned)k0 * (unsigned)ld4 * 16u;      // uniform
#pragma unroll
        for (int i = I0; i < I1; ++i) stage[i] = load_f32x4(cview, my_off, tile + i * step_bytes);
    };
    // the tile of B: rows of D floats, zero-padded to 64 in LDS (the score stage walks all 16 pieces of a row)
    const int d4 = D >> 2;
    unsigned my_boff[kPerB];
    bool my_bpad[kPerB];
#pragma unroll
    for (int i = 0; i < kPerB; ++i) {
        const int e = i * kTileThreads + threadIdx.x;
        const int c4 = e & 15;
        my_bpad[i] = c4 >= d4;
        my_boff[i] = (unsigned)((e >> 4) * d4 + (c4 < d4 ? c4 : d4 - 1)) * 16u;
    }
    auto issue_b = [&](int k0) {
        const unsigned tile = (unsigned)k0 * (unsigned)d4 * 16u;       // uniform
#pragma unroll
        for (int i = 0; i < kPerB; ++i) {
            stageb[i] = load_f32x4(bview, my_boff[i], tile);
            if (my_bpad[i]) stageb[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };
    // registers -> LDS: loads number [I0, I1) of the C tile; the B tile
    auto commit_c = [&](auto i0c, auto i1c) {
        constexpr int I0 = decltype(i0c)::value, I1 = decltype(i1c)::value;
        f32x4 *dst = reinterpret_cast<f32x4 *>(ct);
#pragma unroll
        for (int i = I0; i < I1; ++i) dst[i * kTileThreads + threadIdx.x] = stage[i];
    };
    auto commit_b = [&]() {
        f32x4 *dstb = reinterpret_cast<f32x4 *>(bt);
#pragma unroll
        for (int i = 0; i < kPerB; ++i) {
            const int e = i * kTileThreads + threadIdx.x;
            if (e < KT * 16) dstb[e] = stageb[i];
        }
    };
    using I0 = std::integral_constant<int, 0>;
    // PF = -1: every load of the next tile goes out at the END of the current one, ahead of the barrier that ends it,
    // into registers the arithmetic has just let go of
    constexpr bool kTail = PF < 0;
    using IPF = std::integral_constant<int, (kTail ? 0 : PF)>;
    using IEND = std::integral_constant<int, kPer>;
    constexpr bool kAllAhead = PF == kPer;

    if (ks.kb < ks.ke) {
        if constexpr (kTail) {
            issue(ks.kb, I0{}, IEND{});
            issue_b(ks.kb);
        } else {
            if constexpr (PF > 0) issue(ks.kb, I0{}, IPF{});
            if constexpr (kAllAhead) issue_b(ks.kb);
        }
    }
    clk.start();
    for (int k0 = ks.kb; k0 < ks.ke; k0 += KT) {
        __syncthreads();                    // previous tile fully consumed
        clk.lap(kPhBarrier1);
        if constexpr (!kAllAhead && !kTail) {
            // What was prefetched goes to LDS first, so that those writes drain while the rest - what no register
            // could be spared for during the previous tile's arithmetic - is being requested (requests first: the
            // 16 wavefronts' loads fill the vector-memory queue for about 1000 cycles before a single LDS write is
            // issued; 1.96 -> 1.89 ms at 16384^2 / 20 %).  The fence keeps the compiler from moving the loads up.
            commit_c(I0{}, IPF{});
            __builtin_amdgcn_sched_barrier(0);
            issue(k0, IPF{}, IEND{});
            issue_b(k0);
            clk.lap(kPhIssue);
            commit_c(IPF{}, IEND{});
            commit_b();
        } else {
            commit_c(I0{}, IEND{});
            commit_b();
        }
        if constexpr (TIMED) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        clk.lap(kPhCommit);
        __syncthreads();
        clk.lap(kPhBarrier2);
        // (Issuing these loads later, from a different row's accumulate stage in each wavefront, as the SPMM kernel
        // does with its whole tile, measured level here: with 3 of 8 loads ahead the queue is not what is waited for.)
        if constexpr (PF > 0) {
            if (k0 + KT < ks.ke) {          // lands while this tile is being worked on
                issue(k0 + KT, I0{}, IPF{});
                if constexpr (kAllAhead) issue_b(k0 + KT);
            }
            clk.lap(kPhIssue);
        }
        const int kend = k0 + KT;
        // lane's byte offset in a tile row, minus the tile origin; unsigned so that the products with
        // large column numbers wrap instead of overflowing (the sum below is always a small offset)
        const unsigned lb = (unsigned)(n * 4) - (unsigned)k0 * (unsigned)kRowBytes;

        // entries of this tile = leading lanes of each row's chunk with column < kend.  A row whose whole chunk
        // lies in the tile gets its next chunk (a blocking load: dense rows only) and the tile goes round again
        // for those rows.
        bool fresh[ROWS];                   // this row's chunk has not been counted for this tile yet
        bool moved[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            fresh[r] = true;
            moved[r] = false;
        }
        for (;;) {
        int full[ROWS];                     // ... how many of the chunk's 64
        int most = 0;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            full[r] = fresh[r] ? __builtin_popcountll(__ballot(kc[r] < kend)) : 0;
            most = full[r] > most ? full[r] : most;
            // order check on the chunk, here where it is first used
            if (fresh[r]) bad |= descending_lanes(kc[r]);
        }
        if (most == 0) break;
        // the slots hold SL entries per row: lanes [part, part + SL) of the chunks at a time (one part unless a
        // row has more than SL entries in this tile)
        for (int part = 0; part < most; part += SL) {
        int cnts[ROWS];
        int maxcnt = 0, my_cnt = 0;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            int cnt = full[r] - part;
            cnt = cnt < 0 ? 0 : (cnt < SL ? cnt : SL);
            cnts[r] = cnt;
            maxcnt = cnt > maxcnt ? cnt : maxcnt;
            if (my_r == r) my_cnt = cnt;
            if (lane >= part && lane < part + SL)
                ent[r * SL + lane - part] = make_int2(kc[r], __builtin_bit_cast(int, vc[r]));
        }

        for (int base = 0; base < maxcnt;) {
            // ---- score stage: this lane's entry of this pass
            clk.lap(kPhCompute);
            {
                const int idx = base + my_first;
                const bool on = idx < my_cnt;
                int2 *mine = ent + my_r * SL + (on ? idx : 0);
                const int2 kv = *mine;
                // byte address of piece i16 of the entry's row of B; lanes without an entry walk row 0 of the tile
                const unsigned row_b = (unsigned)(L::kCFloats * 4) + (on ? (unsigned)(kv.x - k0) * 256u : 0u) + i16 * 16;
                const char *base_a = reinterpret_cast<const char *>(lds) + row_b;
                const char *base_b = base_a - 256;
                float dot = 0.f;
                constexpr int GL = 4, NG = 16 / GL;
                float b[2][GL][4];
                auto read_group = [&](auto gc) {
                    constexpr int g = decltype(gc)::value;
                    static_for<0, GL>([&](auto uc) {
                        constexpr int s = g * GL + decltype(uc)::value;
                        // piece (i16 - s) mod 16: 16 * (16 - s) bytes past base_b for lanes i16 >= s, past base_a otherwise
                        const char *p = s == 0 ? base_a : ((i16 >= s ? base_b : base_a) + 16 * (16 - s));
                        load_vec<4>(reinterpret_cast<const float *>(p), b[g & 1][decltype(uc)::value]);
                    });
                };
                read_group(std::integral_constant<int, 0>{});
                static_for<0, NG>([&](auto gc) {
                    constexpr int g = decltype(gc)::value;
                    if constexpr (g + 1 < NG) read_group(std::integral_constant<int, g + 1>{});
                    static_for<0, GL>([&](auto uc) {
                        constexpr int u = decltype(uc)::value;
#pragma unroll
                        for (int c = 0; c < 4; ++c) fma_row_rotated<g * GL + u>(dot, a[c], b[g & 1][u][c]);
                    });
                });
                if (on) reinterpret_cast<int *>(mine)[1] = __builtin_bit_cast(int, __builtin_bit_cast(float, kv.y) * dot);
            }
            // A pass scores kPass entries per row.  The few entries a row has beyond that (a row of a 20 % dense
            // matrix has 13 +- 3 entries in a 64-column tile, a pass takes 16) are not worth another pass - a chain
            // of 16 LDS reads and 64 multiply-adds for the whole wavefront, which also makes the wavefronts that need
            // one arrive late at the tile's barrier: up to kExtra of them per row are scored one at a time instead,
            // each by the 16 lanes of its row's group (lane i: piece i of the row of B times its piece of A, then a
            // sum over the group), the groups working side by side.
            int pass_end = base + kPass;
            if (maxcnt > pass_end && maxcnt <= pass_end + kExtra) {
                for (int idx = pass_end; idx < maxcnt; ++idx) {
                    const bool on = idx < my_cnt;
                    int2 *mine = ent + my_r * SL + (on ? idx : 0);
                    const int2 kv = *mine;
                    float bq[4];
                    load_vec<4>(bt + (on ? kv.x - k0 : 0) * 64 + i16 * 4, bq);
                    float part = a[0] * bq[0];
#pragma unroll
                    for (int v = 1; v < 4; ++v) part = fmaf(a[v], bq[v], part);
                    part = group_sum<16>(part);
                    if (on && my_first == 0) reinterpret_cast<int *>(mine)[1] = __builtin_bit_cast(int, __builtin_bit_cast(float, kv.y) * part);
                }
                pass_end = maxcnt;
            }
            if constexpr (TIMED) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            clk.lap(kPhScore);
            // ---- accumulate stage: entries [base, pass_end) of every row
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const int2 *e = ent + r * SL;
                const int lim = cnts[r] < pass_end ? cnts[r] : pass_end;
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
                int t = base;
                for (; t + 4 <= lim; t += 4) batch(t, std::integral_constant<int, 4>{});
                // the last 1-3 entries as a pair and a single: two plain ifs keep the accumulators in place, where a
                // switch over the three cases made the compiler copy them in and out
                if (lim - t >= 2) {
                    batch(t, std::integral_constant<int, 2>{});
                    t += 2;
                }
                if (lim - t >= 1) batch(t, std::integral_constant<int, 1>{});
            }
            base = pass_end;
        }

        }   // part

        if constexpr (KT <= kWave) {
            // A tile of at most 64 columns holds more than a chunk of one row only if columns repeat, and a full
            // chunk only for a dense row: the simple continuation, one entry at a time, is enough (and keeps the
            // 512-wide kernel free of the bookkeeping of the rounds, which costs it 2 %).
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                pos[r] += full[r];
                moved[r] = full[r] > 0;
                if (full[r] == kWave) {
                    int lastk = __builtin_amdgcn_readlane(kc[r], kWave - 1);
                    while (pos[r] < end[r]) {
                        const int k = uniform(colidx[pos[r]]);
                        if (k < lastk) bad |= 1;     // descending across the chunk boundary or inside this run
                        lastk = k;
                        if (k >= kend) break;
                        float s = vals ? __builtin_bit_cast(float, uniform(__builtin_bit_cast(int, vals[pos[r]]))) : 1.f;
                        float bq[4];
                        load_vec<4>(bt + (k - k0) * 64 + i16 * 4, bq);
                        float part = a[0] * bq[0];
#pragma unroll
                        for (int v = 1; v < 4; ++v) part = fmaf(a[v], bq[v], part);
                        part = group_sum<16>(part);           // the 16 lanes of the row's first group hold its row of A
                        s *= readlane_f(part, r * kGroupsPerRow * 16);
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
            break;
        } else {
            bool again = false;
    #pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                pos[r] += full[r];
                moved[r] |= full[r] > 0;
                fresh[r] = false;
                if (full[r] == kWave) {
                    const int lastk = __builtin_amdgcn_readlane(kc[r], kWave - 1);
                    const bool okn = lane < end[r] - pos[r];
                    kc[r] = okn ? lane_elem(colidx + pos[r], lane_b) : 0x7fffffff;
                    vc[r] = okn ? (vals ? lane_elem(vals + pos[r], lane_b) : 1.f) : 0.f;
                    if (__builtin_amdgcn_readlane(kc[r], 0) < lastk) bad |= 1;   // descending across the chunk boundary
                    fresh[r] = true;
                    moved[r] = false;           // its look-ahead chunk is already the right one
                    again = true;
                }
            }
            if (__builtin_expect(!again, 1)) break;
        }
        }   // rounds of this tile
        clk.lap(kPhCompute);
        // look-ahead chunks for the next tile, all requested here, after the arithmetic
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            if (moved[r]) {
                const bool okn = lane < end[r] - pos[r];
                kc[r] = okn ? lane_elem(colidx + pos[r], lane_b) : 0x7fffffff;          // uniform base + lane
                vc[r] = okn ? (vals ? lane_elem(vals + pos[r], lane_b) : 1.f) : 0.f;
            }
        }
        clk.lap(kPhReload);
        if constexpr (kTail) {
            if (k0 + KT < ks.ke) {
                issue(k0 + KT, I0{}, IEND{});
                issue_b(k0 + KT);
            }
            clk.lap(kPhIssue);
        }
    }
    clk.store(tim, kTileWaves, wave, lane);
    if (bad != 0 && lane == 0) flags[0] = 1;   // the general kernels behind this one redo the call
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int row = rows[r];
        if (row < M) {
            float *out = job_out(job, O, partial, M, ld, RB, wave * LIVE + r, row);   // K cut: a partial row, added up later
#pragma unroll
            for (int tt = 0; tt < T; ++tt)
                if (n + tt * 256 < N) store_vec<4>(out + n + tt * 256, acc[r][tt]);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// FusedMM for narrow outputs (N <= 128, D <= 128): the paper's own shapes.  Score stage exactly as above (lanes
// as entries, a group of 16 lanes per row, rotated walk of the rows of B, which may now be 128 floats = two
// halves of 16 pieces); accumulate stage as in ktile_narrow_kernel: the wavefront is cut into G groups of 64/G
// lanes, a group covers the 256/G-column row of C with one 128-bit read per lane, the G groups work on G
// different entries at once and their G partial rows are added at the very end.
// ---------------------------------------------------------------------------------------------------------
template <int G, int KT, int ROWS, int SL, int DMAX>
struct FusedNarrowLds {
    static constexpr int kRowFloats = 256 / G;
    static constexpr int kCFloats = KT * kRowFloats;            // tile of C
    static constexpr int kBFloats = KT * DMAX;                  // tile of B, rows zero-padded to DMAX floats
    static constexpr int kEntFloats = kTileWaves * ROWS * SL * 2;
    static constexpr int kBytes = (kCFloats + kBFloats + kEntFloats) * 4;
};

template <int G, int KT, int ROWS, int SL, int DMAX, int PF, int LIVE = ROWS>
__global__ __launch_bounds__(kTileThreads) void fused_narrow_kernel(
    int M, int K, int D, int N, int ld, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ vals, const float *__restrict__ A, const float *__restrict__ Bmat,
    const float *__restrict__ Cmat, float *__restrict__ O, int32_t *flags, float *partial, float inline_density,
    int32_t *other_flags, const int32_t *__restrict__ perm = nullptr, const int4 *__restrict__ items = nullptr) {
    using L = FusedNarrowLds<G, KT, ROWS, SL, DMAX>;
    static_assert(SL == 32 || SL == 64, "slot sizes");
    static_assert(ROWS == 1 || ROWS == 2 || ROWS == 4, "a row owns 4 / ROWS groups of 16 lanes");
    static_assert(DMAX == 64 || DMAX == 128, "dot lengths the score stage is laid out for");
    extern __shared__ __attribute__((aligned(16))) float lds[];
    if (!tile_go(M, K, rowptr, inline_density, flags, other_flags, reinterpret_cast<int *>(lds))) return;
    constexpr int LN = kWave / G;           // lanes per entry in the accumulate stage
    constexpr int H = DMAX / 64;            // 16-piece halves of a row of B
    constexpr int kRowBytes = L::kRowFloats * 4;
    constexpr int kBRowBytes = DMAX * 4;
    constexpr int kGroupsPerRow = 4 / ROWS;
    constexpr int kPass = 16 * kGroupsPerRow;      // entries of a row scored per pass
    // Entries are parked in the order the accumulate stage fetches them back: a round is 4 G entries, group g takes
    // entries t+g, t+G+g, t+2G+g, t+3G+g of it, and those four pairs sit next to each other (32 bytes), so a lane
    // gets them with two 128-bit reads instead of four 64-bit ones (the pair reads were half of the accumulate
    // stage's LDS instructions, and LDS issue is what bounds it).  Needs passes of whole rounds.
    constexpr bool kPermuted = kPass % (4 * G) == 0;
    auto parked = [](int q) { return kPermuted ? (q / (4 * G)) * (4 * G) + (q % G) * 4 + (q / G) % 4 : q; };
    const int lane = lane_id();
    const int wave = uniform(threadIdx.x >> 6);
    float *ct = lds;
    float *bt = lds + L::kCFloats;
    int2 *ent = reinterpret_cast<int2 *>(bt + L::kBFloats) + wave * (ROWS * SL);

    // see fused_ktile_kernel: row_ror:s hands lane i the value of lane (i - s) mod 16
    const int i16 = lane & 15;

    static_assert(LIVE >= 1 && LIVE <= ROWS, "rows owned within rows laid out");
    const TileJob job = tile_job(items);
    constexpr int RB = kTileWaves * LIVE;
    const int g = lane / LN;                // accumulate stage: which of the G side-by-side entries
    const int n = (lane % LN) * 4;          // accumulate stage: this lane's first column
    const int my_r = (lane >> 4) / kGroupsPerRow;       // score stage: the row this lane's group scores entries of
    const int my_first = ((lane >> 4) % kGroupsPerRow) * 16 + i16;   // ... and which entry of a pass

    const KSplit ks = job_range<KT>(job, K);    // the whole of K unless the job is one range of several
    if (!job.sched && job.nseg > 1 && ksplit_block_unsorted<RB>(M, rowptr, colidx)) {
        if (lane == 0) flags[0] = 1;        // the reduction stands down, the general kernels redo the call
    }
    int rows[ROWS];
    int pos[ROWS], end[ROWS];
    int kc[ROWS];
    float vc[ROWS];
    float acc[ROWS][4];
    unsigned long long bad = 0;             // lanes that ever saw a descending pair of columns
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int row = r < LIVE ? job_row(job, perm, RB, wave * LIVE + r) : M;
        rows[r] = row;
        const bool live = row < M;
        pos[r] = live ? uniform(rowptr[row]) : 0;
        end[r] = live ? uniform(rowptr[row + 1]) : 0;
        if (job.nseg > 1) pos[r] = first_entry_at_or_after(colidx, pos[r], end[r], ks.kb);
        const int j = pos[r] + lane;
        const bool ok = j < end[r];
        kc[r] = ok ? colidx[j] : 0x7fffffff;
        vc[r] = ok ? (vals ? vals[j] : 1.f) : 0.f;
        acc[r][0] = acc[r][1] = acc[r][2] = acc[r][3] = 0.f;
    }
    float a[H][4];                          // pieces i16 (and 16 + i16) of this group's row of A, zero beyond D
    int my_row = M;                         // the row of S this lane's group scores entries of
#pragma unroll
    for (int r = 0; r < ROWS; ++r) my_row = my_r == r ? rows[r] : my_row;
#pragma unroll
    for (int h = 0; h < H; ++h) {
        a[h][0] = a[h][1] = a[h][2] = a[h][3] = 0.f;
        if (my_row < M && (h * 16 + i16) * 4 < D) load_vec<4>(A + (size_t)my_row * D + (h * 16 + i16) * 4, a[h]);
    }

    // ---- staging of the dense tiles: global -> registers (`issue`), registers -> LDS (`commit`)
    const int n4 = N >> 2;                  // float4s of a row of C that this launch works on ...
    const int ld4 = ld >> 2;                // ... out of this many (a launch may take a slab of the columns)
    constexpr int kRow4 = 64 / G;
    constexpr int kStep = kTileThreads / kRow4;      // tile rows covered by one round of loads
    constexpr int kPer = KT / kStep;
    static_assert(KT % kStep == 0, "tile height must be a whole number of load rounds");
    constexpr int kD4 = DMAX / 4;
    constexpr int kPerB = (KT * kD4 + kTileThreads - 1) / kTileThreads;
    static_assert(PF >= 0 && PF <= kPer, "prefetch depth beyond the tile");
    float4 stage[kPer];
    float4 stageb[kPerB];
    const int my_kk = threadIdx.x / kRow4, my_c4 = threadIdx.x % kRow4;
    const bool my_col = my_c4 < n4;
    const size_t my_off = (size_t)my_kk * ld4 + my_c4;
    const size_t step_off = (size_t)kStep * ld4;
    auto issue = [&](int k0, auto i0c, auto i1c) {
        constexpr int I0 = decltype(i0c)::value, I1 = decltype(i1c)::value;
        const float4 *tile = reinterpret_cast<const float4 *>(Cmat) + (size_t)k0 * ld4;   // uniform
        if (k0 + KT <= K) {
#pragma unroll
            for (int i = I0; i < I1; ++i) stage[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (my_col) {
#pragma unroll
                for (int i = I0; i < I1; ++i) stage[i] = tile[i * step_off + my_off];
            }
        } else {                                      // last, partial tile
#pragma unroll
            for (int i = I0; i < I1; ++i) {
                stage[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (my_col && k0 + i * kStep + my_kk < K) stage[i] = tile[i * step_off + my_off];
            }
        }
    };
    auto issue_b = [&](int k0) {
        const float4 *srcb = reinterpret_cast<const float4 *>(Bmat);
        const int d4 = D >> 2;
#pragma unroll
        for (int i = 0; i < kPerB; ++i) {
            const int e = i * kTileThreads + threadIdx.x;
            const int kk = e / kD4, c4 = e % kD4;
            stageb[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (e < KT * kD4 && k0 + kk < K && c4 < d4) stageb[i] = srcb[(size_t)(k0 + kk) * d4 + c4];
        }
    };
    // registers -> LDS: loads number [I0, I1) of the C tile; the B tile
    auto commit_c = [&](auto i0c, auto i1c) {
        constexpr int I0 = decltype(i0c)::value, I1 = decltype(i1c)::value;
        float4 *dst = reinterpret_cast<float4 *>(ct);
#pragma unroll
        for (int i = I0; i < I1; ++i) dst[i * kTileThreads + threadIdx.x] = stage[i];
    };
    auto commit_b = [&]() {
        float4 *dstb = reinterpret_cast<float4 *>(bt);
#pragma unroll
        for (int i = 0; i < kPerB; ++i) {
            const int e = i * kTileThreads + threadIdx.x;
            if (e < KT * kD4) dstb[e] = stageb[i];
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using IPF = std::integral_constant<int, PF>;
    using IEND = std::integral_constant<int, kPer>;
    constexpr bool kAllAhead = PF == kPer;

    if constexpr (PF > 0) issue(ks.kb, I0{}, IPF{});
    if constexpr (kAllAhead) issue_b(ks.kb);
    for (int k0 = ks.kb; k0 < ks.ke; k0 += KT) {
        __syncthreads();                    // previous tile fully consumed
        if constexpr (!kAllAhead) {
            // what was prefetched goes to LDS before the rest is requested (see fused_ktile_kernel)
            commit_c(I0{}, IPF{});
            __builtin_amdgcn_sched_barrier(0);
            issue(k0, IPF{}, IEND{});
            issue_b(k0);
            commit_c(IPF{}, IEND{});
            commit_b();
        } else {
            commit_c(I0{}, IEND{});
            commit_b();
        }
        __syncthreads();
        if constexpr (PF > 0) {
            if (k0 + KT < ks.ke) {              // lands while this tile is being worked on
                issue(k0 + KT, I0{}, IPF{});
                if constexpr (kAllAhead) issue_b(k0 + KT);
            }
        }
        const int kend = k0 + KT;
        const unsigned lb = (unsigned)(n * 4) - (unsigned)k0 * (unsigned)kRowBytes;

        // entries of this tile = leading lanes of each row's chunk with column < kend.  A row whose whole chunk
        // lies in the tile gets its next chunk (a blocking load: dense rows only) and the tile goes round again
        // for those rows.
        bool fresh[ROWS];                   // this row's chunk has not been counted for this tile yet
        bool moved[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            fresh[r] = true;
            moved[r] = false;
        }
        for (;;) {
        int full[ROWS];                     // ... how many of the chunk's 64
        int most = 0;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            full[r] = fresh[r] ? __builtin_popcountll(__ballot(kc[r] < kend)) : 0;
            most = full[r] > most ? full[r] : most;
            if (fresh[r]) bad |= descending_lanes(kc[r]);
        }
        if (most == 0) break;
        // the slots hold SL entries per row: lanes [part, part + SL) of the chunks at a time
        for (int part = 0; part < most; part += SL) {
            int cnts[ROWS];
            int maxcnt = 0, my_cnt = 0;
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                int cnt = full[r] - part;
                cnt = cnt < 0 ? 0 : (cnt < SL ? cnt : SL);
                cnts[r] = cnt;
                maxcnt = cnt > maxcnt ? cnt : maxcnt;
                if (my_r == r) my_cnt = cnt;
                if (lane >= part && lane < part + SL)
                    ent[r * SL + parked(lane - part)] = make_int2(kc[r], __builtin_bit_cast(int, vc[r]));
            }
            for (int base = 0; base < maxcnt; base += kPass) {
                // ---- score stage: this lane's entry of this pass
                {
                    const int idx = base + my_first;
                    const bool on = idx < my_cnt;
                    int2 *mine = ent + my_r * SL + parked(on ? idx : 0);
                    const int2 kv = *mine;
                    // byte address of piece i16 of the entry's row of B; lanes without an entry walk row 0 of the tile
                    const unsigned row_b = (unsigned)(L::kCFloats * 4) + (on ? (unsigned)(kv.x - k0) * (unsigned)kBRowBytes : 0u) + i16 * 16;
                    const char *base_a = reinterpret_cast<const char *>(lds) + row_b;
                    const char *base_b = base_a - 256;
                    float dot = 0.f;
                    constexpr int GL = 4, NR = 16 * H, NG = NR / GL;     // reads: step s, half h -> number s * H + h
                    float b[2][GL][4];
                    auto read_group = [&](auto gc) {
                        constexpr int gi = decltype(gc)::value;
                        static_for<0, GL>([&](auto uc) {
                            constexpr int q = gi * GL + decltype(uc)::value;
                            constexpr int st = q / H, hh = q % H;
                            // piece (i16 - st) mod 16 of half hh
                            const char *p = (st == 0 ? base_a : ((i16 >= st ? base_b : base_a) + 16 * (16 - st))) + hh * 256;
                            load_vec<4>(reinterpret_cast<const float *>(p), b[gi & 1][decltype(uc)::value]);
                        });
                    };
                    read_group(std::integral_constant<int, 0>{});
                    static_for<0, NG>([&](auto gc) {
                        constexpr int gi = decltype(gc)::value;
                        if constexpr (gi + 1 < NG) read_group(std::integral_constant<int, gi + 1>{});
                        static_for<0, GL>([&](auto uc) {
                            constexpr int u = decltype(uc)::value;
                            constexpr int q = gi * GL + u;
#pragma unroll
                            for (int c = 0; c < 4; ++c) fma_row_rotated<q / H>(dot, a[q % H][c], b[gi & 1][u][c]);
                        });
                    });
                    if (on) reinterpret_cast<int *>(mine)[1] = __builtin_bit_cast(int, __builtin_bit_cast(float, kv.y) * dot);
                }
                // ---- accumulate stage: entries [base, base + kPass) of every row; group g takes entries
                // t+g, t+G+g, t+2G+g, t+3G+g of each round
#pragma unroll
                for (int r = 0; r < ROWS; ++r) {
                    const int2 *e = ent + r * SL;
                    const int lim = cnts[r] < base + kPass ? cnts[r] : base + kPass;
                    int t = base;
                    auto fetch = [&](int2 (&ks4)[4]) {
                        if constexpr (kPermuted) {
                            const int4 lo = *reinterpret_cast<const int4 *>(e + t + 4 * g);
                            const int4 hi = *reinterpret_cast<const int4 *>(e + t + 4 * g + 2);
                            ks4[0] = make_int2(lo.x, lo.y);
                            ks4[1] = make_int2(lo.z, lo.w);
                            ks4[2] = make_int2(hi.x, hi.y);
                            ks4[3] = make_int2(hi.z, hi.w);
                        } else {
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                const int idx = t + u * G + g;
                                ks4[u] = e[idx < lim ? idx : base];
                            }
                        }
                    };
                    for (; t + 4 * G <= lim; t += 4 * G) {
                        int2 ks4[4];
                        float c[4][4];
                        fetch(ks4);
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            load_vec<4>(reinterpret_cast<const float *>(reinterpret_cast<const char *>(ct) +
                                                                        ((unsigned)ks4[u].x * (unsigned)kRowBytes + lb)),
                                        c[u]);
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const float sv = __builtin_bit_cast(float, ks4[u].y);
#pragma unroll
                            for (int v = 0; v < 4; ++v) acc[r][v] = fmaf(sv, c[u][v], acc[r][v]);
                        }
                    }
                    if (t < lim) {                  // last, partial round: lanes whose entry does not exist sit out
                        int2 ks4[4];
                        float c[4][4];
                        fetch(ks4);
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            // an entry that does not exist: read the tile's first row (what its pair holds is anything)
                            const int col = t + u * G + g < lim ? ks4[u].x : k0;
                            load_vec<4>(reinterpret_cast<const float *>(reinterpret_cast<const char *>(ct) +
                                                                        ((unsigned)col * (unsigned)kRowBytes + lb)),
                                        c[u]);
                        }
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            if (t + u * G + g < lim) {
                                const float sv = __builtin_bit_cast(float, ks4[u].y);
#pragma unroll
                                for (int v = 0; v < 4; ++v) acc[r][v] = fmaf(sv, c[u][v], acc[r][v]);
                            }
                        }
                    }
                }
            }
        }   // part

        bool again = false;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            pos[r] += full[r];
            moved[r] |= full[r] > 0;
            fresh[r] = false;
            if (full[r] == kWave) {
                const int lastk = __builtin_amdgcn_readlane(kc[r], kWave - 1);
                const bool okn = lane < end[r] - pos[r];
                kc[r] = okn ? (colidx + pos[r])[lane] : 0x7fffffff;
                vc[r] = okn ? (vals ? (vals + pos[r])[lane] : 1.f) : 0.f;
                if (__builtin_amdgcn_readlane(kc[r], 0) < lastk) bad |= 1;   // descending across the chunk boundary
                fresh[r] = true;
                moved[r] = false;           // its look-ahead chunk is already the right one
                again = true;
            }
        }
        if (__builtin_expect(!again, 1)) break;
        }   // rounds of this tile
        // look-ahead chunks for the next tile, all requested here, after the arithmetic
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            if (moved[r]) {
                const bool okn = lane < end[r] - pos[r];
                kc[r] = okn ? (colidx + pos[r])[lane] : 0x7fffffff;          // uniform base + lane
                vc[r] = okn ? (vals ? (vals + pos[r])[lane] : 1.f) : 0.f;
            }
        }
    }
    if (bad != 0 && lane == 0) flags[0] = 1;   // the general kernels behind this one redo the call
    // add the G partial rows of every row and store
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
#pragma unroll
        for (int off = LN; off < kWave; off <<= 1)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[r][v] += __shfl_xor(acc[r][v], off);
        const int row = rows[r];
        if (row < M && g == 0 && n < N)         // K cut: a partial row, added up later
            store_vec<4>(job_out(job, O, partial, M, ld, RB, wave * LIVE + r, row) + n, acc[r]);
    }
}

}  // namespace csrk
