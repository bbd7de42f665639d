// LDS-tiled SPMM for narrow outputs (N <= 128): the paper's own widths, 32 and 128.  (FusedMM for these
// widths: fused_narrow_kernel in kernels_ktile_fused.hpp, which has the same accumulate stage.)
//
// Same scheme as ktile_kernel (a workgroup of 16 wavefronts owns 16*ROWS rows of S, sweeps K in
// tiles staged in LDS, finds each row's entries of a tile as a prefix of a 64-entry look-ahead
// chunk, fetches (column, scale) pairs back by LDS broadcast), with the lanes laid out for a
// narrow dense row: the wavefront is cut into G groups of 64/G lanes, a group covers the
// 256/G-column row with one 128-bit read per lane, and the G groups work on G different
// entries at once.  Each group accumulates its own partial row; the G partial rows are added
// once, at the very end.  One workgroup per CU (the kernel needs more than 64 registers per lane), so the
// next tile is requested into registers while the current one is worked on (PF of a thread's loads, the
// rest at the start of the tile), and SPMM's tiles are as high as LDS allows (256 rows at 128 columns, 384
// at 64 and 32): more entries per row and tile to spread the per-tile work over.
//
// Two look-ahead chunks per row (128 entries) are kept in registers.  A segment longer than that (dense or
// very long rows) continues chunk by chunk with blocking loads; that path is correct for any length but
// only the first 128 entries of a segment run at full speed.
#pragma once
#include <type_traits>

#include "device_util.hpp"
#include "kernels_ktile.hpp"

namespace csrk {

template <int G, int KT>
struct NarrowLds {
    static constexpr int kRowFloats = 256 / G;
    static constexpr int kCFloats = KT * kRowFloats;
    static constexpr int kEntFloats = kTileWaves * 2 * kWave * 2;     // two 64-entry slots of pairs per wavefront
    static constexpr int kBytes = (kCFloats + kEntFloats) * 4;
};

template <int G, int KT, int ROWS, int PF>
__global__ __launch_bounds__(kTileThreads) void ktile_narrow_kernel(
    int M, int K, int N, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ vals, const float *__restrict__ Cmat, float *__restrict__ O, int32_t *flags,
    float *partial, float inline_density, int32_t *other_flags, const int32_t *__restrict__ perm = nullptr,
    const int4 *__restrict__ items = nullptr) {
    using L = NarrowLds<G, KT>;
    constexpr int LN = kWave / G;           // lanes per entry
    constexpr int kRowBytes = L::kRowFloats * 4;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    if (!tile_go(M, K, rowptr, inline_density, flags, other_flags, reinterpret_cast<int *>(lds))) return;
    const int lane = lane_id();
    const int wave = uniform(threadIdx.x >> 6);
    float *ct = lds;
    int2 *ent = reinterpret_cast<int2 *>(lds + L::kCFloats) + wave * (2 * kWave);

    const TileJob job = tile_job(items);
    constexpr int RB = kTileWaves * ROWS;
    const int g = lane / LN;                // which of the G side-by-side entries
    const int n = (lane % LN) * 4;          // this lane's first column

    const KSplit ks = job_range<KT>(job, K);    // the whole of K unless the job is one range of several
    if (!job.sched && job.nseg > 1 && ksplit_block_unsorted<RB>(M, rowptr, colidx)) {
        if (lane == 0) flags[0] = 1;        // the reduction stands down, the general kernels redo the call
    }
    int rows[ROWS];
    int pos[ROWS], end[ROWS];
    int kc[ROWS], kc2[ROWS];                // look-ahead: columns of the next 64 entries and of the 64 after them
    float vc[ROWS], vc2[ROWS];              // ... and their values
    float acc[ROWS][4];
    unsigned long long bad = 0;
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int row = job_row(job, perm, RB, wave * ROWS + r);
        rows[r] = row;
        pos[r] = row < M ? uniform(rowptr[row]) : 0;
        end[r] = row < M ? uniform(rowptr[row + 1]) : 0;
        if (job.nseg > 1) pos[r] = first_entry_at_or_after(colidx, pos[r], end[r], ks.kb);
        const int j = pos[r] + lane;
        const bool ok = j < end[r];
        kc[r] = ok ? colidx[j] : 0x7fffffff;
        vc[r] = ok ? (vals ? vals[j] : 1.f) : 0.f;
        const bool ok2 = j + kWave < end[r];
        kc2[r] = ok2 ? colidx[j + kWave] : 0x7fffffff;
        vc2[r] = ok2 ? (vals ? vals[j + kWave] : 1.f) : 0.f;
        acc[r][0] = acc[r][1] = acc[r][2] = acc[r][3] = 0.f;
    }
    const int n4 = N >> 2;
    constexpr int kRow4 = 64 / G;                       // float4s per tile row
    constexpr int kStep = kTileThreads / kRow4;         // tile rows per round of loads
    constexpr int kPer = KT / kStep;
    static_assert(KT % kStep == 0, "tile height must be a whole number of load rounds");
    const int my_kk = threadIdx.x / kRow4, my_c4 = threadIdx.x % kRow4;
    const bool my_col = my_c4 < n4;
    const size_t my_off = (size_t)my_kk * n4 + my_c4;
    const size_t step_off = (size_t)kStep * n4;

    static_assert(PF >= 0 && PF <= kPer, "prefetch depth beyond the tile");
    float4 stage[kPer];
    // loads number [I0, I1) of this thread for the C tile that starts at column k0
    auto issue = [&](int k0, auto i0c, auto i1c) {
        constexpr int I0 = decltype(i0c)::value, I1 = decltype(i1c)::value;
        const float4 *tile = reinterpret_cast<const float4 *>(Cmat) + (size_t)k0 * n4;   // uniform
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
    auto commit = [&]() {
        float4 *dst = reinterpret_cast<float4 *>(ct);
#pragma unroll
        for (int i = 0; i < kPer; ++i) dst[i * kTileThreads + threadIdx.x] = stage[i];
    };
    using I0 = std::integral_constant<int, 0>;
    using IPF = std::integral_constant<int, PF>;
    using IEND = std::integral_constant<int, kPer>;

    if constexpr (PF > 0) issue(ks.kb, I0{}, IPF{});
    for (int k0 = ks.kb; k0 < ks.ke; k0 += KT) {
        __syncthreads();                    // previous tile fully consumed
        if constexpr (PF < kPer) issue(k0, IPF{}, IEND{});
        commit();
        __syncthreads();
        if constexpr (PF > 0) {
            if (k0 + KT < ks.ke) issue(k0 + KT, I0{}, IPF{});   // lands while this tile is being worked on
        }
        const int kend = k0 + KT;
        const unsigned lb = (unsigned)(n * 4) - (unsigned)k0 * (unsigned)kRowBytes;
        bool moved[ROWS];

        // one chunk's worth of a row: `cnt` leading entries of (kreg, vreg) belong to this tile
        auto process = [&](int r, int slot, int kreg, float vreg, int cnt) {
            int2 *e = ent + slot * kWave;
            // Entries are parked in the order they are fetched back: a round is 4 G entries, group g takes entries
            // t+g, t+G+g, t+2G+g, t+3G+g of it, and those four pairs sit next to each other (32 bytes), so a lane
            // gets them with two 128-bit reads instead of four 64-bit ones (the pair reads were half of the
            // kernel's LDS instructions, and LDS issue is what bounds it).
            e[(lane / (4 * G)) * (4 * G) + (lane % G) * 4 + (lane / G) % 4] = make_int2(kreg, __builtin_bit_cast(int, vreg));
            int t = 0;
            auto fetch = [&](int2 (&ks)[4]) {
                const int4 lo = *reinterpret_cast<const int4 *>(e + t + 4 * g);
                const int4 hi = *reinterpret_cast<const int4 *>(e + t + 4 * g + 2);
                ks[0] = make_int2(lo.x, lo.y);
                ks[1] = make_int2(lo.z, lo.w);
                ks[2] = make_int2(hi.x, hi.y);
                ks[3] = make_int2(hi.z, hi.w);
            };
            for (; t + 4 * G <= cnt; t += 4 * G) {
                int2 ks[4];
                float c[4][4];
                fetch(ks);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    load_vec<4>(reinterpret_cast<const float *>(reinterpret_cast<const char *>(ct) +
                                                                ((unsigned)ks[u].x * (unsigned)kRowBytes + lb)),
                                c[u]);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float sv = __builtin_bit_cast(float, ks[u].y);
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[r][v] = fmaf(sv, c[u][v], acc[r][v]);
                }
            }
            if (t < cnt) {                  // last, partial round: lanes whose entry does not exist read the tile's
                int2 ks[4];                 // first row (their pair holds a column beyond the tile) and sit out
                float c[4][4];
                fetch(ks);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int col = t + u * G + g < cnt ? ks[u].x : k0;
                    load_vec<4>(reinterpret_cast<const float *>(reinterpret_cast<const char *>(ct) +
                                                                ((unsigned)col * (unsigned)kRowBytes + lb)),
                                c[u]);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (t + u * G + g < cnt) {
                        const float sv = __builtin_bit_cast(float, ks[u].y);
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[r][v] = fmaf(sv, c[u][v], acc[r][v]);
                    }
                }
            }
        };

#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const int cnt = __builtin_popcountll(__ballot(kc[r] < kend));
            bad |= descending_lanes(kc[r]);
            moved[r] = cnt > 0;
            if (cnt > 0) {
                process(r, 0, kc[r], vc[r], cnt);
                pos[r] += cnt;
                if (cnt == kWave) {
                    // the whole first chunk lay in the tile: on to the second one
                    bad |= descending_lanes(kc2[r]);
                    if (__builtin_amdgcn_readlane(kc2[r], 0) < __builtin_amdgcn_readlane(kc[r], kWave - 1)) bad |= 1;
                    const int cntb = __builtin_popcountll(__ballot(kc2[r] < kend));
                    if (cntb > 0) {
                        process(r, 1, kc2[r], vc2[r], cntb);
                        pos[r] += cntb;
                    }
                    if (cntb == kWave) {
                        // rare: more than 128 entries of the row in this tile: chunk by chunk with blocking loads
                        int lastk = __builtin_amdgcn_readlane(kc2[r], kWave - 1);
                        while (pos[r] < end[r]) {
                            const bool ok3 = lane < end[r] - pos[r];
                            const int k3 = ok3 ? (colidx + pos[r])[lane] : 0x7fffffff;
                            const float v3 = ok3 ? (vals ? (vals + pos[r])[lane] : 1.f) : 0.f;
                            bad |= descending_lanes(k3);
                            if (__builtin_amdgcn_readlane(k3, 0) < lastk) bad |= 1;
                            const int cnt3 = __builtin_popcountll(__ballot(k3 < kend));
                            if (cnt3 == 0) break;
                            process(r, 0, k3, v3, cnt3);
                            pos[r] += cnt3;
                            if (cnt3 < kWave) break;
                            lastk = __builtin_amdgcn_readlane(k3, kWave - 1);
                        }
                    }
                }
            }
        }
        // look-ahead chunks for the next tile
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            if (moved[r]) {
                const int left = end[r] - pos[r];
                const bool okn = lane < left, okn2 = lane + kWave < left;
                kc[r] = okn ? (colidx + pos[r])[lane] : 0x7fffffff;
                vc[r] = okn ? (vals ? (vals + pos[r])[lane] : 1.f) : 0.f;
                kc2[r] = okn2 ? (colidx + pos[r] + kWave)[lane] : 0x7fffffff;
                vc2[r] = okn2 ? (vals ? (vals + pos[r] + kWave)[lane] : 1.f) : 0.f;
            }
        }
    }
    // add the G partial rows of every row and store
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
#pragma unroll
        for (int off = LN; off < kWave; off <<= 1)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[r][v] += __shfl_xor(acc[r][v], off);
        const int row = rows[r];
        if (row < M && g == 0 && n < N)         // K cut: a partial row, added up later
            store_vec<4>(job_out(job, O, partial, M, N, RB, wave * ROWS + r, row) + n, acc[r]);
    }
    if (bad != 0 && lane == 0) flags[0] = 1;
}

}  // namespace csrk
