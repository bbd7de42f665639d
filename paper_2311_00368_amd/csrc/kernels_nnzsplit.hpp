// Row-segment kernels that gather dense rows straight from memory (the general path): every kernel here
// works on segments of rows - a run of stored entries of one row - and differs only in who gets which segment.
//
// Two ways of dealing out the work:
//
//  (1) Equal shares of the stored entries (`*_nnzsplit_kernel`).  Each wavefront ("worker") takes an equal
//      share of S's stored entries, whatever the row lengths are, finds the row its share starts in by a
//      wave-wide search of rowptr and walks the rows it touches.  This is the load balancing for skewed row
//      lengths: a row longer than a share is cut into segments handled by consecutive workers.
//       - SPMM / FusedMM: a worker writes the rows that START inside its share straight to O (if such a row
//         continues into later shares this is its first partial sum), and puts the partial sum of the row
//         that was already running when its share began (its "head") into a scratch row;
//         `combine_heads_kernel` then adds the heads to O in worker order, so the result does not depend on
//         timing.
//       - SDDMM: outputs are per stored entry, segments are disjoint, no combine.
//
//  (2) Whole rows (`*_rows_kernel`, and a branch of the kernels of (1) taken when the row analysis found the
//      rows about equally long): the paper's own decomposition, a row per work-item, with 2 or 4 wavefronts
//      of a workgroup sharing a row where there are few rows (its NT, section "SDDMM").  No search, no heads,
//      no combine step; faster wherever there is nothing to balance.
//
// Inside a segment the column indices and values are streamed in coalesced chunks of 64 (one per lane), the
// next chunk being loaded while the current one is consumed.  A group of LG lanes covers the dense width with
// VEC floats per lane, so 64/LG entries are processed side by side; their dense rows are gathered with one
// (128-bit when VEC == 4) load per lane, several steps' gathers in flight together (gather_axpy).
//
// Paper correspondence: the chunked index stream with look-ahead is the role of the VLC-sized blocks and
// prefetches in the paper's kernels (section "ESIMD Implementation"); the per-row arithmetic is
// Algorithms 1-3.
#pragma once
#include "device_util.hpp"
#include "kernels_ktile.hpp"

namespace csrk {

constexpr int kBlockThreads = 256;
constexpr int kWavesPerBlock = kBlockThreads / kWave;

// f(t) for t = t0, t0+stride, ... < t1, in blocks of U statically unrolled calls and a
// one-at-a-time remainder.
template <int U, typename F>
__device__ __forceinline__ void for_unrolled(int t0, int t1, int stride, F &&f) {
    int t = t0;
    for (; t + U * stride <= t1; t += U * stride) {
#pragma unroll
        for (int u = 0; u < U; ++u) f(t + u * stride);
    }
    for (; t < t1; t += stride) f(t);
}

// ---------------------------------------------------------------------------------
// Gather-and-accumulate over the entries [t0, t1) of one chunk (entry t: column in lane t
// of `kc`, scale in lane t of `sc`):
//     acc[tt][v] += sc_t * Mat[kc_t, n + tt*TW + v]
// A group of LG lanes covers the dense width, NPAR = 64/LG entries go side by side.
//
// The gathers of a block of U steps are all requested before the first is used.  That
// only happens if no load sits under a condition (the compiler waits for such a load on
// the spot, which would put the U gathers one after the other): every lane loads in every
// step, with columns beyond N moved to column 0 and steps beyond the chunk's end moved
// to entry t0, and the condition is applied to the multiply-adds instead.
// ---------------------------------------------------------------------------------
template <int VEC, int LG, int T, typename E>
__device__ __forceinline__ void gather_axpy(int kc, float sc, int t0, int t1, const E *__restrict__ Mat, int N,
                                            int n, float (&acc)[T][VEC]) {
    constexpr int NPAR = kWave / LG;
    constexpr int TW = LG * VEC;
    constexpr int U = NPAR == 1 ? 8 : 4;         // steps per full block
    constexpr int UR = NPAR == 1 ? 4 : 2;        // steps per block of the remainder
    const int g = lane_id() / LG;
    int off[T];
    bool col_ok[T];
#pragma unroll
    for (int tt = 0; tt < T; ++tt) {
        col_ok[tt] = n + tt * TW < N;
        off[tt] = col_ok[tt] ? n + tt * TW : 0;
    }
    auto block = [&](int t, auto uc) {
        constexpr int UU = decltype(uc)::value;
        float s[UU];
        bool on[UU];
        float b[UU][T][VEC];
#pragma unroll
        for (int u = 0; u < UU; ++u) {
            const int idx = t + u * NPAR + g;
            on[u] = idx >= t0 && idx < t1;
            const int src = on[u] ? idx : t0;
            int k;
            if constexpr (NPAR == 1) {
                const int su = uniform(src);
                k = __builtin_amdgcn_readlane(kc, su);
                s[u] = readlane_f(sc, su);
            } else {
                k = __shfl(kc, src);
                s[u] = __shfl(sc, src);
            }
            const E *row = Mat + (size_t)k * N;
#pragma unroll
            for (int tt = 0; tt < T; ++tt) load_vec<VEC>(row + off[tt], b[u][tt]);
        }
#pragma unroll
        for (int u = 0; u < UU; ++u)
#pragma unroll
            for (int tt = 0; tt < T; ++tt)
                if (on[u] && col_ok[tt]) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[tt][v] = fmaf(s[u], b[u][tt][v], acc[tt][v]);
                }
    };
    int t = t0 - (t0 % NPAR);
    for (; t + U * NPAR <= t1; t += U * NPAR) block(t, std::integral_constant<int, U>{});
    for (; t < t1; t += UR * NPAR) block(t, std::integral_constant<int, UR>{});
}

// ---------------------------------------------------------------------------------
// SPMM segment: acc[t][v] += sum_{j in [s0,s1)} vals[j] * Bmat[colidx[j], n + t*TW + v]
// ---------------------------------------------------------------------------------
template <int VEC, int LG, int T, typename E>
__device__ __forceinline__ void spmm_segment(int s0, int s1, const int32_t *__restrict__ colidx,
                                             const float *__restrict__ vals,
                                             const E *__restrict__ Bmat, int N, int n,
                                             float (&acc)[T][VEC]) {
    const int lane = lane_id();
    if (s1 <= s0) return;
    int base = s0 & ~(kWave - 1);
    int j = base + lane;
    bool ok = j >= s0 && j < s1;
    int kc = ok ? colidx[j] : 0;
    float vc = ok ? (vals ? vals[j] : 1.f) : 0.f;
    for (; base < s1; base += kWave) {
        // look-ahead: next chunk of the index/value stream
        const int jn = base + kWave + lane;
        const bool okn = jn < s1;
        const int kn = okn ? colidx[jn] : 0;
        const float vn = okn ? (vals ? vals[jn] : 1.f) : 0.f;
        const int t0 = s0 > base ? s0 - base : 0;
        const int t1 = (s1 - base) < kWave ? (s1 - base) : kWave;
        gather_axpy<VEC, LG, T>(kc, vc, t0, t1, Bmat, N, n, acc);
        kc = kn;
        vc = vn;
    }
}

// Sum the NPAR side-by-side partial rows of a wave into lanes [0, LG).
template <int VEC, int LG, int T>
__device__ __forceinline__ void fold_groups(float (&acc)[T][VEC]) {
#pragma unroll
    for (int off = LG; off < kWave; off <<= 1)
#pragma unroll
        for (int tt = 0; tt < T; ++tt)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[tt][v] += __shfl_xor(acc[tt][v], off);
}

template <int VEC, int LG, int T>
__device__ __forceinline__ void store_row(float *dst, int N, int n, const float (&acc)[T][VEC]) {
    constexpr int TW = LG * VEC;
    if (lane_id() < LG) {
#pragma unroll
        for (int tt = 0; tt < T; ++tt)
            if (n + tt * TW < N) store_vec<VEC>(dst + n + tt * TW, acc[tt]);
    }
}

// A row per wavefront - or per 2 or 4 wavefronts of a workgroup (`wpr`), which then take consecutive parts of
// the row and whose partial rows the first of them adds in order through LDS: the paper's own decomposition (a row
// per work-item, NT work-items per row for short matrices; Algorithms 1-3 and section "SDDMM").  No shares, no
// search, no heads and so no combine step: a call is one launch whose wavefronts go through three or four
// dependent memory round trips.  For sparse matrices so small that this chain, not throughput, is the whole
// cost; no balancing of long rows (the host picks it only where a row can hold few chunks).
template <int VEC, int LG, int T>
struct RowParts {
    static constexpr int kWidth = LG * VEC * T;      // columns one workgroup covers
    float part[kWavesPerBlock][kWidth];
};

// this wavefront's part [s0, s1) of the row [rs, re)
__device__ __forceinline__ void row_part(int rs, int re, int sub, int wpr, int &s0, int &s1) {
    const long long len = re - rs;
    s0 = rs + (int)(len * sub / wpr);
    s1 = rs + (int)(len * (sub + 1) / wpr);
}

// acc of the `wpr` wavefronts of a row -> O[r, :], added in the order of the parts (wpr > 1 only; all wavefronts
// of the workgroup come through here together)
template <int VEC, int LG, int T>
__device__ __forceinline__ void add_row_parts(RowParts<VEC, LG, T> &lds, int wv, int sub, int wpr, bool valid,
                                              float *orow, int N, int n, float (&acc)[T][VEC]) {
    constexpr int TW = LG * VEC;
    const int lane = lane_id();
    const int nl = (lane % LG) * VEC;
    if (sub != 0 && lane < LG) {
#pragma unroll
        for (int tt = 0; tt < T; ++tt) store_vec<VEC>(&lds.part[wv][tt * TW + nl], acc[tt]);
    }
    __syncthreads();
    if (sub == 0 && valid) {
        if (lane < LG) {
            for (int p = 1; p < wpr; ++p)
#pragma unroll
                for (int tt = 0; tt < T; ++tt) {
                    float q[VEC];
                    load_vec<VEC>(&lds.part[wv + p][tt * TW + nl], q);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[tt][v] += q[v];
                }
        }
        store_row<VEC, LG, T>(orow, N, n, acc);
    }
    __syncthreads();
}

// instantiations of the general SPMM kernel whose whole-row branch shares rows between wavefronts whatever M is
template <int VEC, int LG, int T>
constexpr bool kSpmmRowsAnyM = VEC >= 4 && T == 1;

// wavefronts per row when the kernel decides for itself (the whole-row branch of the general SPMM and SDDMM
// kernels): W is the number of wavefronts in the grid
__device__ __forceinline__ int rows_wpr_for(int M, int W) { return 2ll * M > W ? 1 : (4ll * M > W ? 2 : 4); }

template <int VEC, int LG, int T, typename E>
__device__ __forceinline__ void spmm_rows_body(int M, int N, const int32_t *__restrict__ rowptr,
                                               const int32_t *__restrict__ colidx, const float *__restrict__ vals,
                                               const E *__restrict__ Bmat, float *__restrict__ O, int wpr,
                                               RowParts<VEC, LG, T> &lds) {
    constexpr int TW = LG * VEC;
    const int lane = lane_id();
    const int wv = uniform(threadIdx.x >> 6);
    const int sub = wv % wpr, rows_per_block = kWavesPerBlock / wpr;
    const int n = blockIdx.y * (TW * T) + (lane % LG) * VEC;
    for (long long r0 = (long long)blockIdx.x * rows_per_block; r0 < M; r0 += (long long)gridDim.x * rows_per_block) {
        const long long r = r0 + wv / wpr;
        const bool valid = r < M;
        const int rs = valid ? uniform(rowptr[r]) : 0;
        const int re = valid ? uniform(rowptr[r + 1]) : 0;
        int s0, s1;
        row_part(rs, re, sub, wpr, s0, s1);
        float acc[T][VEC] = {};
        spmm_segment<VEC, LG, T>(s0, s1, colidx, vals, Bmat, N, n, acc);
        fold_groups<VEC, LG, T>(acc);
        if (wpr == 1) {
            if (valid) store_row<VEC, LG, T>(O + (size_t)r * N, N, n, acc);
        } else {
            add_row_parts<VEC, LG, T>(lds, wv, sub, wpr, valid, O + (size_t)(valid ? r : 0) * N, N, n, acc);
        }
    }
}

template <int VEC, int LG, int T, typename E = float>
__global__ __launch_bounds__(kBlockThreads) void spmm_rows_kernel(
    int M, int N, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ vals, const E *__restrict__ Bmat, float *__restrict__ O, int wpr) {
    __shared__ RowParts<VEC, LG, T> lds;
    spmm_rows_body<VEC, LG, T>(M, N, rowptr, colidx, vals, Bmat, O, wpr, lds);
}

template <int VEC, int LG, int T, typename E = float>
__global__ __launch_bounds__(kBlockThreads) void spmm_nnzsplit_kernel(
    int M, int N, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ vals, const E *__restrict__ Bmat, float *__restrict__ O,
    float *__restrict__ head, int32_t *__restrict__ head_row, const int32_t *__restrict__ gate,
    const int32_t *__restrict__ even) {
    constexpr int TW = LG * VEC;
    if (gate && ktile_ok(gate)) return;     // the LDS-tiled kernel has done this call
    const int lane = lane_id();
    const int W = gridDim.x * kWavesPerBlock;
    const int w = uniform(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    const int n = blockIdx.y * (TW * T) + (lane % LG) * VEC;
    if (even && *even != 0) {
        // The row analysis found no row much longer than the mean: nothing to balance, so whole rows are dealt out
        // (1, 2 or 4 wavefronts per row, whatever keeps the wavefronts of the grid busy) - no search for a share's
        // first row, no heads (combine_heads_kernel stands down on the same flag).  Measured 10-60 % faster than
        // the equal-nonzero split on such matrices.
        // (Sharing rows between wavefronts only where it costs no occupancy: not in the 512-wide instantiation,
        // 91 -> 99 VGPRs; that one takes whole rows with more than half as many rows as wavefronts.)
        if constexpr (kSpmmRowsAnyM<VEC, LG, T>) {
            __shared__ RowParts<VEC, LG, T> lds;
            spmm_rows_body<VEC, LG, T>(M, N, rowptr, colidx, vals, Bmat, O, rows_wpr_for(M, W), lds);
            return;
        } else if (2ll * M > W) {
            for (int r = w; r < M; r += W) {
                const int rs = uniform(rowptr[r]);
                const int re = uniform(rowptr[r + 1]);
                float acc[T][VEC] = {};
                spmm_segment<VEC, LG, T>(rs, re, colidx, vals, Bmat, N, n, acc);
                fold_groups<VEC, LG, T>(acc);
                store_row<VEC, LG, T>(O + (size_t)r * N, N, n, acc);
            }
            return;
        }
    }
    const Share sh = make_share(rowptr, M, w, W);
    if (!sh.active) {
        if (blockIdx.y == 0 && lane == 0) head_row[w] = -1;
        return;
    }
    int r = wave_lower_bound(rowptr, M, sh.lo);
    int hr = -1;
    if (sh.lo < sh.nnz) {
        const int start = uniform(rowptr[r]);      // r <= M and rowptr[M] = nnz
        if (start != sh.lo) {                      // share begins inside row r-1
            hr = r - 1;
            float acc[T][VEC] = {};
            spmm_segment<VEC, LG, T>(sh.lo, start < sh.hi ? start : sh.hi, colidx, vals, Bmat, N, n, acc);
            fold_groups<VEC, LG, T>(acc);
            store_row<VEC, LG, T>(head + (size_t)w * N, N, n, acc);
        }
    }
    if (blockIdx.y == 0 && lane == 0) head_row[w] = hr;
    for (; r < M; ++r) {
        const int rs = uniform(rowptr[r]);
        if (!sh.last && rs >= sh.hi) break;
        const int re = uniform(rowptr[r + 1]);
        float acc[T][VEC] = {};
        spmm_segment<VEC, LG, T>(rs, re < sh.hi ? re : sh.hi, colidx, vals, Bmat, N, n, acc);
        fold_groups<VEC, LG, T>(acc);
        store_row<VEC, LG, T>(O + (size_t)r * N, N, n, acc);
    }
}

// O[r, :] += head[w, :] + head[w+1, :] + ... for the run of workers whose head is row r.
// One wavefront per worker, lanes over the output columns; only the first worker of a run does the
// adding, in worker order, so sums are reproducible.  `vec4`: N is a multiple of 4 and O and head
// are 16-byte aligned.
// This is the last kernel of every SPMM / FusedMM call.  If a tiled kernel did the call there are no heads;
// if that kernel's launch was K-split (S > 1) its S partial outputs (`partial`, count4 float4s each) still
// have to be added into O, which this grid then does instead.
__global__ __launch_bounds__(kBlockThreads) void combine_heads_kernel(int M, int N, int W, float *__restrict__ O,
                                                                       const float *__restrict__ head,
                                                                       const int32_t *__restrict__ head_row,
                                                                       const int32_t *__restrict__ gate, int vec4,
                                                                       size_t count4, int S, const float4 *partial,
                                                                       const int32_t *__restrict__ even, int any_m) {
    if (gate && ktile_ok(gate)) {
        if (S > 1) ksplit_reduce(count4, S, partial, reinterpret_cast<float4 *>(O));
        return;
    }
    // the general kernel dealt out whole rows (SPMM: whenever the rows are even; FusedMM: with enough rows too)
    if (even && *even != 0 && (any_m || 2ll * M > W)) return;
    const int w = uniform(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    if (w >= W) return;
    const int r = uniform(head_row[w]);
    if (r < 0) return;
    if (w > 0 && uniform(head_row[w - 1]) == r) return;
    int wend = w + 1;
    while (wend < W && uniform(head_row[wend]) == r) ++wend;
    const int lane = lane_id();
    float *orow = O + (size_t)r * N;
    if (vec4) {
        for (int n = lane * 4; n < N; n += kWave * 4) {
            float s[4];
            load_vec<4>(orow + n, s);
            for (int ww = w; ww < wend; ++ww) {
                float h[4];
                load_vec<4>(head + (size_t)ww * N + n, h);
#pragma unroll
                for (int v = 0; v < 4; ++v) s[v] += h[v];
            }
            store_vec<4>(orow + n, s);
        }
    } else {
        for (int n = lane; n < N; n += kWave) {
            float s = orow[n];
            for (int ww = w; ww < wend; ++ww) s += head[(size_t)ww * N + n];
            orow[n] = s;
        }
    }
}

// ---------------------------------------------------------------------------------
// SDDMM chunk: dot products of one row of A with the gathered rows of Bmat for the
// entries of one chunk; results land in `slot[0..64)` (LDS, one slot array per wave)
// ---------------------------------------------------------------------------------
// T > 0: the A row sits in registers (`a`, T tiles of LG*VEC columns).  T == 0: any D,
// tiles are walked at run time and the A row is re-read from memory (it stays in L1).
template <int VEC, int LG, int T, typename E>
__device__ __forceinline__ void sddmm_chunk(int kc, int t0, int t1, const E *__restrict__ Bmat, int D,
                                            int d, const E *__restrict__ arow,
                                            const float (&a)[T > 0 ? T : 1][VEC], float *slot) {
    constexpr int NPAR = kWave / LG;
    constexpr int TW = LG * VEC;
    const int lane = lane_id();
    const int g = lane / LG;
    if constexpr (T > 0) {
        // Blocks of U steps whose gathers are all requested before the first dot product starts; loads in every
        // lane and step, conditions on the arithmetic only (see gather_axpy).
        constexpr int U = 4, UR = 2;
        int off[T];
        bool col_ok[T];
#pragma unroll
        for (int tt = 0; tt < T; ++tt) {
            col_ok[tt] = d + tt * TW < D;
            off[tt] = col_ok[tt] ? d + tt * TW : 0;
        }
        auto block = [&](int t, auto uc) {
            constexpr int UU = decltype(uc)::value;
            float b[UU][T][VEC];
#pragma unroll
            for (int u = 0; u < UU; ++u) {
                const int idx = t + u * NPAR + g;
                const int src = (idx >= t0 && idx < t1) ? idx : t0;
                const int k = (NPAR == 1) ? __builtin_amdgcn_readlane(kc, uniform(src)) : __shfl(kc, src);
                const E *brow = Bmat + (size_t)k * D;
#pragma unroll
                for (int tt = 0; tt < T; ++tt) load_vec<VEC>(brow + off[tt], b[u][tt]);
            }
#pragma unroll
            for (int u = 0; u < UU; ++u) {
                const int idx = t + u * NPAR + g;
                float part = 0.f;
#pragma unroll
                for (int tt = 0; tt < T; ++tt)
                    if (col_ok[tt]) {
#pragma unroll
                        for (int v = 0; v < VEC; ++v) part = fmaf(a[tt][v], b[u][tt][v], part);
                    }
                part = group_sum<LG>(part);
                if (idx >= t0 && idx < t1 && (lane % LG) == 0) slot[idx] = part;
            }
        };
        int t = t0 - (t0 % NPAR);
        for (; t + U * NPAR <= t1; t += U * NPAR) block(t, std::integral_constant<int, U>{});
        for (; t < t1; t += UR * NPAR) block(t, std::integral_constant<int, UR>{});
    } else {
        for_unrolled<4>(t0 - (t0 % NPAR), t1, NPAR, [&](int t) {
            const int idx = t + g;
            const int k = (NPAR == 1) ? __builtin_amdgcn_readlane(kc, t) : __shfl(kc, idx);
            const bool act = idx >= t0 && idx < t1;
            float part = 0.f;
            if (act) {
                const E *brow = Bmat + (size_t)k * D + d;
                for (int dd = 0; d + dd < D; dd += TW) {
                    float b[VEC], av[VEC];
                    load_vec<VEC>(brow + dd, b);
                    load_vec<VEC>(arow + d + dd, av);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) part = fmaf(av[v], b[v], part);
                }
            }
            part = group_sum<LG>(part);
            if (act && (lane % LG) == 0) slot[idx] = part;
        });
    }
}

template <int VEC, int LG, int T, typename E>
__device__ __forceinline__ void load_a_row(const E *__restrict__ arow, int D, int d,
                                           float (&a)[T > 0 ? T : 1][VEC]) {
    constexpr int TW = LG * VEC;
    if constexpr (T > 0) {
#pragma unroll
        for (int tt = 0; tt < T; ++tt) {
            if (d + tt * TW < D) {
                load_vec<VEC>(arow + d + tt * TW, a[tt]);
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) a[tt][v] = 0.f;
            }
        }
    } else {
#pragma unroll
        for (int v = 0; v < VEC; ++v) a[0][v] = 0.f;
    }
}

// P[j] = vals[j] * <A[r, :], Bmat[colidx[j], :]> for the stored entries [s0, s1) of row r (Algorithm 1's inner
// loops), a chunk of 64 entries at a time.  P may alias vals.
template <int VEC, int LG, int T, typename E>
__device__ __forceinline__ void sddmm_segment(int r, int s0, int s1, const int32_t *__restrict__ colidx,
                                              const float *vals, const E *__restrict__ A,
                                              const E *__restrict__ Bmat, float *P, int D, int d, float *slot) {
    if (s1 <= s0) return;
    const int lane = lane_id();
    const E *arow = A + (size_t)r * D;
    float a[T > 0 ? T : 1][VEC];
    load_a_row<VEC, LG, T>(arow, D, d, a);
    for (int base = s0 & ~(kWave - 1); base < s1; base += kWave) {
        const int j = base + lane;
        const bool ok = j >= s0 && j < s1;
        const int kc = ok ? colidx[j] : 0;
        const float vc = (ok && vals) ? vals[j] : 1.f;
        const int t0 = s0 > base ? s0 - base : 0;
        const int t1 = (s1 - base) < kWave ? (s1 - base) : kWave;
        sddmm_chunk<VEC, LG, T>(kc, t0, t1, Bmat, D, d, arow, a, slot);
        __builtin_amdgcn_wave_barrier();
        if (ok) P[j] = vc * slot[lane];
        __builtin_amdgcn_wave_barrier();
    }
}

// SDDMM with a row per 1, 2 or 4 wavefronts (consecutive parts of the row; outputs are per stored entry, so
// nothing to add up): see spmm_rows_kernel.
template <int VEC, int LG, int T, typename E>
__device__ __forceinline__ void sddmm_rows_body(int M, int D, const int32_t *__restrict__ rowptr,
                                                const int32_t *__restrict__ colidx, const float *vals,
                                                const E *__restrict__ A, const E *__restrict__ Bmat, float *P,
                                                int wpr, float *slot) {
    const int lane = lane_id();
    const int wv = uniform(threadIdx.x >> 6);
    const int sub = wv % wpr, rows_per_block = kWavesPerBlock / wpr;
    const int d = (lane % LG) * VEC;
    for (long long r = (long long)blockIdx.x * rows_per_block + wv / wpr; r < M; r += (long long)gridDim.x * rows_per_block) {
        const int rs = uniform(rowptr[r]);
        const int re = uniform(rowptr[r + 1]);
        int s0, s1;
        row_part(rs, re, sub, wpr, s0, s1);
        sddmm_segment<VEC, LG, T>((int)r, s0, s1, colidx, vals, A, Bmat, P, D, d, slot);
    }
}

template <int VEC, int LG, int T, typename E = float>
__global__ __launch_bounds__(kBlockThreads) void sddmm_rows_kernel(
    int M, int D, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx, const float *vals,
    const E *__restrict__ A, const E *__restrict__ Bmat, float *P, int wpr) {
    __shared__ float slots[kWavesPerBlock][kWave];
    sddmm_rows_body<VEC, LG, T>(M, D, rowptr, colidx, vals, A, Bmat, P, wpr, slots[threadIdx.x >> 6]);
}

// P may alias vals, so neither is __restrict__.
template <int VEC, int LG, int T, typename E = float>
__global__ __launch_bounds__(kBlockThreads) void sddmm_nnzsplit_kernel(
    int M, int D, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *vals, const E *__restrict__ A, const E *__restrict__ Bmat, float *P,
    const int32_t *__restrict__ gate, const int32_t *__restrict__ even) {
    __shared__ float slots[kWavesPerBlock][kWave];
    if (gate && ktile_ok(gate)) return;     // the LDS-tiled kernel has done this call
    const int lane = lane_id();
    const int W = gridDim.x * kWavesPerBlock;
    const int wv = threadIdx.x >> 6;
    const int w = uniform(blockIdx.x * kWavesPerBlock + wv);
    const int d = (lane % LG) * VEC;
    if (even && *even != 0) {               // whole rows: see spmm_nnzsplit_kernel
        sddmm_rows_body<VEC, LG, T>(M, D, rowptr, colidx, vals, A, Bmat, P, rows_wpr_for(M, W), slots[wv]);
        return;
    }
    const Share sh = make_share(rowptr, M, w, W);
    if (!sh.active || sh.lo >= sh.nnz) return;
    float *slot = slots[wv];
    // row containing entry lo: the last row that starts at or before lo
    int r = wave_lower_bound(rowptr, M, sh.lo);
    if (uniform(rowptr[r]) != sh.lo) --r;
    for (; r < M; ++r) {
        const int rs = uniform(rowptr[r]);
        if (rs >= sh.hi) break;
        const int re = uniform(rowptr[r + 1]);
        const int s0 = rs > sh.lo ? rs : sh.lo;
        const int s1 = re < sh.hi ? re : sh.hi;
        if (s1 <= s0) continue;
        sddmm_segment<VEC, LG, T>(r, s0, s1, colidx, vals, A, Bmat, P, D, d, slot);
    }
}

// ---------------------------------------------------------------------------------
// FusedMM: per chunk, the SDDMM stage leaves the 64 scores in LDS slots, each lane
// picks up "its" score (scaled by vals) into a register, and the SPMM stage consumes
// them from there; scores never reach device memory (Algorithm 3's `arow`).
// Dot stage uses (VD, LD, TD) over D, the accumulate stage (VN, LN, TN) over N.
// ---------------------------------------------------------------------------------
template <int VD, int LD, int TD, int VN, int LN, int TN, typename E>
__device__ __forceinline__ void fused_segment(int row, int s0, int s1, const int32_t *__restrict__ colidx,
                                              const float *__restrict__ vals, const E *__restrict__ A,
                                              const E *__restrict__ Bmat, const E *__restrict__ Cmat,
                                              int D, int N, int d, int n, float *slot, float (&acc)[TN][VN]) {
    if (s1 <= s0) return;
    const int lane = lane_id();
    const E *arow = A + (size_t)row * D;
    float a[TD > 0 ? TD : 1][VD];
    load_a_row<VD, LD, TD>(arow, D, d, a);
    for (int base = s0 & ~(kWave - 1); base < s1; base += kWave) {
        const int j = base + lane;
        const bool ok = j >= s0 && j < s1;
        const int kc = ok ? colidx[j] : 0;
        const float vc = (ok && vals) ? vals[j] : 1.f;
        const int t0 = s0 > base ? s0 - base : 0;
        const int t1 = (s1 - base) < kWave ? (s1 - base) : kWave;
        sddmm_chunk<VD, LD, TD>(kc, t0, t1, Bmat, D, d, arow, a, slot);
        __builtin_amdgcn_wave_barrier();
        const float sc = ok ? vc * slot[lane] : 0.f;
        __builtin_amdgcn_wave_barrier();
        gather_axpy<VN, LN, TN>(kc, sc, t0, t1, Cmat, N, n, acc);
    }
}

// FusedMM with a row per 1, 2 or 4 wavefronts: see spmm_rows_kernel.
template <int VD, int LD, int TD, int VN, int LN, int TN, typename E>
__device__ __forceinline__ void fusedmm_rows_body(int M, int D, int N, const int32_t *__restrict__ rowptr,
                                                  const int32_t *__restrict__ colidx, const float *__restrict__ vals,
                                                  const E *__restrict__ A, const E *__restrict__ Bmat,
                                                  const E *__restrict__ Cmat, float *__restrict__ O, int wpr,
                                                  float *slot, RowParts<VN, LN, TN> &lds) {
    constexpr int TWN = LN * VN;
    const int lane = lane_id();
    const int wv = uniform(threadIdx.x >> 6);
    const int sub = wv % wpr, rows_per_block = kWavesPerBlock / wpr;
    const int d = (lane % LD) * VD;
    const int n = blockIdx.y * (TWN * TN) + (lane % LN) * VN;
    for (long long r0 = (long long)blockIdx.x * rows_per_block; r0 < M; r0 += (long long)gridDim.x * rows_per_block) {
        const long long r = r0 + wv / wpr;
        const bool valid = r < M;
        const int rs = valid ? uniform(rowptr[r]) : 0;
        const int re = valid ? uniform(rowptr[r + 1]) : 0;
        int s0, s1;
        row_part(rs, re, sub, wpr, s0, s1);
        float acc[TN][VN] = {};
        fused_segment<VD, LD, TD, VN, LN, TN>((int)(valid ? r : 0), s0, s1, colidx, vals, A, Bmat, Cmat, D, N, d, n, slot,
                                              acc);
        fold_groups<VN, LN, TN>(acc);
        if (wpr == 1) {
            if (valid) store_row<VN, LN, TN>(O + (size_t)r * N, N, n, acc);
        } else {
            add_row_parts<VN, LN, TN>(lds, wv, sub, wpr, valid, O + (size_t)(valid ? r : 0) * N, N, n, acc);
        }
    }
}

template <int VD, int LD, int TD, int VN, int LN, int TN, typename E = float>
__global__ __launch_bounds__(kBlockThreads) void fusedmm_rows_kernel(
    int M, int D, int N, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ vals, const E *__restrict__ A, const E *__restrict__ Bmat,
    const E *__restrict__ Cmat, float *__restrict__ O, int wpr) {
    __shared__ float slots[kWavesPerBlock][kWave];
    __shared__ RowParts<VN, LN, TN> lds;
    fusedmm_rows_body<VD, LD, TD, VN, LN, TN>(M, D, N, rowptr, colidx, vals, A, Bmat, Cmat, O, wpr,
                                              slots[threadIdx.x >> 6], lds);
}

template <int VD, int LD, int TD, int VN, int LN, int TN, typename E = float>
__global__ __launch_bounds__(kBlockThreads) void fusedmm_nnzsplit_kernel(
    int M, int D, int N, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ vals, const E *__restrict__ A, const E *__restrict__ Bmat,
    const E *__restrict__ Cmat, float *__restrict__ O, float *__restrict__ head,
    int32_t *__restrict__ head_row, const int32_t *__restrict__ gate, const int32_t *__restrict__ even) {
    __shared__ float slots[kWavesPerBlock][kWave];
    constexpr int TWN = LN * VN;
    if (gate && ktile_ok(gate)) return;
    const int lane = lane_id();
    const int W = gridDim.x * kWavesPerBlock;
    const int wv = threadIdx.x >> 6;
    const int w = uniform(blockIdx.x * kWavesPerBlock + wv);
    const int d = (lane % LD) * VD;
    const int n = blockIdx.y * (TWN * TN) + (lane % LN) * VN;
    float *slot = slots[wv];
    // Whole rows, round robin (see spmm_nnzsplit_kernel) - here only with more than half as many rows as wavefronts
    // and one wavefront per row: sharing rows between wavefronts costs registers that the equal-share branch below,
    // the one skewed matrices take, needs for full occupancy (62 -> 70 VGPRs, 12 % slower on `fused8k_skew`).
    if (even && *even != 0 && 2ll * M > W) {
        for (int r = w; r < M; r += W) {
            const int rs = uniform(rowptr[r]);
            const int re = uniform(rowptr[r + 1]);
            float acc[TN][VN] = {};
            fused_segment<VD, LD, TD, VN, LN, TN>(r, rs, re, colidx, vals, A, Bmat, Cmat, D, N, d, n, slot, acc);
            fold_groups<VN, LN, TN>(acc);
            store_row<VN, LN, TN>(O + (size_t)r * N, N, n, acc);
        }
        return;
    }
    const Share sh = make_share(rowptr, M, w, W);
    if (!sh.active) {
        if (blockIdx.y == 0 && lane == 0) head_row[w] = -1;
        return;
    }
    int r = wave_lower_bound(rowptr, M, sh.lo);
    int hr = -1;
    if (sh.lo < sh.nnz) {
        const int start = uniform(rowptr[r]);
        if (start != sh.lo) {
            hr = r - 1;
            float acc[TN][VN] = {};
            fused_segment<VD, LD, TD, VN, LN, TN>(hr, sh.lo, start < sh.hi ? start : sh.hi, colidx, vals, A, Bmat,
                                                  Cmat, D, N, d, n, slot, acc);
            fold_groups<VN, LN, TN>(acc);
            store_row<VN, LN, TN>(head + (size_t)w * N, N, n, acc);
        }
    }
    if (blockIdx.y == 0 && lane == 0) head_row[w] = hr;
    for (; r < M; ++r) {
        const int rs = uniform(rowptr[r]);
        if (!sh.last && rs >= sh.hi) break;
        const int re = uniform(rowptr[r + 1]);
        float acc[TN][VN] = {};
        fused_segment<VD, LD, TD, VN, LN, TN>(r, rs, re < sh.hi ? re : sh.hi, colidx, vals, A, Bmat, Cmat, D, N, d,
                                              n, slot, acc);
        fold_groups<VN, LN, TN>(acc);
        store_row<VN, LN, TN>(O + (size_t)r * N, N, n, acc);
    }
}

}  // namespace csrk
