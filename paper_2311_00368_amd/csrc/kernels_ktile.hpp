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
// length is a ballot + popcount.  The chunk for the next tile is requested before the
// multiply-adds of the current one start.
//
// Requirements (checked on the device by analyze_kernel, else the general kernels run):
// columns of every row non-decreasing; S dense enough for the LDS copy to pay.
//
// FusedMM adds a dot stage per segment: 4 entries at a time, 16 lanes x 4 floats over
// D <= 64, rows of the first dense operand B also staged in LDS, DPP reduction, scores
// parked in a 64-float LDS slot per wavefront and picked up one per lane, exactly as in
// the general kernel.  Scores never leave the CU (Algorithm 3's `arow`).
#pragma once
#include "device_util.hpp"

namespace csrk {

constexpr int kTileThreads = 1024;
constexpr int kTileWaves = kTileThreads / kWave;

// flags[0] != 0: some row has descending columns.  flags[1] != 0: dense enough.
__device__ __forceinline__ bool ktile_ok(const int32_t *flags) { return flags[0] == 0 && flags[1] != 0; }

__global__ void reset_flags_kernel(int32_t *flags) {
    if (threadIdx.x < 4) flags[threadIdx.x] = 0;
}

// One pass over colidx: are all rows ascending?  Also records whether nnz reaches
// `min_density` of M*K.  (The row analysis step of the hot path.)
__global__ __launch_bounds__(256) void analyze_kernel(int M, int K, const int32_t *__restrict__ rowptr,
                                                      const int32_t *__restrict__ colidx, float min_density,
                                                      int32_t *__restrict__ flags) {
    const int lane = lane_id();
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    if (wave == 0 && lane == 0) {
        const double nnz = (double)rowptr[M];
        if (nnz >= (double)min_density * (double)M * (double)K) flags[1] = 1;
    }
    bool bad = false;
    for (int r = wave; r < M; r += nwaves) {
        const int rs = rowptr[r], re = rowptr[r + 1];
        for (int j = rs + 1 + lane; j < re; j += kWave) bad |= colidx[j - 1] > colidx[j];
    }
    if (__ballot(bad) != 0 && lane == 0) flags[0] = 1;
}

template <int T, int KT, int ROWS, bool FUSED>
struct KTileLds {
    static constexpr int kRowFloats = T * 256;
    static constexpr int kCFloats = KT * kRowFloats;
    static constexpr int kDFloats = FUSED ? KT * 64 : 0;
    static constexpr int kSlotFloats = FUSED ? kTileWaves * kWave : 0;
    static constexpr int kBytes = (kCFloats + kDFloats + kSlotFloats) * 4;
};

template <int T, int KT, int ROWS, bool FUSED>
__global__ __launch_bounds__(kTileThreads) void ktile_kernel(
    int M, int K, int D, int N, const int32_t *__restrict__ rowptr, const int32_t *__restrict__ colidx,
    const float *__restrict__ vals, const float *__restrict__ A, const float *__restrict__ Bmat,
    const float *__restrict__ Cmat, float *__restrict__ O, const int32_t *__restrict__ flags) {
    using L = KTileLds<T, KT, ROWS, FUSED>;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    if (!ktile_ok(flags)) return;
    float *ct = lds;                        // KT x (T*256)
    float *bt = lds + L::kCFloats;          // KT x 64        (FUSED)
    float *slots = bt + L::kDFloats;        // 16 x 64        (FUSED)

    const int lane = lane_id();
    const int wave = uniform(threadIdx.x >> 6);
    const int row0 = blockIdx.x * (kTileWaves * ROWS) + wave * ROWS;
    const int n = lane * 4;                 // this lane's first column inside each 256-wide tile
    const int d = (lane & 15) * 4;          // FUSED: this lane's slice of the dot length
    const int g = lane >> 4;                // FUSED: which of 4 side-by-side entries

    int pos[ROWS], end[ROWS];
    int kc[ROWS];
    float vc[ROWS];
    float a[FUSED ? ROWS : 1][4];
    float acc[ROWS][T][4];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int row = row0 + r;
        pos[r] = row < M ? uniform(rowptr[row]) : 0;
        end[r] = row < M ? uniform(rowptr[row + 1]) : 0;
        const int j = pos[r] + lane;
        const bool ok = j < end[r];
        kc[r] = ok ? colidx[j] : 0x7fffffff;
        vc[r] = ok ? (vals ? vals[j] : 1.f) : 0.f;
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[r][t][v] = 0.f;
        if constexpr (FUSED) {
            if (row < M && d < D) {
                load_vec<4>(A + (size_t)row * D + d, a[r]);
            } else {
                a[r][0] = a[r][1] = a[r][2] = a[r][3] = 0.f;
            }
        }
    }

    const int n4 = N >> 2;                  // float4s per dense row
    for (int k0 = 0; k0 < K; k0 += KT) {
        __syncthreads();                    // previous tile fully consumed
        // ---- stage C[k0:k0+KT, 0:N] (and B[k0:k0+KT, 0:D]) in LDS
        {
            const float4 *src = reinterpret_cast<const float4 *>(Cmat);
            float4 *dst = reinterpret_cast<float4 *>(ct);
            constexpr int kRow4 = T * 64;
#pragma unroll
            for (int i = 0; i < KT * kRow4 / kTileThreads; ++i) {
                const int e = i * kTileThreads + threadIdx.x;
                const int kk = e / kRow4, c4 = e % kRow4;
                if (k0 + kk < K && c4 < n4) dst[e] = src[(size_t)(k0 + kk) * n4 + c4];
            }
            if constexpr (FUSED) {
                const float4 *srcb = reinterpret_cast<const float4 *>(Bmat);
                float4 *dstb = reinterpret_cast<float4 *>(bt);
                const int d4 = D >> 2;
#pragma unroll
                for (int i = 0; i < (KT * 16 + kTileThreads - 1) / kTileThreads; ++i) {
                    const int e = i * kTileThreads + threadIdx.x;
                    const int kk = e >> 4, c4 = e & 15;
                    if (e < KT * 16 && k0 + kk < K && c4 < d4) dstb[e] = srcb[(size_t)(k0 + kk) * d4 + c4];
                }
            }
        }
        __syncthreads();
        const int kend = k0 + KT;
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            while (true) {
                // entries of this tile = leading lanes of the chunk with column < kend
                const int cnt = __builtin_popcountll(__ballot(kc[r] < kend));
                if (cnt == 0) break;
                // request the chunk that follows before doing the arithmetic
                const int npos = pos[r] + cnt;
                const int jn = npos + lane;
                const bool okn = jn < end[r];
                const int kn = okn ? colidx[jn] : 0x7fffffff;
                const float vn = okn ? (vals ? vals[jn] : 1.f) : 0.f;
                float sc = vc[r];
                if constexpr (FUSED) {
                    float *slot = slots + wave * kWave;
                    for (int t = 0; t < cnt; t += 4) {
                        const int idx = t + g;
                        const int kk = __shfl(kc[r], idx) - k0;
                        float part = 0.f;
                        if (idx < cnt && d < D) {
                            float b[4];
                            load_vec<4>(bt + kk * 64 + d, b);
                            part = a[r][0] * b[0];
                            part = fmaf(a[r][1], b[1], part);
                            part = fmaf(a[r][2], b[2], part);
                            part = fmaf(a[r][3], b[3], part);
                        }
                        part = group_sum<16>(part);
                        if (idx < cnt && (lane & 15) == 0) slot[idx] = part;
                    }
                    __builtin_amdgcn_wave_barrier();
                    sc = lane < cnt ? vc[r] * slot[lane] : 0.f;
                    __builtin_amdgcn_wave_barrier();
                }
                const int kcur = kc[r];
                auto step = [&](int t) {
                    const int kk = __builtin_amdgcn_readlane(kcur, t) - k0;
                    const float s = readlane_f(sc, t);
                    const float *crow = ct + kk * L::kRowFloats + n;
#pragma unroll
                    for (int tt = 0; tt < T; ++tt) {
                        float c[4];
                        load_vec<4>(crow + tt * 256, c);
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[r][tt][v] = fmaf(s, c[v], acc[r][tt][v]);
                    }
                };
                int t = 0;
                for (; t + 4 <= cnt; t += 4) {
                    step(t);
                    step(t + 1);
                    step(t + 2);
                    step(t + 3);
                }
                for (; t < cnt; ++t) step(t);
                pos[r] = npos;
                kc[r] = kn;
                vc[r] = vn;
                if (cnt < kWave) break;
            }
        }
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int row = row0 + r;
        if (row < M) {
#pragma unroll
            for (int tt = 0; tt < T; ++tt)
                if (n + tt * 256 < N) store_vec<4>(O + (size_t)row * N + n + tt * 256, acc[r][tt]);
        }
    }
}

}  // namespace csrk
