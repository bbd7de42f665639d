// Device-side helpers shared by the gfx950 kernels: wave64 lane utilities, DPP
// reductions, vector loads, the equal-nonzero work partition and the wave-wide
// search that maps a nonzero position to its row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace csrk {

constexpr int kWave = 64;

// four floats as one 128-bit register value: loads and stores of it are plain moves (an array of HIP's float4
// structs filled through a casted pointer can end up copied through private memory instead)
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ float readlane_f(float v, int l) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

// Sum over groups of LG consecutive lanes (LG a power of two, <= 64); every lane of
// a group ends up with the group's sum.  The first four steps stay inside a row of 16
// lanes and use DPP (quad permutes, half-row mirror, row mirror); wider groups finish
// with cross-row exchanges.
template <int LG>
__device__ __forceinline__ float group_sum(float v) {
    if (LG >= 2) v += dpp_f<0xB1>(v);    // quad_perm [1,0,3,2]
    if (LG >= 4) v += dpp_f<0x4E>(v);    // quad_perm [2,3,0,1]
    if (LG >= 8) v += dpp_f<0x141>(v);   // row_half_mirror
    if (LG >= 16) v += dpp_f<0x140>(v);  // row_mirror
    if (LG >= 32) v += __shfl_xor(v, 16);
    if (LG >= 64) v += __shfl_xor(v, 32);
    return v;
}

// f(std::integral_constant<int, i>) for i = I0 .. I1-1, unrolled at compile time.
template <int I0, int I1, typename F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I0 < I1) {
        f(std::integral_constant<int, I0>{});
        static_for<I0 + 1, I1>(f);
    }
}

// acc += a' * b, where a' is the value of `a` in the lane that the rotation row_ror:S of a row of 16 lanes
// pairs with this one.  Written as the one DPP multiply-add it is meant to be: left to the compiler, the
// rotated values (loop invariants) are hoisted out of the loop as hundreds of extra live registers.
template <int S>
__device__ __forceinline__ void fma_row_rotated(float &acc, float a, float b) {
    if constexpr (S == 0) {
        acc = fmaf(a, b, acc);
    } else {
        asm("v_fmac_f32_dpp %0, %1, %2 row_ror:%3 row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(a), "v"(b), "n"(S));
    }
}

// VEC consecutive floats; VEC a multiple of 4: 128-bit accesses (address must be 16-byte aligned).
template <int VEC>
__device__ __forceinline__ void load_vec(const float *p, float (&d)[VEC]) {
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int i = 0; i < VEC; i += 4) {
            const float4 t = *reinterpret_cast<const float4 *>(p + i);
            d[i] = t.x; d[i + 1] = t.y; d[i + 2] = t.z; d[i + 3] = t.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) d[i] = p[i];
    }
}

// bfloat16 as stored (the upper half of an IEEE single); arithmetic is always done in FP32
using bf16_t = uint16_t;

// VEC consecutive bfloat16 widened to floats; VEC == 8 is one 128-bit access (16-byte aligned address).
// Widening is exact: the 16 bits become the upper half of the float.
template <int VEC>
__device__ __forceinline__ void load_vec(const bf16_t *p, float (&d)[VEC]) {
    if constexpr (VEC == 8) {
        const uint4 t = *reinterpret_cast<const uint4 *>(p);
        const unsigned w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            d[2 * i] = __builtin_bit_cast(float, w[i] << 16);
            d[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) d[i] = __builtin_bit_cast(float, (unsigned)p[i] << 16);
    }
}

// VEC a multiple of 4: 128-bit accesses (16-byte aligned address)
template <int VEC>
__device__ __forceinline__ void store_vec(float *p, const float (&d)[VEC]) {
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int i = 0; i < VEC; i += 4)
            *reinterpret_cast<float4 *>(p + i) = make_float4(d[i], d[i + 1], d[i + 2], d[i + 3]);
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) p[i] = d[i];
    }
}

// A dense operand seen through a buffer descriptor: loads take the descriptor and a scalar byte offset (the part of
// the address that is the same for the whole wavefront: tile and load number) from scalar registers and ONE 32-bit
// vector register with the lane's own byte offset.  Plain global loads need a 64-bit address per lane and load, and
// since a thread's offsets inside a tile never change the compiler keeps all of them - two vector registers per load
// of a tile - alive through the whole kernel: 16 registers out of 128 in the 512-column kernels.  Loads past `bytes`
// return zeros instead of faulting, which is what the rows past K of a last, partial tile should read as.
// `bytes` must be below 4 GB (the launcher checks).
struct DenseView {
    __amdgpu_buffer_rsrc_t rsrc;
};
__device__ __forceinline__ DenseView dense_view(const void *base, unsigned bytes) {
    // word 3: 32-bit data format, no swizzle (the value the gfx9 family's untyped buffer loads expect)
    return DenseView{__builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000)};
}
__device__ __forceinline__ f32x4 load_f32x4(const DenseView &v, unsigned lane_bytes, unsigned uniform_bytes) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(v.rsrc, lane_bytes, uniform_bytes, 0));
}

// Element number `lane` behind a wave-uniform pointer, for a lane-wide load of a chunk of colidx or vals: the
// pointer from scalar registers, the lane's byte offset (unsigned) from one vector register.  The empty asm pins the
// pointer to scalar registers as it is: otherwise the compiler re-associates base + position + lane into
// (base + lane) + position and keeps the loop-invariant per-lane 64-bit address in two vector registers per
// stream, registers the tiled kernels do not have.
template <typename E>
__device__ __forceinline__ E lane_elem(const E *uniform_base, unsigned lane_bytes) {
    asm("" : "+s"(uniform_base));
    return *reinterpret_cast<const E *>(reinterpret_cast<const char *>(uniform_base) + lane_bytes);
}

// First r in [0, M) with rowptr[r] >= x, or M if there is none.  All 64 lanes of the
// wave probe at once, so a search over M rows takes ceil(log64 M) rounds.
__device__ __forceinline__ int wave_lower_bound(const int32_t *rowptr, int M, int x) {
    const int lane = lane_id();
    int a = 0, b = M;
    while (b > a) {
        const int step = (b - a + kWave - 1) / kWave;
        const long long idx = (long long)a + (long long)lane * step;
        const bool ge = (idx < b) ? (rowptr[idx] >= x) : true;
        const unsigned long long m = __ballot(ge);
        const int f = m ? __builtin_ctzll(m) : kWave;
        const int na = (f > 0) ? a + (f - 1) * step + 1 : a;
        const long long nb = (long long)a + (long long)f * step;
        b = (int)(nb < b ? nb : b);
        a = na;
        if (f == 0) b = a;
    }
    return uniform(a);
}

// Equal-nonzero partition: worker w of W takes the stored entries [lo, hi), a share
// rounded up to whole chunks of 64 so chunk loads stay aligned.  Workers past the last
// entry are idle; the last active worker also owns the trailing rows that have no
// entries.  With nnz == 0 worker 0 owns every row.
struct Share {
    int lo, hi;     // this worker's entries
    int nnz;
    bool active;    // has entries or owns rows
    bool last;      // last active worker
};

__device__ __forceinline__ Share make_share(const int32_t *rowptr, int M, int w, int W) {
    Share s;
    s.nnz = rowptr[M];
    long long per = ((long long)s.nnz + W - 1) / W;
    per = (per + kWave - 1) / kWave * kWave;
    if (per == 0) per = kWave;
    const long long wl = s.nnz > 0 ? (s.nnz - 1) / per : 0;
    const long long lo = (long long)w * per;
    s.active = (long long)w <= wl;
    s.last = (long long)w == wl;
    s.lo = s.active ? (int)lo : s.nnz;
    const long long hi = lo + per;
    s.hi = (int)(hi < s.nnz ? hi : s.nnz);
    if (!s.active) s.hi = s.nnz;
    return s;
}

}  // namespace csrk
