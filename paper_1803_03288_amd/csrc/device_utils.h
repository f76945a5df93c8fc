// Wave- and block-level helpers shared by the TAC and simulation kernels (wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tictac {

#define TT_INF (__builtin_huge_val())

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// ordering point for LDS traffic between the lanes of one wave (LDS operations of a wave
// complete in issue order; this only keeps the compiler from moving them across)
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ double wave_min_f64(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmin(v, __shfl_xor(v, off));
    return v;
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

__device__ __forceinline__ double wave_max_f64(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off));
    return v;
}

// ---- the same reductions and scans through data-parallel-primitive moves (no LDS traffic) ----
// A wave64 is four rows of 16 lanes.  row_shr:n moves a value n lanes up inside a row;
// row_bcast:15 hands lane 15 of every row to the whole next row, row_bcast:31 hands lane 31
// to rows 2 and 3.  A lane without a source keeps `identity`.  Four shifts (1, 2, 4, 8) scan
// the rows, the two broadcasts (applied to rows 1 and 3, then to rows 2 and 3) add the totals
// of the rows before; lane 63 ends with the reduction over the wave.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_i32(int identity, int v)
{
    return __builtin_amdgcn_update_dpp(identity, v, CTRL, ROW_MASK, 0xf, false);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double identity, double v)
{
    const int lo = __builtin_amdgcn_update_dpp(__double2loint(identity), __double2loint(v), CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(__double2hiint(identity), __double2hiint(v), CTRL, ROW_MASK, 0xf, false);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double readlane_f64(double v, int l)      // l wave-uniform
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), l),
                            __builtin_amdgcn_readlane(__double2loint(v), l));
}

__device__ __forceinline__ double lane63_f64(double v)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63),
                            __builtin_amdgcn_readlane(__double2loint(v), 63));
}

#define TT_DPP_SCAN(T, DPP, OP, ID)                                                       \
    v = OP(v, DPP<0x111, 0xf>(ID, v));                                                    \
    v = OP(v, DPP<0x112, 0xf>(ID, v));                                                    \
    v = OP(v, DPP<0x114, 0xf>(ID, v));                                                    \
    v = OP(v, DPP<0x118, 0xf>(ID, v));                                                    \
    v = OP(v, DPP<0x142, 0xa>(ID, v));                                                    \
    v = OP(v, DPP<0x143, 0xc>(ID, v));

__device__ __forceinline__ double tt_add_f64(double a, double b) { return a + b; }
__device__ __forceinline__ int tt_add_i32(int a, int b) { return a + b; }
__device__ __forceinline__ int tt_min_i32(int a, int b) { return min(a, b); }
__device__ __forceinline__ int tt_max_i32(int a, int b) { return max(a, b); }

// inclusive prefix sum over the lanes of a wave
__device__ __forceinline__ double wave_incl_scan_f64_dpp(double v)
{
    TT_DPP_SCAN(double, dpp_f64, tt_add_f64, 0.0)
    return v;
}
__device__ __forceinline__ double wave_sum_f64_dpp(double v)
{
    TT_DPP_SCAN(double, dpp_f64, tt_add_f64, 0.0)
    return lane63_f64(v);
}
__device__ __forceinline__ double wave_max_f64_dpp(double v)
{
    TT_DPP_SCAN(double, dpp_f64, fmax, -TT_INF)
    return lane63_f64(v);
}
__device__ __forceinline__ double wave_min_f64_dpp(double v)
{
    TT_DPP_SCAN(double, dpp_f64, fmin, TT_INF)
    return lane63_f64(v);
}
__device__ __forceinline__ int wave_min_i32_dpp(int v)
{
    TT_DPP_SCAN(int, dpp_i32, tt_min_i32, INT32_MAX)
    return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ int wave_max_i32_dpp(int v)
{
    TT_DPP_SCAN(int, dpp_i32, tt_max_i32, INT32_MIN)
    return __builtin_amdgcn_readlane(v, 63);
}
#undef TT_DPP_SCAN

// A row of a timing array that is stored as float64 or as float32.  A float32 value is converted
// when it is loaded; every sum and comparison is float64.
struct TimeRow {
    const void *p;
    bool f32;
    __device__ __forceinline__ double operator[](int j) const
    {
        return f32 ? (double)static_cast<const float *>(p)[j] : static_cast<const double *>(p)[j];
    }
    __device__ __forceinline__ const float *as_f32() const { return static_cast<const float *>(p); }
    __device__ __forceinline__ const double *as_f64() const { return static_cast<const double *>(p); }
};
__device__ __forceinline__ TimeRow time_row(const void *base, size_t first, bool f32)
{
    return TimeRow{f32 ? static_cast<const void *>(static_cast<const float *>(base) + first)
                       : static_cast<const void *>(static_cast<const double *>(base) + first), f32};
}

// Four consecutive elements with one load (two for float64).  Rows start at any element, so the
// vector types carry the alignment of one element; the class table is read the same way.
typedef float tt_f32x4 __attribute__((ext_vector_type(4), aligned(4)));
typedef double tt_f64x2 __attribute__((ext_vector_type(2), aligned(8)));
typedef int tt_i32x4 __attribute__((ext_vector_type(4), aligned(4)));

__device__ __forceinline__ void load4(const double *__restrict__ q, double (&x)[4])
{
    const tt_f64x2 a = *reinterpret_cast<const tt_f64x2 *>(q), b = *reinterpret_cast<const tt_f64x2 *>(q + 2);
    x[0] = a.x; x[1] = a.y; x[2] = b.x; x[3] = b.y;
}
__device__ __forceinline__ void load4(const float *__restrict__ q, double (&x)[4])
{
    const tt_f32x4 a = *reinterpret_cast<const tt_f32x4 *>(q);
    x[0] = (double)a.x; x[1] = (double)a.y; x[2] = (double)a.z; x[3] = (double)a.w;
}

// totals[cls_of[j]] += row[j] for j in [0, N), totals in LDS, by one wave.  A lane takes four
// consecutive columns at a time and first adds up runs of equal class in registers: columns of
// one class tend to sit next to each other, and every LDS add of several lanes to one address
// is served one lane after the other.
template <typename T>
__device__ __forceinline__ void class_totals(double *totals, const T *__restrict__ row,
                                             const int32_t *__restrict__ cls_of, int N, int lane)
{
    for (int j0 = lane * 4; j0 < N; j0 += 64 * 4 * 2) {          // two groups of four in flight per lane
        double x[2][4];
        int c[2][4];
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            const int j = j0 + g * 256;
            if (j + 3 < N) {
                load4(row + j, x[g]);
                const tt_i32x4 q = *reinterpret_cast<const tt_i32x4 *>(cls_of + j);
                c[g][0] = q.x; c[g][1] = q.y; c[g][2] = q.z; c[g][3] = q.w;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    x[g][i] = j + i < N ? (double)row[j + i] : 0.0;
                    c[g][i] = j + i < N ? cls_of[j + i] : -1;
                }
            }
        }
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            double acc = x[g][0];
            int cur = c[g][0];
#pragma unroll
            for (int i = 1; i < 4; ++i) {
                if (c[g][i] == cur) {
                    acc += x[g][i];
                } else {
                    if (cur >= 0) atomicAdd(&totals[cur], acc);
                    cur = c[g][i];
                    acc = x[g][i];
                }
            }
            if (cur >= 0) atomicAdd(&totals[cur], acc);
        }
    }
}

__device__ __forceinline__ void class_totals(double *totals, const TimeRow &row, const int32_t *__restrict__ cls_of,
                                             int N, int lane)
{
    if (row.f32) class_totals(totals, row.as_f32(), cls_of, N, lane);
    else class_totals(totals, row.as_f64(), cls_of, N, lane);
}

__device__ __forceinline__ int wave_min_i32(int v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = min(v, __shfl_xor(v, off));
    return v;
}

// Block-wide reductions; every thread of the block must call them (uniform control
// flow).  `red` is LDS scratch of at least BS/64 elements of the reduced type; two
// barriers make it reusable right after the call.
template <int BS>
__device__ __forceinline__ double block_min_f64(double v, double *red)
{
    v = wave_min_f64(v);
    if (BS == 64) return v;
    __syncthreads();
    if (lane_id() == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = red[0];
#pragma unroll
    for (int k = 1; k < BS / 64; ++k) r = fmin(r, red[k]);
    return r;
}

template <int BS>
__device__ __forceinline__ double block_sum_f64(double v, double *red)
{
    v = wave_sum_f64(v);
    if (BS == 64) return v;
    __syncthreads();
    if (lane_id() == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = red[0];
#pragma unroll
    for (int k = 1; k < BS / 64; ++k) r += red[k];
    return r;
}

template <int BS>
__device__ __forceinline__ int block_min_i32(int v, double *red)
{
    v = wave_min_i32(v);
    if (BS == 64) return v;
    int *ri = reinterpret_cast<int *>(red);
    __syncthreads();
    if (lane_id() == 0) ri[threadIdx.x >> 6] = v;
    __syncthreads();
    int r = ri[0];
#pragma unroll
    for (int k = 1; k < BS / 64; ++k) r = min(r, ri[k]);
    return r;
}

// arr[idx] += v for the threads with `active`, arr in LDS.  With one wave per block the
// additions are applied one after the other in lane order by lane 0 (a fixed order, so
// the result is reproducible bit for bit); with several waves LDS atomics are used.
// Must be called by all threads of a wave together.
template <int BS>
__device__ __forceinline__ void lds_scatter_add(double *arr, int idx, double v, bool active)
{
    if (BS == 64) {
        unsigned long long m = __ballot(active);
        while (m) {
            const int l = __builtin_ctzll(m);
            m &= m - 1;
            const int i = __shfl(idx, l);
            const double x = __shfl(v, l);
            if (threadIdx.x == 0) arr[i] += x;
        }
    } else {
        if (active) atomicAdd(&arr[idx], v);
    }
}

}  // namespace tictac
