// Average distortion (1/N) sum_i ||theta_i - theta_bar||^2, theta_bar the mean
// over all N rows (left-hand side of the equation of Thm 3.2; the error
// measure of Sec. 4.1), for gfx950.
//
// The state is read exactly once.  For every column c the kernel accumulates,
// in binary64, s1 = sum_i (x_ic - x_0c) and s2 = sum_i (x_ic - x_0c)^2 and uses
// sum_i (x_ic - mean_c)^2 = s2 - s1^2 / N.  Shifting by row 0 keeps the
// subtraction harmless once the peers have (nearly) agreed: all differences
// are then tiny and exact in binary64.  With a `present` mask (a partly filled
// grid) the same runs over the rows that hold a peer, shifted by the first one.
//
// Mapping.  A block owns a tile of 64 vectors (one 128-bit vector per lane,
// 1 KiB per row); its W waves (W chosen so that a wave sees about 256 rows) take
// rows w, w+W, ... with 8 non-temporal row loads in flight each, then combine their per-column sums through LDS, reduce across lanes
// and write ONE partial per block.  A second one-block kernel adds the partials
// in a fixed order, so the result does not depend on scheduling.
#include <mutex>

#include "moshpit_internal.h"

// Partial sums of the allocation-free entry point: one double per block of the
// first kernel, kept in the code object so that no call ever allocates.  Every
// GPU the library runs on holds its own copy (1 MiB) at its own address until
// the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the kernels get the address that call returns.
static __device__ __align__(256) double scratch[moshpit::kStaticPartials];

namespace moshpit {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double *g_scratch_ptr[kMaxDevices] = {};     // device address of `scratch`, per device

constexpr int kMaxWaves = 16;      // waves per block: 1, 2, 4, 8 or 16
constexpr int kRowsInFlight = 8;   // row loads issued before the first use

template <int DT, int VE> struct Wide;

template <> struct Wide<0, 4> {
    typedef f32x4 mem_t;
    static constexpr int NE = 4;
    static __device__ __forceinline__ void widen(const mem_t &m, double (&f)[NE])
    {
        f[0] = m.x; f[1] = m.y; f[2] = m.z; f[3] = m.w;
    }
};
template <> struct Wide<0, 1> {
    typedef float mem_t;
    static constexpr int NE = 1;
    static __device__ __forceinline__ void widen(const mem_t &m, double (&f)[NE]) { f[0] = m; }
};
template <> struct Wide<1, 8> {
    typedef u32x4 mem_t;
    static constexpr int NE = 8;
    static __device__ __forceinline__ void widen(const mem_t &m, double (&f)[NE])
    {
        const uint32_t w[4] = {m.x, m.y, m.z, m.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f[2 * k] = __uint_as_float(w[k] << 16);
            f[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u);
        }
    }
};
template <> struct Wide<1, 1> {
    typedef uint16_t mem_t;
    static constexpr int NE = 1;
    static __device__ __forceinline__ void widen(const mem_t &m, double (&f)[NE])
    {
        f[0] = __uint_as_float(static_cast<uint32_t>(m) << 16);
    }
};

// X         byte pointer to element (row 0, first column of this launch)
// nvec      vectors of VE elements per row covered by this launch
// partials  one double per block: sum over the block's columns of s2 - s1^2/n
// present   nullptr, or N bytes: rows with 0 are left out of mean and sum
//           (vertices of a partly filled grid that hold no peer)
// first     index of the first row that counts; n = number of rows that count
template <int DT, int VE, int kWaves>
__global__ __launch_bounds__(kWaves * 64) void dist_partial_kernel(const char *__restrict__ X, int64_t row_bytes,
                                                                    int64_t nvec, int64_t N,
                                                                    double *__restrict__ partials,
                                                                    const uint8_t *__restrict__ present,
                                                                    int64_t first, int64_t n)
{
    typedef Wide<DT, VE> V;
    typedef typename V::mem_t mem_t;
    constexpr int NE = V::NE;
    __shared__ double sh[2][kWaves][64];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t v = static_cast<int64_t>(blockIdx.x) * 64 + lane;
    const bool valid = v < nvec;
    const char *col = X + v * static_cast<int64_t>(sizeof(mem_t));

    double x0[NE], s1[NE], s2[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) { x0[e] = 0.0; s1[e] = 0.0; s2[e] = 0.0; }
    if (valid) V::widen(*reinterpret_cast<const mem_t *>(col + first * row_bytes), x0);

    for (int64_t i0 = wave; i0 < N; i0 += kWaves * kRowsInFlight) {
        mem_t buf[kRowsInFlight];
        bool have[kRowsInFlight];
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u) {
            const int64_t i = i0 + static_cast<int64_t>(u) * kWaves;
            have[u] = valid && i < N && (present == nullptr || present[i] != 0);
            if (have[u]) buf[u] = __builtin_nontemporal_load(reinterpret_cast<const mem_t *>(col + i * row_bytes));
        }
#pragma unroll
        for (int u = 0; u < kRowsInFlight; ++u) {
            if (have[u]) {
                double x[NE];
                V::widen(buf[u], x);
#pragma unroll
                for (int e = 0; e < NE; ++e) {
                    const double dlt = x[e] - x0[e];
                    s1[e] += dlt;
                    s2[e] = fma(dlt, dlt, s2[e]);
                }
            }
        }
    }

    // combine the waves' per-column sums, one element of the vector at a time
    double colsum = 0.0;
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        sh[0][wave][lane] = s1[e];
        sh[1][wave][lane] = s2[e];
        __syncthreads();
        if (wave == 0) {
            double t1 = 0.0, t2 = 0.0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) { t1 += sh[0][w][lane]; t2 += sh[1][w][lane]; }
            if (valid) colsum += t2 - t1 * t1 / static_cast<double>(n);
        }
        __syncthreads();
    }
    if (wave == 0) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) colsum += __shfl_down(colsum, off, 64);
        if (lane == 0) partials[blockIdx.x] = colsum;
    }
}

__global__ __launch_bounds__(256) void dist_final_kernel(const double *__restrict__ partials, int64_t count,
                                                         int64_t n, double *__restrict__ out)
{
    __shared__ double sh[256];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < count; i += 256) acc += partials[i];
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (static_cast<int>(threadIdx.x) < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = sh[0] / static_cast<double>(n);
}

struct Split {
    int64_t nvec;       // 128-bit vectors per row
    int64_t tail0;      // first element-wise column
    int64_t blocks_vec, blocks_tail;
};

Split split_row(int dtype, int64_t P, int64_t row_stride, const void *X)
{
    const int64_t esize = dtype == 0 ? 4 : 2;
    const int64_t ve = dtype == 0 ? 4 : 8;
    const bool aligned = (reinterpret_cast<uintptr_t>(X) % 16 == 0) && ((row_stride * esize) % 16 == 0);
    Split s;
    s.nvec = aligned ? P / ve : 0;
    s.tail0 = s.nvec * ve;
    s.blocks_vec = (s.nvec + 63) / 64;
    s.blocks_tail = (P - s.tail0 + 63) / 64;
    return s;
}

}  // namespace

int64_t dist_partials_count(int dtype, int64_t P, int64_t row_stride, const void *X)
{
    const Split s = split_row(dtype, P, row_stride, X);
    return s.blocks_vec + s.blocks_tail;
}

hipError_t launch_dist_to_mean(const void *X, int dtype, int64_t N, int64_t P, int64_t row_stride,
                               double *partials, double *out, const uint8_t *present, int64_t first, int64_t n,
                               hipStream_t stream)
{
    const Split s = split_row(dtype, P, row_stride, X);
    if (s.blocks_vec > 0x7fffffffLL || s.blocks_tail > 0x7fffffffLL) return hipErrorInvalidValue;
    const int64_t esize = dtype == 0 ? 4 : 2;
    const int64_t row_bytes = row_stride * esize;
    const char *base = static_cast<const char *>(X);
    // about 256 rows per wave (measured best on MI355X for 64 <= N <= 4096)
    int waves = 1;
    while (waves < kMaxWaves && N / (waves * 2) >= 256) waves *= 2;
    const char *tbase = base + s.tail0 * esize;
    double *tpart = partials + s.blocks_vec;
#define MOSHPIT_DIST(W)                                                                                        \
    if (waves == W) {                                                                                          \
        const dim3 block(W * 64);                                                                              \
        if (s.blocks_vec > 0) {                                                                                \
            const dim3 grid(static_cast<uint32_t>(s.blocks_vec));                                              \
            if (dtype == 0)                                                                                    \
                dist_partial_kernel<0, 4, W><<<grid, block, 0, stream>>>(base, row_bytes, s.nvec, N, partials, present, first, n); \
            else                                                                                               \
                dist_partial_kernel<1, 8, W><<<grid, block, 0, stream>>>(base, row_bytes, s.nvec, N, partials, present, first, n); \
        }                                                                                                      \
        if (s.blocks_tail > 0) {                                                                               \
            const dim3 grid(static_cast<uint32_t>(s.blocks_tail));                                             \
            if (dtype == 0)                                                                                    \
                dist_partial_kernel<0, 1, W><<<grid, block, 0, stream>>>(tbase, row_bytes, P - s.tail0, N, tpart, present, first, n); \
            else                                                                                               \
                dist_partial_kernel<1, 1, W><<<grid, block, 0, stream>>>(tbase, row_bytes, P - s.tail0, N, tpart, present, first, n); \
        }                                                                                                      \
    }
    MOSHPIT_DIST(1)
    MOSHPIT_DIST(2)
    MOSHPIT_DIST(4)
    MOSHPIT_DIST(8)
    MOSHPIT_DIST(16)
#undef MOSHPIT_DIST
    {
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    dist_final_kernel<<<dim3(1), dim3(256), 0, stream>>>(partials, s.blocks_vec + s.blocks_tail, n, out);
    return hipGetLastError();
}

hipError_t static_scratch(double **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (ptr == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<double *>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace moshpit
