// Calibration of the static per-tensor step on the device (Sec. 3 "Initialization of
// Quantization Parameters": max-min initialisation, and an MSE-based grid search over the
// quantization parameter for per-tensor static quantization).  Offline work, not the hot path:
// three small launches, every sum taken in a fixed order so that the result is reproducible.
//
//   1. per row: rotate (as the quantizer kernels do), row maximum of |y|          -> ws[row]
//   2. per row: global maximum = max over ws; for every candidate step
//      s_i = fp32(gamma_i * max|y| / qmax), the row's squared error
//      sum_k (y - s_i * clamp(round(y / s_i)))^2                                   -> ws[T + row*n + i]
//   3. one workgroup: per candidate, the sum over rows in fp64, the arg-min (lowest index wins a
//      tie), and the result record.
#include "pq_rotate.h"

namespace pq {
namespace {

using rq::kChunk;
using rq::kThreads;

constexpr int kMaxGrid = 128;

__device__ __forceinline__ float wave_max(float a)
{
    a = fmaxf(a, rq::lane_xor<0>(a));
    a = fmaxf(a, rq::lane_xor<1>(a));
    a = fmaxf(a, rq::lane_xor<2>(a));
    a = fmaxf(a, rq::lane_xor<3>(a));
    a = fmaxf(a, rq::lane_xor<4>(a));
    a = fmaxf(a, rq::lane_xor<5>(a));
    return a;
}

__device__ __forceinline__ float wave_sum(float a)
{
    a += rq::lane_xor<0>(a);
    a += rq::lane_xor<1>(a);
    a += rq::lane_xor<2>(a);
    a += rq::lane_xor<3>(a);
    a += rq::lane_xor<4>(a);
    a += rq::lane_xor<5>(a);
    return a;
}

// A step provider that quantizes nothing: it hands the rotated values back to the kernel (the
// shared routine is then run in its store-nothing mode, BITS = 0).
struct Capture {
    float* dst;   // G * 8 floats of the calling thread
    template <int NV>
    __device__ __forceinline__ void prepare(const float (&v)[NV])
    {
#pragma unroll
        for (int i = 0; i < NV; ++i) dst[i] = v[i];
    }
    __device__ __forceinline__ void get(int64_t, float& m, float& s) const { m = 0.0f; s = 0.0f; }
    __device__ __forceinline__ int zero_offset() const { return 0; }
};

// Rotated (unnormalised) values of one row, NC chunks of 2048 channels, into v; dead entries zero.
template <int NC>
__device__ __forceinline__ void rotated_row(const __half* x_row, int64_t K, int log2h, rq::lds_f32_ptr xch, int tid,
                                            float (&v)[NC * 8])
{
    v4i raw[NC];
    bool live[NC];
    rq::load_chunk<NC>(x_row, K, 0, tid, true, raw, live);
    rq::rotate_quant_regs_with<NC, false, 0>(raw, live, 0, log2h, Capture{v}, static_cast<uint32_t*>(nullptr), xch, tid,
                                             true);
}

template <int NC>
__global__ __launch_bounds__(kThreads) void k_cal_rowmax(const __half* __restrict__ x, int64_t K, int log2h,
                                                        float* __restrict__ ws)
{
    extern __shared__ float xch_cal[];
    __shared__ float red[4];
    const int tid = threadIdx.x;
    float v[NC * 8];
    rotated_row<NC>(x + (int64_t)blockIdx.x * K, K, log2h, (rq::lds_f32_ptr)xch_cal, tid, v);
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < NC * 8; ++i) amax = fmaxf(amax, fabsf(v[i]));
    amax = wave_max(amax);
    if ((tid & 63) == 0) red[tid >> 6] = amax;
    __syncthreads();
    if (tid == 0) ws[blockIdx.x] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

template <int NC>
__global__ __launch_bounds__(kThreads) void k_cal_rowerr(const __half* __restrict__ x, int64_t T, int64_t K, int log2h,
                                                        double inv_sqrt_h, int bits, int n_grid, double gamma_min,
                                                        float* __restrict__ ws)
{
    extern __shared__ float xch_cal[];
    __shared__ float red[4];
    __shared__ float part[kMaxGrid][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float v[NC * 8];
    rotated_row<NC>(x + (int64_t)blockIdx.x * K, K, log2h, (rq::lds_f32_ptr)xch_cal, tid, v);

    // global maximum of the unnormalised values: every workgroup reduces the T row maxima itself
    float amax = 0.0f;
    for (int64_t r = tid; r < T; r += kThreads) amax = fmaxf(amax, ws[r]);
    amax = wave_max(amax);
    if (lane == 0) red[wave] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));

    const double qmax = (double)((1 << (bits - 1)) - 1);
    const float lo = -(float)(1 << (bits - 1)), hi = (float)((1 << (bits - 1)) - 1);
    const float inv_f = (float)inv_sqrt_h;
    const double amax_y = (double)amax * inv_sqrt_h;
    for (int i = 0; i < n_grid; ++i) {
        const double gamma = 1.0 - (double)i * (1.0 - gamma_min) / (double)(n_grid - 1);
        float s = (float)(gamma * amax_y / qmax);
        if (!(s > 0.0f)) s = 1.0f;
        const float mult = (float)(inv_sqrt_h / (double)s);
        float err = 0.0f;
#pragma unroll
        for (int k = 0; k < NC * 8; ++k) {
            const float q = rintf(__builtin_amdgcn_fmed3f(v[k] * mult, lo, hi));
            const float d = fmaf(-q, s, v[k] * inv_f);
            err = fmaf(d, d, err);
        }
        err = wave_sum(err);
        if (lane == 0) part[i][wave] = err;
    }
    __syncthreads();
    if (tid < n_grid)
        ws[T + (int64_t)blockIdx.x * n_grid + tid] = (part[tid][0] + part[tid][1]) + (part[tid][2] + part[tid][3]);
}

__global__ __launch_bounds__(kMaxGrid) void k_cal_pick(const float* __restrict__ ws, int64_t T, int n_grid,
                                                      double inv_sqrt_h, int bits, double gamma_min,
                                                      float* __restrict__ result)
{
    __shared__ double tot[kMaxGrid];
    __shared__ float amax_s;
    const int i = threadIdx.x;
    if (i == 0) {
        float a = 0.0f;
        for (int64_t r = 0; r < T; ++r) a = fmaxf(a, ws[r]);
        amax_s = a;
    }
    if (i < n_grid) {
        double s = 0.0;
        for (int64_t r = 0; r < T; ++r) s += (double)ws[T + r * n_grid + i];
        tot[i] = s;
        result[3 + i] = (float)s;
    }
    __syncthreads();
    if (i == 0) {
        int best = 0;
        for (int j = 1; j < n_grid; ++j)
            if (tot[j] < tot[best]) best = j;
        const double qmax = (double)((1 << (bits - 1)) - 1);
        const double amax_y = (double)amax_s * inv_sqrt_h;
        const double gamma = 1.0 - (double)best * (1.0 - gamma_min) / (double)(n_grid - 1);
        float s_best = (float)(gamma * amax_y / qmax), s_max = (float)(amax_y / qmax);
        if (!(s_best > 0.0f)) s_best = 1.0f;
        if (!(s_max > 0.0f)) s_max = 1.0f;
        result[0] = s_best;
        result[1] = s_max;
        result[2] = (float)gamma;
    }
}

// ---- the same search for Eq. 1 with a zero-point: candidates are pairs of clipping factors
// (gamma_i on max(y, 0), beta_j on min(y, 0)), s and z follow from Eq. 1; index = i * n_beta + j.
__device__ __forceinline__ float wave_min(float a)
{
    a = fminf(a, rq::lane_xor<0>(a));
    a = fminf(a, rq::lane_xor<1>(a));
    a = fminf(a, rq::lane_xor<2>(a));
    a = fminf(a, rq::lane_xor<3>(a));
    a = fminf(a, rq::lane_xor<4>(a));
    a = fminf(a, rq::lane_xor<5>(a));
    return a;
}

// Eq. 1's parameters for candidate (i, j); hi >= 0 >= lo are the extremes of the normalised values.
__device__ __forceinline__ void zp_candidate(int i, int j, int ng, int nb, double gmin, double bmin, double hi, double lo,
                                             float& s, int& z)
{
    const double gamma = ng > 1 ? 1.0 - (double)i * (1.0 - gmin) / (double)(ng - 1) : 1.0;
    const double beta = nb > 1 ? 1.0 - (double)j * (1.0 - bmin) / (double)(nb - 1) : 1.0;
    s = (float)((gamma * hi - beta * lo) / 15.0);
    if (!(s > 0.0f)) { s = 1.0f; z = 0; return; }
    double zz = -rint(beta * lo / (double)s);
    zz = zz < 0.0 ? 0.0 : (zz > 15.0 ? 15.0 : zz);
    z = (int)zz;
}

template <int NC>
__global__ __launch_bounds__(kThreads) void k_cal_rowminmax(const __half* __restrict__ x, int64_t T, int64_t K,
                                                           int log2h, float* __restrict__ ws)
{
    extern __shared__ float xch_cal[];
    __shared__ float red[8];
    const int tid = threadIdx.x;
    float v[NC * 8];
    rotated_row<NC>(x + (int64_t)blockIdx.x * K, K, log2h, (rq::lds_f32_ptr)xch_cal, tid, v);
    float hi = 0.0f, lo = 0.0f;   // dead entries are zero, and zero takes part by definition
#pragma unroll
    for (int i = 0; i < NC * 8; ++i) { hi = fmaxf(hi, v[i]); lo = fminf(lo, v[i]); }
    hi = wave_max(hi);
    lo = wave_min(lo);
    if ((tid & 63) == 0) { red[tid >> 6] = hi; red[4 + (tid >> 6)] = lo; }
    __syncthreads();
    if (tid == 0) {
        ws[blockIdx.x] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        ws[T + blockIdx.x] = fminf(fminf(red[4], red[5]), fminf(red[6], red[7]));
    }
}

template <int NC>
__global__ __launch_bounds__(kThreads) void k_cal_rowerr_zp(const __half* __restrict__ x, int64_t T, int64_t K,
                                                           int log2h, double inv_sqrt_h, int ng, int nb, double gmin,
                                                           double bmin, float* __restrict__ ws)
{
    extern __shared__ float xch_cal[];
    __shared__ float red[8];
    __shared__ float part[kMaxGrid][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float v[NC * 8];
    rotated_row<NC>(x + (int64_t)blockIdx.x * K, K, log2h, (rq::lds_f32_ptr)xch_cal, tid, v);
    float hi = 0.0f, lo = 0.0f;
    for (int64_t r = tid; r < T; r += kThreads) { hi = fmaxf(hi, ws[r]); lo = fminf(lo, ws[T + r]); }
    hi = wave_max(hi);
    lo = wave_min(lo);
    if (lane == 0) { red[wave] = hi; red[4 + wave] = lo; }
    __syncthreads();
    const double hid = (double)fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) * inv_sqrt_h;
    const double lod = (double)fminf(fminf(red[4], red[5]), fminf(red[6], red[7])) * inv_sqrt_h;
    const float inv_f = (float)inv_sqrt_h;
    const int n = ng * nb;
    for (int c = 0; c < n; ++c) {
        float s;
        int z;
        zp_candidate(c / nb, c % nb, ng, nb, gmin, bmin, hid, lod, s, z);
        const float mult = (float)(inv_sqrt_h / (double)s), zf = (float)z;
        float err = 0.0f;
#pragma unroll
        for (int k = 0; k < NC * 8; ++k) {
            const float q = __builtin_amdgcn_fmed3f(rintf(v[k] * mult) + zf, 0.0f, 15.0f) - zf;
            const float d = fmaf(-q, s, v[k] * inv_f);
            err = fmaf(d, d, err);
        }
        err = wave_sum(err);
        if (lane == 0) part[c][wave] = err;
    }
    __syncthreads();
    if (tid < n) ws[2 * T + (int64_t)blockIdx.x * n + tid] = (part[tid][0] + part[tid][1]) + (part[tid][2] + part[tid][3]);
}

__global__ __launch_bounds__(kMaxGrid) void k_cal_pick_zp(const float* __restrict__ ws, int64_t T, int ng, int nb,
                                                         double inv_sqrt_h, double gmin, double bmin,
                                                         float* __restrict__ result)
{
    __shared__ double tot[kMaxGrid];
    __shared__ float ext[2];
    const int i = threadIdx.x, n = ng * nb;
    if (i == 0) {
        float hi = 0.0f, lo = 0.0f;
        for (int64_t r = 0; r < T; ++r) { hi = fmaxf(hi, ws[r]); lo = fminf(lo, ws[T + r]); }
        ext[0] = hi;
        ext[1] = lo;
    }
    if (i < n) {
        double s = 0.0;
        for (int64_t r = 0; r < T; ++r) s += (double)ws[2 * T + r * n + i];
        tot[i] = s;
        result[6 + i] = (float)s;
    }
    __syncthreads();
    if (i == 0) {
        int best = 0;
        for (int j = 1; j < n; ++j)
            if (tot[j] < tot[best]) best = j;
        const double hid = (double)ext[0] * inv_sqrt_h, lod = (double)ext[1] * inv_sqrt_h;
        float s, s0;
        int z, z0;
        zp_candidate(best / nb, best % nb, ng, nb, gmin, bmin, hid, lod, s, z);
        zp_candidate(0, 0, ng, nb, gmin, bmin, hid, lod, s0, z0);
        result[0] = s;
        result[1] = (float)z;
        result[2] = s0;
        result[3] = (float)z0;
        result[4] = (float)(best / nb);
        result[5] = (float)(best % nb);
    }
}

template <int NC>
int launch_cal_zp_nc(const __half* xp, int64_t T, int64_t K, int log2h, double inv_sqrt_h, int ng, int nb, double gmin,
                     double bmin, float* result, float* ws, hipStream_t st)
{
    const size_t lds = log2h > 9 ? (size_t)NC * kChunk * sizeof(float) : 0;
    static std::atomic<uint64_t> lds_a{0}, lds_b{0};
    if (lds > 32 * 1024) {
        const size_t mx = (size_t)NC * kChunk * sizeof(float);
        if (allow_dynamic_lds(reinterpret_cast<const void*>(k_cal_rowminmax<NC>), mx, lds_a) != PQ_OK ||
            allow_dynamic_lds(reinterpret_cast<const void*>(k_cal_rowerr_zp<NC>), mx, lds_b) != PQ_OK)
            return PQ_ERR_HIP;
    }
    hipLaunchKernelGGL(k_cal_rowminmax<NC>, dim3((unsigned)T), dim3(kThreads), lds, st, xp, T, K, log2h, ws);
    hipLaunchKernelGGL(k_cal_rowerr_zp<NC>, dim3((unsigned)T), dim3(kThreads), lds, st, xp, T, K, log2h, inv_sqrt_h, ng, nb,
                       gmin, bmin, ws);
    hipLaunchKernelGGL(k_cal_pick_zp, dim3(1), dim3(kMaxGrid), 0, st, ws, T, ng, nb, inv_sqrt_h, gmin, bmin, result);
    return hip_status(hipGetLastError());
}

template <int NC>
int launch_cal_nc(const __half* xp, int64_t T, int64_t K, int log2h, double inv_sqrt_h, int bits, int n_grid,
                  double gamma_min, float* result, float* ws, hipStream_t st)
{
    const size_t lds = log2h > 9 ? (size_t)NC * kChunk * sizeof(float) : 0;
    static std::atomic<uint64_t> lds_a{0}, lds_b{0};
    if (lds > 32 * 1024) {
        const size_t mx = (size_t)NC * kChunk * sizeof(float);
        if (allow_dynamic_lds(reinterpret_cast<const void*>(k_cal_rowmax<NC>), mx, lds_a) != PQ_OK ||
            allow_dynamic_lds(reinterpret_cast<const void*>(k_cal_rowerr<NC>), mx, lds_b) != PQ_OK)
            return PQ_ERR_HIP;
    }
    hipLaunchKernelGGL(k_cal_rowmax<NC>, dim3((unsigned)T), dim3(kThreads), lds, st, xp, K, log2h, ws);
    hipLaunchKernelGGL(k_cal_rowerr<NC>, dim3((unsigned)T), dim3(kThreads), lds, st, xp, T, K, log2h, inv_sqrt_h, bits,
                       n_grid, gamma_min, ws);
    hipLaunchKernelGGL(k_cal_pick, dim3(1), dim3(kMaxGrid), 0, st, ws, T, n_grid, inv_sqrt_h, bits, gamma_min, result);
    return hip_status(hipGetLastError());
}

}  // namespace

int max_calibration_grid() { return kMaxGrid; }

int launch_calibrate(const void* x, int64_t T, int64_t K, int32_t h, int32_t bits, int32_t n_grid, float gamma_min,
                     float* result, float* ws, hipStream_t st)
{
    if (K > 16 * kChunk || T > 0x7fffffff) return PQ_ERR_UNSUPPORTED;
    int log2h = 0;
    while ((1 << log2h) < h) ++log2h;
    const double inv_sqrt_h = h > 1 ? 1.0 / sqrt((double)h) : 1.0;
    const __half* xp = static_cast<const __half*>(x);
    const int nc = (int)((K + kChunk - 1) / kChunk);
    if (nc <= 1) return launch_cal_nc<1>(xp, T, K, log2h, inv_sqrt_h, bits, n_grid, gamma_min, result, ws, st);
    if (nc <= 2) return launch_cal_nc<2>(xp, T, K, log2h, inv_sqrt_h, bits, n_grid, gamma_min, result, ws, st);
    if (nc <= 4) return launch_cal_nc<4>(xp, T, K, log2h, inv_sqrt_h, bits, n_grid, gamma_min, result, ws, st);
    if (nc <= 8) return launch_cal_nc<8>(xp, T, K, log2h, inv_sqrt_h, bits, n_grid, gamma_min, result, ws, st);
    return launch_cal_nc<16>(xp, T, K, log2h, inv_sqrt_h, bits, n_grid, gamma_min, result, ws, st);
}

int launch_calibrate_zp(const void* x, int64_t T, int64_t K, int32_t h, int32_t ng, int32_t nb, float gamma_min,
                        float beta_min, float* result, float* ws, hipStream_t st)
{
    if (K > 16 * kChunk || T > 0x7fffffff) return PQ_ERR_UNSUPPORTED;
    int log2h = 0;
    while ((1 << log2h) < h) ++log2h;
    const double inv_sqrt_h = h > 1 ? 1.0 / sqrt((double)h) : 1.0;
    const __half* xp = static_cast<const __half*>(x);
    const int nc = (int)((K + kChunk - 1) / kChunk);
    if (nc <= 1) return launch_cal_zp_nc<1>(xp, T, K, log2h, inv_sqrt_h, ng, nb, gamma_min, beta_min, result, ws, st);
    if (nc <= 2) return launch_cal_zp_nc<2>(xp, T, K, log2h, inv_sqrt_h, ng, nb, gamma_min, beta_min, result, ws, st);
    if (nc <= 4) return launch_cal_zp_nc<4>(xp, T, K, log2h, inv_sqrt_h, ng, nb, gamma_min, beta_min, result, ws, st);
    if (nc <= 8) return launch_cal_zp_nc<8>(xp, T, K, log2h, inv_sqrt_h, ng, nb, gamma_min, beta_min, result, ws, st);
    return launch_cal_zp_nc<16>(xp, T, K, log2h, inv_sqrt_h, ng, nb, gamma_min, beta_min, result, ws, st);
}

}  // namespace pq
