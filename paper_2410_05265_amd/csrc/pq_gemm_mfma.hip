// Tiled 4-bit x 4-bit product on the CDNA4 INT8 matrix pipe, with the dequantising
// epilogue (Sec. 3 of the paper: weight + activation quantization enable low-bit matrix
// multiplication for the compute-bound prefill; Table 1 row O2: per-tensor activation
// step, per-channel weight step).
//
//   acc[m,n] = sum_k xq[m,k] * wq[n,k]        out[m,n] = fp16(acc * (s_x * s_w[n]))
//
// Both operands are K-contiguous ("row" x "row"), which is what the matrix instruction
// wants: every lane feeds 16 consecutive bytes of one row.  Packed nibbles travel
// HBM -> registers -> LDS unchanged (half the LDS traffic of int8); a lane reads 16 packed
// bytes (32 channels) back and expands them in registers into two operands holding
// 16*code: the even channels and the odd channels.  A dot product does not care about the
// order of its terms as long as both operands use the same order, so "evens, then odds"
// needs no interleave.  The accumulator ends up as 256 * acc and is shifted back exactly.
//
// v_mfma_i32_32x32x32_i8 operand layout used here (lane l, r = l % 32, g = l / 32):
//   A: row r of the 32 x 32 tile, bytes k = 16 g .. 16 g + 15
//   B: column r, same bytes
//   D: register v holds D[8 (v / 4) + 4 g + v % 4][r]
#include "pq_internal.h"

#include <hip/hip_fp16.h>
#include <stdlib.h>

namespace pq {
namespace {

constexpr int kRowBytes = 64;  // packed bytes per tile row per K stage (128 channels)

__device__ __forceinline__ int swz(int row) { return ((row >> 1) ^ (row >> 3)) & 3; }

// Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous run of
// tiles so that the tiles sharing a weight panel hit the same L2.
__device__ __forceinline__ int xcd_remap(int b, int total)
{
    const int x = b & 7, idx = b >> 3;
    const int q = total >> 3, rem = total & 7;
    return x * q + (x < rem ? x : rem) + idx;
}

template <int BM, int BN, int WR, int WC>
__global__ __launch_bounds__(256) void k_gemm_mfma(const uint8_t* __restrict__ xq, const uint8_t* __restrict__ wq,
                                                 const float* __restrict__ sw, float sx, int M, int N, int K,
                                                 int GM, __half* __restrict__ out, int32_t* __restrict__ acc_out)
{
    static_assert(WR * WC == 4, "four wavefronts");
    constexpr int WM = BM / WR, WN = BN / WC, TM = WM / 32, TN = WN / 32;
    constexpr int LA = BM / 64, LB = BN / 64;
    constexpr int A_STAGE = BM * kRowBytes, STAGE = (BM + BN) * kRowBytes;
    extern __shared__ __align__(16) uint8_t smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WC, wn = wave % WC;
    const int r = lane & 31, g = lane >> 5;

    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int m0 = (tile % GM) * BM, n0 = (tile / GM) * BN;
    const int Kb = K >> 1;
    const int nk = (Kb + kRowBytes - 1) / kRowBytes;

    // loader: 4 threads per row, 64 rows per pass
    const int lc = tid & 3, lr = tid >> 2;
    const int wr_off = lr * kRowBytes + ((lc ^ swz(lr)) << 4);
    v4i ga[LA], gb[LB];

    auto load_stage = [&](int kt) {
        const int boff = kt * kRowBytes + lc * 16;
        const bool kin = boff < Kb;
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int row = m0 + lr + 64 * i;
            ga[i] = (v4i){0, 0, 0, 0};
            if (kin && row < M) ga[i] = *reinterpret_cast<const v4i*>(xq + (int64_t)row * Kb + boff);
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int row = n0 + lr + 64 * i;
            gb[i] = (v4i){0, 0, 0, 0};
            if (kin && row < N) gb[i] = *reinterpret_cast<const v4i*>(wq + (int64_t)row * Kb + boff);
        }
    };
    auto store_stage = [&](int buf) {
        uint8_t* base = smem + buf * STAGE;
#pragma unroll
        for (int i = 0; i < LA; ++i) *reinterpret_cast<v4i*>(base + wr_off + i * 64 * kRowBytes) = ga[i];
#pragma unroll
        for (int i = 0; i < LB; ++i) *reinterpret_cast<v4i*>(base + A_STAGE + wr_off + i * 64 * kRowBytes) = gb[i];
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    const int sz = swz(r);
    const int a_rd = (wm * WM + r) * kRowBytes;
    const int b_rd = A_STAGE + (wn * WN + r) * kRowBytes;

    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) load_stage(kt + 1);
        const uint8_t* base = smem + (kt & 1) * STAGE;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int coff = ((kk * 2 + g) ^ sz) << 4;
            v4i ae[TM], ao[TM], be[TN], bo[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                unpack16(*reinterpret_cast<const v4i*>(base + a_rd + i * 32 * kRowBytes + coff), ae[i], ao[i]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                unpack16(*reinterpret_cast<const v4i*>(base + b_rd + j * 32 * kRowBytes + coff), be[j], bo[j]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ae[i], be[j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ao[i], bo[j], acc[i][j], 0, 0, 0);
                }
        }
        if (kt + 1 < nk) store_stage((kt + 1) & 1);
        __syncthreads();
    }

    // epilogue: lane owns column n = ... + r and 16 rows per 32 x 32 tile
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WN + j * 32 + r;
        if (n >= N) continue;
        const float sc = sx * sw[n];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * WM + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                if (m < M) {
                    const int a = acc[i][j][v] >> 8;
                    if (acc_out) acc_out[(int64_t)m * N + n] = a;
                    if (out) out[(int64_t)m * N + n] = __float2half_rn((float)a * sc);
                }
            }
        }
    }
}

template <int BM, int BN, int WR, int WC>
int launch_cfg(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
               void* out, int32_t* acc, hipStream_t st)
{
    const int GM = (int)((M + BM - 1) / BM), GN = (int)((N + BN - 1) / BN);
    const size_t lds = 2 * (size_t)(BM + BN) * kRowBytes;
    auto kern = k_gemm_mfma<BM, BN, WR, WC>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return PQ_ERR_HIP;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(GM * GN)), dim3(256), lds, st, static_cast<const uint8_t*>(xq),
                       static_cast<const uint8_t*>(wq), sw, sx, (int)M, (int)N, (int)K, GM,
                       static_cast<__half*>(out), acc);
    return hip_status(hipGetLastError());
}

struct TileCfg { int bm, bn; double eff; };
// relative efficiency guesses per tile (larger wave tiles amortise unpacking and LDS reads)
constexpr TileCfg kCfgs[] = {{256, 256, 1.00}, {256, 128, 0.90}, {128, 128, 0.75}};

int pick_cfg(int64_t M, int64_t N)
{
    if (const char* f = getenv("PQ_GEMM_TILE")) {
        const int v = atoi(f);
        if (v >= 0 && v < 3) return v;
    }
    int best = 0;
    double best_cost = 1e300;
    for (int c = 0; c < 3; ++c) {
        const int64_t tiles = ((M + kCfgs[c].bm - 1) / kCfgs[c].bm) * ((N + kCfgs[c].bn - 1) / kCfgs[c].bn);
        const int64_t rounds = (tiles + 255) / 256;
        const double cost = (double)rounds * kCfgs[c].bm * kCfgs[c].bn / kCfgs[c].eff;
        if (cost < best_cost) { best_cost = cost; best = c; }
    }
    return best;
}

}  // namespace

int launch_gemm_mfma(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
                     void* out, int32_t* acc, hipStream_t st)
{
    if (M > (1 << 30) || N > (1 << 30) || K > (1 << 30)) return PQ_ERR_UNSUPPORTED;
    switch (pick_cfg(M, N)) {
        case 0: return launch_cfg<256, 256, 2, 2>(xq, wq, sw, sx, M, N, K, out, acc, st);
        case 1: return launch_cfg<256, 128, 2, 2>(xq, wq, sw, sx, M, N, K, out, acc, st);
        default: return launch_cfg<128, 128, 2, 2>(xq, wq, sw, sx, M, N, K, out, acc, st);
    }
}

}  // namespace pq
