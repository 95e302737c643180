// Tiled 4-bit x 4-bit product on the CDNA4 INT8 matrix pipe, with the dequantising
// epilogue (Sec. 3 of the paper: weight + activation quantization enable low-bit matrix
// multiplication for the compute-bound prefill; Table 1 row O2: per-tensor activation
// step, per-channel weight step).
//
//   acc[m,n] = sum_k xq[m,k] * wq[n,k]        out[m,n] = fp16(acc * (s_x * s_w[n]))
//
// Both operands are K-contiguous, which is what the matrix instruction wants: every lane
// feeds 16 consecutive bytes of one row.  Packed nibbles are loaded from HBM with 16-byte
// loads (64 contiguous bytes per row per stage), expanded ONCE per workgroup to int8 in
// registers and written to LDS; the wavefronts then read ready-made operands.  The
// expansion produces 16*code (the odd-channel nibble is already in the high half of its
// byte, the even-channel nibble is shifted there), so no sign extension is needed; the
// accumulator becomes 256 * acc and is shifted back exactly.  A dot product does not care
// about the order of its terms as long as both operands use the same order, so the even
// and the odd channels of a 32-channel group simply feed two different matrix steps.
//
// v_mfma_i32_32x32x32_i8 operand layout (lane l, r = l % 32, g = l / 32):
//   A: row r of the 32 x 32 tile, bytes k = 16 g .. 16 g + 15;  B: column r, same bytes;
//   D: register v holds D[8 (v / 4) + 4 g + v % 4][r].
//
// LDS layout of one K stage (128 channels = 64 packed bytes = 4 packed 16-byte chunks c per
// row, 4 matrix steps s): for every 32-row fragment and every step one 1 KiB block that is
// read linearly, lane l taking bytes [16 l, 16 l + 16) up to an XOR on the row slot:
//   step s uses chunk c = 2 (s / 2) + g, its even channels if s is even, else its odd ones;
//   block offset = g * 512 + ((r ^ 4 c) * 16).
// The XOR keeps the 16-byte stores of the loader (4 lanes per row, one chunk each)
// spread over all banks; the reads stay a permutation inside aligned groups of 16 lanes.
#include "pq_internal.h"

#include <hip/hip_fp16.h>
#include <stdlib.h>

namespace pq {
namespace {

// Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous run of
// tiles so that the tiles sharing a weight panel hit the same L2.
__device__ __forceinline__ int xcd_remap(int b, int total)
{
    const int x = b & 7, idx = b >> 3;
    const int q = total >> 3, rem = total & 7;
    return x * q + (x < rem ? x : rem) + idx;
}

// LDS-only barrier: wait for this wave's LDS traffic, then meet the other waves.  Global
// loads that are still in flight stay in flight.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int BM, int BN, int WR, int WC>
__global__ __launch_bounds__(WR * WC * 64) void k_gemm_i8(const uint8_t* __restrict__ xq,
                                                         const uint8_t* __restrict__ wq,
                                                         const float* __restrict__ sw, float sx, int M, int N,
                                                         int K, int GM, __half* __restrict__ out,
                                                         int32_t* __restrict__ acc_out)
{
    constexpr int NT = WR * WC * 64;
    constexpr int WM = BM / WR, WN = BN / WC, TM = WM / 32, TN = WN / 32;
    constexpr int FA = BM / 32, FB = BN / 32;
    constexpr int A_BYTES = FA * 4096, STAGE = (FA + FB) * 4096;
    constexpr int RPP = NT / 4;  // rows covered by one loader pass (4 lanes per row)
    constexpr int LA = BM / RPP, LB = BN / RPP, L = LA + LB;
    static_assert(BM % RPP == 0 && BN % RPP == 0 && RPP % 32 == 0, "loader shape");
    extern __shared__ __align__(16) uint8_t smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WC, wn = wave % WC;
    const int r = lane & 31, g = lane >> 5;

    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int m0 = (tile % GM) * BM, n0 = (tile / GM) * BN;
    const int Kb = K >> 1;
    const int nk = K >> 7;

    // ---- loader: lane -> (row, packed chunk); rows past the end are clamped (their
    // products are computed and never stored)
    const int lc = tid & 3, lrow = tid >> 2;
    const uint8_t* gp[L];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        int row = m0 + lrow + RPP * i;
        row = row < M ? row : M - 1;
        gp[i] = xq + (int64_t)row * Kb + lc * 16;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        int row = n0 + lrow + RPP * i;
        row = row < N ? row : N - 1;
        gp[LA + i] = wq + (int64_t)row * Kb + lc * 16;
    }
    const int wr0 = ((lrow >> 5) * 4 + 2 * (lc >> 1)) * 1024 + (lc & 1) * 512 + (((lrow & 31) ^ (4 * lc)) << 4);
    auto wr_off = [&](int idx) {  // byte offset inside a stage of staged load idx
        return idx < LA ? wr0 + idx * (RPP / 32) * 4096 : A_BYTES + wr0 + (idx - LA) * (RPP / 32) * 4096;
    };
    v4i gr[L];
    auto gload = [&](int idx, int kt) { gr[idx] = *reinterpret_cast<const v4i*>(gp[idx] + kt * 64); };
    auto expand_store = [&](int idx, uint8_t* stage) {
        v4i e, o;
        unpack16(gr[idx], e, o);
        *reinterpret_cast<v4i*>(stage + wr_off(idx)) = e;
        *reinterpret_cast<v4i*>(stage + wr_off(idx) + 1024) = o;
    };

    // ---- reader offsets (two values: steps 0-1 use chunks 0/1, steps 2-3 chunks 2/3)
    const int rd0 = g * 512 + ((r ^ (4 * g)) << 4);
    const int rd1 = g * 512 + ((r ^ (4 * (2 + g))) << 4);
    const int a_base = wm * TM * 4096, b_base = A_BYTES + wn * TN * 4096;

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    v4i fa[2][TM], fb[2][TN];
    auto read_frags = [&](const uint8_t* stage, int s, int set) {
        const int off = (s >> 1) ? rd1 : rd0;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[set][i] = *reinterpret_cast<const v4i*>(stage + a_base + (i * 4 + s) * 1024 + off);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[set][j] = *reinterpret_cast<const v4i*>(stage + b_base + (j * 4 + s) * 1024 + off);
    };
    auto mfma_step = [&](int set) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
    };

    // ---- prologue: stage 0 into buffer 0, stage 1 into the staging registers
#pragma unroll
    for (int idx = 0; idx < L; ++idx) gload(idx, 0);
#pragma unroll
    for (int idx = 0; idx < L; ++idx) expand_store(idx, smem);
    {
        const int k1 = nk > 1 ? 1 : 0;
#pragma unroll
        for (int idx = 0; idx < L; ++idx) gload(idx, k1);
    }
    lds_barrier();
    read_frags(smem, 0, 0);

    for (int kt = 0; kt < nk; ++kt) {
        uint8_t* cur = smem + (kt & 1) * STAGE;
        uint8_t* nxt = smem + ((kt & 1) ^ 1) * STAGE;
        const int k2 = (kt + 2 < nk) ? kt + 2 : nk - 1;
        // steps 0..2: operands of the next step are fetched while this step multiplies;
        // a third of the staged stage kt+1 is expanded into the other buffer per step and
        // its registers are refilled with stage kt+2
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            read_frags(cur, s + 1, (s + 1) & 1);
            mfma_step(s & 1);
#pragma unroll
            for (int idx = 0; idx < L; ++idx)
                if (idx % 3 == s) {
                    expand_store(idx, nxt);
                    gload(idx, k2);
                }
        }
        lds_barrier();  // stage kt+1 complete in nxt; nobody reads cur any more
        read_frags(nxt, 0, 0);
        mfma_step(1);
    }

    // ---- epilogue: lane owns column n = ... + r and 16 rows per 32 x 32 tile
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

// ---------------------------------------------------------------------------------------
// Generic variant for K % 128 != 0: nibbles stay packed in LDS and are expanded per
// wavefront after the read; loads are predicated so that a ragged last stage is zero.
constexpr int kRowBytes = 64;

__device__ __forceinline__ int swz(int row) { return ((row >> 1) ^ (row >> 3)) & 3; }

template <int BM, int BN, int WR, int WC>
__global__ __launch_bounds__(256) void k_gemm_ragged(const uint8_t* __restrict__ xq, const uint8_t* __restrict__ wq,
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
int launch_i8(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K, void* out,
              int32_t* acc, hipStream_t st)
{
    const int GM = (int)((M + BM - 1) / BM), GN = (int)((N + BN - 1) / BN);
    constexpr size_t lds = 2 * (size_t)(BM + BN) * 128;
    auto kern = k_gemm_i8<BM, BN, WR, WC>;
    static bool attr_set = false;  // benign race: the call is idempotent
    if (lds > 48 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return PQ_ERR_HIP;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(GM * GN)), dim3(WR * WC * 64), lds, st,
                       static_cast<const uint8_t*>(xq), static_cast<const uint8_t*>(wq), sw, sx, (int)M, (int)N,
                       (int)K, GM, static_cast<__half*>(out), acc);
    return hip_status(hipGetLastError());
}

int launch_ragged(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
                  void* out, int32_t* acc, hipStream_t st)
{
    constexpr int BM = 128, BN = 128;
    const int GM = (int)((M + BM - 1) / BM), GN = (int)((N + BN - 1) / BN);
    const size_t lds = 2 * (size_t)(BM + BN) * kRowBytes;
    hipLaunchKernelGGL((k_gemm_ragged<BM, BN, 2, 2>), dim3((unsigned)(GM * GN)), dim3(256), lds, st,
                       static_cast<const uint8_t*>(xq), static_cast<const uint8_t*>(wq), sw, sx, (int)M, (int)N,
                       (int)K, GM, static_cast<__half*>(out), acc);
    return hip_status(hipGetLastError());
}

struct TileCfg { int bm, bn; double eff; };
// relative efficiency guesses per tile (larger wave tiles need fewer LDS reads per multiply)
constexpr int kNumCfg = 4;
constexpr TileCfg kCfgs[kNumCfg] = {{256, 256, 1.00}, {256, 128, 0.92}, {128, 128, 0.80}, {256, 256, 1.0}};

int pick_cfg(int64_t M, int64_t N)
{
    if (const char* f = getenv("PQ_GEMM_TILE")) {
        const int v = atoi(f);
        if (v >= 0 && v < kNumCfg) return v;
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
    if (K % 128 != 0) return launch_ragged(xq, wq, sw, sx, M, N, K, out, acc, st);
    switch (pick_cfg(M, N)) {
        case 0: return launch_i8<256, 256, 2, 2>(xq, wq, sw, sx, M, N, K, out, acc, st);
        case 1: return launch_i8<256, 128, 2, 2>(xq, wq, sw, sx, M, N, K, out, acc, st);
        case 2: return launch_i8<128, 128, 2, 2>(xq, wq, sw, sx, M, N, K, out, acc, st);
        default: return launch_i8<256, 256, 2, 4>(xq, wq, sw, sx, M, N, K, out, acc, st);
    }
}

}  // namespace pq
