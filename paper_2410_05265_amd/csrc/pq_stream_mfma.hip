// Weight-streaming product for a few tokens (M <= 16) on the matrix cores: the packed weight
// matrix is read from HBM exactly once and nothing else matters at these shapes (Sec. 3 of the
// paper: weight quantization speeds up memory-bound computation; Sec. 5.4, decoding column).
//
// One workgroup of 16 wavefronts per CU.  A "row group" is 16 consecutive output channels; a
// task is 16 / S row groups, and the wavefronts of the workgroup split K of each into S slices (as
// few as leave enough tasks for the chip), so that every wavefront has the same few loads.
//   - Memory side: a "unit" is 16 rows x 128 contiguous bytes, fetched by two wavefront-loads of
//     8 rows each (lane l: row l / 8, bytes 16 (l % 8) ..): every request is a whole 128-byte
//     line (half lines measured 20 % slower).  A ring of DEPTH units per lane stays in flight
//     across tasks.  Every load is unconditional (slots without work re-read the wavefront's
//     first unit), so the compiler counts outstanding loads exactly and a unit is consumed as soon
//     as it has arrived.
//   - Matrix side: v_mfma_i32_16x16x64_i8 wants lane 16 g + i to hold row i, bytes 16 g .. of a
//     64-byte block.  Two lane-shifted moves interleave the two loads so that one register set holds
//     the first 64-byte block of all 16 rows and another the second, and the transpose to the
//     matrix layout is then the same four ds_bpermute_b32 for either.
//   - The activation codes (given; 4-bit packed or int8 in the even/odd-grouped order) are staged
//     once per workgroup in LDS, token rows padded by 16 bytes, which makes the operand reads
//     (lane 16 g + j: token j, bytes 16 g ..) conflict-free.  Their loads (only the instructions
//     that some lane needs: each one delays the weight stream, loads return in order) go out
//     first, then the first unit of weights; the staging barrier follows at once.  What makes a
//     barrier expensive in this kernel is a wavefront that still waits for the memory pipeline to
//     accept its loads: with the whole ring requested before the barrier that is most of the
//     kernel's duration (measured), with one unit per wavefront it is nothing, and the rest of
//     the ring is requested right behind the barrier.  Tokens >= M read token M - 1 and their
//     columns are never stored.
//   - Both 4-bit operands are expanded to bytes of 16 * code (sum carries 256, shifted out
//     exactly); with int8 activations only the weights are (factor 16).
//   - No barrier after that: a wavefront adds its partial 16 x 16 tile to the row group's tile
//     in LDS with atomic adds, then bumps the tile's counter; the wavefront that finds the counter
//     at S - 1 has the complete sums (every other one finished its adds before its bump, and the
//     LDS executes a wavefront's operations in order) and writes the outputs.  With a barrier
//     per row group every wavefront waits for the slowest load of the workgroup before anything
//     is multiplied.
//     The weight steps and zero-point corrections of the epilogue come through the scalar cache
//     (the row group is uniform over the wavefront), so they never queue behind the weight
//     stream; the first ones are touched early so that the tail of the kernel finds them cached.
//
// v_mfma_i32_16x16x64_i8 layout used (lane l, r = l % 16, g = l / 16):
//   A: row r, bytes k = 16 g .. 16 g + 15;  B: column r, same bytes;  D: register v holds D[4 g + v][r].
#include "pq_internal.h"

#include <hip/hip_fp16.h>

namespace pq {
namespace {

constexpr int kTiles = 16;                      // row-group tiles of partial sums open at a time
constexpr int kSumBytes = kTiles * 1024 + 64;   // the tiles and their counters
constexpr int kXB = 8;                          // 16-byte pieces of activation codes a lane requests up front
constexpr int kEarly = 1;                       // units a wavefront requests before the staging barrier (2 and 4 measured slower)

typedef __attribute__((address_space(3))) v4i* lds_v4;
typedef __attribute__((address_space(3))) const v4i* lds_cv4;
typedef __attribute__((address_space(3))) int* lds_i;

__device__ __forceinline__ void lds_sync() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// lanes 4-7 and 12-15 of every 16 take `b` from four lanes below, the others keep `a`
__device__ __forceinline__ int low_blocks(int a, int b) { return __builtin_amdgcn_update_dpp(a, b, 0x114, 0xF, 0xA, false); }
// lanes 0-3 and 8-11 of every 16 take `a` from four lanes above, the others keep `b`
__device__ __forceinline__ int high_blocks(int a, int b) { return __builtin_amdgcn_update_dpp(b, a, 0x104, 0xF, 0x5, false); }

// this lane's group of four channels (g = lane / 16) out of the row group's sixteen
template <typename V>
__device__ __forceinline__ V pick4(const V s0, const V s1, const V s2, const V s3, int g)
{
    V r;
    r.x = g & 2 ? (g & 1 ? s3.x : s2.x) : (g & 1 ? s1.x : s0.x);
    r.y = g & 2 ? (g & 1 ? s3.y : s2.y) : (g & 1 ? s1.y : s0.y);
    r.z = g & 2 ? (g & 1 ? s3.z : s2.z) : (g & 1 ? s1.z : s0.z);
    r.w = g & 2 ? (g & 1 ? s3.w : s2.w) : (g & 1 ? s1.w : s0.w);
    return r;
}

// DEPTH: units (2 x 16 bytes per lane) a lane keeps in flight; the launcher picks the smallest
// that covers a wavefront's units, so that no slot of the ring is loaded without being used
// except in a workgroup's last round.
template <int ABITS, int DEPTH>
__global__ __launch_bounds__(1024) void k_stream_mfma(const uint8_t* __restrict__ xq, const uint8_t* __restrict__ wq,
                                                    const float* __restrict__ sw, float sx, int M, int N, int K,
                                                    int log2S, __half* __restrict__ out,
                                                    int32_t* __restrict__ acc_out, const float* __restrict__ srow,
                                                    const int32_t* __restrict__ zcorr)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // sums and counters start at zero (the staging barrier below orders this before the first add)
    lds_i counters = (lds_i)(smem + kTiles * 1024);
    auto clear = [&]() {
        ((lds_v4)smem)[tid] = (v4i){0, 0, 0, 0};
        if (tid < 16) counters[tid] = 0;
    };
    clear();

    const int Kb = K >> 1;
    const int Ka = ABITS == 8 ? K : Kb;     // bytes per row of activation codes
    const int S = 1 << log2S;               // slices of K per row group
    const int RG = 16 >> log2S;             // row groups per task
    const int P = Kb >> 7;                  // units (128 bytes) per weight row
    const int upt = (P + S - 1) >> log2S;   // units per slice = per task (the same for every wavefront)
    const int q = wave >> log2S, s = wave & (S - 1);
    const int p0 = s * upt;
    const int p1 = p0 + upt < P ? p0 + upt : P;      // this wavefront's units: [p0, p1), possibly empty
    const int R = N >> 4;
    const int T = (R + RG - 1) / RG;
    const int my_tasks = (int)blockIdx.x < T ? (T - 1 - (int)blockIdx.x) / (int)gridDim.x + 1 : 0;
    const int tpe = kTiles >> (4 - log2S);   // tasks per epoch: their tiles fit in LDS together
    const int r = lane & 15, g = lane >> 4;
    // this lane's token step (the load is unconditional so that outstanding loads can be counted)
    const float tstep = (srow ? srow : sw)[srow ? (r < M ? r : M - 1) : 0];

    // ---- every token's codes go to LDS, rows padded by 16 bytes (conflict-free operand reads).
    // The first kXB pieces per lane are requested before any weight (loads complete in order, so
    // they can be waited for without waiting for weights); a wavefront none of whose lanes has a
    // piece issues no load, since each one delays the weight stream.
    const int xstride = Ka + 16;
    uint8_t* xs = smem + kSumBytes;
    const int ppr = Ka >> 4, pieces = M * ppr;       // 16-byte pieces per row, in all
    v4i xr[kXB];
#pragma unroll
    for (int u = 0; u < kXB; ++u) {
        const int i = tid + 1024 * u;
        xr[u] = (v4i){0, 0, 0, 0};
        if (wave * 64 + 1024 * u < pieces) xr[u] = *reinterpret_cast<const v4i*>(xq + (int64_t)(i < pieces ? i : 0) * 16);
    }

    // ---- ring of weight loads: the first kEarly units now, the others behind the staging barrier
    v4i w[DEPTH][2];
    const uint8_t* wlane = wq + (int64_t)(lane >> 3) * Kb + (lane & 7) * 16;
    // a slot without work re-reads this wavefront's first unit (in bounds, and its own cache lines)
    const int64_t idle_off = ((int)blockIdx.x * RG + q < R && p0 < p1)
                                 ? (int64_t)((int)blockIdx.x * RG + q) * 16 * Kb + p0 * 128 : 0;
    auto issue = [&](int d, int task, int b) {
        const int rg = ((int)blockIdx.x + task * (int)gridDim.x) * RG + q;
        const bool valid = task < my_tasks && rg < R && p0 + b < p1;
        const uint8_t* base = wlane + (valid ? (int64_t)rg * 16 * Kb + (p0 + b) * 128 : idle_off);
        w[d][0] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(base));
        w[d][1] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(base + 8 * (int64_t)Kb));
    };
    constexpr int EARLY = DEPTH < kEarly ? DEPTH : kEarly;
    int it = 0, ib = 0;   // task and unit of the next load
#pragma unroll
    for (int d = 0; d < EARLY; ++d) {
        issue(d, it, ib);
        if (++ib == upt) { ib = 0; ++it; }
    }

    auto put = [&](int i, const v4i v) {
        if (i < pieces) {
            const int row = i / ppr, col = i - row * ppr;
            *(lds_v4)(xs + row * xstride + col * 16) = v;
        }
    };
#pragma unroll
    for (int u = 0; u < kXB; ++u) put(tid + 1024 * u, xr[u]);
    for (int i = tid + 1024 * kXB; i < pieces; i += 1024)   // very long rows: the rest waits behind the early weights
        put(i, *reinterpret_cast<const v4i*>(xq + (int64_t)i * 16));
    // the only barrier (apart from tile reuse): one unit per wavefront is in flight, so no
    // wavefront is still waiting for the memory pipeline to accept its loads
    lds_sync();
#pragma unroll
    for (int d = EARLY; d < DEPTH; ++d) {
        issue(d, it, ib);
        if (++ib == upt) { ib = 0; ++it; }
    }
    // the weight steps of this workgroup's first row groups, fetched once now so that the scalar
    // loads of the epilogue (the tail of the kernel) find them in the cache
    float warm = 0.f;
    {
        const int task = wave >> (4 - log2S), rgw = ((int)blockIdx.x + task * (int)gridDim.x) * RG + (wave & (RG - 1));
        if (task < my_tasks && rgw < R) warm = sw[rgw * 16];
    }
    const float st = srow ? tstep : sx;
    asm volatile("" ::"s"(warm));

    // ---- units in order; a task ends with this wavefront's contribution to the row group's tile
    // lane 16 g + i of the matrix operand takes (row i, block piece g) from the lane that holds it
    // after the interleave: rows 0-7 at lanes 8 i + g, rows 8-15 at lanes 8 (i - 8) + 4 + g
    const int src = (8 * (r & 7) + 4 * (r >> 3) + g) * 4;
    const uint8_t* xlane = xs + (r < M ? r : M - 1) * xstride + g * (ABITS == 8 ? 32 : 16);
    v4i acc = {0, 0, 0, 0};
    int ct = 0, cb = 0;   // task and unit being consumed
    auto consume = [&](int d) {
        const bool live = ct < my_tasks;   // uniform; slots past the last unit hold nothing
        const int rg = ((int)blockIdx.x + ct * (int)gridDim.x) * RG + q;
        const v4i a = w[d][0], b = w[d][1];
        if (live && rg < R && p0 + cb < p1) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                v4i u, t, we, wo, xe, xo;
                if (kb == 0) {
                    u.x = low_blocks(a.x, b.x); u.y = low_blocks(a.y, b.y);
                    u.z = low_blocks(a.z, b.z); u.w = low_blocks(a.w, b.w);
                } else {
                    u.x = high_blocks(a.x, b.x); u.y = high_blocks(a.y, b.y);
                    u.z = high_blocks(a.z, b.z); u.w = high_blocks(a.w, b.w);
                }
                t.x = __builtin_amdgcn_ds_bpermute(src, u.x);
                t.y = __builtin_amdgcn_ds_bpermute(src, u.y);
                t.z = __builtin_amdgcn_ds_bpermute(src, u.z);
                t.w = __builtin_amdgcn_ds_bpermute(src, u.w);
                unpack16(t, we, wo);
                const int p = p0 + cb;
                if constexpr (ABITS == 8) {
                    xe = *(lds_cv4)(xlane + p * 256 + kb * 128);
                    xo = *(lds_cv4)(xlane + p * 256 + kb * 128 + 16);
                } else {
                    const v4i xv = *(lds_cv4)(xlane + p * 128 + kb * 64);
                    unpack16(xv, xe, xo);
                }
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(we, xe, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wo, xo, acc, 0, 0, 0);
            }
        }
        if (live && ++cb == upt) {
            if (rg < R) {
                // this wavefront's share of the row group's sums; register v of lane l at word 4 l + v
                const int tile = (ct % tpe) * RG + q;
                lds_i sums = (lds_i)smem + tile * 256 + lane * 4;
                __hip_atomic_fetch_add(sums + 0, acc.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                __hip_atomic_fetch_add(sums + 1, acc.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                __hip_atomic_fetch_add(sums + 2, acc.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                __hip_atomic_fetch_add(sums + 3, acc.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the adds are done before the counter moves
                int before = 0;
                if (lane == 0)
                    before = __hip_atomic_fetch_add(counters + tile, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                before = __builtin_amdgcn_readfirstlane(before);
                if (before == S - 1) {
                    // last one in: the tile is complete.  Lane (token r, channels 4 g .. 4 g + 3)
                    asm volatile("" ::: "memory");
                    v4i sum = *(lds_cv4)(sums);
                    const float4* sp = reinterpret_cast<const float4*>(sw + rg * 16);   // uniform address
                    const float4 sc = pick4(sp[0], sp[1], sp[2], sp[3], g);
                    v4i zc = {0, 0, 0, 0};
                    if (zcorr) {
                        const v4i* zp = reinterpret_cast<const v4i*>(zcorr + rg * 16);
                        zc = pick4(zp[0], zp[1], zp[2], zp[3], g);
                    }
                    constexpr int SH = ABITS == 8 ? 4 : 8;
                    sum.x >>= SH; sum.y >>= SH; sum.z >>= SH; sum.w >>= SH;
                    if (r < M) {
                        const int64_t o = (int64_t)r * N + rg * 16 + 4 * g;
                        if (acc_out) *reinterpret_cast<v4i*>(acc_out + o) = sum;
                        if (out) {
                            sum.x += zc.x; sum.y += zc.y; sum.z += zc.z; sum.w += zc.w;   // correction of Eq. 1, if any
                            const __half2 lo = __floats2half2_rn(mul_rn((float)sum.x, st * sc.x),
                                                                 mul_rn((float)sum.y, st * sc.y));
                            const __half2 hi = __floats2half2_rn(mul_rn((float)sum.z, st * sc.z),
                                                                 mul_rn((float)sum.w, st * sc.w));
                            uint2 pk;
                            pk.x = *reinterpret_cast<const uint32_t*>(&lo);
                            pk.y = *reinterpret_cast<const uint32_t*>(&hi);
                            *reinterpret_cast<uint2*>(out + o) = pk;
                        }
                    }
                }
            }
            acc = (v4i){0, 0, 0, 0};
            cb = 0;
            ++ct;
            if (ct % tpe == 0 && ct < my_tasks) {   // uniform over the workgroup: the tiles are reused
                lds_sync();
                clear();
                lds_sync();
            }
        }
    };
    const int rounds = (my_tasks * upt + DEPTH - 1) / DEPTH;
    for (int rnd = 1; rnd < rounds; ++rnd) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            consume(d);
            issue(d, it, ib);
            if (++ib == upt) { ib = 0; ++it; }
        }
    }
    if (rounds > 0) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) consume(d);
    }
}

}  // namespace

// M <= 16 tokens of given codes (abits 4: packed; 8: grouped bytes), K a multiple of 256 up to 65536,
// N a multiple of 16, and the codes of half the tokens fit in LDS beside the tiles of sums
namespace {
// slices of K per row group (log2), units per slice and LDS bytes of a launch
void stream_plan(int64_t M, int64_t N, int64_t K, int32_t abits, int* log2S, int* upt, size_t* lds)
{
    const int P = (int)(K / 256);   // units of 128 bytes per weight row
    const int64_t R = N / 16;
    int lmax = 2;                   // at least 4 slices, at most one per unit, at most 16
    while (lmax < 4 && (2 << lmax) <= P) ++lmax;
    // as few slices as leave enough tasks for the chip: a task then covers more row groups, a
    // workgroup runs through fewer of them, and every task ends with a round of atomics and an
    // epilogue (measured at 14336 x 4096: 4 slices 8.3 us, 8 slices 8.8, 16 slices 9.5)
    int l2 = 2;
    while (l2 < lmax && (R + (16 >> l2) - 1) / (16 >> l2) < 176) ++l2;
    *log2S = l2;
    *upt = (P + (1 << l2) - 1) >> l2;
    *lds = (size_t)kSumBytes + (size_t)M * ((abits == 8 ? K : K / 2) + 16);
}
}  // namespace

namespace {
bool fits_in_lds(int64_t M, int64_t N, int64_t K, int32_t abits)
{
    int log2S, upt;
    size_t lds;
    stream_plan(M, N, K, abits, &log2S, &upt, &lds);
    return lds <= 160 * 1024;
}

int launch_tokens(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K, void* out,
                  int32_t* acc, hipStream_t st, const float* srow, int32_t abits, const int32_t* zcorr)
{
    int log2S, upt;
    size_t lds;
    stream_plan(M, N, K, abits, &log2S, &upt, &lds);
    const int RG = 16 >> log2S;
    const int64_t T = (N / 16 + RG - 1) / RG;
    const unsigned grid = (unsigned)(T < 256 ? T : 256);
    // units a wavefront has at most: the ring is as deep as that, up to 4
    const int64_t units = ((T + grid - 1) / grid) * upt;
    auto launch = [&](auto kern) {
        static std::atomic<uint64_t> lds_ok{0};
        if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), 160 * 1024, lds_ok) != PQ_OK) return (int)PQ_ERR_HIP;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(1024), lds, st, static_cast<const uint8_t*>(xq),
                           static_cast<const uint8_t*>(wq), sw, sx, (int)M, (int)N, (int)K, log2S,
                           static_cast<__half*>(out), acc, srow, zcorr);
        return hip_status(hipGetLastError());
    };
    if (abits == 8) {
        if (units <= 1) return launch(k_stream_mfma<8, 1>);
        if (units <= 2) return launch(k_stream_mfma<8, 2>);
        return launch(k_stream_mfma<8, 4>);
    }
    if (units <= 1) return launch(k_stream_mfma<4, 1>);
    if (units <= 2) return launch(k_stream_mfma<4, 2>);
    return launch(k_stream_mfma<4, 4>);
}
}  // namespace

// The kernel takes up to 16 tokens whose codes fit in LDS together.  Up to 32 tokens, or tokens whose
// codes do not fit, go in several launches (blocks of 16 tokens, halved where they do not fit): the
// weights are then streamed once per launch; the caller weighs that against the tiled kernel, whose
// few tiles walk K one after the other (stream_mfma_launches says how many launches it would be).
bool stream_mfma_supported(int64_t M, int64_t N, int64_t K, int32_t abits)
{
    if (!(M >= 1 && M <= 32 && N >= 16 && (N % 16) == 0 && N <= (1 << 30) && K >= 256 && (K % 256) == 0 && K <= 65536))
        return false;
    const int64_t block = M < 16 ? M : 16;
    return fits_in_lds((block + 1) / 2, N, K, abits);
}

// Launches launch_stream_mfma makes for a supported shape (each streams the whole matrix).
int stream_mfma_launches(int64_t M, int64_t N, int64_t K, int32_t abits)
{
    if (M <= 16 && fits_in_lds(M, N, K, abits)) return 1;
    const int64_t m1 = M > 16 ? 16 : (M + 1) / 2;
    return stream_mfma_launches(m1, N, K, abits) + stream_mfma_launches(M - m1, N, K, abits);
}

int launch_stream_mfma(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
                       void* out, int32_t* acc, hipStream_t st, const float* srow, int32_t abits,
                       const int32_t* zcorr)
{
    if (!stream_mfma_supported(M, N, K, abits)) return PQ_ERR_UNSUPPORTED;
    if (M <= 16 && fits_in_lds(M, N, K, abits))
        return launch_tokens(xq, wq, sw, sx, M, N, K, out, acc, st, srow, abits, zcorr);
    // first part: 16 tokens of more than 16, else the first half
    const int64_t m1 = M > 16 ? 16 : (M + 1) / 2, ka = abits == 8 ? K : K / 2;
    int rc = launch_stream_mfma(xq, wq, sw, sx, m1, N, K, out, acc, st, srow, abits, zcorr);
    if (rc != PQ_OK) return rc;
    return launch_stream_mfma(static_cast<const uint8_t*>(xq) + m1 * ka, wq, sw, sx, M - m1, N, K,
                              out ? static_cast<__half*>(out) + m1 * N : nullptr, acc ? acc + m1 * N : nullptr, st,
                              srow ? srow + m1 : nullptr, abits, zcorr);
}

}  // namespace pq
