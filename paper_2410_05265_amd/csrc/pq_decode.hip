// Decode in ONE launch of one workgroup per CU: rotate + quantize the few activation rows
// (M <= 4) into LDS, or take given codes (M <= 8; 4-bit packed or 8-bit), and stream the packed
// weight matrix once (Sec. 3 of the paper: weight quantization speeds up memory-bound computation;
// Sec. 5.4, decoding column).  Per-token steps and the zero-point correction of Eq. 1 enter in the
// epilogue when given.
//
// At these sizes a linear is 8-30 MB of weights, i.e. 32-112 KB per CU: the kernel is a single
// burst of loads and its duration is launch + memory latency + bytes / bandwidth, so
//   - the first weight loads of a wavefront (at least four per lane) are issued before anything
//     else happens, the others as soon as the activation rows are staged;
//   - the activation rows are rotated, quantized and packed by every workgroup (= every CU)
//     for itself while those loads are in flight (a second launch would cost more than the
//     redundant arithmetic); rows of up to 32768 channels in all go from the registers they were
//     loaded into straight through the quantizer, 8 to 32 channels per thread;
//   - a wavefront-load is 1 KiB of ONE weight row (lane l: bytes 16 l .. 16 l + 15), the most
//     contiguous access the canonical layout allows;
//   - the products use v_dot8_i32_i4 directly on packed nibbles (no expansion), and the 64
//     per-lane partial sums of each row are folded with a halving butterfly.
#include "pq_rotate.h"

namespace pq {
namespace {

using rq::kChunk;



// Fold V per-lane values over the 64 lanes.  Stage b halves the number of values a lane keeps
// (lanes with bit b clear keep the first half, the others the second half), so the whole
// reduction costs about V + log2(64 / V) exchange-add pairs instead of 6 V.  On return lane l
// holds in v[0] the total of value index bitrev_{log2 V}(l mod V).
template <int V, int B = 0>
__device__ __forceinline__ void fold(int (&v)[V], int lane)
{
    if constexpr (V > 1) {
        const bool up = (lane >> B) & 1;
        int keep[V / 2];
#pragma unroll
        for (int i = 0; i < V / 2; ++i) {
            const int send = up ? v[i] : v[i + V / 2];
            const int mine = up ? v[i + V / 2] : v[i];
            keep[i] = mine + rq::lane_xor_i<B>(send);
        }
        fold<V / 2, B + 1>(keep, lane);
        v[0] = keep[0];
    } else {
        if constexpr (B < 6) {
            int one[1] = {v[0] + rq::lane_xor_i<B>(v[0])};
            fold<1, B + 1>(one, lane);
            v[0] = one[0];
        }
    }
}

__host__ __device__ constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v / 2); }
__device__ __forceinline__ int bitrev(int x, int bits)
{
    int r = 0;
    for (int i = 0; i < bits; ++i) r |= ((x >> i) & 1) << (bits - 1 - i);
    return r;
}

// MODE 0: packed codes are given (xq_in); 1: rows are fp16, quantized with exact ties (log2h == 0)
// or rotated with blocks of 2^log2h <= 2048 first; 2: rotated with blocks of 4096.
// One workgroup of 16 wavefronts per CU; a wavefront owns RPW weight rows at a time and has
// RPW * CB 16-byte loads in flight; MP = padded M.
// ABITS = 8 (given codes only): the activation codes are int8 in the grouped order (16 even
// channels, then 16 odd ones per 32), the weight nibbles are expanded to 16 * code bytes and the
// products are 4-way byte dot products; the sums carry a factor 16, shifted out at the end.
template <int RPW, int CB, int MP, int MODE, int ABITS = 4>
__global__ __launch_bounds__(1024) void k_decode(const __half* __restrict__ x, const uint8_t* __restrict__ xq_in,
                                               const uint8_t* __restrict__ wq, const float* __restrict__ sw,
                                               float sx, float mult, int log2h, int M, int N, int K,
                                               __half* __restrict__ out, int32_t* __restrict__ acc_out,
                                               uint8_t* __restrict__ xq_out, const float* __restrict__ srow,
                                               const int32_t* __restrict__ zcorr, DecodeSecond two)
{
    constexpr int G = MODE == 2 ? 2 : 1;
    static_assert(ABITS == 4 || (ABITS == 8 && MODE == 0), "8-bit activations: given codes only");
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int Kb = K >> 1;
    const int Ka = ABITS == 8 ? K : Kb;   // bytes per row of activation codes
    const int cpr = (Kb + 1023) >> 10;   // KiB chunks per row
    const int groups = N / RPW, gstride = gridDim.x * 16;
    int gid = blockIdx.x * 16 + wave;
    // LDS: [MP][Ka] codes | rotation scratch | [M][K] fp16 rows (fused modes only)
    uint8_t* xs = smem;
    const int xch_off = (MP * Ka + 15) & ~15;
    const int xraw_off = xch_off + (MODE == 0 ? 16 : G * kChunk * 4);

    // ---- 1. first pieces of the activation rows (ordinary loads, issued before the weights:
    // loads complete in order, so waiting for these leaves the weight loads in flight)
    constexpr int XB = 4;   // enough for 32768 channels in all (e.g. one token of 28672); more pieces wait behind the weights
    const uint8_t* xsrc = MODE == 0 ? xq_in : reinterpret_cast<const uint8_t*>(x);
    const int pieces = (MODE == 0 ? M * Ka : M * K * 2) >> 4;   // 16-byte pieces
    uint8_t* xdst = MODE == 0 ? xs : smem + xraw_off;
    v4i xr[XB];
#pragma unroll
    for (int u = 0; u < XB; ++u) {
        const int i = tid + 1024 * u;
        if (u < 2 || 1024 * u < pieces)                                            // (workgroup-uniform)
            xr[u] = *reinterpret_cast<const v4i*>(xsrc + (i < pieces ? i : 0) * 16);   // lanes: clamped, no branch
        else
            xr[u] = (v4i){0, 0, 0, 0};
    }
    // The channel step this lane will need in the epilogue of the wavefront's first row group, requested with the
    // activation rows (branch-free, clamped): asked for after the fold it would put a whole memory latency at the
    // end of a kernel that takes three to seven microseconds.
    constexpr int VV = RPW * MP;
    float sw_first;
    {
        const int idx = bitrev(lane, ilog2(VV));
        int n = gid * RPW + idx / MP;
        n = n < N ? n : N - 1;
        sw_first = *(n >= two.n1 ? two.sw + (n - two.n1) : sw + n);
    }
    __builtin_amdgcn_sched_barrier(0);
    // every wavefront has issued its row loads before any weight load enters the memory pipeline:
    // the rows arrive early and are quantized while the weights stream in
    asm volatile("s_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);

    // ---- 2. weight loads of the first row group (branch-free: lanes past the row's end and
    // wavefronts past the last group read in bounds and are ignored below)
    v4i w[RPW][CB];
    auto load_weights = [&](int g, int cb, int c0 = 0, int c1 = CB) {
        const int gc = g < groups ? g : groups - 1;
#pragma unroll
        for (int j = 0; j < RPW; ++j)
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                if (c < c0 || c >= c1) continue;
                int off = (cb + c) * 1024 + lane * 16;
                off = off < Kb ? off : 0;
                // (two matrices behind one another: a group of RPW rows never straddles them, n1 % 16 == 0)
                const int row = gc * RPW + j;
                const uint8_t* rp = row < two.n1 ? wq + (int64_t)row * Kb : two.wq + (int64_t)(row - two.n1) * Kb;
                w[j][c] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(rp + off));
            }
    };
    // Only the first loads (at least four per lane) go out before the activation rows are staged:
    // the barriers of the staging then come early, while the memory pipeline still accepts loads
    // at once.  With every load issued first, the slowest wavefront gets its last load accepted when
    // most of the matrix has arrived, the barrier behind it holds all products back until then, and
    // they all run in the tail of the kernel (gate_proj, fused linear: 7.7 -> 7.1 us at one token,
    // 10.6 -> 9.5 us at four).
    constexpr int EARLY = (4 + RPW - 1) / RPW < CB ? (4 + RPW - 1) / RPW : CB;
    load_weights(gid, 0, 0, EARLY);
    __builtin_amdgcn_sched_barrier(0);

    // ---- 3. the codes of the activation rows into LDS.
    // Short rows (all pieces in registers already, rotation blocks inside a wavefront: up to 512 channels):
    // every thread rotates and quantizes the pieces it loaded, straight from its registers (lane l of a
    // wavefront holds channels 8 l .. 8 l + 7 of 512 consecutive ones, which is what the register form of
    // the quantizer expects), and writes the packed dword: no staging of the fp16 rows, one barrier.
    // Otherwise: rows into LDS (later pieces, if any, wait behind the weights), then chunk by chunk.
    const bool in_registers = MODE == 1 && log2h <= 9 && pieces <= 1024 * XB;
    if (in_registers) {
        if constexpr (MODE == 1) {
#pragma unroll
            for (int u = 0; u < XB; ++u) {
                const int i = tid + 1024 * u;
                if (1024 * u < pieces) {                      // wavefront-uniform up to the last partial wavefront
                    const v4i raw1[1] = {xr[u]};
                    const bool live1[1] = {i < pieces};
                    auto dst = (rq::lds_u32_ptr)xs;           // piece i -> dword i: rows are contiguous, K / 8 dwords each
                    if (log2h == 0)
                        rq::rotate_quant_regs_with<1, true, 4>(raw1, live1, 0, 0, rq::StaticStep{mult, sx}, dst,
                                                               (rq::lds_f32_ptr) nullptr, i, live1[0]);
                    else
                        rq::rotate_quant_regs_with<1, false, 4>(raw1, live1, 0, log2h, rq::StaticStep{mult, sx}, dst,
                                                                (rq::lds_f32_ptr) nullptr, i, live1[0]);
                }
            }
        }
        rq::lds_sync();
    } else {
#pragma unroll
    for (int u = 0; u < XB; ++u) {
        const int i = tid + 1024 * u;   // pieces past the end land in the (still unused) scratch: no branch
        uint8_t* d = i < pieces ? xdst + i * 16 : smem + xch_off;
        *(__attribute__((address_space(3))) v4i*)d = xr[u];
    }
    for (int base = 1024 * XB; base < pieces; base += 1024 * XB) {
#pragma unroll
        for (int u = 0; u < XB; ++u) {
            const int i = base + tid + 1024 * u;
            xr[u] = *reinterpret_cast<const v4i*>(xsrc + (i < pieces ? i : 0) * 16);
        }
#pragma unroll
        for (int u = 0; u < XB; ++u) {
            const int i = base + tid + 1024 * u;
            uint8_t* d = i < pieces ? xdst + i * 16 : smem + xch_off;
            *(__attribute__((address_space(3))) v4i*)d = xr[u];
        }
    }
    rq::lds_sync();
    if constexpr (MODE != 0) {
        // four groups of 256 threads take chunks in turn; with a cross-wavefront exchange
        // (blocks > 512) the scratch is shared, so only the first group works
        const int sg = wave >> 2, stid = tid & 255;
        const int nch = (K + G * kChunk - 1) / (G * kChunk), items = M * nch;
        const bool serial = log2h > 9;
        for (int it0 = 0; it0 < items; it0 += serial ? 1 : 4) {
            const int it = serial ? it0 : it0 + sg;
            const bool active = serial ? sg == 0 : it < items;
            const int m = active ? it / nch : 0, c = active ? it % nch : 0;
            auto src = (__attribute__((address_space(3))) const __half*)(smem + xraw_off + m * K * 2);
            auto dst = (rq::lds_u32_ptr)(xs + m * Kb);
            auto scratch = (rq::lds_f32_ptr)(smem + xch_off);
            if (!serial && !active) continue;   // no barriers inside: idle groups skip the arithmetic
            if (log2h == 0)
                rq::rotate_quant_chunk<G, true>(src, K, (int64_t)c * G * kChunk, 0, mult, sx, dst, scratch, stid, active);
            else
                rq::rotate_quant_chunk<G, false>(src, K, (int64_t)c * G * kChunk, log2h, mult, sx, dst, scratch, stid,
                                                 active);
        }
        rq::lds_sync();
    }
    }
    if constexpr (MODE != 0) {
        if (xq_out != nullptr && blockIdx.x == 0) {
            for (int i = tid * 16; i < M * Kb; i += 1024 * 16)
                *reinterpret_cast<v4i*>(xq_out + i) = *(__attribute__((address_space(3))) const v4i*)(xs + i);
        }
    }

    if constexpr (EARLY < CB) {
        load_weights(gid, 0, EARLY, CB);
        __builtin_amdgcn_sched_barrier(0);
    }
    // ---- 4. row groups: dot products on packed nibbles, fold over lanes, dequantise, store
    for (bool first = true; gid < groups; gid += gstride, first = false) {
        int p[RPW * MP];
#pragma unroll
        for (int i = 0; i < RPW * MP; ++i) p[i] = 0;
        for (int cb = 0; cb < cpr; cb += CB) {
            if (!first || cb > 0) load_weights(gid, cb);
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                const int off = (cb + c) * 1024 + lane * 16;
                if (off < Kb) {
                    if constexpr (ABITS == 8) {
                        v4i we[RPW], wo[RPW];
#pragma unroll
                        for (int j = 0; j < RPW; ++j) unpack16(w[j][c], we[j], wo[j]);
#pragma unroll
                        for (int m = 0; m < MP; ++m) {
                            if (m < M) {
                                const v4i xe = *(__attribute__((address_space(3))) const v4i*)(xs + m * Ka + 2 * off);
                                const v4i xo = *(__attribute__((address_space(3))) const v4i*)(xs + m * Ka + 2 * off + 16);
#pragma unroll
                                for (int j = 0; j < RPW; ++j) {
                                    int a = p[j * MP + m];
                                    a = __builtin_amdgcn_sdot4(we[j].x, xe.x, a, false);
                                    a = __builtin_amdgcn_sdot4(we[j].y, xe.y, a, false);
                                    a = __builtin_amdgcn_sdot4(we[j].z, xe.z, a, false);
                                    a = __builtin_amdgcn_sdot4(we[j].w, xe.w, a, false);
                                    a = __builtin_amdgcn_sdot4(wo[j].x, xo.x, a, false);
                                    a = __builtin_amdgcn_sdot4(wo[j].y, xo.y, a, false);
                                    a = __builtin_amdgcn_sdot4(wo[j].z, xo.z, a, false);
                                    a = __builtin_amdgcn_sdot4(wo[j].w, xo.w, a, false);
                                    p[j * MP + m] = a;
                                }
                            }
                        }
                    } else {
#pragma unroll
                    for (int m = 0; m < MP; ++m) {
                        if (m < M) {
                            const v4i xv = *(__attribute__((address_space(3))) const v4i*)(xs + m * Kb + off);
#pragma unroll
                            for (int j = 0; j < RPW; ++j) {
                                int a = p[j * MP + m];
                                a = __builtin_amdgcn_sdot8(w[j][c].x, xv.x, a, false);
                                a = __builtin_amdgcn_sdot8(w[j][c].y, xv.y, a, false);
                                a = __builtin_amdgcn_sdot8(w[j][c].z, xv.z, a, false);
                                a = __builtin_amdgcn_sdot8(w[j][c].w, xv.w, a, false);
                                p[j * MP + m] = a;
                            }
                        }
                    }
                    }
                }
            }
        }
        constexpr int V = RPW * MP;
        fold<V>(p, lane);
        if (lane < V) {
            const int idx = bitrev(lane, ilog2(V));
            const int j = idx / MP, m = idx % MP;
            if (m < M) {
                const int n = gid * RPW + j;
                const int total = ABITS == 8 ? p[0] >> 4 : p[0];
                if (n >= two.n1) {   // the second matrix: its own channel steps and output
                    const int n2 = n - two.n1;
                    const float sw_n = first ? sw_first : two.sw[n2];
                    two.out[(int64_t)m * (N - two.n1) + n2] = __float2half_rn(mul_rn((float)total, sx * sw_n));
                } else {
                    if (acc_out) acc_out[(int64_t)m * two.n1 + n] = total;
                    const int shifted = total + (zcorr ? zcorr[n] : 0);   // zero-point correction of Eq. 1, if any
                    const float sw_n = first ? sw_first : sw[n];
                    if (out) out[(int64_t)m * two.n1 + n] = __float2half_rn(mul_rn((float)shifted, (srow ? srow[m] : sx) * sw_n));
                }
            }
        }
    }
}

template <int RPW, int CB, int MP, int MODE, int ABITS = 4>
int launch_one(const __half* x, const uint8_t* xq_in, const uint8_t* wq, const float* sw, float sx, float mult,
               int log2h, int M, int N, int K, __half* out, int32_t* acc, uint8_t* xq_out, hipStream_t st,
               const float* srow, const int32_t* zcorr, const DecodeSecond& two)
{
    constexpr int G = MODE == 2 ? 2 : 1;
    const size_t lds = (((size_t)MP * (ABITS == 8 ? K : K / 2) + 15) & ~(size_t)15) +
                       (MODE == 0 ? 16 : (size_t)G * kChunk * 4 + (size_t)M * K * 2);
    auto kern = k_decode<RPW, CB, MP, MODE, ABITS>;
    static std::atomic<uint64_t> lds_ok{0};
    if (lds > 48 * 1024 && allow_dynamic_lds(reinterpret_cast<const void*>(kern), 160 * 1024, lds_ok) != PQ_OK)
        return PQ_ERR_HIP;
    const int groups = N / RPW;
    int grid = (groups + 15) / 16;
    grid = grid > 256 ? 256 : grid;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(1024), lds, st, x, xq_in, wq, sw, sx, mult, log2h, M, N, K, out,
                       acc, xq_out, srow, zcorr, two);
    return hip_status(hipGetLastError());
}

template <int RPW, int CB, int MP, int ABITS = 4>
int launch_mode(const __half* x, const uint8_t* xq_in, const uint8_t* wq, const float* sw, float sx, int h, int M,
                int N, int K, __half* out, int32_t* acc, uint8_t* xq_out, hipStream_t st, const float* srow,
                const int32_t* zcorr, const DecodeSecond& two)
{
    if constexpr (ABITS == 8) {
        if constexpr (RPW > 2 || (MP > 1 && RPW * CB > 8)) return PQ_ERR_UNSUPPORTED;   // never chosen
        else if (x != nullptr) return PQ_ERR_UNSUPPORTED;                               // given codes only
        else return launch_one<RPW, CB, MP, 0, 8>(x, xq_in, wq, sw, sx, 0.f, 0, M, N, K, out, acc, xq_out, st, srow, zcorr, two);
    } else
    if constexpr (MP > 4 && (RPW > 2 || RPW * CB > 8)) return PQ_ERR_UNSUPPORTED;   // never chosen: too many registers
    else if (x == nullptr) return launch_one<RPW, CB, MP, 0>(x, xq_in, wq, sw, sx, 0.f, 0, M, N, K, out, acc, xq_out, st, srow, zcorr, two);
    if constexpr (MP > 4) return PQ_ERR_UNSUPPORTED;   // more than 4 tokens: codes only, no fused quantizer
    else if (h <= 1) {
        const float inv = (float)(1.0 / (double)sx);
        return launch_one<RPW, CB, MP, 1>(x, xq_in, wq, sw, sx, inv, 0, M, N, K, out, acc, xq_out, st, srow, zcorr, two);
    }
    else {
        int log2h = 0;
        while ((1 << log2h) < h) ++log2h;
        const float mult = (float)(1.0 / ((double)sx * sqrt((double)h)));
        if (h <= kChunk)
            return launch_one<RPW, CB, MP, 1>(x, xq_in, wq, sw, sx, mult, log2h, M, N, K, out, acc, xq_out, st, srow, zcorr, two);
        return launch_one<RPW, CB, MP, 2>(x, xq_in, wq, sw, sx, mult, log2h, M, N, K, out, acc, xq_out, st, srow, zcorr, two);
    }
}

template <int MP, int ABITS = 4>
int launch_shape(int rpw, int cb, const __half* x, const uint8_t* xi, const uint8_t* w, const float* sw, float sx,
                 int h, int m, int n, int k, __half* o, int32_t* acc, uint8_t* xo, hipStream_t st, const float* srow,
                 const int32_t* zcorr, const DecodeSecond& two)
{
    switch (rpw * 100 + cb) {
        case 102: return launch_mode<1, 2, MP, ABITS>(x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
        case 202: return launch_mode<2, 2, MP, ABITS>(x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
        case 402: return launch_mode<4, 2, MP, ABITS>(x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
        case 104: return launch_mode<1, 4, MP, ABITS>(x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
        case 204: return launch_mode<2, 4, MP, ABITS>(x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
        case 404: return launch_mode<4, 4, MP, ABITS>(x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
        case 108: return launch_mode<1, 8, MP, ABITS>(x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
        default: return launch_mode<2, 8, MP, ABITS>(x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
    }
}

}  // namespace

// h < 0: the packed codes are given; h >= 0: fused rotate + quantize from fp16 rows
bool decode_supported(int64_t M, int64_t N, int64_t K, int32_t h, int32_t abits)
{
    if (abits == 8) {   // int8 codes given: [MP][K] bytes of LDS
        if (!(h < 0 && M >= 1 && M <= 8 && (N % 16) == 0 && (K % 32) == 0 && K <= 131072 && N <= (1 << 30))) return false;
        const int64_t mp8 = M == 1 ? 1 : (M <= 4 ? 4 : 8);
        return mp8 * K + 32 <= 160 * 1024;
    }
    if (!(M >= 1 && M <= (h < 0 ? 8 : 4) && (N % 16) == 0 && K <= 131072 && h <= 2 * kChunk && N <= (1 << 30)))
        return false;
    const int64_t mp = M == 1 ? 1 : (M <= 4 ? 4 : 8), g = h <= kChunk ? 1 : 2;
    const int64_t fused = h >= 0 ? M * K * 2 + g * kChunk * 4 : 16;
    return mp * (K / 2) + 16 + fused <= 160 * 1024;
}

// x_f16 != NULL: fused rotate + quantize (codes also written to xq_out if it is not NULL);
// x_f16 == NULL: packed codes are read from xq_in.  srow != NULL: per-token steps replace sx in the
// epilogue (per-token dynamic quantization; only with given codes).
int launch_decode(const void* x_f16, const void* xq_in, const void* wq, const float* sw, float sx, int32_t h,
                  int64_t M, int64_t N, int64_t K, void* out, int32_t* acc, void* xq_out, hipStream_t st,
                  const float* srow, int32_t abits, const int32_t* zcorr, const DecodeSecond* second)
{
    if (!decode_supported(M, N, K, x_f16 ? h : -1, abits)) return PQ_ERR_UNSUPPORTED;
    // N counts the rows of both matrices when a second one follows; alone, all N rows are the first's
    DecodeSecond two{nullptr, nullptr, nullptr, (int)N};
    if (second) {
        if (second->n1 <= 0 || second->n1 >= N || (second->n1 % 16) != 0 || acc || zcorr || srow) return PQ_ERR_UNSUPPORTED;
        two = *second;
    }
    const __half* x = static_cast<const __half*>(x_f16);
    const uint8_t* xi = static_cast<const uint8_t*>(xq_in);
    const uint8_t* w = static_cast<const uint8_t*>(wq);
    __half* o = static_cast<__half*>(out);
    uint8_t* xo = static_cast<uint8_t*>(xq_out);
    const int cpr = (int)((K / 2 + 1023) / 1024);
    // chunks per batch, then rows per wavefront: up to 16 loads in flight per lane, and few
    // enough row groups that the 4096 wavefronts of the chip take them in one pass if possible
    const int cb = cpr <= 2 ? 2 : (cpr <= 4 ? 4 : 8);
    int rpw = 1;
    while (rpw < 4 && rpw * 2 * cb <= 16 && N / rpw > 4096) rpw *= 2;
    if (rpw == 4 && cb == 8) rpw = 2;
    const int m = (int)M, n = (int)N, k = (int)K;
    if (abits == 8) {
        if (rpw > 2) rpw = 2;
        if (M == 1) return launch_shape<1, 8>(rpw, cb, x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
        if (cb == 8) rpw = 1;   // more tokens: fewer rows per wavefront keep the accumulators in registers
        if (M <= 4) return launch_shape<4, 8>(rpw, cb, x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
        return launch_shape<8, 8>(rpw, cb, x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
    }
    if (M == 1) return launch_shape<1>(rpw, cb, x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
    if (M <= 4) return launch_shape<4>(rpw, cb, x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
    // 5..8 tokens: fewer rows per wavefront so that the accumulators stay in registers
    if (rpw > 2) rpw = 2;
    if (cb == 8) rpw = 1;
    return launch_shape<8>(rpw, cb, x, xi, w, sw, sx, h, m, n, k, o, acc, xo, st, srow, zcorr, two);
}

}  // namespace pq
