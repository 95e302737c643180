// The integer product of Eq. 1's codes on the 6-bit floating-point matrix instruction
// (v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in E3M2, fp32 accumulate).  Every code -8..7 is
// exact in E3M2 (1, 2, 3 = 1.5 x 2, 4..7 = {1, 1.25, 1.5, 1.75} x 4, 8), a product is at most 64 and
// fp32 adds integers exactly below 2^24, so for K <= 262080 the accumulators are the exact integer
// sums; the instruction runs at twice the nominal rate of the INT8 one and is less held back by the
// chip's power limit.
//
// Both operands arrive repacked ("f6 tiles", k_repack_f6): for every block of 32 rows and every 128
// channels (two steps of the instruction) the register images of a wavefront, 3072 bytes; the blocks of
// all row blocks for one group of 128 channels lie side by side, group after group.  The image
// of lane l for step s holds row 32 rb + l % 32 and the 32 channels 64 (2 kt + s) + 32 (l / 32) + i as
// a little-endian stream of 6-bit values, 24 bytes = six dwords.  A block stores them as four planes,
// each lane after lane: bytes 0-15 of the first step's images (64 x 16 bytes), their bytes 16-23
// (64 x 8), bytes 0-7 of the second step's (64 x 8), their bytes 8-23 (64 x 16).  Every plane is what
// one load instruction of a wavefront fetches (16 or 8 bytes per lane, consecutive lanes adjacent:
// whole cache lines from memory, conflict-free from LDS), and its destination is a run of registers
// inside the six of an image, so no instruction is spent on rearranging.
//
// At twice the INT8 rate the matrix pipe outruns the LDS if both operands pass through it (a 256 x 256
// tile reads 96 KiB and writes 48 KiB of LDS per 128 channels, in the 1024 clocks its matrix
// instructions take).  So only the tokens go through LDS: a workgroup's tile is 128 tokens x 4 wavefronts x
// 32 CI channels, the 128 tokens' images (12 KiB per 128 channels) are shared by the four
// wavefronts, and every wavefront streams the weights of its own 32 CI channels from memory straight
// into the registers the matrix instruction reads (a ring of three stages, refilled image by image
// right behind the last instruction that uses it): 48 KiB of LDS reads and 12 KiB of writes per 128
// channels for the same 1024 clocks of matrix work.
#include <hip/hip_fp16.h>
#include <math.h>
#include <stdlib.h>

#include <atomic>
#include <type_traits>

#include "pq_internal.h"
#include "pq_rotate.h"

namespace pq {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kImage = 24, kStep = 64 * kImage, kChunkF6 = 2 * kStep;   // 1536 B per (row block, step); 3072 per stage
// stages in flight (LDS slots of the tokens, register sets of the weights); deeper rings for the narrow tiles
// (6 stages at CI = 2, 4 at CI = 3: the same 144 registers) measured no faster with cold weights and 1-2 us
// slower per tile with warm ones
constexpr int ring_of(int) { return 3; }
constexpr int kPersistentWorkgroups = 256;                               // one per CU

// Offsets of the four planes of a block, and an image's 24 bytes (three qwords) into its two planes.
constexpr int kP0 = 0, kP1 = 1024, kP2 = 1536, kP3 = 2048;

// STREAM: non-temporal stores (a compile-time choice: a run-time branch around the stores cost the quantizers 5 %).  The activation images a quantizer writes are read next by every XCD of the
// product launch, from the memory side in any case (the L2s are not coherent with one another).  While all of
// a launch's images fit the L2s (rq::kStreamBelow), ordinary stores would leave in one burst at the end of the
// kernel; written through at once they leave during it and do not push the weights out of the memory-side cache
// (2048 x 14336, 22 MB of images: 21.7 -> 21.3 us, the step with cold weights 344 -> 339 us).  A larger output is
// evicted as the kernel goes anyway and streaming costs time (8192 x 14336, 88 MB: 58 -> 65 us).
template <bool STREAM>
__device__ __forceinline__ void store_image(uint8_t* block, int lane, int step, const uint64_t (&w)[3])
{
    typedef uint64_t v2u __attribute__((ext_vector_type(2)));
    v2u* wide = reinterpret_cast<v2u*>(block + (step == 0 ? kP0 : kP3) + lane * 16);
    uint64_t* narrow = reinterpret_cast<uint64_t*>(block + (step == 0 ? kP1 : kP2) + lane * 8);
    const v2u two = step == 0 ? (v2u){w[0], w[1]} : (v2u){w[1], w[2]};
    const uint64_t one = step == 0 ? w[2] : w[0];
    if constexpr (STREAM) {
        __builtin_nontemporal_store(two, wide);
        __builtin_nontemporal_store(one, narrow);
    } else {
        *wide = two;
        *narrow = one;
    }
}

// Eight packed two's complement nibbles (channel i in bits 4 i ..) -> their eight E3M2 codes as a 48-bit
// little-endian stream.  The 16-entry table look-up runs on four codes at a time: v_perm_b32 picks bytes
// of an 8-entry table by the low three bits of each nibble, once from the table of 0..7 and once from that
// of -8..-1, and bit 3 selects between the two per byte; then bytes are paired into 12-bit and 24-bit runs.
__device__ __forceinline__ uint64_t e3m2_stream8(uint32_t w)
{
    constexpr uint32_t T0 = 0u | (12u << 8) | (16u << 16) | (18u << 24);    // 0, 1, 2, 3
    constexpr uint32_t T1 = 20u | (21u << 8) | (22u << 16) | (23u << 24);   // 4, 5, 6, 7
    constexpr uint32_t T2 = 56u | (55u << 8) | (54u << 16) | (53u << 24);   // -8, -7, -6, -5
    constexpr uint32_t T3 = 52u | (50u << 8) | (48u << 16) | (44u << 24);   // -4, -3, -2, -1
    auto lut = [](uint32_t x) {      // four nibbles, one per byte -> four codes
        const uint32_t sel = x & 0x07070707u;
        const uint32_t a = __builtin_amdgcn_perm(T1, T0, sel);   // selector 0-3: second operand, 4-7: first
        const uint32_t b = __builtin_amdgcn_perm(T3, T2, sel);
        const uint32_t m = (x >> 3) & 0x01010101u;
        const uint32_t mask = (m << 8) - m;                      // 0xFF in every byte whose nibble has bit 3 set
        return a ^ ((a ^ b) & mask);
    };
    const uint32_t ev = lut(w & 0x0F0F0F0Fu);            // codes of channels 0, 2, 4, 6
    const uint32_t od = lut((w >> 4) & 0x0F0F0F0Fu);     // codes of channels 1, 3, 5, 7
    // 16-bit lanes: (c0 | c1 << 6), (c2 | c3 << 6) and (c4 | c5 << 6), (c6 | c7 << 6); selector 0x0c = a zero byte
    const uint32_t a = __builtin_amdgcn_perm(0u, ev, 0x0c010c00u) | (__builtin_amdgcn_perm(0u, od, 0x0c010c00u) << 6);
    const uint32_t b = __builtin_amdgcn_perm(0u, ev, 0x0c030c02u) | (__builtin_amdgcn_perm(0u, od, 0x0c030c02u) << 6);
    const uint32_t h0 = (a & 0xFFFu) | ((a >> 4) & 0xFFF000u);   // c0 .. c3: 24 bits
    const uint32_t h1 = (b & 0xFFFu) | ((b >> 4) & 0xFFF000u);   // c4 .. c7
    return (uint64_t)h0 | ((uint64_t)h1 << 24);
}

// 32 codes of one row (16 bytes of packed nibbles) -> their register image, 24 bytes as three qwords.
__device__ __forceinline__ void image_of_nibbles(const v4i p, uint64_t (&w)[3])
{
    const uint64_t s0 = e3m2_stream8((uint32_t)p.x), s1 = e3m2_stream8((uint32_t)p.y);
    const uint64_t s2 = e3m2_stream8((uint32_t)p.z), s3 = e3m2_stream8((uint32_t)p.w);
    w[0] = s0 | (s1 << 48);
    w[1] = (s1 >> 16) | (s2 << 32);
    w[2] = (s2 >> 32) | (s3 << 16);
}

// One thread per register image: 32 codes (16 bytes of nibbles) of one row -> 24 bytes.
__global__ __launch_bounds__(256) void k_repack_f6(const uint8_t* __restrict__ codes, int R, int K, int64_t images,
                                                  uint8_t* __restrict__ out)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= images) return;
    const int KS = K >> 6, lane = (int)(t & 63);
    const int64_t blk = t >> 6;
    const int ks = (int)(blk % KS), rb = (int)(blk / KS);
    const int row = rb * 32 + (lane & 31), k0 = ks * 64 + (lane >> 5) * 32;
    uint64_t w[3] = {0, 0, 0};
    if (row < R) image_of_nibbles(*reinterpret_cast<const v4i*>(codes + (int64_t)row * (K >> 1) + (k0 >> 1)), w);
    store_image<false>(out + ((int64_t)(ks >> 1) * ((R + 31) >> 5) + rb) * kChunkF6, lane, ks & 1, w);
}

// Rotation (blocks of up to 512 channels) + static quantizer that writes f6 tiles: one launch instead of
// quantizer + repack, loads and stores both in whole cache lines.  A workgroup owns 32 tokens x C channels
// (C = 128, 256 or 512: the rotation block, at least one block of the tiles), i.e. C / 128 blocks of 3072
// bytes.  First every wavefront takes eight of the tokens, 512 / C of them at a time, all loads issued before
// the arithmetic: a lane holds 8 consecutive channels (16 bytes), rotates and quantizes them exactly as
// pq_rotate_quant does (the same device code, the same codes bit for bit) and leaves the packed dword in LDS.
// Then one thread per register image (32 channels of a token) turns it into its 24 bytes and stores them: a
// wavefront's store covers a whole plane of a block.  Optionally the canonical nibbles go out as well.
// The narrow variants are what keeps the GPU busy on a 2048 x 4096 input (2048 workgroups of C = 128 instead
// of 512 of C = 512): short workgroups at different phases hide one another's load latency.
template <bool EXACT, int C, bool STREAM>
__global__ __launch_bounds__(256) void k_rotate_quant_f6(const __half* __restrict__ x, int M, int K, int log2h,
                                                        rq::StaticStep steps, uint8_t* __restrict__ tiles,
                                                        uint8_t* __restrict__ nibbles)
{
    constexpr int LPR = C / 8, RPP = 64 / LPR, PASSES = 8 / RPP;     // lanes per token, tokens per pass, passes
    constexpr int kPitch = C / 2 + 16;                                // staged row: nibbles, padded (bank spread)
    __shared__ __align__(16) uint8_t stage[32 * kPitch];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lrow = lane / LPR, lcol = lane % LPR;                   // token within a pass, group of 8 channels
    const int rb = blockIdx.y, chunk0 = blockIdx.x * C;
    const int64_t krel = K - chunk0;                                  // channels from chunk0 to the end of the row
    v4i raw[PASSES][1];
    bool live[PASSES][1];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int64_t row = (int64_t)rb * 32 + wave * 8 + p * RPP + lrow;
        const bool in = row < M;
        rq::load_chunk<1>(static_cast<const __half*>(x + (in ? row : 0) * K + chunk0), krel, 0, lcol, in, raw[p], live[p]);
    }
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        rq::lds_u32_ptr dst = (rq::lds_u32_ptr)(stage + (wave * 8 + p * RPP + lrow) * kPitch);
        if (!live[p][0]) dst[lcol] = 0u;                              // tokens past the end, channels past K: zero codes
        // (lane stages of the rotation pair lanes inside a token's LPR lanes: bit b of lcol is bit b of the lane)
        rq::rotate_quant_regs_with<1, EXACT, 4>(raw[p], live[p], 0, log2h, steps, dst, (rq::lds_f32_ptr) nullptr, lcol,
                                                live[p][0]);
    }
    __syncthreads();
    // images of the workgroup: C / 128 blocks x 2 steps x 64 lanes
    const int nk = K >> 7;
#pragma unroll
    for (int i = threadIdx.x; i < (C / 128) * 128; i += 256) {
        const int blk = i >> 7, st = (i >> 6) & 1, l = i & 63, kt = blockIdx.x * (C / 128) + blk;
        if (kt < nk) {
            const v4i p = *(__attribute__((address_space(3))) const v4i*)(stage + (l & 31) * kPitch + blk * 64 + st * 32 +
                                                                          (l >> 5) * 16);
            uint64_t w[3];
            image_of_nibbles(p, w);
            store_image<STREAM>(tiles + ((int64_t)kt * gridDim.y + rb) * kChunkF6, l, st, w);
        }
    }
    if (nibbles) {
        constexpr int PPR = C / 32;                                   // 16-byte pieces per staged row
#pragma unroll
        for (int i = threadIdx.x; i < 32 * PPR; i += 256) {
            const int row = i / PPR, c16 = i % PPR;
            const int64_t grow = (int64_t)rb * 32 + row;
            if (grow < M && chunk0 + c16 * 32 < K)
                *reinterpret_cast<v4i*>(nibbles + grow * (K >> 1) + (chunk0 >> 1) + c16 * 16) =
                    *(__attribute__((address_space(3))) const v4i*)(stage + row * kPitch + c16 * 16);
        }
    }
}

template <int I, int N, typename F>
__device__ __forceinline__ void static_for6(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for6<I + 1, N>(f);
    }
}

// The 128-point block rotation as a product on the matrix pipe, fused with the quantizer (App. B "Online
// Rotation" + Eq. 1).  Butterflies cost about 25 vector instructions per element with conversion and
// quantizer, which bounds the kernel above (2048 x 14336: 23.6 us for 81 MB); here Y^T = H X^T runs on
// v_mfma_f32_32x32x16_f16 (the fp16 inputs as they are, the +-1 of H exact in fp16, fp32 accumulate: the same
// sums of 128 terms as the butterflies, in another order, so codes can differ from theirs only where the
// rotated value sits within fp32 rounding of a tie) and the vector pipe is left with the quantizer and the images.
//
// One wavefront = 32 tokens x 128 channels = one rotation block = one block of the tiles, no barriers:
//  - 8 coalesced 16-byte loads per lane (4 tokens x 256 bytes per instruction) into a padded LDS tile of its own;
//  - per 16-channel step the token operand (lane = token l % 32, 8 channels 16 s + 8 (l / 32) ...) is one LDS
//    read; the H operand (lane = output channel j = 32 n + l % 32, same 8 input channels i) is +-1 with sign
//    parity(popcount(i & j)): the low three bits of i give a per-lane pattern, the bits above flip all eight
//    together, by lane for bits 3 and 4 and by (n, s) at compile time for bits 5 and 6: four register sets
//    prepared once serve all 32 matrix instructions;
//  - the accumulators leave a lane with one token and, per 32 channels, the channels 8 q + 4 (l / 32) + 0..3:
//    four codes make 16 bits; one exchange between the two half-wavefronts (v_permlane32_swap) pairs them to
//    dwords of eight channels, a second one hands each half-wavefront the four dwords of its own 32 channels,
//    which is the 16 bytes of canonical nibbles (stored if asked for) and the input of the register image.
constexpr int kXPitch = 272;      // LDS row of 128 fp16 + 16 bytes: the 16-byte operand reads of 32 rows spread over all banks
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

// (at least four wavefronts per SIMD: with that bound the compiler keeps the accumulators in ordinary registers,
// which the quantizer reads directly, instead of accumulation registers that cost a move per value)
// TILES: blocks a wavefront takes, one after the other (neighbours along K); the loads of all of them are
// issued before the first is worked on, so a wavefront's next block is on its way while it rotates one.
template <int WAVES, int TILES, bool STREAM>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(4, 8))) void k_rotate128_quant_mfma(
    const __half* __restrict__ x, int M, int K, rq::StaticStep steps, uint8_t* __restrict__ tiles, uint8_t* __restrict__ nibbles)
{
    __shared__ __align__(16) uint8_t stage_all[WAVES * 32 * kXPitch];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nk = K >> 7, kt0 = (blockIdx.x * WAVES + wave) * TILES, rb = blockIdx.y;
    if (kt0 >= nk) return;                                  // (no barriers below: wavefronts are independent)
    uint8_t* stg = stage_all + wave * (32 * kXPitch);
    const int t = lane & 31, g = lane >> 5;
    const int r4 = lane >> 4, c = lane & 15;
    v4i raw[TILES][8];
#pragma unroll
    for (int b = 0; b < TILES; ++b) {
        // (wavefront-uniform 64-bit base, 32-bit lane offsets: 32 rows of at most 2^24 channels; a block past
        // the end of the row re-reads the last one and is not worked on)
        const int kb = kt0 + b < nk ? kt0 + b : nk - 1;
        const uint8_t* base = reinterpret_cast<const uint8_t*>(x + ((int64_t)rb * 32 * K + (int64_t)kb * 128));
        const int rows_left = M - rb * 32;                  // >= 1
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int r = 4 * p + r4;
            const bool in = r < rows_left;
            const uint32_t off = ((uint32_t)(in ? r : 0) * (uint32_t)K + (uint32_t)c * 8u) * 2u;
            raw[b][p] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(base + off));
            if (!in) raw[b][p] = (v4i){0, 0, 0, 0};          // tokens past the end: zero codes
        }
    }
    // ---- the H operand: hreg[s & 1][flip by (n, s)][4 dwords of two fp16 each]
    uint32_t hreg[2][2][4];
    {
        const int j = t;                                    // low five bits of the output channel
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t lo = __builtin_popcount((2 * d) & j & 7) & 1, hi = __builtin_popcount((2 * d + 1) & j & 7) & 1;
            const uint32_t base = 0x3C003C00u ^ (lo << 15) ^ (hi << 31);
            const uint32_t f0 = (uint32_t)(g & (j >> 3)) & 1u;              // input bit 3 = half-wavefront
            const uint32_t f1 = f0 ^ ((uint32_t)(j >> 4) & 1u);            // input bit 4 = s & 1
            hreg[0][0][d] = base ^ (f0 * 0x80008000u);
            hreg[0][1][d] = hreg[0][0][d] ^ 0x80008000u;
            hreg[1][0][d] = base ^ (f1 * 0x80008000u);
            hreg[1][1][d] = hreg[1][0][d] ^ 0x80008000u;
        }
    }
    static_for6<0, TILES>([&](auto bc) {
        constexpr int b = decltype(bc)::value;
        const int kt = kt0 + b;
        if (kt >= nk) return;
        // ---- tokens into LDS (the wavefront's own region; its LDS operations execute in order)
#pragma unroll
        for (int p = 0; p < 8; ++p)
            *(__attribute__((address_space(3))) v4i*)(stg + (4 * p + r4) * kXPitch + c * 16) = raw[b][p];
        const int64_t row = (int64_t)rb * 32 + t;
        uint8_t* block = tiles ? tiles + ((int64_t)kt * gridDim.y + rb) * kChunkF6 : nullptr;
        // p: this lane's 32 channels of step st as nibbles (channels 0-7, 8-15, 16-23, 24-31)
        auto emit = [&](int st, const v4i p) {
            if (nibbles && row < M) {
                v4i* at = reinterpret_cast<v4i*>(nibbles + row * (K >> 1) + (int64_t)kt * 64 + st * 32 + g * 16);
                if constexpr (STREAM) __builtin_nontemporal_store(p, at);
                else *at = p;
            }
            if (block) {
                uint64_t w[3];
                image_of_nibbles(p, w);
                store_image<STREAM>(block, lane, st, w);
            }
        };
        v16f acc[4];
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[n][v] = 0.0f;
        static_for6<0, 8>([&](auto sc) {
            constexpr int s = decltype(sc)::value;
            const v4i xi = *(__attribute__((address_space(3))) const v4i*)(stg + t * kXPitch + 32 * s + 16 * g);
            const v8h xop = __builtin_bit_cast(v8h, xi);
            static_for6<0, 4>([&](auto nc) {
                constexpr int n = decltype(nc)::value;
                constexpr int flip = __builtin_popcount((s >> 1) & n) & 1;     // input bits 5, 6 against output bits 5, 6
                const v4i hi4 = {(int)hreg[s & 1][flip][0], (int)hreg[s & 1][flip][1], (int)hreg[s & 1][flip][2], (int)hreg[s & 1][flip][3]};
                acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, hi4), xop, acc[n], 0, 0, 0);
            });
        });
        // ---- quantize, pair, exchange
        uint32_t lo2[4], hi2[4];                        // per 32 channels: dwords of channels 8 q .. for q = 2 g, 2 g + 1
        static_for6<0, 4>([&](auto nc) {
            constexpr int n = decltype(nc)::value;
            float v01[8], v23[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) { v01[i] = acc[n][i]; v23[i] = acc[n][8 + i]; }
            // low half: four channels of group q = 0 (2), high half: of q = 1 (3), all of this lane's half 4 g ..
            uint32_t w01 = rq::quant_pack8<false>(v01, v01, steps.mult, steps.step);
            uint32_t w23 = rq::quant_pack8<false>(v23, v23, steps.mult, steps.step);
            // after the swap the lower half-wavefront holds (w01 of its own, w01 of the upper), the upper (w23 of the lower, its own w23)
            const auto sw = __builtin_amdgcn_permlane32_swap(w01, w23, false, false);
            const uint32_t mine = sw[0], theirs = sw[1];        // channels 4 * 0 .. of two groups, channels 4 * 1 .. of the same two
            lo2[n] = __builtin_amdgcn_perm(theirs, mine, 0x05040100u);   // group 2 g:     mine.lo16 | theirs.lo16 << 16
            hi2[n] = __builtin_amdgcn_perm(theirs, mine, 0x07060302u);   // group 2 g + 1: mine.hi16 | theirs.hi16 << 16
        });
        static_for6<0, 2>([&](auto stc) {
            constexpr int st = decltype(stc)::value;
            // tiles 2 st (for the lower half-wavefront) and 2 st + 1 (for the upper): the lower half gives its dwords of
            // the odd tile and takes the upper half's dwords of the even one
            uint32_t ea = lo2[2 * st], eb = hi2[2 * st], oa = lo2[2 * st + 1], ob = hi2[2 * st + 1];
            const auto sa = __builtin_amdgcn_permlane32_swap(ea, oa, false, false);
            const auto sb = __builtin_amdgcn_permlane32_swap(eb, ob, false, false);
            emit(st, (v4i){(int)sa[0], (int)sb[0], (int)sa[1], (int)sb[1]});
        });
    });
}

__device__ __forceinline__ int xcd_run(int b, int total)   // each XCD takes a contiguous run of tiles
{
    const int x = b & 7, idx = b >> 3, q = total >> 3, rem = total & 7;
    return x * q + (x < rem ? x : rem) + idx;
}

#define PQ6_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define PQ6_GLB(p) ((const __attribute__((address_space(1))) void*)(p))

// 16 bytes per lane from global memory straight into LDS (lane l lands at lds_addr + 16 l); base and
// lds_addr are wavefront-uniform.  Issued as inline assembly on purpose: the compiler's bookkeeping of
// outstanding loads treats a direct load to LDS as a memory operation of unknown kind and from then on
// waits for *all* outstanding loads at the next register it needs, which would empty the ring of weight
// loads every time.  Unknown to the compiler, these loads only make its waits for the weight registers
// stricter than needed (more loads are in flight than it counts, and vmcnt waits for the oldest first);
// the waits for the LDS data itself are placed by hand and count every load.
__device__ __forceinline__ void lds_dma16(const uint8_t* base, uint32_t lane_offset, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_offset), "s"(base), "s"(lds_addr)
                 : "memory");     // (m0 is written here and used by nothing else in these kernels: the compiler keeps
                                  // no value in it and sets it itself right in front of the instructions that read it)
}

constexpr int kTokBlocks = 4;                       // 128 tokens per workgroup tile
constexpr int kStageA = kTokBlocks * kChunkF6;      // their images for 128 channels: 12 KiB of LDS
constexpr int kLoadsA = kStageA / 1024 / 4;         // direct loads to LDS per wavefront and stage: 3

// Waits as instructions the compiler knows (not inline asm): its own bookkeeping of outstanding loads,
// which places the waits for the weight registers, then counts from these.  gfx9 encoding of s_waitcnt:
// vmcnt in bits 3:0 and 15:14, expcnt in 6:4, lgkmcnt in 11:8; all ones = no wait on that counter.
template <int N> __device__ __forceinline__ void wait_vm6()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
__device__ __forceinline__ void wait_lds6() { __builtin_amdgcn_s_waitcnt(15 | (3 << 14) | (7 << 4) | (0 << 8)); }

// One workgroup's share of the product: the tiles b, b + G, b + 2 G ... of a list of GM x GN tiles of 128 CI
// channels that starts at channel n_base (row tiles fastest; inside a round of G tiles each XCD takes a
// contiguous run, so the tiles that share a weight panel meet in one L2); b = bid, G = workgroups on the list.
// A tile is 128 tokens x 128 CI channels (CI = 2, 3 or 4); wavefront w holds all 128 tokens x the 32 CI
// channels n0 + 32 CI w ..., i.e. CI x 4 matrix tiles.  The weights are the first operand: a lane ends with
// one token (l % 32) and, per matrix tile, the channels 8 (v / 4) + 4 (l / 32) + v % 4 in register v.
// LDS: ring_of(CI) stages of token images, a staging region per wavefront for the epilogue, the channel steps.
// Between two tiles the order is: main loop of tile t, first loads of tile t + G (both rings), epilogue of
// tile t.  Waits count memory operations in issue order, oldest first: with the next tile's loads issued
// ahead of this tile's output stores, its first stages never wait for stores, and the stores drain under
// its main loop.
template <int CM>
__device__ __forceinline__ void f6_persistent(const uint8_t* __restrict__ x6, const uint8_t* __restrict__ w6,
                                              const float* __restrict__ sw, float sx, int M, int N, int K, int GM,
                                              int GN, int n_base, int bid, int G, __half* __restrict__ out,
                                              int32_t* __restrict__ acc_out)
{
    extern __shared__ __align__(16) uint8_t smem[];
    constexpr int R = ring_of(CM);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t l16 = (uint32_t)lane * 16u, l8 = (uint32_t)lane * 8u;   // unsigned: scalar base + 32-bit lane offset
    const int nk = K >> 7;
    const int RBX = (M + 31) >> 5, RBW = (N + 31) >> 5;
    const uint32_t lds_ring = (uint32_t)(uintptr_t)PQ6_LDS(smem);
    const int total = GM * GN;
    // Workgroup b runs on XCD b % 8.  XCDs that multiply the same tokens or the same weight panels walk K in step;
    // each starts an eighth of K further on (integer sums do not care in which order the stages are added), so a
    // line is fetched from HBM by one L2 and found in the memory-side cache by the others, not asked for by
    // several L2s at once.
    const int k_first = (int)(((int64_t)(bid & 7) * nk) >> 3);

    // tile t of the list: workgroup-uniform
    auto tile_of = [&](int seq) {             // seq-th tile of this workgroup, -1 past the end
        const int base = seq * G;
        if (base >= total) return -1;
        const int cnt = total - base < G ? total - base : G;
        return bid < cnt ? base + xcd_run(bid, cnt) : -1;
    };

    // ---- state of the tile whose loads are in flight / whose main loop runs
    uint32_t aoff[kLoadsA];                   // tokens: piece q = wave + 4 t of a stage is KiB q % 3 of token block q / 3
    const uint8_t* wrow[CM];                  // weights: the wavefront's own row blocks
    v8i bw[R][2][CM];                         // [ring slot][step][row block]; six dwords of each count
    v8i a0[kTokBlocks], a1[kTokBlocks];       // token images of the first / second step
    v16f acc[CM][kTokBlocks];
#pragma unroll
    for (int j = 0; j < kTokBlocks; ++j) { a0[j] = (v8i){0, 0, 0, 0, 0, 0, 0, 0}; a1[j] = a0[j]; }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int i = 0; i < CM; ++i) bw[r][st][i] = (v8i){0, 0, 0, 0, 0, 0, 0, 0};

    auto load_a = [&](int t, int kt, int slot) {
        int k = (kt < nk ? kt : nk - 1) + k_first;      // (past the last stage: harmless re-reads)
        k = k >= nk ? k - nk : k;
        lds_dma16(x6 + (size_t)k * ((size_t)RBX * kChunkF6), aoff[t], lds_ring + slot * kStageA + (wave + 4 * t) * 1024);
    };
    auto load_b = [&](auto slotc, auto stepc, auto ic, int kt) {
        constexpr int slot = decltype(slotc)::value, st = decltype(stepc)::value, i = decltype(ic)::value;
        int k = (kt < nk ? kt : nk - 1) + k_first;
        k = k >= nk ? k - nk : k;
        const uint8_t* blk = wrow[i] + (size_t)k * ((size_t)RBW * kChunkF6);
        v8i& d = bw[slot][st][i];
        if constexpr (st == 0) {
            const v4i t = *reinterpret_cast<const v4i*>(blk + kP0 + l16);
            const v2i u = *reinterpret_cast<const v2i*>(blk + kP1 + l8);
            d[0] = t.x; d[1] = t.y; d[2] = t.z; d[3] = t.w; d[4] = u.x; d[5] = u.y;
        } else {
            const v2i u = *reinterpret_cast<const v2i*>(blk + kP2 + l8);
            const v4i t = *reinterpret_cast<const v4i*>(blk + kP3 + l16);
            d[0] = u.x; d[1] = u.y; d[2] = t.x; d[3] = t.y; d[4] = t.z; d[5] = t.w;
        }
    };
    // token images of one step from LDS: two reads per image
    auto read_a = [&](int slot, int st, int j, int kind, v8i (&a)[kTokBlocks]) {
        const uint8_t* blk = smem + slot * kStageA + j * kChunkF6;
        v8i& d = a[j];
        if (st == 0) {
            if (kind == 0) {
                const v4i t = *(__attribute__((address_space(3))) const v4i*)(blk + kP0 + l16);
                d[0] = t.x; d[1] = t.y; d[2] = t.z; d[3] = t.w;
            } else {
                const v2i u = *(__attribute__((address_space(3))) const v2i*)(blk + kP1 + l8);
                d[4] = u.x; d[5] = u.y;
            }
        } else {
            if (kind == 0) {
                const v4i t = *(__attribute__((address_space(3))) const v4i*)(blk + kP3 + l16);
                d[2] = t.x; d[3] = t.y; d[4] = t.z; d[5] = t.w;
            } else {
                const v2i u = *(__attribute__((address_space(3))) const v2i*)(blk + kP2 + l8);
                d[0] = u.x; d[1] = u.y;
            }
        }
    };

    // The channel steps of a tile travel through LDS: requested as the first of the tile's first loads (one
    // direct load per wavefront: lane l fetches the steps of channels 4 l ... of the wavefront's 32 CI, lanes
    // past them a clamped address), read back in the epilogue.  Held in registers they would cost 16 CI of
    // them while the next tile's weight ring is filling, and loaded in the epilogue they would queue behind
    // that tile's first loads (loads complete in order).  Two regions, used in turn: the next tile's request
    // is issued before this tile's epilogue reads.
    const int scales_at = R * kStageA + 4 * 32 * (64 * CM + 16);
    auto request_scales = [&](int n0, int parity) {
        int n = n0 + wave * (32 * CM) + 4 * lane;
        n = n + 4 <= N ? n : N - 4;
        lds_dma16(reinterpret_cast<const uint8_t*>(sw), (uint32_t)n * 4u, lds_ring + scales_at + parity * 4096 + wave * 1024);
    };

    // ---- first loads of a tile: addresses, then both rings filled stage by stage.  (The waits count loads
    // in program order: every stage's group is pinned in place.)  Vector memory operations per wavefront
    // and stage: kLoadsA direct loads to LDS + 4 CI register loads.
    auto prefetch = [&](int m0, int n0, int parity) {
        constexpr int CI = CM;
#pragma unroll
        for (int t = 0; t < kLoadsA; ++t) {
            const int q = wave + 4 * t, j = q / 3, part = q % 3;
            int rb = (m0 >> 5) + j;
            rb = rb < RBX - 1 ? rb : RBX - 1;
            aoff[t] = ((uint32_t)rb * (uint32_t)kChunkF6 + part * 1024) + l16;   // (wavefront-uniform) + lane
        }
#pragma unroll
        for (int i = 0; i < CI; ++i) {
            int rb = (n0 >> 5) + wave * CI + i;
            rb = rb < RBW - 1 ? rb : RBW - 1;
            wrow[i] = w6 + (size_t)rb * kChunkF6;
        }
        if (out) request_scales(n0, parity);
        __builtin_amdgcn_sched_barrier(0);
        static_for6<0, R>([&](auto rc) {
            constexpr int r = decltype(rc)::value;
#pragma unroll
            for (int t = 0; t < kLoadsA; ++t) load_a(t, r, r);
            static_for6<0, CI>([&](auto ic) {
                load_b(std::integral_constant<int, r>{}, std::integral_constant<int, 0>{}, ic, r);
                load_b(std::integral_constant<int, r>{}, std::integral_constant<int, 1>{}, ic, r);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // ---- main loop of a tile whose first loads have been issued
    auto compute = [&](int parity) {
        constexpr int CI = CM;
        constexpr int V = 4 * CI + kLoadsA;                  // vector memory operations of a wavefront per stage
#pragma unroll
        for (int i = 0; i < CI; ++i)
#pragma unroll
            for (int j = 0; j < kTokBlocks; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
        // One step of a stage: CI x 4 matrix instructions, row block by row block.  Between them: the LDS
        // reads of the other step's token images (one per instruction, first eight), the refill of this
        // step's weight images for stage kt + R (right behind the last instruction that reads an image), and
        // in the second step the refill of the stage's LDS slot.  A wavefront issues in order: what is to
        // overlap the matrix pipe has to sit between its instructions.
        auto step = [&](auto slotc, auto stepc, int kt) {
            constexpr int slot = decltype(slotc)::value, st = decltype(stepc)::value;
            constexpr int rslot = st == 0 ? slot : (slot + 1) % R;      // where the other step's token images lie
            static_for6<0, CI * kTokBlocks>([&](auto nc) {
                constexpr int n = decltype(nc)::value, i = n / kTokBlocks, j = n % kTokBlocks;
                // formats 3, 3: E3M2 both; scale bytes 127 = 2^0
                if constexpr (st == 0)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bw[slot][0][i], a0[j], acc[i][j], 3, 3, 0, 127, 0, 127);
                else
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bw[slot][1][i], a1[j], acc[i][j], 3, 3, 0, 127, 0, 127);
                if constexpr (n < 2 * kTokBlocks) {
                    if constexpr (st == 0) read_a(rslot, 1, n >> 1, n & 1, a1);
                    else read_a(rslot, 0, n >> 1, n & 1, a0);
                }
                if constexpr (st == 1 && n < kLoadsA) load_a(n, kt + R, slot);
                if constexpr (j == kTokBlocks - 1)
                    load_b(std::integral_constant<int, slot>{}, std::integral_constant<int, st>{}, std::integral_constant<int, i>{}, kt + R);
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        auto stage = [&](auto slotc, int kt) {
            constexpr int slot = decltype(slotc)::value;
            step(std::integral_constant<int, slot>{}, std::integral_constant<int, 0>{}, kt);
            // The token images of stage kt + 1 were requested in the second step of stage kt + 1 - R; behind
            // them this wavefront has issued the second-step weights of that stage (2 CI), R - 2 whole stages
            // and the first-step weights of this one (2 CI).  (In the first R - 1 stages more lies behind
            // them, the previous tile's output stores included, so there the count is only stricter than needed.)
            wait_lds6();
            wait_vm6<4 * CI + (R - 2) * V>();
            asm volatile("s_barrier" ::: "memory");          // all have read stage kt; all of stage kt + 1 is in LDS
            __builtin_amdgcn_sched_barrier(0);
            step(std::integral_constant<int, slot>{}, std::integral_constant<int, 1>{}, kt);
            wait_lds6();
            __builtin_amdgcn_sched_barrier(0);
        };
        // Stage 0 has landed when all but the (R - 1) V newest operations are complete: behind its own V
        // operations lie the other R - 1 stages of the first loads and, if a tile preceded, that tile's
        // output stores (then more than stage 0 is waited for, but never a store: there are at most 8 CI <
        // (R - 1) V of them).
        static_assert(8 * CI <= (R - 1) * V, "the first wait of a tile would wait for output stores");
        wait_vm6<(R - 1) * V>();
        asm volatile("s_barrier" ::: "memory");
        if (out && lane < 8 * CI) {
            // The channel steps have landed (they were requested ahead of stage 0).  Turn them, in place, into
            // what the epilogue multiplies by: fl(sw * (sx / 256)), the INT8 tiled kernel's factor for its
            // accumulators of 256 acc, times 256 (exact), so that acc * factor has the same real value, hence
            // the same rounding, as that kernel's (256 acc) * fl(sw * (sx / 256)).
            float* mine = reinterpret_cast<float*>(smem + scales_at + parity * 4096 + wave * 1024) + 4 * lane;
            v4f c = *(__attribute__((address_space(3))) const v4f*)mine;
            const float f = sx * (1.0f / 256.0f);
            c.x = mul_rn(c.x, f) * 256.0f; c.y = mul_rn(c.y, f) * 256.0f; c.z = mul_rn(c.z, f) * 256.0f; c.w = mul_rn(c.w, f) * 256.0f;
            *(__attribute__((address_space(3))) v4f*)mine = c;
        }
#pragma unroll
        for (int p = 0; p < 2 * kTokBlocks; ++p) read_a(0, 0, p >> 1, p & 1, a0);
        wait_lds6();
        __builtin_amdgcn_sched_barrier(0);
        // the ring slot of a stage is a compile-time constant (its weights live in registers): the loop body
        // is R stages, the remaining nk % R stages follow one by one
        int kt = 0;
        for (; kt + R <= nk; kt += R)
            static_for6<0, R>([&](auto uc) { stage(uc, kt + decltype(uc)::value); });
        const int rem = nk - kt;
        static_for6<0, R - 1>([&](auto uc) {
            if (decltype(uc)::value < rem) stage(uc, kt + decltype(uc)::value);
        });
        wait_vm6<0>();      // the loads past the last stage: none may still be writing LDS or registers
    };

    // ---- epilogue: out = fp16(fp32(acc * factor)) with the factors prepared in LDS: the same real product,
    // rounded once to fp32 and once to fp16, as the INT8 tiled kernel's fp32(256 acc) * (sw[n] * (sx / 256)).
    // A lane owns one token and groups of four channels; stored like that one instruction would touch 32
    // token rows with 8 bytes each.  Each wavefront turns its 32 tokens x 32 CI channels through a private,
    // padded LDS region (behind the ring, which the next tile's loads are filling meanwhile) and stores
    // whole rows of 64 CI contiguous bytes.
    auto epilogue = [&](auto cic, int m0, int n0, int parity) {
        constexpr int CI = decltype(cic)::value;
        // (the lane number is taken afresh: kept in a register across the main loop, which uses every one,
        // the values derived from it would be spilled there and reloaded here, and a reload waits for all
        // memory operations in flight, the next tile's first loads and this tile's stores included)
        int lane;
        asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane));
        const int g = lane >> 5, r = lane & 31;
        constexpr int kRowPitch = 64 * CI + 16;
        uint8_t* stg = smem + R * kStageA + wave * (32 * kRowPitch);
        const int nw = n0 + wave * (32 * CI);
        const float* scl = reinterpret_cast<const float*>(smem + scales_at + parity * 4096 + wave * 1024);
#pragma unroll
        for (int j = 0; j < kTokBlocks; ++j) {
            const int mb = m0 + j * 32;
            if (acc_out) {
                const int m = mb + r;
#pragma unroll
                for (int i = 0; i < CI; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n = nw + i * 32 + 8 * q + 4 * g;
                        const v4i iv = {(int)acc[i][j][4 * q], (int)acc[i][j][4 * q + 1], (int)acc[i][j][4 * q + 2],
                                        (int)acc[i][j][4 * q + 3]};
                        if (m < M && n + 4 <= N) *reinterpret_cast<v4i*>(acc_out + (int64_t)m * N + n) = iv;
                    }
            }
            if (out) {
#pragma unroll
                for (int i = 0; i < CI; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const v4f c = *(__attribute__((address_space(3))) const v4f*)(scl + i * 32 + 8 * q + 4 * g);
                        const __half2 lo = __floats2half2_rn(mul_rn(acc[i][j][4 * q], c.x), mul_rn(acc[i][j][4 * q + 1], c.y));
                        const __half2 hi = __floats2half2_rn(mul_rn(acc[i][j][4 * q + 2], c.z), mul_rn(acc[i][j][4 * q + 3], c.w));
                        v2i val;
                        val.x = *reinterpret_cast<const int*>(&lo);
                        val.y = *reinterpret_cast<const int*>(&hi);
                        *(__attribute__((address_space(3))) v2i*)(stg + r * kRowPitch + (i * 32 + 8 * q + 4 * g) * 2) = val;
                    }
                // LDS operations of a wavefront execute in order: the reads below see the writes above, and
                // the next token block's writes come after these reads.  A pass stores RP whole rows: 4 CI
                // lanes of 16 bytes per row (CI = 3: 48 of the 64 lanes take part).
                constexpr int RP = CI == 3 ? 4 : 16 / CI;
                const int lrow = lane / (4 * CI), lu = lane % (4 * CI);
                const bool live = lrow < RP && nw + lu * 8 + 8 <= N;
                __half* dst = out + (int64_t)(mb + lrow) * N + nw + lu * 8;
                const uint8_t* src = stg + lrow * kRowPitch + lu * 16;
#pragma unroll
                for (int t = 0; t < 32 / RP; ++t) {
                    const v4i val = *(__attribute__((address_space(3))) const v4i*)(src + t * RP * kRowPitch);
                    // (the output is written once and not read here again: stored non-temporal, it does not take the place of
                    // weight panels and token images in the L2, nor of the weights in the memory-side cache)
                    if (live && mb + lrow + t * RP < M)
                        __builtin_nontemporal_store(val, reinterpret_cast<v4i*>(dst + (int64_t)t * RP * N));
                }
            }
        }
    };

    // Position of tile t of the list.  Plain order: row tiles fastest, so the 32 tiles an XCD holds at a time are
    // 2 panels x 16 row tiles when GM = 16: every XCD fetches all tokens, the panels once.  Where the list
    // divides into blocks of 8 row tiles x 4 panels, an XCD's 32 tiles are such a block: half of the tokens and
    // 4 panels, which is the smaller sum when a panel is at least as large as a row tile's tokens.
    const bool blocked = G == kPersistentWorkgroups && (GM % 8) == 0 && (GN % 4) == 0;
    auto pos_of = [&](int t, int& mt, int& nt) {
        if (blocked) {
            const int blk = t >> 5, in = t & 31, rows_of_blocks = GM >> 3;
            mt = (blk % rows_of_blocks) * 8 + (in & 7);
            nt = (blk / rows_of_blocks) * 4 + (in >> 3);
        } else {
            mt = t % GM;
            nt = t / GM;
        }
    };
    auto m0_of = [&](int t) { int mt, nt; pos_of(t, mt, nt); return mt * 128; };
    auto n0_of = [&](int t) { int mt, nt; pos_of(t, mt, nt); return n_base + nt * (128 * CM); };
    int t = tile_of(0);
    if (t < 0) return;
    prefetch(m0_of(t), n0_of(t), 0);
    int next = tile_of(1), parity = 0;
    for (int seq = 2; next >= 0; ++seq) {
        compute(parity);
        prefetch(m0_of(next), n0_of(next), parity ^ 1);
        epilogue(std::integral_constant<int, CM>{}, m0_of(t), n0_of(t), parity);
        t = next;
        next = tile_of(seq);
        parity ^= 1;
    }
    compute(parity);
    epilogue(std::integral_constant<int, CM>{}, m0_of(t), n0_of(t), parity);
}

// Persistent workgroups, one per CU and list.  MIXED: the first GA workgroups walk a list of GM x nA tiles 512
// channels wide, the others a list of GM x nB tiles 384 wide behind it; workgroups are dispatched in index
// order, so with GM x nA = GM x nB = the number of CUs every CU computes one tile of each width and none idles
// through a partial last round (gate/up: 14336 = 16 x 512 + 16 x 384); a workgroup of the second list starts as
// soon as one of the first has issued its last stores, and loads while those drain.
template <int CM, bool MIXED>
__global__ __launch_bounds__(256) void k_gemm_f6(const uint8_t* __restrict__ x6, const uint8_t* __restrict__ w6,
                                                const float* __restrict__ sw, float sx, int M, int N, int K,
                                                int GM, int nA, int nB, int GA, __half* __restrict__ out,
                                                int32_t* __restrict__ acc_out)
{
    if constexpr (MIXED) {
        if ((int)blockIdx.x < GA)
            f6_persistent<CM>(x6, w6, sw, sx, M, N, K, GM, nA, 0, (int)blockIdx.x, GA, out, acc_out);
        else
            f6_persistent<CM - 1>(x6, w6, sw, sx, M, N, K, GM, nB, nA * (128 * CM), (int)blockIdx.x - GA,
                                  (int)gridDim.x - GA, out, acc_out);
    } else {
        f6_persistent<CM>(x6, w6, sw, sx, M, N, K, GM, nA, 0, (int)blockIdx.x, (int)gridDim.x, out, acc_out);
    }
}

}  // namespace

namespace {
// Forced tile width (2, 3 = the mix, 4; -1 none): set by pq_set_gemm_f6_tile, and before the first such
// call by the environment variable PQ_GEMM_F6_TILE, which is read once.
constexpr int kF6Unread = -100;
std::atomic<int> g_forced_f6{kF6Unread};

int forced_f6_tile()
{
    int v = g_forced_f6.load(std::memory_order_relaxed);
    if (v == kF6Unread) {
        const char* f = getenv("PQ_GEMM_F6_TILE");
        v = f ? atoi(f) : -1;
        if (v < 2 || v > 4) v = -1;
        int expected = kF6Unread;
        g_forced_f6.compare_exchange_strong(expected, v);
        v = g_forced_f6.load(std::memory_order_relaxed);
    }
    return v;
}
}  // namespace

int set_gemm_f6_tile(int tile)
{
    if (tile != -1 && (tile < 2 || tile > 4)) return -2;
    const int prev = forced_f6_tile();
    g_forced_f6.store(tile);
    return prev;
}

size_t f6_tiles_bytes(int64_t R, int64_t K) { return (size_t)((R + 31) / 32) * (size_t)(K / 64) * kStep; }

// had_block: 0 or 1 = no rotation, else a power of two up to 512 that divides K (validated by the caller;
// larger blocks take pq_rotate_quant + repack).  nibbles: NULL, or where the canonical codes go as well.
bool quant_f6_supported(int64_t R, int64_t K, int32_t h) { return h <= 512 && (K % 128) == 0 && (R + 31) / 32 <= 65535 && K <= (1 << 30); }

template <bool EXACT>
static void launch_quant_f6_c(int c, const void* x, int64_t R, int64_t K, int log2h, rq::StaticStep steps, void* out,
                              void* nibbles, hipStream_t st)
{
    const dim3 grid((unsigned)((K + c - 1) / c), (unsigned)((R + 31) / 32));
    const __half* xp = static_cast<const __half*>(x);
    uint8_t *op = static_cast<uint8_t*>(out), *np = static_cast<uint8_t*>(nibbles);
    auto launch = [&](auto streamc) {
        constexpr bool S = decltype(streamc)::value;
        if (c == 128) hipLaunchKernelGGL((k_rotate_quant_f6<EXACT, 128, S>), grid, dim3(256), 0, st, xp, (int)R, (int)K, log2h, steps, op, np);
        else if (c == 256) hipLaunchKernelGGL((k_rotate_quant_f6<EXACT, 256, S>), grid, dim3(256), 0, st, xp, (int)R, (int)K, log2h, steps, op, np);
        else hipLaunchKernelGGL((k_rotate_quant_f6<EXACT, 512, S>), grid, dim3(256), 0, st, xp, (int)R, (int)K, log2h, steps, op, np);
    };
    if ((int64_t)f6_tiles_bytes(R, K) <= rq::kStreamBelow) launch(std::true_type{});      // (the tiles are the larger output)
    else launch(std::false_type{});
}

// 128-point blocks: rotation on the matrix pipe.  out (tiles) or nibbles may be NULL, not both.
bool rotate128_mfma_supported(int64_t R, int64_t K, int32_t h) { return h == 128 && (K % 128) == 0 && (R + 31) / 32 <= 65535 && K <= (1 << 24) && R >= 1; }

int launch_rotate128_mfma(const void* x, int64_t R, int64_t K, float act_scale, void* tiles, void* nibbles, hipStream_t st)
{
    constexpr int W = 4;      // wavefronts per workgroup (1, 2 and 4 measured level)
    const int64_t nk = K / 128, rbs = (R + 31) / 32;
    // the 1/sqrt(128) of the rotation is folded into the reciprocal step, as in pq_rotate_quant
    const rq::StaticStep steps{(float)(1.0 / ((double)act_scale * sqrt(128.0))), act_scale};
    const bool stream = (tiles ? (int64_t)f6_tiles_bytes(R, K) : R * (K / 2)) <= rq::kStreamBelow;   // (the larger output)
    uint8_t *tp = static_cast<uint8_t*>(tiles), *np = static_cast<uint8_t*>(nibbles);
    const __half* xp = static_cast<const __half*>(x);
    // Two blocks per wavefront where that still leaves a CU a dozen wavefronts and the output is streamed: the
    // second block's loads are in flight while the first is rotated (2048 x 14336, 7168 blocks: 21.3 -> 19.0 us;
    // with ordinary stores, i.e. on larger inputs, it gains nothing); on a small input one block each, so that
    // there are wavefronts enough.
    if (stream && nk * rbs >= 6144) {
        const dim3 grid((unsigned)((nk + 2 * W - 1) / (2 * W)), (unsigned)rbs);
        hipLaunchKernelGGL((k_rotate128_quant_mfma<W, 2, true>), grid, dim3(64 * W), 0, st, xp, (int)R, (int)K, steps, tp, np);
    } else {
        const dim3 grid((unsigned)((nk + W - 1) / W), (unsigned)rbs);
        if (stream) hipLaunchKernelGGL((k_rotate128_quant_mfma<W, 1, true>), grid, dim3(64 * W), 0, st, xp, (int)R, (int)K, steps, tp, np);
        else hipLaunchKernelGGL((k_rotate128_quant_mfma<W, 1, false>), grid, dim3(64 * W), 0, st, xp, (int)R, (int)K, steps, tp, np);
    }
    return hip_status(hipGetLastError());
}

int launch_quant_f6(const void* x, int64_t R, int64_t K, int32_t h, float act_scale, void* out, void* nibbles, hipStream_t st)
{
    if (!quant_f6_supported(R, K, h)) return PQ_ERR_UNSUPPORTED;
    if (rotate128_mfma_supported(R, K, h)) return launch_rotate128_mfma(x, R, K, act_scale, out, nibbles, st);
    const int c = h <= 128 ? 128 : h;                    // channels per workgroup: the rotation block, at least 128
    if (h <= 1) {
        launch_quant_f6_c<true>(c, x, R, K, 0, rq::StaticStep{(float)(1.0 / (double)act_scale), act_scale}, out, nibbles, st);
    } else {
        int log2h = 0;
        while ((1 << log2h) < h) ++log2h;
        // the 1/sqrt(h) of the rotation is folded into the reciprocal step, as in pq_rotate_quant
        launch_quant_f6_c<false>(c, x, R, K, log2h, rq::StaticStep{(float)(1.0 / ((double)act_scale * sqrt((double)h))), act_scale},
                                 out, nibbles, st);
    }
    return hip_status(hipGetLastError());
}

int launch_repack_f6(const void* codes, int64_t R, int64_t K, void* out, hipStream_t st)
{
    const int64_t images = ((R + 31) / 32) * (K / 64) * 64;
    hipLaunchKernelGGL(k_repack_f6, dim3((unsigned)((images + 255) / 256)), dim3(256), 0, st,
                       static_cast<const uint8_t*>(codes), (int)R, (int)K, images, static_cast<uint8_t*>(out));
    return hip_status(hipGetLastError());
}

namespace {
constexpr size_t lds_bytes_f6(int ci) { return (size_t)ring_of(ci) * kStageA + 4 * 32 * (64 * ci + 16) + 2 * 4096; }   // ring, staging, channel steps (two regions)

template <int CM, bool MIXED>
int launch_f6(const void* x6, const void* w6, const float* sw, float sx, int64_t M, int64_t N, int64_t K, int nA, int nB,
              void* out, int32_t* acc, hipStream_t st)
{
    const int GM = (int)((M + 127) / 128);
    const int64_t ta = (int64_t)GM * nA, tb = (int64_t)GM * nB;
    const int GA = (int)(ta < kPersistentWorkgroups ? ta : kPersistentWorkgroups);
    const int GB = (int)(tb < kPersistentWorkgroups ? tb : kPersistentWorkgroups);
    constexpr size_t lds = lds_bytes_f6(CM);
    static_assert(lds <= 160 * 1024, "LDS ring and staging too large");
    static std::atomic<uint64_t> lds_ok{0};
    if (allow_dynamic_lds(reinterpret_cast<const void*>(k_gemm_f6<CM, MIXED>), lds, lds_ok) != PQ_OK) return PQ_ERR_HIP;
    hipLaunchKernelGGL((k_gemm_f6<CM, MIXED>), dim3((unsigned)(GA + GB)), dim3(256), lds, st, static_cast<const uint8_t*>(x6),
                       static_cast<const uint8_t*>(w6), sw, sx, (int)M, (int)N, (int)K, GM, nA, nB, GA,
                       static_cast<__half*>(out), acc);
    return hip_status(hipGetLastError());
}
}  // namespace

// Channels per tile: 512, 384 or 256 (CI = 4, 3, 2), or a mix of 512 and 384 in one launch where N = 512 a +
// 384 b; the choice minimises the estimated time of the busiest CU (a tile costs a fixed part plus a part
// proportional to its width).
// pq_set_gemm_f6_tile: 2, 4 force one width, 3 the mix where N allows one (else 384 wide).
int launch_gemm_f6(const void* x6, const void* w6, const float* sw, float sx, int64_t M, int64_t N, int64_t K, void* out,
                   int32_t* acc, hipStream_t st)
{
    const int64_t gm = (M + 127) / 128;
    const int forced_tile = forced_f6_tile();
    auto cost_of = [](int ci) { return 0.35 + 0.1625 * ci; };      // relative to a 512-wide tile = 1
    auto makespan = [&](int64_t tiles_a, double ca, int64_t tiles_b, double cb) {
        // each list is dealt round-robin to its (up to) 256 workgroups; a CU hosts one workgroup of each list in turn
        const int64_t G = kPersistentWorkgroups;
        return (double)((tiles_a + G - 1) / G) * ca + (double)((tiles_b + G - 1) / G) * cb;
    };
    int best_ci = 4, best_a = 0, best_b = 0;
    double best = 1e300;
    for (int ci = 2; ci <= 4; ++ci) {
        if (forced_tile != -1 && forced_tile != 3 && forced_tile != ci) continue;
        const int64_t gn = (N + 128 * ci - 1) / (128 * ci);
        if (gm * gn > (1 << 24)) continue;
        const double c = makespan(gm * gn, cost_of(ci), 0, 0.0);
        if (c < best) { best = c; best_ci = ci; }
    }
    if (forced_tile == -1 || forced_tile == 3) {
        double bar = forced_tile == 3 ? 1e300 : best * 0.97;       // the mixed launch has to win by a margin
        for (int64_t b = 1; 384 * b < N; ++b) {
            if ((N - 384 * b) % 512 != 0) continue;
            const int64_t a = (N - 384 * b) / 512;
            if (a < 1 || gm * (a + b) > (1 << 24)) continue;
            const double c = makespan(gm * a, cost_of(4), gm * b, cost_of(3));
            if (c < bar) { bar = c; best_a = (int)a; best_b = (int)b; }
        }
    }
    if (best_a > 0) return launch_f6<4, true>(x6, w6, sw, sx, M, N, K, best_a, best_b, out, acc, st);
    const int gn = (int)((N + 128 * best_ci - 1) / (128 * best_ci));
    if (best_ci == 2) return launch_f6<2, false>(x6, w6, sw, sx, M, N, K, gn, 0, out, acc, st);
    if (best_ci == 3) return launch_f6<3, false>(x6, w6, sw, sx, M, N, K, gn, 0, out, acc, st);
    return launch_f6<4, false>(x6, w6, sw, sx, M, N, K, gn, 0, out, acc, st);
}

}  // namespace pq
