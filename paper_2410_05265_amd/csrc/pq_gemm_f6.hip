// The integer product of Eq. 1's codes on the 6-bit floating-point matrix instruction
// (v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in E3M2, fp32 accumulate).  Every code -8..7 is
// exact in E3M2 (1, 2, 3 = 1.5 x 2, 4..7 = {1, 1.25, 1.5, 1.75} x 4, 8), a product is at most 64 and
// fp32 adds integers exactly below 2^24, so for K <= 262080 the accumulators are the exact integer
// sums; the instruction runs at twice the nominal rate of the INT8 one and is less held back by the
// chip's power limit.
//
// Both operands arrive repacked ("f6 tiles", k_repack_f6): for every block of 32 rows and every 128
// channels (two steps of the instruction) the register images of a wavefront, lane after lane, 48
// bytes per lane: the image of the first step (24 bytes), then that of the second.  An image of lane
// l holds row 32 rb + l % 32 and the 32 channels 64 ks + 32 (l / 32) + i as a little-endian stream of
// 6-bit values.  Such a block is 3072 contiguous bytes and is one row block's share of a ring stage:
// the loads are straight copies into LDS, the main loop has no expansion work at all, and a lane
// reads an image as one 16-byte and one 8-byte piece at a stride of 48 bytes (conflict-free).
#include <hip/hip_fp16.h>
#include <stdlib.h>

#include <atomic>

#include "pq_internal.h"
#include "pq_rotate.h"

namespace pq {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kImage = 24, kStep = 64 * kImage, kChunkF6 = 2 * kStep;   // 1536 B per (row block, step); 3072 per stage
constexpr int kRing = 3;                                                 // stages in LDS

// two's complement nibble -> E3M2 (bias 3): two tables of eight 6-bit entries, for 0..7 and for -8..-1
__device__ __forceinline__ uint32_t e3m2_of_nibble(uint32_t nib)
{
    constexpr uint64_t pos = 0ull | (12ull << 6) | (16ull << 12) | (18ull << 18) | (20ull << 24) | (21ull << 30) | (22ull << 36) |
                             (23ull << 42);                                            // 0, 1, ..., 7
    constexpr uint64_t neg = 56ull | (55ull << 6) | (54ull << 12) | (53ull << 18) | (52ull << 24) | (50ull << 30) |
                             (48ull << 36) | (44ull << 42);                            // -8, -7, ..., -1
    return (uint32_t)(((nib & 8u) ? neg : pos) >> (6u * (nib & 7u))) & 63u;
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
    if (row < R) {
        const v4i p = *reinterpret_cast<const v4i*>(codes + (int64_t)row * (K >> 1) + (k0 >> 1));
        const uint32_t d[4] = {(uint32_t)p.x, (uint32_t)p.y, (uint32_t)p.z, (uint32_t)p.w};
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const uint64_t e = e3m2_of_nibble((d[i >> 3] >> (4 * (i & 7))) & 15u);
            const int bit = 6 * i;
            w[bit / 64] |= e << (bit % 64);
            if (bit % 64 > 58) w[bit / 64 + 1] |= e >> (64 - bit % 64);
        }
    }
    uint64_t* o = reinterpret_cast<uint64_t*>(out + ((int64_t)rb * (KS >> 1) + (ks >> 1)) * kChunkF6 + lane * 48 + (ks & 1) * kImage);
    o[0] = w[0]; o[1] = w[1]; o[2] = w[2];
}

// Quantizer for unrotated input that writes f6 tiles directly (one launch instead of quantizer + repack):
// one thread per register image, i.e. 32 consecutive channels of one token: four times the exact-tie
// quantizer of the nibble path (the same codes bit for bit), then the same conversion as k_repack_f6.
// Optionally also stores the canonical nibbles (the layer's workspace contract).
__global__ __launch_bounds__(256) void k_quant_f6(const __half* __restrict__ x, int R, int K, int64_t images, float mult,
                                                 float step, uint8_t* __restrict__ out, uint8_t* __restrict__ nibbles)
{
    const int64_t t0 = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t t = t0 < images ? t0 : images - 1;     // every lane runs the quantizer (it votes across the wavefront)
    const int KS = K >> 6, lane = (int)(t & 63);
    const int64_t blk = t >> 6;
    const int ks = (int)(blk % KS), rb = (int)(blk / KS);
    const int row = rb * 32 + (lane & 31), k0 = ks * 64 + (lane >> 5) * 32;
    const bool live = row < R;
    const __half* src = x + (int64_t)(live ? row : 0) * K + k0;
    uint32_t d[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const v4i raw = *reinterpret_cast<const v4i*>(src + 8 * c);
        const __half2* h2 = reinterpret_cast<const __half2*>(&raw);
        float v[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float2 f = __half22float2(h2[i]);
            v[2 * i] = f.x;
            v[2 * i + 1] = f.y;
        }
        d[c] = rq::quant_pack8<true>(v, v, mult, step, 0);
    }
    if (t0 >= images) return;
    uint64_t w[3] = {0, 0, 0};
    if (live) {
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const uint64_t e = e3m2_of_nibble((d[i >> 3] >> (4 * (i & 7))) & 15u);
            const int bit = 6 * i;
            w[bit / 64] |= e << (bit % 64);
            if (bit % 64 > 58) w[bit / 64 + 1] |= e >> (64 - bit % 64);
        }
        if (nibbles) {
            const v4i nb = {(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
            *reinterpret_cast<v4i*>(nibbles + (int64_t)row * (K >> 1) + (k0 >> 1)) = nb;
        }
    }
    uint64_t* o = reinterpret_cast<uint64_t*>(out + ((int64_t)rb * (KS >> 1) + (ks >> 1)) * kChunkF6 + lane * 48 + (ks & 1) * kImage);
    o[0] = w[0]; o[1] = w[1]; o[2] = w[2];
}

__device__ __forceinline__ int xcd_run(int b, int total)   // each XCD takes a contiguous run of tiles
{
    const int x = b & 7, idx = b >> 3, q = total >> 3, rem = total & 7;
    return x * q + (x < rem ? x : rem) + idx;
}

#define PQ6_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define PQ6_GLB(p) ((const __attribute__((address_space(1))) void*)(p))

// Tile of 64 CI channels x 256 tokens (CI = 4 or 2); wavefront (wr, wc): 32 CI channels x 128 tokens =
// CI x 4 matrix tiles.  The weights are the first operand: a lane ends with one token (l % 32) and, per
// matrix tile, the channels 8 (v / 4) + 4 (l / 32) + v % 4 in register v.
template <int CI>
__device__ __forceinline__ void f6_tile(const uint8_t* __restrict__ x6, const uint8_t* __restrict__ w6,
                                        const float* __restrict__ sw, float sx, int M, int N, int K, int m0, int n0,
                                        __half* __restrict__ out, int32_t* __restrict__ acc_out)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wr = wave >> 1, wc = wave & 1;
    constexpr int kWB = 2 * CI;                          // weight row blocks of the tile; 8 token row blocks follow
    constexpr int kStageF6 = (kWB + 8) * kChunkF6;       // 48, 42 or 36 KiB
    constexpr int kPieces = (kWB + 8) * 3;               // 1 KiB pieces of a stage
    constexpr int kLoads = (kPieces + 3) / 4;            // direct loads per wavefront per stage: 12, 11 or 9 (CI = 3:
                                                         // 42 pieces, two wavefronts repeat the last one)
    constexpr int NM = 4 * CI;                           // matrix instructions of a step
    const int KS = K >> 6, nk = K >> 7;
    const int RBX = (M + 31) >> 5, RBW = (N + 31) >> 5;

    // loader: load q = wave + 4 t of a stage is part q % 3 (1 KiB) of chunk q / 3
    uint32_t goff[kLoads];
    bool is_w[kLoads];
#pragma unroll
    for (int t = 0; t < kLoads; ++t) {
        const int q = wave + 4 * t < kPieces ? wave + 4 * t : kPieces - 1, chunk = q / 3, part = q % 3;
        int rb = chunk < kWB ? (n0 >> 5) + chunk : (m0 >> 5) + chunk - kWB;
        const int last = chunk < kWB ? RBW - 1 : RBX - 1;
        rb = rb < last ? rb : last;
        is_w[t] = chunk < kWB;
        goff[t] = (uint32_t)rb * (uint32_t)KS * (uint32_t)kStep + part * 1024 + lane * 16;
    }
    auto load_stage = [&](int kt, int buf) {
        const int k = kt < nk ? kt : nk - 1;
#pragma unroll
        for (int t = 0; t < kLoads; ++t) {
            const int q = wave + 4 * t < kPieces ? wave + 4 * t : kPieces - 1;
            const uint8_t* src = (is_w[t] ? w6 : x6) + (size_t)goff[t] + (size_t)k * kChunkF6;
            __builtin_amdgcn_global_load_lds(PQ6_GLB(src), PQ6_LDS(smem + buf * kStageF6 + q * 1024), 16, 0, 0);
        }
    };
    v16f acc[CI][4];
#pragma unroll
    for (int i = 0; i < CI; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // One of the 2 (CI + 4) LDS reads that fetch the images of a 64-channel step: piece p = 2 * operand +
    // kind, operands 0..CI-1 = weights (the row blocks of this wavefront), CI..CI+3 = tokens; kind 0 = the
    // 16-byte part of the image, 1 = the 8-byte part.  First step: bytes 0..23 of a lane's 48 (16 + 8),
    // second step: bytes 24..47 (8 + 16).
    constexpr int NP = 2 * (CI + 4);
    auto read_piece = [&](int buf, int s, int p, v8i (&a)[CI], v8i (&b)[4]) {
        const int o = p >> 1, kind = p & 1;
        const int chunk = o < CI ? wr * CI + o : kWB + wc * 4 + (o - CI);
        const uint8_t* src = smem + buf * kStageF6 + lane * 48 + chunk * kChunkF6;
        v8i& d = o < CI ? a[o < CI ? o : 0] : b[o < CI ? 0 : o - CI];
        if (kind == 0) {
            const v4i t = *(__attribute__((address_space(3))) const v4i*)(src + (s ? 32 : 0));
            if (s == 0) { d[0] = t.x; d[1] = t.y; d[2] = t.z; d[3] = t.w; }
            else { d[2] = t.x; d[3] = t.y; d[4] = t.z; d[5] = t.w; }
        } else {
            const v2i t = *(__attribute__((address_space(3))) const v2i*)(src + (s ? 24 : 16));
            if (s == 0) { d[4] = t.x; d[5] = t.y; }
            else { d[0] = t.x; d[1] = t.y; }
        }
    };
    auto read_images = [&](int buf, int s, v8i (&a)[CI], v8i (&b)[4]) {
#pragma unroll
        for (int p = 0; p < NP; ++p) read_piece(buf, s, p, a, b);
    };
    // One step: NM matrix instructions on the images (ca, cb); between them the reads of the next step's
    // images into (na, nb), spread over the first half of the instructions, and the direct loads of the
    // refill, spread over the last three quarters (a wavefront issues in order: what overlaps the matrix
    // pipe has to sit between its instructions).
    auto step = [&](const v8i (&ca)[CI], const v8i (&cb)[4], int rbuf, int rs, v8i (&na)[CI], v8i (&nb)[4], bool refill,
                    int refill_kt, int refill_buf) {
        constexpr int RS = NM / 2, D0 = NM / 4, DS = NM - D0;
#pragma unroll
        for (int n = 0; n < NM; ++n) {
            const int i = n >> 2, j = n & 3;   // formats 3, 3: E3M2 both; scale bytes 127 = 2^0
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ca[i], cb[j], acc[i][j], 3, 3, 0, 127, 0, 127);
            if (n < RS) {
#pragma unroll
                for (int p = n * NP / RS; p < (n + 1) * NP / RS; ++p) read_piece(rbuf, rs, p, na, nb);
            }
            if (refill && n >= D0) {
#pragma unroll
                for (int t = (n - D0) * kLoads / DS; t < (n - D0 + 1) * kLoads / DS; ++t) {
                    const int q = wave + 4 * t < kPieces ? wave + 4 * t : kPieces - 1;
                    const int k = refill_kt < nk ? refill_kt : nk - 1;
                    const uint8_t* src = (is_w[t] ? w6 : x6) + (size_t)goff[t] + (size_t)k * kChunkF6;
                    __builtin_amdgcn_global_load_lds(PQ6_GLB(src), PQ6_LDS(smem + refill_buf * kStageF6 + q * 1024), 16, 0, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- prologue: fill the ring, read the first step's images
#pragma unroll
    for (int st = 0; st < kRing; ++st) load_stage(st, st);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kRing - 1) * kLoads) : "memory");
    asm volatile("s_barrier" ::: "memory");
    v8i pa[CI], pb[4], qa[CI], qb[4];     // (only the first six dwords of an image count; the rest stays zero)
#pragma unroll
    for (int i = 0; i < 4; ++i) { pb[i] = (v8i){0, 0, 0, 0, 0, 0, 0, 0}; qb[i] = pb[i]; }
#pragma unroll
    for (int i = 0; i < CI; ++i) { pa[i] = (v8i){0, 0, 0, 0, 0, 0, 0, 0}; qa[i] = pa[i]; }
    read_images(0, 0, pa, pb);

    // ---- main loop: while one step multiplies, the next step's images are read; a stage's buffer is
    // free once every wavefront has read its second step, which is where the barrier sits
    int buf = 0;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    for (int kt = 0; kt < nk; ++kt) {
        // first step of stage kt; its second step's images are read meanwhile
        step(pa, pb, buf, 1, qa, qb, false, 0, 0);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kRing - 2) * kLoads) : "memory");   // own loads of stage kt + 1 landed
        asm volatile("s_barrier" ::: "memory");          // all have read stage kt; all of stage kt + 1 is in LDS
        __builtin_amdgcn_sched_barrier(0);
        // second step; the next stage's first images are read and the freed buffer is refilled meanwhile
        const int nbuf = buf + 1 == kRing ? 0 : buf + 1;
        step(qa, qb, nbuf, 0, pa, pb, true, kt + kRing, buf);   // (past the last stage: harmless re-reads)
        buf = nbuf;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // no direct load may still be writing LDS at the end
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    asm volatile("s_barrier" ::: "memory");              // the ring is free: every wavefront is past its last read

    // ---- epilogue: out = fp16(fp32(256 acc) * (sw[n] * (sx / 256))), the tiled kernel's expression.
    // A lane owns one token and groups of four channels; stored like that one instruction would touch 32
    // token rows with 8 bytes each.  Each wavefront turns its 32 tokens x 128 channels through a private,
    // padded LDS region and stores whole rows of 64 CI contiguous bytes.
    const int g = lane >> 5, r = lane & 31;
    const float f = sx * (1.0f / 256.0f);
    constexpr int kRowPitch = 64 * CI + 16;
    uint8_t* stg = smem + wave * (32 * kRowPitch);
    float4 sc[CI][4];
#pragma unroll
    for (int i = 0; i < CI; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int n = n0 + (wr * CI + i) * 32 + 8 * q + 4 * g;
            n = n + 4 <= N ? n : N - 4;
            sc[i][q] = *reinterpret_cast<const float4*>(sw + n);
            sc[i][q].x *= f; sc[i][q].y *= f; sc[i][q].z *= f; sc[i][q].w *= f;
        }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int mb = m0 + (wc * 4 + j) * 32;
        if (acc_out) {
            const int m = mb + r;
#pragma unroll
            for (int i = 0; i < CI; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = n0 + (wr * CI + i) * 32 + 8 * q + 4 * g;
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
                    const __half2 lo = __floats2half2_rn(mul_rn(acc[i][j][4 * q] * 256.0f, sc[i][q].x),
                                                         mul_rn(acc[i][j][4 * q + 1] * 256.0f, sc[i][q].y));
                    const __half2 hi = __floats2half2_rn(mul_rn(acc[i][j][4 * q + 2] * 256.0f, sc[i][q].z),
                                                         mul_rn(acc[i][j][4 * q + 3] * 256.0f, sc[i][q].w));
                    v2i val;
                    val.x = *reinterpret_cast<const int*>(&lo);
                    val.y = *reinterpret_cast<const int*>(&hi);
                    *(__attribute__((address_space(3))) v2i*)(stg + r * kRowPitch + (i * 32 + 8 * q + 4 * g) * 2) = val;
                }
            // LDS operations of a wavefront execute in order: the reads below see the writes above, and
            // the next token block's writes come after these reads
#pragma unroll
            for (int t = 0; t < 2 * CI; ++t) {
                const int id = 64 * t + lane, row = id / (4 * CI), u = id % (4 * CI);
                const v4i val = *(__attribute__((address_space(3))) const v4i*)(stg + row * kRowPitch + u * 16);
                const int m = mb + row, n = n0 + wr * (32 * CI) + u * 8;
                if (m < M && n + 8 <= N) *reinterpret_cast<v4i*>(out + (int64_t)m * N + n) = val;
            }
        }
    }
}

template <int CI>
__global__ __launch_bounds__(256) void k_gemm_f6(const uint8_t* __restrict__ x6, const uint8_t* __restrict__ w6,
                                                const float* __restrict__ sw, float sx, int M, int N, int K,
                                                int GM, __half* __restrict__ out, int32_t* __restrict__ acc_out)
{
    const int tile = xcd_run(blockIdx.x, gridDim.x);
    f6_tile<CI>(x6, w6, sw, sx, M, N, K, (tile % GM) * 256, (tile / GM) * (64 * CI), out, acc_out);
}

// Two tile widths in one launch: the first GM * n1 workgroups take 256-channel tiles of the columns
// [0, 256 n1), the others 192-channel tiles of the rest.  Workgroups are dispatched in index order, so
// with GM * n1 = GM * n2 = number of CUs every CU computes one tile of each width and none idles through
// a partial last round (gate/up: 14336 = 32 x 256 + 32 x 192).
__global__ __launch_bounds__(256) void k_gemm_f6_dual(const uint8_t* __restrict__ x6, const uint8_t* __restrict__ w6,
                                                     const float* __restrict__ sw, float sx, int M, int N, int K,
                                                     int GM, int n1, int n2, __half* __restrict__ out,
                                                     int32_t* __restrict__ acc_out)
{
    const int first = GM * n1;
    if ((int)blockIdx.x < first) {
        const int tile = xcd_run(blockIdx.x, first);
        f6_tile<4>(x6, w6, sw, sx, M, N, K, (tile % GM) * 256, (tile / GM) * 256, out, acc_out);
    } else {
        const int tile = xcd_run(blockIdx.x - first, GM * n2);
        f6_tile<3>(x6, w6, sw, sx, M, N, K, (tile % GM) * 256, n1 * 256 + (tile / GM) * 192, out, acc_out);
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

int launch_quant_f6(const void* x, int64_t R, int64_t K, float act_scale, void* out, void* nibbles, hipStream_t st)
{
    const int64_t images = ((R + 31) / 32) * (K / 64) * 64;
    hipLaunchKernelGGL(k_quant_f6, dim3((unsigned)((images + 255) / 256)), dim3(256), 0, st, static_cast<const __half*>(x),
                       (int)R, (int)K, images, (float)(1.0 / (double)act_scale), act_scale, static_cast<uint8_t*>(out),
                       static_cast<uint8_t*>(nibbles));
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
template <int CI>
int launch_f6(const void* x6, const void* w6, const float* sw, float sx, int64_t M, int64_t N, int64_t K, void* out,
              int32_t* acc, hipStream_t st)
{
    const int GM = (int)((M + 255) / 256), GN = (int)((N + 64 * CI - 1) / (64 * CI));
    constexpr size_t lds = (size_t)kRing * (2 * CI + 8) * kChunkF6;
    static_assert(lds <= 160 * 1024, "LDS ring too large");
    static_assert(4 * 32 * (64 * CI + 16) <= lds, "epilogue staging does not fit the ring");
    static std::atomic<uint64_t> lds_ok{0};
    if (allow_dynamic_lds(reinterpret_cast<const void*>(k_gemm_f6<CI>), lds, lds_ok) != PQ_OK) return PQ_ERR_HIP;
    hipLaunchKernelGGL(k_gemm_f6<CI>, dim3((unsigned)(GM * GN)), dim3(256), lds, st, static_cast<const uint8_t*>(x6),
                       static_cast<const uint8_t*>(w6), sw, sx, (int)M, (int)N, (int)K, GM, static_cast<__half*>(out), acc);
    return hip_status(hipGetLastError());
}
}  // namespace

// 256 channels per tile unless 128 fill the chip better (rounds of 256 tiles; the narrow tile costs
// about 0.6 of the wide one), or a mix of 256 and 192 in one launch where that saves a partial round.
// PQ_GEMM_F6_TILE = 2 or 4 forces one width, 3 the mix where N allows one (sweeps and tests).
int launch_gemm_f6(const void* x6, const void* w6, const float* sw, float sx, int64_t M, int64_t N, int64_t K, void* out,
                   int32_t* acc, hipStream_t st)
{
    const int64_t gm = (M + 255) / 256;
    const double wide = (double)((gm * ((N + 255) / 256) + 255) / 256) * 1.0;
    const double narrow = (double)((gm * ((N + 127) / 128) + 255) / 256) * 0.6;
    int ci = narrow < wide ? 2 : 4;
    const int forced_tile = forced_f6_tile();
    const bool forced = forced_tile != -1;
    if (forced_tile == 2 || forced_tile == 4) ci = forced_tile;
    // mixed widths: 256 n1 + 192 n2 = N; rounds of wide tiles, then rounds of 192-wide ones at 0.75 each
    if (!forced || forced_tile == 3) {
        double best = (narrow < wide ? narrow : wide) * 0.97;
        int b1 = 0, b2 = 0;
        for (int64_t n2 = 1; 192 * n2 < N; ++n2) {
            if ((N - 192 * n2) % 256 != 0) continue;
            const int64_t n1 = (N - 192 * n2) / 256;
            if (n1 < 1 || gm * (n1 + n2) > (1 << 20)) continue;
            const double cost = (double)((gm * n1 + 255) / 256) + 0.75 * (double)((gm * n2 + 255) / 256);
            if (cost < best || (forced && b1 == 0)) { best = cost; b1 = (int)n1; b2 = (int)n2; }
        }
        if (b1 > 0) {
            constexpr size_t lds = (size_t)kRing * 16 * kChunkF6;
            static std::atomic<uint64_t> lds_ok{0};
            if (allow_dynamic_lds(reinterpret_cast<const void*>(k_gemm_f6_dual), lds, lds_ok) != PQ_OK) return PQ_ERR_HIP;
            hipLaunchKernelGGL(k_gemm_f6_dual, dim3((unsigned)(gm * (b1 + b2))), dim3(256), lds, st,
                               static_cast<const uint8_t*>(x6), static_cast<const uint8_t*>(w6), sw, sx, (int)M, (int)N, (int)K,
                               (int)gm, b1, b2, static_cast<__half*>(out), acc);
            return hip_status(hipGetLastError());
        }
    }
    return ci == 2 ? launch_f6<2>(x6, w6, sw, sx, M, N, K, out, acc, st) : launch_f6<4>(x6, w6, sw, sx, M, N, K, out, acc, st);
}

}  // namespace pq
