// Tiled 4-bit x 4-bit product on the CDNA4 INT8 matrix pipe, with the dequantising
// epilogue (Sec. 3 of the paper: weight + activation quantization enable low-bit matrix
// multiplication for the compute-bound prefill; Table 1 row O2: per-tensor activation
// step, per-channel weight step).
//
//   acc[m,n] = sum_k xq[m,k] * wq[n,k]        out[m,n] = fp16(acc * (s_x * s_w[n]))
//
// Both operands are K-contiguous, which is what the matrix instruction wants: every lane
// feeds 16 consecutive bytes of one row.  Packed nibbles go from HBM straight into LDS
// (global_load_lds_dwordx4: no staging registers, no LDS store instruction), a ring of NS
// stages deep; every wavefront expands what it reads in registers into two operands holding
// 16*code: the odd-channel nibble is already in the high half of its byte, the even-channel
// nibble is shifted there, so no sign extension is needed.  The accumulator becomes
// 256 * acc and is shifted back exactly.  A dot product does not care about the order of
// its terms as long as both operands use the same order, so the even and the odd channels
// of a 32-channel group simply feed two different matrix instructions.
//
// v_mfma_i32_32x32x32_i8 operand layout (lane l, r = l % 32, g = l / 32):
//   A: row r of the 32 x 32 tile, bytes k = 16 g .. 16 g + 15;  B: column r, same bytes;
//   D: register v holds D[8 (v / 4) + 4 g + v % 4][r].
// The weights are the row operand and the activations the column operand, so a lane ends
// up with one token and groups of four consecutive output channels (16-byte stores after
// one exchange between the two half-waves).
//
// LDS layout of a stage (128 channels): plain rows of 64 packed bytes; the 16-byte chunk c
// of row q sits at chunk position c ^ ((q >> 2) & 3), which makes the 16-byte reads of 32
// consecutive rows conflict-free.  One direct load of a wavefront fills 1 KiB = 16 rows,
// lane l fetching row l / 4, position l % 4 (so 4 lanes read 64 contiguous bytes of HBM).
//
// On this chip the kernel is power-limited as much as issue-limited: with all 256 CUs busy
// on random codes the shader clock settles near 1.8 GHz, so everything that is not a matrix
// instruction (expansion, LDS traffic) costs twice: issue slots and clock.
#include "pq_internal.h"

#include <hip/hip_fp16.h>
#include <stdlib.h>
#include <atomic>
#include <type_traits>

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

// Compile-time instruction schedule of one half stage (64 channels) of a wavefront tile
// of TM x TN matrix tiles.  A wavefront issues in order, so expansion work (VALU) only
// overlaps the matrix pipe if it sits between matrix instructions in program order.  The
// half stage has two phases (even channels, odd channels) of TM*TN matrix instructions
// each.  Tiles are visited in a growing-square order so that a new operand is needed only
// every other instruction; the expansion micro-operations (2 per dword for an even
// operand: shift, mask; 1 per dword for an odd one: mask) are listed in the order the
// operands are needed and spread evenly over the slots, running `lead` micro-operations
// ahead of the instruction that needs them (into the next half stage at the end).
// With 8-bit activations (A8) only the weight operands are expanded.
template <int TM, int TN, bool A8>
struct MmaSched {
    static constexpr int NM = TM * TN, NOP = A8 ? TN : TM + TN, NSLOT = 2 * NM, PER = 12 * NOP;
    int mi[NM], mj[NM], op_is_a[NOP], op_idx[NOP], need[NSLOT], lead;
    constexpr MmaSched() : mi{}, mj{}, op_is_a{}, op_idx{}, need{}, lead(0)
    {
        int nm = 0, no = 0, before[NM] = {};
        const int D = TM > TN ? TM : TN;
        for (int d = 0; d < D; ++d) {
            if (d < TN) {
                op_is_a[no] = 0; op_idx[no] = d; ++no;
                for (int i = 0; i < (d < TM ? d : TM); ++i) { mi[nm] = i; mj[nm] = d; before[nm] = no; ++nm; }
            }
            if (d < TM) {
                if (!A8) { op_is_a[no] = 1; op_idx[no] = d; ++no; }
                for (int j = 0; j <= (d < TN - 1 ? d : TN - 1); ++j) { mi[nm] = d; mj[nm] = j; before[nm] = no; ++nm; }
            }
        }
        for (int k = 0; k < NM; ++k) { need[k] = 8 * before[k]; need[NM + k] = 8 * NOP + 4 * before[k]; }
        for (int n = 0; n < NSLOT; ++n) {
            const int def = need[n] - n * PER / NSLOT;
            if (def > lead) lead = def;
        }
    }
    // With weight operand j read in slot b_slot0 + j and activation operand i in slot a_slot0 + i of
    // the preceding half stage: is every operand read before the first micro-operation that uses it?
    constexpr bool reads_precede_expansion(int b_slot0, int a_slot0) const
    {
        for (int o = 0; o < NOP; ++o) {
            const int rs = (op_is_a[o] ? a_slot0 : b_slot0) + op_idx[o];
            if (lead + rs * PER / NSLOT > PER + 8 * o) return false;   // slot rs starts after that micro-operation
            if (lead + rs * PER / NSLOT > PER + 8 * NOP + 4 * o) return false;
        }
        return true;
    }
};
template <int TM, int TN, bool A8> inline constexpr MmaSched<TM, TN, A8> kSched{};

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

#define PQ_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define PQ_GLB(p) ((const __attribute__((address_space(1))) void*)(p))

template <int N> __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// One output tile [m0, m0 + BM) x [n0, n0 + BN) by the whole workgroup (the LDS ring is the
// workgroup's dynamic shared memory).
// SPLIT: the tile covers only the ring stages [kt0, kt0 + nk_part) of the K dimension and leaves
// its accumulators (shift undone) in acc_out, a partial-sum plane of M x N int32; nothing else is
// written.  Without SPLIT the two arguments are ignored and the whole of K is covered.
template <int BM, int BN, int WR, int WC, int NS, int SUBS, int ABITS, int ASHIFT, bool SPLIT = false>
__device__ __forceinline__ void gemm_tile(const uint8_t* xq, const uint8_t* wq, const float* sw, float sx, int M, int N,
                                          int K, int m0, int n0, __half* out, int32_t* acc_out, const float* srow,
                                          const int32_t* zcorr, int kt0 = 0, int nk_part = 0)
{
    extern __shared__ __align__(16) uint8_t smem[];
    constexpr int NW = WR * WC;
    constexpr int WM = BM / WR, WN = BN / WC, TM = WM / 32, TN = WN / 32;
    // srow: per-token step sizes [M] (per-token dynamic quantization) or NULL (one static step sx)
    // a ring stage is SUBS sub-stages of 128 channels each (one barrier per stage)
    // ABITS = 4: activations are packed nibbles like the weights.  ABITS = 8: one int8 per channel
    // (128 bytes per row per stage), in the order "even channels, then odd channels" inside every
    // group of 32, so that a 16-byte read is an operand as it stands; the accumulator then carries
    // a factor 2^ASHIFT (16 from the weights, times whatever the activation bytes carry).
    constexpr bool A8 = ABITS == 8;
    constexpr int A_ROW = A8 ? 128 : 64;
    constexpr int A_BYTES = BM * A_ROW, SUB_BYTES = A_BYTES + BN * 64, STAGE = SUBS * SUB_BYTES;
    constexpr int ABLK = A_BYTES / 1024, BLK = ABLK + BN / 16;   // 1 KiB blocks per sub-stage
    constexpr int LW = BLK / NW;          // direct loads per wavefront per sub-stage
    static_assert(BLK % NW == 0 && ABLK % NW == 0, "loader shape");
    constexpr int LWA = ABLK / NW;        // of which for the activation rows

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps LDS targets in scalar registers
    const int wm = wave / WC, wn = wave % WC;
    const int r = lane & 31, g = lane >> 5;

    const int Kb = K >> 1;
    const int nk = SPLIT ? nk_part : K / (128 * SUBS);
    if constexpr (SPLIT) {
        xq += (size_t)kt0 * SUBS * (ABITS == 8 ? 128 : 64);
        wq += (size_t)kt0 * SUBS * 64;
    }

    // ---- loader
    const int lrow = lane >> 2, lpos = lane & 3;
    const int lchunk = lpos ^ ((lrow >> 2) & 3);
    // int8 activation rows: 8 lanes per 128-byte row, 8 rows per block; the 16-byte unit at position p
    // of tile row t holds unit p ^ ((t >> 1) & 7).  Block b = wave + NW * i holds rows 8 b .. 8 b + 7 and
    // NW is even, so bit 3 of t is the wave's parity for every i.
    static_assert(NW % 2 == 0, "unit swizzle assumes an even number of wavefronts");
    const int lrow8 = lane >> 3, lchunk8 = (lane & 7) ^ (((wave & 1) << 2) | (lrow8 >> 1));
    uint32_t goff[LW];
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        const int blk = wave + NW * i;  // blocks [0, ABLK) hold activation rows, the rest weight rows
        if (i < LWA) {
            int row = m0 + (A8 ? blk * 8 + lrow8 : blk * 16 + lrow);
            row = row < M ? row : M - 1;
            goff[i] = A8 ? (uint32_t)row * (uint32_t)K + lchunk8 * 16 : (uint32_t)row * (uint32_t)Kb + lchunk * 16;
        } else {
            int row = n0 + (blk - ABLK) * 16 + lrow;
            row = row < N ? row : N - 1;
            goff[i] = (uint32_t)row * (uint32_t)Kb + lchunk * 16;
        }
    }
    auto dma_one = [&](int d, int kt, int buf) {   // d-th direct load of a stage, d < SUBS * LW
        const int sub = d / LW, i = d % LW;
        const uint8_t* src = (i < LWA ? xq + (size_t)(kt * SUBS + sub) * A_ROW : wq + (size_t)(kt * SUBS + sub) * 64) + goff[i];
        __builtin_amdgcn_global_load_lds(PQ_GLB(src),
                                         PQ_LDS(smem + buf * STAGE + sub * SUB_BYTES + (wave + NW * i) * 1024), 16, 0, 0);
    };
    auto dma_stage = [&](int kt, int buf) {
        static_for<0, SUBS * LW>([&](auto dc) { dma_one(decltype(dc)::value, kt, buf); });
    };

    // ---- reader
    const int swr = (r >> 2) & 3;
    const int rdA0 = (wm * WM + r) * 64 + (((0 + g) ^ swr) << 4), rdA1 = (wm * WM + r) * 64 + (((2 + g) ^ swr) << 4);
    // int8 rows: matrix step s of a stage reads unit 2 (2 (s / 2) + g) + (s & 1) of the row's eight
    int rdA8[4];
#pragma unroll
    for (int st = 0; st < 4; ++st)
        rdA8[st] = (wm * WM + r) * 128 + (((2 * (2 * (st >> 1) + g) + (st & 1)) ^ ((r >> 1) & 7)) << 4);
    const int rdB0 = A_BYTES + (wn * WN + r) * 64 + (((0 + g) ^ swr) << 4);
    const int rdB1 = A_BYTES + (wn * WN + r) * 64 + (((2 + g) ^ swr) << 4);

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    using SC = MmaSched<TM, TN, A8>;
    v4i pa[2][TM], pb[2][TN];         // packed operands of the current / next half stage
    v4i xa[2][2][TM], xb[2][2][TN];   // expanded: [half-stage parity][even, odd][tile]
    constexpr int MASK = (int)0xF0F0F0F0u;

    // LDS reads of one half stage: NRD of them, one per slot.  Packed activations: TM + TN reads;
    // int8 activations: two per activation tile (they are operands as they stand) + TN.
    constexpr int NRD = A8 ? 2 * TM + TN : TM + TN;
    auto read_frag = [&](const uint8_t* stage, int kk, int set, int f) {
        if constexpr (A8) {
            // weights first: their expansion starts while the previous half stage is still running
            if (f < TN)
                pb[set][f] = *reinterpret_cast<const v4i*>(stage + (kk ? rdB1 : rdB0) + f * 2048);
            else
                xa[set][(f - TN) & 1][(f - TN) >> 1] =
                    *reinterpret_cast<const v4i*>(stage + rdA8[2 * kk + ((f - TN) & 1)] + ((f - TN) >> 1) * 4096);
        } else {
            if (f < TM)
                pa[set][f] = *reinterpret_cast<const v4i*>(stage + (kk ? rdA1 : rdA0) + f * 2048);
            else
                pb[set][f - TM] = *reinterpret_cast<const v4i*>(stage + (kk ? rdB1 : rdB0) + (f - TM) * 2048);
        }
    };
    // expansion micro-operation u (0 <= u < PER) of the half stage with parity `set`
    auto micro = [&](auto setc, auto uc) {
        constexpr int set = decltype(setc)::value, u = decltype(uc)::value;
        if constexpr (u < 8 * SC::NOP) {
            constexpr int o = u / 8, d = (u % 8) / 2, kind = u % 2;
            constexpr int idx = kSched<TM, TN, A8>.op_idx[o];
            if constexpr (kSched<TM, TN, A8>.op_is_a[o]) {
                if constexpr (kind == 0) xa[set][0][idx][d] = pa[set][idx][d] << 4; else xa[set][0][idx][d] &= MASK;
            } else {
                if constexpr (kind == 0) xb[set][0][idx][d] = pb[set][idx][d] << 4; else xb[set][0][idx][d] &= MASK;
            }
        } else {
            constexpr int v = u - 8 * SC::NOP, o = v / 4, d = v % 4;
            constexpr int idx = kSched<TM, TN, A8>.op_idx[o];
            if constexpr (kSched<TM, TN, A8>.op_is_a[o]) xa[set][1][idx][d] = pa[set][idx][d] & MASK;
            else xb[set][1][idx][d] = pb[set][idx][d] & MASK;
        }
    };
    // one half stage: slot n = micro-operations [lead + n*PER/NSLOT, lead + (n+1)*PER/NSLOT), one LDS read
    // of the next half stage's operands (first TM+TN slots), optionally one direct load, one matrix instruction
    auto half_stage = [&](auto setc, const uint8_t* next_stage, int next_kk, bool dma, int dma_kt, int dma_buf) {
        constexpr int set = decltype(setc)::value;
        static_assert(SUBS * LW <= SC::NSLOT && NRD <= SC::NSLOT, "one direct load and one LDS read per slot");
        // a packed operand must be read in a slot no later than the one that runs its first
        // micro-operation (those of the next half stage's first operands run at the end of this one)
        static_assert(kSched<TM, TN, A8>.reads_precede_expansion(A8 ? 0 : TM, 0), "operand read too late");
        static_for<0, SC::NSLOT>([&](auto nc) {
            constexpr int n = decltype(nc)::value;
            if constexpr (n < NRD) read_frag(next_stage, next_kk, set ^ 1, n);
            constexpr int u0 = kSched<TM, TN, A8>.lead + n * SC::PER / SC::NSLOT, u1 = kSched<TM, TN, A8>.lead + (n + 1) * SC::PER / SC::NSLOT;
            static_for<u0, u1>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                if constexpr (u < SC::PER) micro(std::integral_constant<int, set>{}, std::integral_constant<int, u>{});
                else micro(std::integral_constant<int, set ^ 1>{}, std::integral_constant<int, u - SC::PER>{});
            });
            if constexpr (n < SUBS * LW) {
                if (dma) dma_one(n, dma_kt, dma_buf);
            }
            constexpr int ph = n / SC::NM, k = n % SC::NM;
            constexpr int i = kSched<TM, TN, A8>.mi[k], j = kSched<TM, TN, A8>.mj[k];
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xb[set][ph][j], xa[set][ph][i], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // ---- prologue: fill the ring, fetch the first operands and run the expansion `lead` ahead
#pragma unroll
    for (int st = 0; st < NS; ++st) dma_stage(st < nk ? st : nk - 1, st);
    wait_vm<(NS - 1) * SUBS * LW>();
    lds_barrier();
    static_for<0, NRD>([&](auto fc) { read_frag(smem, 0, 0, decltype(fc)::value); });
    static_for<0, kSched<TM, TN, A8>.lead>([&](auto uc) { micro(std::integral_constant<int, 0>{}, uc); });
    __builtin_amdgcn_sched_barrier(0);

    int buf = 0;
    for (int kt = 0; kt < nk; ++kt) {
        const uint8_t* cur = smem + buf * STAGE;
        const int nbuf = (buf + 1 == NS) ? 0 : buf + 1;
        // all half stages but the last: operands of the next half come from this ring stage
        static_for<0, 2 * SUBS - 1>([&](auto hc) {
            constexpr int hi = decltype(hc)::value;
            half_stage(std::integral_constant<int, hi & 1>{}, cur + ((hi + 1) / 2) * SUB_BYTES, (hi + 1) & 1, false, 0, 0);
        });
        // stage kt+1 has landed (its loads were issued NS-1 stages ago); after the barrier all
        // reads of stage kt are done, so its buffer can be refilled
        wait_vm<(NS - 2) * SUBS * LW>();
        lds_barrier();
        __builtin_amdgcn_sched_barrier(0);
        half_stage(std::integral_constant<int, 1>{}, smem + nbuf * STAGE, 0, true, kt + NS < nk ? kt + NS : nk - 1, buf);
        buf = nbuf;
    }
    wait_vm<0>();  // no direct load may still be writing LDS when the wavefront ends

    // ---- epilogue.  The weights were fed as the row operand, so a lane owns one token
    // (m = ... + r) and, per 32 x 32 tile, 16 output channels in groups of four consecutive
    // ones: register v holds channel 8 (v / 4) + 4 g + v % 4.  After scaling and conversion,
    // lanes r and r + 32 trade halves so that each holds 8 consecutive channels (16 bytes).
    // Stored like that, one instruction would touch 32 token rows with 32 bytes each; the output
    // burst of all CUs then runs at about 3 TB/s.  Instead each wavefront turns its 32 x WN block
    // through a private LDS region (rows padded by 16 bytes: conflict-free both ways) and stores
    // whole rows of WN * 2 contiguous bytes: about 4.2 TB/s.  The ring is free by now: every
    // wavefront has passed its last operand read once the barrier below is behind it.
    constexpr int UPR = TN * 4;                 // 16-byte units per row of the wavefront's block
    constexpr int ROWB = UPR * 16 + 16;         // padded row pitch in LDS
    constexpr int REGION = 32 * ROWB;
    static_assert((size_t)NW * REGION <= (size_t)NS * STAGE, "epilogue staging does not fit the ring");
    if constexpr (SPLIT) {
        // a lane's registers 4 q .. 4 q + 3 are four consecutive channels: 16-byte stores
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + wm * WM + i * 32 + r;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = n0 + wn * WN + j * 32 + 8 * q + 4 * g;
                    const v4i val = {acc[i][j][4 * q] >> ASHIFT, acc[i][j][4 * q + 1] >> ASHIFT,
                                     acc[i][j][4 * q + 2] >> ASHIFT, acc[i][j][4 * q + 3] >> ASHIFT};
                    if (m < M && n + 4 <= N) *reinterpret_cast<v4i*>(acc_out + (int64_t)m * N + n) = val;
                }
        }
        return;
    }
    lds_barrier();
    uint8_t* stg = smem + wave * REGION;
    if (acc_out) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + wm * WM + i * 32 + r;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int n = n0 + wn * WN + j * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                    if (m < M && n < N) acc_out[(int64_t)m * N + n] = acc[i][j][v] >> ASHIFT;
                }
        }
    }
    // DYN = false: one static step, folded into the channel scales once per tile column;
    // DYN = true: the token's own step (the lane owns one token per tile row) times the channel scale
    // ZP: a per-channel integer zcorr[n] joins the accumulator before scaling (zero-point of Eq. 1:
    // sum_k (c_k + 8 - z) w_k = acc + (8 - z) sum_k w_k)
    auto store_out = [&](auto dync, auto zpc) {
        constexpr bool DYN = decltype(dync)::value, ZP = decltype(zpc)::value;
        constexpr float kUnshift = 1.0f / (float)(1 << ASHIFT);   // the accumulators hold 2^ASHIFT * acc: exact
        float fm[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + wm * WM + i * 32 + r;
            fm[i] = DYN ? srow[m < M ? m : M - 1] * kUnshift : 0.0f;
        }
        float4 sc[TN][4];  // scales of this lane's channels: [8 q + 4 g, +4) for q = 0..3, per tile column
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int nb = n0 + wn * WN + j * 32;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int n = nb + 8 * q + 4 * g;
                n = n + 4 <= N ? n : N - 4;
                sc[j][q] = *reinterpret_cast<const float4*>(sw + n);
                if constexpr (!DYN) {
                    const float f = sx * kUnshift;
                    sc[j][q].x *= f; sc[j][q].y *= f; sc[j][q].z *= f; sc[j][q].w *= f;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
#pragma unroll
                for (int qp = 0; qp < 2; ++qp) {
                    uint32_t pk[4];
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2) {
                        const int q = 2 * qp + h2;
                        v4i zc = {0, 0, 0, 0};
                        if constexpr (ZP) {   // re-read per use (cache hit): keeps the static path's registers
                            int n = n0 + wn * WN + j * 32 + 8 * q + 4 * g;
                            n = n + 4 <= N ? n : N - 4;
                            zc = *reinterpret_cast<const v4i*>(zcorr + n);
                            zc.x <<= ASHIFT; zc.y <<= ASHIFT; zc.z <<= ASHIFT; zc.w <<= ASHIFT;
                        }
                        const float f0 = mul_rn((float)(acc[i][j][4 * q + 0] + zc.x), DYN ? sc[j][q].x * fm[i] : sc[j][q].x);
                        const float f1 = mul_rn((float)(acc[i][j][4 * q + 1] + zc.y), DYN ? sc[j][q].y * fm[i] : sc[j][q].y);
                        const float f2 = mul_rn((float)(acc[i][j][4 * q + 2] + zc.z), DYN ? sc[j][q].z * fm[i] : sc[j][q].z);
                        const float f3 = mul_rn((float)(acc[i][j][4 * q + 3] + zc.w), DYN ? sc[j][q].w * fm[i] : sc[j][q].w);
                        const __half2 lo = __floats2half2_rn(f0, f1), hi = __floats2half2_rn(f2, f3);
                        pk[2 * h2 + 0] = *reinterpret_cast<const uint32_t*>(&lo);
                        pk[2 * h2 + 1] = *reinterpret_cast<const uint32_t*>(&hi);
                    }
                    // pk[0..1]: channels 16 qp + 4 g + (0..3); pk[2..3]: 16 qp + 8 + 4 g + (0..3)
                    const auto s0 = __builtin_amdgcn_permlane32_swap(pk[0], pk[2], false, false);
                    const auto s1 = __builtin_amdgcn_permlane32_swap(pk[1], pk[3], false, false);
                    // lanes < 32 now hold channels 16 qp + (0..7), lanes >= 32 channels 16 qp + 8 + (0..7)
                    const v4i val = {(int)s0[0], (int)s1[0], (int)s0[1], (int)s1[1]};
                    *(__attribute__((address_space(3))) v4i*)(stg + r * ROWB + (j * 4 + 2 * qp + g) * 16) = val;
                }
            }
            // LDS operations of a wavefront execute in order: the reads below see the writes above, and
            // the next token block's writes come after these reads
#pragma unroll
            for (int t = 0; t < 2 * TN; ++t) {
                const int id = 64 * t + lane, row = id / UPR, u = id % UPR;
                const v4i val = *(__attribute__((address_space(3))) const v4i*)(stg + row * ROWB + u * 16);
                const int m = m0 + wm * WM + i * 32 + row, n = n0 + wn * WN + u * 8;
                // (non-temporal: the output is not read here again.  The same launch repeated on hot operands is
                // 20-25 % slower with them; in a sequence of layers whose weights come from HBM they leave the L2 and
                // the memory-side cache to the operands and the step is 1.5 % faster)
                if (m < M && n < N) __builtin_nontemporal_store(val, reinterpret_cast<v4i*>(out + (int64_t)m * N + n));
            }
        }
    };
    if (out) {
        if (zcorr) store_out(std::false_type{}, std::true_type{});   // (static steps only)
        else if (srow) store_out(std::true_type{}, std::false_type{});
        else store_out(std::false_type{}, std::false_type{});
    }
}

template <int BM, int BN, int WR, int WC, int NS, int SUBS, int ABITS, int ASHIFT>
__global__ __launch_bounds__(WR * WC * 64) void k_gemm_dma(const uint8_t* __restrict__ xq,
                                                          const uint8_t* __restrict__ wq,
                                                          const float* __restrict__ sw, float sx, int M, int N,
                                                          int K, int GM, __half* __restrict__ out,
                                                          int32_t* __restrict__ acc_out,
                                                          const float* __restrict__ srow,
                                                          const int32_t* __restrict__ zcorr)
{
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    gemm_tile<BM, BN, WR, WC, NS, SUBS, ABITS, ASHIFT>(xq, wq, sw, sx, M, N, K, (tile % GM) * BM, (tile / GM) * BN, out,
                                                       acc_out, srow, zcorr);
}

// Two tile widths in one launch: the first GM * n1 workgroups take tiles BM x BN1 of the columns
// [0, n1 * BN1), the others tiles BM x BN2 of the rest.  Workgroups are dispatched in index order,
// so with GM * n1 = GM * n2 = number of CUs every CU computes one tile of each width and no CU idles
// through a partial last round (gate/up: 14336 = 32 x 256 + 32 x 192).
template <int BM, int BN1, int BN2, int WR, int WC, int NS, int ABITS, int ASHIFT>
__global__ __launch_bounds__(WR * WC * 64) void k_gemm_dual(const uint8_t* __restrict__ xq,
                                                           const uint8_t* __restrict__ wq,
                                                           const float* __restrict__ sw, float sx, int M, int N,
                                                           int K, int GM, int n1, int n2, __half* __restrict__ out,
                                                           int32_t* __restrict__ acc_out,
                                                           const float* __restrict__ srow,
                                                           const int32_t* __restrict__ zcorr)
{
    const int first = GM * n1;
    if ((int)blockIdx.x < first) {
        const int tile = xcd_remap(blockIdx.x, first);
        gemm_tile<BM, BN1, WR, WC, NS, 1, ABITS, ASHIFT>(xq, wq, sw, sx, M, N, K, (tile % GM) * BM, (tile / GM) * BN1, out, acc_out,
                                                srow, zcorr);
    } else {
        const int tile = xcd_remap(blockIdx.x - first, GM * n2);
        gemm_tile<BM, BN2, WR, WC, NS, 1, ABITS, ASHIFT>(xq, wq, sw, sx, M, N, K, (tile % GM) * BM, n1 * BN1 + (tile / GM) * BN2, out,
                                                acc_out, srow, zcorr);
    }
}

template <int BM, int BN1, int BN2, int WR, int WC, int NS, int ABITS = 4, int ASHIFT = 8>
int launch_dual(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K, int n1,
                int n2, void* out, int32_t* acc, hipStream_t st, const float* srow = nullptr,
                const int32_t* zcorr = nullptr)
{
    const int GM = (int)((M + BM - 1) / BM);
    constexpr size_t lds = (size_t)NS * (BM * (ABITS == 8 ? 128 : 64) + (BN1 > BN2 ? BN1 : BN2) * 64);
    static_assert(lds <= 160 * 1024, "LDS ring too large");
    auto kern = k_gemm_dual<BM, BN1, BN2, WR, WC, NS, ABITS, ASHIFT>;
    static std::atomic<uint64_t> lds_ok{0};
    if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds, lds_ok) != PQ_OK) return PQ_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3((unsigned)(GM * (n1 + n2))), dim3(WR * WC * 64), lds, st,
                       static_cast<const uint8_t*>(xq), static_cast<const uint8_t*>(wq), sw, sx, (int)M, (int)N,
                       (int)K, GM, n1, n2, static_cast<__half*>(out), acc, srow, zcorr);
    return hip_status(hipGetLastError());
}

template <int BM, int BN, int WR, int WC, int NS, int SUBS, int ABITS = 4, int ASHIFT = 8>
int launch_dma(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K, void* out,
               int32_t* acc, hipStream_t st, const float* srow = nullptr, const int32_t* zcorr = nullptr)
{
    const int GM = (int)((M + BM - 1) / BM), GN = (int)((N + BN - 1) / BN);
    constexpr size_t lds = (size_t)NS * SUBS * (BM * (ABITS == 8 ? 128 : 64) + BN * 64);
    static_assert(lds <= 160 * 1024, "LDS ring too large");
    auto kern = k_gemm_dma<BM, BN, WR, WC, NS, SUBS, ABITS, ASHIFT>;
    static std::atomic<uint64_t> lds_ok{0};
    if (lds > 48 * 1024 && allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds, lds_ok) != PQ_OK)
        return PQ_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3((unsigned)(GM * GN)), dim3(WR * WC * 64), lds, st,
                       static_cast<const uint8_t*>(xq), static_cast<const uint8_t*>(wq), sw, sx, (int)M, (int)N,
                       (int)K, GM, static_cast<__half*>(out), acc, srow, zcorr);
    return hip_status(hipGetLastError());
}

// ---------------------------------------------------------------------------------------
// Split K: for a few dozen to a few hundred tokens the output has far fewer tiles than the chip has
// CUs and a tile's time is set by K alone.  Workgroup (tile, s) covers the s-th of S nearly equal
// runs of 128-channel stages and leaves an int32 plane of partial sums in the caller's workspace;
// k_splitk_reduce adds the planes and applies the same epilogue arithmetic as the tiled kernel
// (integer sums are exact in any order, so accumulators and outputs equal the unsplit ones).
template <int BM, int BN, int WR, int WC, int NS, int ABITS, int ASHIFT>
__global__ __launch_bounds__(WR * WC * 64) void k_gemm_splitk(const uint8_t* __restrict__ xq,
                                                             const uint8_t* __restrict__ wq, int M, int N, int K,
                                                             int GM, int tiles, int S, int32_t* __restrict__ part)
{
    // each XCD takes a contiguous run of (run, tile) pairs, row tiles fastest: the row tiles of one
    // column panel meet in one L2 and fetch its weights once
    const int w = xcd_remap(blockIdx.x, gridDim.x);
    const int tile = w % tiles, s = w / tiles;
    const int nk = K / 128;
    const int kt0 = (int)((int64_t)nk * s / S), kt1 = (int)((int64_t)nk * (s + 1) / S);
    gemm_tile<BM, BN, WR, WC, NS, 1, ABITS, ASHIFT, true>(xq, wq, nullptr, 0.0f, M, N, K, (tile % GM) * BM, (tile / GM) * BN,
                                                          nullptr, part + (int64_t)s * M * N, nullptr, nullptr, kt0,
                                                          kt1 - kt0);
}

// 4 consecutive channels of one token per thread: sum of the S planes (four loads in flight), then
// acc and / or the tiled kernel's epilogue expression: with u = 2^shift (the factor its accumulators
// carry) out = fp16(fp32(u (acc + zcorr[n])) * (sw[n] * (step / u))), step = sx or the token's own.
__global__ __launch_bounds__(256) void k_splitk_reduce(const int32_t* __restrict__ part, int S, int64_t plane,
                                                       const float* __restrict__ sw, float sx, int N, int shift,
                                                       const float* __restrict__ srow,
                                                       const int32_t* __restrict__ zcorr, __half* __restrict__ out,
                                                       int32_t* __restrict__ acc_out)
{
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= plane) return;
    const int n = (int)(e % N);
    const int32_t* p = part + e;
    v4i a = {0, 0, 0, 0};
    int s = 0;
    for (; s + 4 <= S; s += 4) {
        const v4i t0 = *reinterpret_cast<const v4i*>(p + (s + 0) * plane), t1 = *reinterpret_cast<const v4i*>(p + (s + 1) * plane);
        const v4i t2 = *reinterpret_cast<const v4i*>(p + (s + 2) * plane), t3 = *reinterpret_cast<const v4i*>(p + (s + 3) * plane);
        a += (t0 + t1) + (t2 + t3);
    }
    for (; s < S; ++s) a += *reinterpret_cast<const v4i*>(p + s * plane);
    if (acc_out) *reinterpret_cast<v4i*>(acc_out + e) = a;
    if (out) {
        if (zcorr) a += *reinterpret_cast<const v4i*>(zcorr + n);
        const float f = (srow ? srow[e / N] : sx) * (1.0f / (float)(1 << shift));
        float4 s0 = *reinterpret_cast<const float4*>(sw + n);
        s0.x *= f; s0.y *= f; s0.z *= f; s0.w *= f;
        const __half2 h0 = __floats2half2_rn(mul_rn((float)(a.x << shift), s0.x), mul_rn((float)(a.y << shift), s0.y));
        const __half2 h1 = __floats2half2_rn(mul_rn((float)(a.z << shift), s0.z), mul_rn((float)(a.w << shift), s0.w));
        uint2 val;
        val.x = *reinterpret_cast<const uint32_t*>(&h0);
        val.y = *reinterpret_cast<const uint32_t*>(&h1);
        *reinterpret_cast<uint2*>(out + e) = val;
    }
}

struct SplitArgs {   // what the epilogue needs beyond the channel scales
    float sx;
    const float* srow;
    const int32_t* zcorr;
};

template <int BM, int ABITS>
int launch_splitk(const void* xq, const void* wq, const float* sw, SplitArgs ep, int64_t M, int64_t N, int64_t K, int S,
                  void* out, int32_t* acc, int32_t* part, hipStream_t st)
{
    // (a ring of 4 or 6 stages measured the same as 3)
    constexpr int BN = 128, NS = 3, ASHIFT = ABITS == 8 ? 4 : 8;
    const int GM = (int)((M + BM - 1) / BM), GN = (int)((N + BN - 1) / BN);
    constexpr size_t lds = (size_t)NS * (BM * (ABITS == 8 ? 128 : 64) + BN * 64);
    static_assert(lds <= 160 * 1024, "LDS ring too large");
    auto kern = k_gemm_splitk<BM, BN, 2, 2, NS, ABITS, ASHIFT>;
    static std::atomic<uint64_t> lds_ok{0};
    if (lds > 48 * 1024 && allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds, lds_ok) != PQ_OK)
        return PQ_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3((unsigned)(GM * GN * S)), dim3(256), lds, st, static_cast<const uint8_t*>(xq),
                       static_cast<const uint8_t*>(wq), (int)M, (int)N, (int)K, GM, GM * GN, S, part);
    if (hipGetLastError() != hipSuccess) return PQ_ERR_HIP;
    const int64_t plane = M * N;
    hipLaunchKernelGGL(k_splitk_reduce, dim3((unsigned)((plane / 4 + 255) / 256)), dim3(256), 0, st, part, S, plane, sw,
                       ep.sx, (int)N, ASHIFT, ep.srow, ep.zcorr, static_cast<__half*>(out), acc);
    return hip_status(hipGetLastError());
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
                    if (out) out[(int64_t)m * N + n] = __float2half_rn(mul_rn((float)a, sc));
                }
            }
        }
    }
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

constexpr int64_t kMaxK4 = 131072;   // first K at which 256 * 64 * K no longer fits int32

struct TileCfg { int bm, bn; double eff, stage_us; };   // stage_us: one 128-channel stage of one tile, all CUs busy
// tile shapes the automatic choice considers, with measured relative efficiencies (a larger
// wavefront tile needs fewer LDS reads and less expansion per matrix instruction; 64 x 128 is for
// outputs of at most 256 such tiles, where a tile's time is the walk over K: 14.8 against 16.9 us
// for 128 x 128 at K = 4096, 40.7 against 46.5 at K = 14336)
constexpr int kNumAuto = 5, kNumCfg = 9;
constexpr TileCfg kCfgs[kNumCfg] = {{256, 256, 1.00, 1.35}, {256, 128, 0.85, 0.77}, {128, 128, 0.72, 0.42},
                                    {256, 192, 0.95, 1.05}, {64, 128, 0.41, 0.33},  {256, 256, 1.0, 1.35},
                                    {256, 256, 1.0, 1.35},  {256, 128, 1.0, 0.77},  {256, 128, 1.0, 0.77}};

// PQ_GEMM_TILE=0..8 forces a configuration (sweeps only): 0 256x256, 1 256x128, 2 128x128,
// 3 256x192, 4 64x128, 5 256x256 with 8 wavefronts, 6 256x256 with a 4-stage ring, 7 and 8 256x128
// with 8 wavefronts (4x2 and 2x4).
// Forced tile configuration: -1 none; set by pq_set_gemm_tile, and before the first such call by the
// environment variable PQ_GEMM_TILE, which is read once (no getenv on the per-call path).
constexpr int kTileUnread = -100;
std::atomic<int> g_forced_tile{kTileUnread};

int forced_tile()
{
    int v = g_forced_tile.load(std::memory_order_relaxed);
    if (v == kTileUnread) {
        const char* f = getenv("PQ_GEMM_TILE");
        v = f ? atoi(f) : -1;
        if (v < -1 || v >= kNumCfg) v = -1;
        int expected = kTileUnread;
        g_forced_tile.compare_exchange_strong(expected, v);   // a concurrent pq_set_gemm_tile wins
        v = g_forced_tile.load(std::memory_order_relaxed);
    }
    return v;
}

int pick_cfg(int64_t M, int64_t N)
{
    if (forced_tile() >= 0) return forced_tile();
    int best = 0;
    double best_cost = 1e300;
    for (int c = 0; c < kNumAuto; ++c) {
        const int64_t tiles = ((M + kCfgs[c].bm - 1) / kCfgs[c].bm) * ((N + kCfgs[c].bn - 1) / kCfgs[c].bn);
        const int64_t rounds = (tiles + 255) / 256;
        const double cost = (double)rounds * kCfgs[c].bm * kCfgs[c].bn / kCfgs[c].eff;
        if (cost < best_cost) { best_cost = cost; best = c; }
    }
    return best;
}

// Is a launch of n1 column panels of 256 and n2 of 192 (256 n1 + 192 n2 = N) cheaper than the best
// single width?  Tiles go to the earliest free CU in index order; a tile's cost is its area over the
// width's efficiency (the same model as pick_cfg).  PQ_GEMM_TILE switches the mixed launch off.
bool pick_dual(int64_t M, int64_t N, int* n1_out, int* n2_out)
{
    if (forced_tile() != -1 || (N % 64) != 0 || M < 256) return false;
    const int64_t GM = (M + 255) / 256;
    double single = 1e300;
    for (int c = 0; c < kNumAuto; ++c) {
        const int64_t tiles = ((M + kCfgs[c].bm - 1) / kCfgs[c].bm) * ((N + kCfgs[c].bn - 1) / kCfgs[c].bn);
        const double cost = (double)((tiles + 255) / 256) * kCfgs[c].bm * kCfgs[c].bn / kCfgs[c].eff;
        if (cost < single) single = cost;
    }
    const double t1 = 256.0 * 256.0 / kCfgs[0].eff, t2 = 256.0 * 192.0 / kCfgs[3].eff;
    double best = single * 0.97;   // the mixed launch has to win by a margin
    bool found = false;
    for (int64_t n2 = 1; 192 * n2 < N; ++n2) {
        if ((N - 192 * n2) % 256 != 0) continue;
        const int64_t n1 = (N - 192 * n2) / 256;
        if (n1 < 1 || GM * (n1 + n2) > 1 << 20) continue;
        // 256 CUs take tiles in order: all wide tiles first
        const int64_t a = GM * n1, b = GM * n2;
        const int64_t ra = a / 256, xa = a % 256;        // full rounds of wide tiles, CUs with one more
        // after the wide tiles, xa CUs are busy until (ra + 1) t1 and 256 - xa until ra t1; narrow tiles fill in order
        double finish;
        if (xa == 0) {
            finish = ra * t1 + (double)((b + 255) / 256) * t2;
        } else {
            const int64_t early = 256 - xa;               // CUs free at ra * t1
            // narrow tiles: the early CUs take floor(t1 / t2) + ... ; model conservatively by time steps of t2
            int64_t left = b;
            double t_early = ra * t1, t_late = (ra + 1) * t1;
            // hand tiles to whichever group frees first until none are left
            while (left > 0) {
                if (t_early <= t_late) { left -= early < left ? early : left; t_early += t2; }
                else { left -= xa < left ? xa : left; t_late += t2; }
            }
            finish = t_early > t_late ? t_early : t_late;
            if (finish < (ra + 1) * t1) finish = (ra + 1) * t1;
        }
        if (finish < best) { best = finish; *n1_out = (int)n1; *n2_out = (int)n2; found = true; }
    }
    return found;
}

// Tile height and number of K runs of the split launch, from a cost model in microseconds
// (per 128-channel stage: 0.27-0.33 for a 64 x 128 tile, 0.42 for 128 x 128, 0.77 for 256 x 128, 1.35
// for 256 x 256; 3.5 fixed for the unsplit launch, 5.8 for the split pair; partial planes written
// and read back at ~4 TB/s).  S = 1: the unsplit kernel is cheaper or the workspace holds no two planes.
void plan_splitk(int64_t M, int64_t N, int64_t K, size_t ws_bytes, bool force, int* bm_out, int* s_out)
{
    *bm_out = 128;
    *s_out = 1;
    if (K % 128 != 0 || N % 8 != 0 || M * N >= ((int64_t)1 << 31)) return;
    const int64_t nk = K / 128;
    if (force) {   // as many runs as fit, up to 5 (an odd count: uneven runs); the lowest tile that covers M
        int S = 5;
        while (S > 1 && ((int64_t)S * 2 > nk || (size_t)S * (size_t)M * N * 4 > ws_bytes)) --S;
        *bm_out = M > 128 ? 256 : (M > 64 ? 128 : 64);
        *s_out = S;
        return;
    }
    double best = gemm_unsplit_cost_us(M, N, K) - 1.0;   // the split pair has to win by a margin
    const size_t plane_bytes = (size_t)M * N * 4;
    for (int bm = M <= 128 ? 64 : 128; bm <= 256; bm *= 2) {   // (four row tiles of 64: down_proj measured 5 us slower)
        const int64_t tiles = ((M + bm - 1) / bm) * ((N + 127) / 128);
        const double tk = bm == 64 ? 0.27 : (bm == 128 ? 0.42 : 0.77);
        for (int S = 2; S <= 32 && (int64_t)S * 2 <= nk && (size_t)S * plane_bytes <= ws_bytes; ++S) {
            const int64_t rounds = (tiles * S + 255) / 256;
            const double cost = 5.8 + (double)rounds * (double)((nk + S - 1) / S) * tk +
                                (2.0 * S * plane_bytes + (double)M * N * 2) / 4.0e6;
            if (cost < best) { best = cost; *bm_out = bm; *s_out = S; }
        }
    }
}

}  // namespace

int launch_gemm_mfma(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
                     void* out, int32_t* acc, hipStream_t st)
{
    // the accumulators carry 256 * acc in int32 and |acc| <= 64 K: exact for K < 2^17 only
    if (M > (1 << 30) || N > (1 << 30) || K >= kMaxK4) return PQ_ERR_UNSUPPORTED;
    if (M * (K / 2) >= ((int64_t)1 << 32) || N * (K / 2) >= ((int64_t)1 << 32)) return PQ_ERR_UNSUPPORTED;
    if (K % 128 != 0) return launch_ragged(xq, wq, sw, sx, M, N, K, out, acc, st);
    // (two 128-channel sub-stages per ring stage, i.e. one barrier per 256 channels with a 2-deep
    // ring, measured 3-10 % slower than a 3-deep ring of single sub-stages: depth wins)
    int n1 = 0, n2 = 0;
    if (pick_dual(M, N, &n1, &n2)) return launch_dual<256, 256, 192, 2, 2, 3>(xq, wq, sw, sx, M, N, K, n1, n2, out, acc, st);
    switch (pick_cfg(M, N)) {
        case 0: return launch_dma<256, 256, 2, 2, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st);
        case 1: return launch_dma<256, 128, 2, 2, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st);
        case 2: return launch_dma<128, 128, 2, 2, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st);
        case 3: return launch_dma<256, 192, 2, 2, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st);
        case 4: return launch_dma<64, 128, 2, 2, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st);
        case 5: return launch_dma<256, 256, 2, 4, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st);
        case 7: return launch_dma<256, 128, 4, 2, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st);
        case 8: return launch_dma<256, 128, 2, 4, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st);
        default: return launch_dma<256, 256, 2, 2, 4, 1>(xq, wq, sw, sx, M, N, K, out, acc, st);
    }
}

int set_gemm_tile(int tile)
{
    if (tile < -1 || tile >= kNumCfg) return -2;
    const int prev = forced_tile();
    g_forced_tile.store(tile);
    return prev;
}

// The cost model's figure for the unsplit tiled launch, in microseconds (the best automatic tile;
// K % 128 != 0 takes the generic kernel, which is not modelled: a large number).
double gemm_unsplit_cost_us(int64_t M, int64_t N, int64_t K)
{
    if (K % 128 != 0) return 1e9;
    const int64_t nk = K / 128;
    double best = 1e300;
    for (int c = 0; c < kNumAuto; ++c) {
        const int64_t tiles = ((M + kCfgs[c].bm - 1) / kCfgs[c].bm) * ((N + kCfgs[c].bn - 1) / kCfgs[c].bn);
        const double cost = 3.5 + (double)((tiles + 255) / 256) * nk * kCfgs[c].stage_us + (double)M * N * 2 / 4.2e6;
        if (cost < best) best = cost;
    }
    return best;
}

size_t gemm_splitk_workspace_bytes(int64_t M, int64_t N, int64_t K, bool force)
{
    int bm, S;
    plan_splitk(M, N, K, ~(size_t)0, force, &bm, &S);
    return S > 1 ? (size_t)S * (size_t)M * (size_t)N * 4 : 0;
}

namespace {
// The split launch if the plan has one for this workspace; -1: the caller runs the unsplit kernel.
template <int ABITS>
int try_splitk(const void* xq, const void* wq, const float* sw, SplitArgs ep, int64_t M, int64_t N, int64_t K, void* out,
               int32_t* acc, void* ws, size_t ws_bytes, bool force, hipStream_t st)
{
    int bm = 128, S = 1;
    if (ws) plan_splitk(M, N, K, ws_bytes, force, &bm, &S);
    if (S <= 1) return force ? PQ_ERR_UNSUPPORTED : -1;
    int32_t* part = static_cast<int32_t*>(ws);
    if (bm == 64) return launch_splitk<64, ABITS>(xq, wq, sw, ep, M, N, K, S, out, acc, part, st);
    if (bm == 128) return launch_splitk<128, ABITS>(xq, wq, sw, ep, M, N, K, S, out, acc, part, st);
    return launch_splitk<256, ABITS>(xq, wq, sw, ep, M, N, K, S, out, acc, part, st);
}
}  // namespace

int launch_gemm_mfma_ws(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
                        void* out, int32_t* acc, void* ws, size_t ws_bytes, bool force, hipStream_t st)
{
    if (M <= (1 << 30) && N <= (1 << 30) && K < kMaxK4 && M * (K / 2) < ((int64_t)1 << 32) &&
        N * (K / 2) < ((int64_t)1 << 32)) {
        const int rc = try_splitk<4>(xq, wq, sw, SplitArgs{sx, nullptr, nullptr}, M, N, K, out, acc, ws, ws_bytes, force, st);
        if (rc >= 0) return rc;
    } else if (force) {
        return PQ_ERR_UNSUPPORTED;
    }
    return launch_gemm_mfma(xq, wq, sw, sx, M, N, K, out, acc, st);
}

// 4-bit weights x 8-bit activations (codes in the even/odd-grouped byte order written by the
// 8-bit quantizer): the same kernel with the activation operand taken from LDS as it stands.
int launch_gemm_w4a8(const void* xq8, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
                     void* out, int32_t* acc, hipStream_t st, void* ws, size_t ws_bytes, bool force)
{
    if (M > (1 << 30) || N > (1 << 30) || K > 65536 || K % 128 != 0) return PQ_ERR_UNSUPPORTED;
    if (M * K >= ((int64_t)1 << 32) || N * (K / 2) >= ((int64_t)1 << 32)) return PQ_ERR_UNSUPPORTED;
    const int rc = try_splitk<8>(xq8, wq, sw, SplitArgs{sx, nullptr, nullptr}, M, N, K, out, acc, ws, ws_bytes, force, st);
    if (rc >= 0) return rc;
    int n1 = 0, n2 = 0;
    if (pick_dual(M, N, &n1, &n2))
        return launch_dual<256, 256, 192, 2, 2, 3, 8, 4>(xq8, wq, sw, sx, M, N, K, n1, n2, out, acc, st);
    switch (pick_cfg(M, N)) {
        case 0: return launch_dma<256, 256, 2, 2, 3, 1, 8, 4>(xq8, wq, sw, sx, M, N, K, out, acc, st);
        case 1: return launch_dma<256, 128, 2, 2, 3, 1, 8, 4>(xq8, wq, sw, sx, M, N, K, out, acc, st);
        case 3: return launch_dma<256, 192, 2, 2, 3, 1, 8, 4>(xq8, wq, sw, sx, M, N, K, out, acc, st);
        case 4: return launch_dma<64, 128, 2, 2, 3, 1, 8, 4>(xq8, wq, sw, sx, M, N, K, out, acc, st);
        default: return launch_dma<128, 128, 2, 2, 3, 1, 8, 4>(xq8, wq, sw, sx, M, N, K, out, acc, st);
    }
}

// Per-token dynamic quantization (Table 1 row O1): out = acc * row_scale[m] * w_scale[n].  bits = 4
// (packed codes) or 8 (grouped bytes).
int launch_gemm_dynamic(const void* xq, int32_t bits, const void* wq, const float* sw, const float* srow, int64_t M,
                        int64_t N, int64_t K, void* out, int32_t* acc, hipStream_t st, void* ws, size_t ws_bytes,
                        bool force)
{
    if (M > (1 << 30) || N > (1 << 30) || K > 65536 || K % 128 != 0) return PQ_ERR_UNSUPPORTED;
    if (M * K >= ((int64_t)1 << 32) || N * (K / 2) >= ((int64_t)1 << 32)) return PQ_ERR_UNSUPPORTED;
    {
        const SplitArgs ep{1.0f, srow, nullptr};
        const int rc = bits == 8 ? try_splitk<8>(xq, wq, sw, ep, M, N, K, out, acc, ws, ws_bytes, force, st)
                                 : try_splitk<4>(xq, wq, sw, ep, M, N, K, out, acc, ws, ws_bytes, force, st);
        if (rc >= 0) return rc;
    }
    const int cfg = pick_cfg(M, N);
    int n1 = 0, n2 = 0;
    const bool dual = pick_dual(M, N, &n1, &n2);
    if (bits == 8) {
        if (dual) return launch_dual<256, 256, 192, 2, 2, 3, 8, 4>(xq, wq, sw, 1.0f, M, N, K, n1, n2, out, acc, st, srow);
        switch (cfg) {
            case 0: return launch_dma<256, 256, 2, 2, 3, 1, 8, 4>(xq, wq, sw, 1.0f, M, N, K, out, acc, st, srow);
            case 1: return launch_dma<256, 128, 2, 2, 3, 1, 8, 4>(xq, wq, sw, 1.0f, M, N, K, out, acc, st, srow);
            case 3: return launch_dma<256, 192, 2, 2, 3, 1, 8, 4>(xq, wq, sw, 1.0f, M, N, K, out, acc, st, srow);
            case 4: return launch_dma<64, 128, 2, 2, 3, 1, 8, 4>(xq, wq, sw, 1.0f, M, N, K, out, acc, st, srow);
            default: return launch_dma<128, 128, 2, 2, 3, 1, 8, 4>(xq, wq, sw, 1.0f, M, N, K, out, acc, st, srow);
        }
    }
    if (dual) return launch_dual<256, 256, 192, 2, 2, 3>(xq, wq, sw, 1.0f, M, N, K, n1, n2, out, acc, st, srow);
    switch (cfg) {
        case 0: return launch_dma<256, 256, 2, 2, 3, 1>(xq, wq, sw, 1.0f, M, N, K, out, acc, st, srow);
        case 1: return launch_dma<256, 128, 2, 2, 3, 1>(xq, wq, sw, 1.0f, M, N, K, out, acc, st, srow);
        case 3: return launch_dma<256, 192, 2, 2, 3, 1>(xq, wq, sw, 1.0f, M, N, K, out, acc, st, srow);
        case 4: return launch_dma<64, 128, 2, 2, 3, 1>(xq, wq, sw, 1.0f, M, N, K, out, acc, st, srow);
        default: return launch_dma<128, 128, 2, 2, 3, 1>(xq, wq, sw, 1.0f, M, N, K, out, acc, st, srow);
    }
}

// Static steps with a zero-point (Eq. 1): out = (acc + zcorr[n]) * s_x * s_w[n].
int launch_gemm_zp(const void* xq, const void* wq, const float* sw, float sx, const int32_t* zcorr, int64_t M, int64_t N,
                   int64_t K, void* out, int32_t* acc, hipStream_t st, void* ws, size_t ws_bytes, bool force)
{
    if (M > (1 << 30) || N > (1 << 30) || K > 32768 || K % 128 != 0) return PQ_ERR_UNSUPPORTED;
    if (M * (K / 2) >= ((int64_t)1 << 32) || N * (K / 2) >= ((int64_t)1 << 32)) return PQ_ERR_UNSUPPORTED;
    const int rc = try_splitk<4>(xq, wq, sw, SplitArgs{sx, nullptr, zcorr}, M, N, K, out, acc, ws, ws_bytes, force, st);
    if (rc >= 0) return rc;
    int n1 = 0, n2 = 0;
    if (pick_dual(M, N, &n1, &n2))
        return launch_dual<256, 256, 192, 2, 2, 3>(xq, wq, sw, sx, M, N, K, n1, n2, out, acc, st, nullptr, zcorr);
    switch (pick_cfg(M, N)) {
        case 0: return launch_dma<256, 256, 2, 2, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st, nullptr, zcorr);
        case 1: return launch_dma<256, 128, 2, 2, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st, nullptr, zcorr);
        case 3: return launch_dma<256, 192, 2, 2, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st, nullptr, zcorr);
        case 4: return launch_dma<64, 128, 2, 2, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st, nullptr, zcorr);
        default: return launch_dma<128, 128, 2, 2, 3, 1>(xq, wq, sw, sx, M, N, K, out, acc, st, nullptr, zcorr);
    }
}

}  // namespace pq
