// Device-side building blocks of the online rotation + quantizer, shared by the stand-alone
// kernels, the fused decode kernel and the calibration kernels (App. B "Online Rotation" and Eq. 1
// of the paper).  A workgroup of 256 threads transforms one chunk of a row; what the quantizer's
// step is (static, per head, per token, per group, with a zero-point) comes from a step provider,
// and an input transform can fuse an elementwise producer in front.
#pragma once

#include "pq_internal.h"

#include <hip/hip_fp16.h>
#include <type_traits>

namespace pq {
namespace rq {

constexpr int kThreads = 256;
constexpr int kChunk = 2048;  // channels per workgroup per group index

// ---- partner exchange between lanes: returns the value held by lane (id ^ (1 << B)).
template <int B>
__device__ __forceinline__ int lane_xor_i(int iv)
{
    int r;
    if constexpr (B == 0) {
        r = __builtin_amdgcn_update_dpp(iv, iv, 0xB1, 0xF, 0xF, false);  // quad_perm [1,0,3,2]
    } else if constexpr (B == 1) {
        r = __builtin_amdgcn_update_dpp(iv, iv, 0x4E, 0xF, 0xF, false);  // quad_perm [2,3,0,1]
    } else if constexpr (B == 2) {
        // lanes 0-3 and 8-11 of each row of 16 take lane+4, the others lane-4
        r = __builtin_amdgcn_update_dpp(iv, iv, 0x104, 0xF, 0x5, false);  // row_shl:4
        r = __builtin_amdgcn_update_dpp(r, iv, 0x114, 0xF, 0xA, false);   // row_shr:4
    } else if constexpr (B == 3) {
        r = __builtin_amdgcn_update_dpp(iv, iv, 0x128, 0xF, 0xF, false);  // row_ror:8
    } else if constexpr (B == 4) {
        r = __builtin_amdgcn_ds_swizzle(iv, 0x401F);  // bit-mask mode: and 0x1F, xor 0x10
    } else {
        r = __shfl_xor(iv, 32, 64);
    }
    return r;
}

template <int B>
__device__ __forceinline__ float lane_xor(float v)
{
    return __int_as_float(lane_xor_i<B>(__float_as_int(v)));
}

template <int B, int NV>
__device__ __forceinline__ void lane_stage(float (&v)[NV], int lane)
{
    const bool upper = (lane >> B) & 1;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const float p = lane_xor<B>(v[i]);
        v[i] = upper ? (p - v[i]) : (p + v[i]);
    }
}

// d = 1, 2, 4 inside one group of 8
__device__ __forceinline__ void reg_stages8(float* v, int nstages)
{
    if (nstages >= 1) {
#pragma unroll
        for (int i = 0; i < 8; i += 2) { float a = v[i], b = v[i + 1]; v[i] = a + b; v[i + 1] = a - b; }
    }
    if (nstages >= 2) {
#pragma unroll
        for (int i = 0; i < 8; i += 4)
#pragma unroll
            for (int j = 0; j < 2; ++j) { float a = v[i + j], b = v[i + j + 2]; v[i + j] = a + b; v[i + j + 2] = a - b; }
    }
    if (nstages >= 3) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { float a = v[j], b = v[j + 4]; v[j] = a + b; v[j + 4] = a - b; }
    }
}

// Round-to-nearest-even of eight scaled values, clamp to [-8,7], pack low nibble first.
// `magic` puts round(t) + 8 into the low mantissa bits of an fp32 in [2^23, 2^24).
constexpr float kMagic = 12582920.0f;            // 1.5 * 2^23 + 8, bit pattern 0x4B400008
constexpr uint32_t kMagicSum = 0x4B400000u * 0x11111111u;  // sum of (pattern - offset part) << 4i

// zo = zero-point - 8 (Eq. 1 with a zero-point z: stored code = clamp(round(t) + z, 0, 15) - 8); 0 for
// the symmetric quantizer, in which case the compiler drops every trace of it.
template <bool EXACT>
__device__ __forceinline__ uint32_t quant_pack8(const float* v, const float* raw, float mult, float step, int zo = 0)
{
    float t[8];
    uint32_t bits[8];
    bool suspect = false;
    const float lo = -8.0f - (float)zo, hi = 7.0f - (float)zo;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        t[i] = v[i] * mult;
        const float c = __builtin_amdgcn_fmed3f(t[i], lo, hi);
        const float r = c + kMagic;                 // fp32 add rounds to an integer, ties to even
        bits[i] = __float_as_uint(r) + (uint32_t)zo;   // the offset enters after the rounding (integer add)
        if constexpr (EXACT) {
            const float f = c - (r - kMagic);       // exact; |f| <= 0.5
            suspect |= (fabsf(f) > 0.5f - 0x1.0p-18f);
        }
    }
    if constexpr (EXACT) {
        // t carries two fp32 roundings (reciprocal and product), so a quotient within
        // ~1e-6 of k + 1/2 may have been rounded to the wrong side.  Decide those from
        // the sign of (k + 1/2) * step - x, which one fused multiply-add gives exactly.
        if (__builtin_amdgcn_ballot_w64(suspect) != 0) {   // wave-uniform: a real branch, taken rarely
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float c = __builtin_amdgcn_fmed3f(t[i], lo, hi);
                const float r = c + kMagic;
                const float f = c - (r - kMagic);
                if (fabsf(f) > 0.5f - 0x1.0p-18f) {
                    const float k = floorf(t[i]);
                    const float d = fmaf(k + 0.5f, step, -raw[i]);
                    const int ki = (int)k;
                    int q = (d > 0.0f ? ki : (d < 0.0f ? ki + 1 : ((ki & 1) ? ki + 1 : ki))) + zo;
                    q = q < -8 ? -8 : (q > 7 ? 7 : q);
                    bits[i] = 0x4B400008u + (uint32_t)q;
                }
            }
        }
    }
    uint32_t s = bits[7];
#pragma unroll
    for (int i = 6; i >= 0; --i) s = (s << 4) + bits[i];
    return (s - kMagicSum) ^ 0x88888888u;   // offset-binary nibbles -> two's complement
}

// 8-bit variant: codes in [-128, 127], one byte each.  The four even-channel bytes and the four
// odd-channel bytes of the thread's eight channels are returned as two dwords.
constexpr float kMagic8 = 12582912.0f;   // 1.5 * 2^23, bit pattern 0x4B400000: low byte = code

template <bool EXACT>
__device__ __forceinline__ void quant_bytes8(const float* v, const float* raw, float mult, float step, uint32_t& even4,
                                             uint32_t& odd4)
{
    float t[8];
    uint32_t bits[8];
    bool suspect = false;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        t[i] = v[i] * mult;
        const float c = __builtin_amdgcn_fmed3f(t[i], -128.0f, 127.0f);
        const float r = c + kMagic8;
        bits[i] = __float_as_uint(r);
        if constexpr (EXACT) {
            const float f = c - (r - kMagic8);
            suspect |= (fabsf(f) > 0.5f - 0x1.0p-14f);   // |t| <= 128: two roundings move t by < 2^-15
        }
    }
    if constexpr (EXACT) {
        if (__builtin_amdgcn_ballot_w64(suspect) != 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float c = __builtin_amdgcn_fmed3f(t[i], -128.0f, 127.0f);
                const float r = c + kMagic8;
                const float f = c - (r - kMagic8);
                if (fabsf(f) > 0.5f - 0x1.0p-14f) {
                    const float k = floorf(t[i]);
                    const float d = fmaf(k + 0.5f, step, -raw[i]);
                    const int ki = (int)k;
                    int q = d > 0.0f ? ki : (d < 0.0f ? ki + 1 : ((ki & 1) ? ki + 1 : ki));
                    q = q < -128 ? -128 : (q > 127 ? 127 : q);
                    bits[i] = 0x4B400000u + (uint32_t)q;
                }
            }
        }
    }
    // byte 0 of bits[i] is the code; gather bytes with v_perm_b32 (selector: 0-3 second operand, 4-7 first)
    even4 = __builtin_amdgcn_perm(bits[2], bits[0], 0x0c0c0400u) | __builtin_amdgcn_perm(bits[6], bits[4], 0x04000c0cu);
    odd4 = __builtin_amdgcn_perm(bits[3], bits[1], 0x0c0c0400u) | __builtin_amdgcn_perm(bits[7], bits[5], 0x04000c0cu);
}

// BITS = 0: no output.  BITS = 16: no quantizer, fp16 out (global memory only).
// BITS = 4: eight codes packed into dst_row[channel / 8].  BITS = 8: one byte per code; inside every
// group of 32 channels the 16 even channels come first, then the 16 odd ones (the order in which
// the matrix kernel consumes them), so a thread stores two dwords.
// A row of codes in global memory whose writer chooses how the dwords leave: STREAM = written through at once
// (non-temporal), else ordinary stores that wait in this XCD's L2.  The codes are read next by another launch,
// on every XCD, i.e. from the memory side in any case.  While all of a launch's codes fit the L2s, ordinary
// stores leave in one burst at the end of the kernel, and streaming them out during it is faster (canonical
// step of the five 2048-token linears with cold weights 415 -> 406 us); a larger output is evicted as the kernel
// goes anyway, and streaming costs 1 % (8192 tokens: 1419 -> 1434 us).  kStreamBelow is the sum of the eight L2s.
// (A compile-time choice: a run-time branch around every store cost the kernels 5 %.)
template <bool STREAM>
struct GlobalCodes {
    uint32_t* p;
};
constexpr int64_t kStreamBelow = 32ll << 20;

template <typename DST>
__device__ __forceinline__ void put_codes(DST dst_row, int64_t at, uint32_t w)
{
    if constexpr (std::is_same<DST, GlobalCodes<true>>::value) {
        __builtin_nontemporal_store(w, dst_row.p + at);
    } else if constexpr (std::is_same<DST, GlobalCodes<false>>::value) {
        dst_row.p[at] = w;
    } else {
        dst_row[at] = w;
    }
}

template <int BITS, bool EXACT, typename DST>
__device__ __forceinline__ void store_codes(const float* v, float mult, float step, DST dst_row, int64_t e0, int zo = 0)
{
    if constexpr (BITS == 0) {
        // nothing is stored: the caller took the values through its step provider
    } else if constexpr (BITS == 16) {
        // rotation only: the normalised values go out as fp16 (round to nearest even), 16 bytes
        v4i o;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const __half2 h = __floats2half2_rn(v[2 * i] * mult, v[2 * i + 1] * mult);
            o[i] = *reinterpret_cast<const int*>(&h);
        }
        *reinterpret_cast<v4i*>(&dst_row[e0 >> 1]) = o;
    } else if constexpr (BITS == 4) {
        put_codes(dst_row, e0 >> 3, quant_pack8<EXACT>(v, v, mult, step, zo));
    } else {
        uint32_t ev, od;
        quant_bytes8<EXACT>(v, v, mult, step, ev, od);
        const int64_t d = (e0 >> 5) * 8 + ((e0 >> 3) & 3);
        put_codes(dst_row, d, ev);
        put_codes(dst_row, d + 4, od);
    }
}

// Rotate (block size 2^log2h, 0 = none), quantize and pack the channels [chunk0, chunk0 + 2048 G)
// of one row.  x_row points at the row's first channel; packed dwords go to dst_row[channel / 8]
// (global or LDS).  xch: LDS scratch of 2048 G floats, touched only when log2h > 9.  Must be
// called by all threads of the workgroup (it contains LDS barriers when log2h > 9): `tid` is
// the thread's index 0..255 inside the group of 256 that owns the chunk, and threads of other
// groups, or groups without a chunk, pass active = false and only take part in the barriers.
// LDS-only barrier: global loads that are still in flight stay in flight.
__device__ __forceinline__ void lds_sync() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

typedef __attribute__((address_space(3))) const v4i* lds_cv4_ptr;
typedef __attribute__((address_space(3))) uint32_t* lds_u32_ptr;
typedef __attribute__((address_space(3))) float* lds_f32_ptr;

// SRC: const __half* (global) or an LDS pointer to fp16; DST: uint32_t* (global) or
// lds_u32_ptr.  Explicit LDS pointers keep the accesses off the vector-memory counter.
//
// load_chunk only issues the loads (branch-free: threads without data read the row's first
// bytes), so a caller can have several chunks in flight before the arithmetic starts.
template <int G, typename SRC>
__device__ __forceinline__ void load_chunk(SRC x_row, int64_t K, int64_t chunk0, int tid, bool active, v4i (&raw)[G],
                                           bool (&live)[G])
{
    using src_v4 = std::conditional_t<std::is_same<SRC, const __half*>::value, const v4i*, lds_cv4_ptr>;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int64_t e0 = chunk0 + (int64_t)g * kChunk + tid * 8;
        live[g] = active && e0 < K;
        // (activations in global memory are read once: non-temporal, they leave the caches to what is read again)
        if constexpr (std::is_same<SRC, const __half*>::value)
            raw[g] = __builtin_nontemporal_load((src_v4)(x_row + (live[g] ? e0 : 0)));
        else
            raw[g] = *(src_v4)(x_row + (live[g] ? e0 : 0));
    }
}

// The step of a per-tensor static quantizer: known before the rotation, the same everywhere.
struct StaticStep {
    float mult, step;
    template <int NV>
    __device__ __forceinline__ void prepare(const float (&)[NV]) {}
    __device__ __forceinline__ void get(int64_t, float& m, float& s) const { m = mult; s = step; }
    __device__ __forceinline__ int zero_offset() const { return 0; }
};

// Per-tensor static step with a zero-point (Eq. 1 in its general form): zo = zero-point - 8.
struct StaticStepZp {
    float mult, step;
    int zo;
    template <int NV>
    __device__ __forceinline__ void prepare(const float (&)[NV]) {}
    __device__ __forceinline__ void get(int64_t, float& m, float& s) const { m = mult; s = step; }
    __device__ __forceinline__ int zero_offset() const { return zo; }
};

// Per-head static steps (one per block of 2^log2d consecutive channels), read from device memory;
// the reciprocal carries the 1/sqrt(h) of the rotation.
struct HeadStep {
    const float* scales;
    int log2d;
    double inv_sqrt_h;
    template <int NV>
    __device__ __forceinline__ void prepare(const float (&)[NV]) {}
    __device__ __forceinline__ void get(int64_t e0, float& m, float& s) const
    {
        s = scales[e0 >> log2d];
        m = (float)(inv_sqrt_h / (double)s);
    }
    __device__ __forceinline__ int zero_offset() const { return 0; }
};

// A step provider has `prepare(values)`, called once after the rotation by every thread of the
// workgroup with its G * 8 rotated (unnormalised) values (a dynamic quantizer derives its step
// there and may synchronise the workgroup), and `get(channel, mult, step)`, called per group of 8
// channels, which sets the quantizer's reciprocal step and step for that group.
//
// An input transform `xf.apply(g, values)` may rewrite the 8 fp32 values of group g right after
// they are converted from fp16 (before the rotation): the identity for a plain input, or the
// fusion of an elementwise producer (see SiluGate).
struct NoTransform {
    __device__ __forceinline__ void apply(int, float (&)[8]) const {}
};

// Producer fusion for down_proj: the layer input is silu(gate) * up, elementwise.  The values
// passed in are the gate's; the matching 16 bytes of `up` were loaded by the caller.
struct SiluGate {
    const v4i* up_raw;   // G loaded groups of the calling thread
    __device__ __forceinline__ void apply(int g, float (&v)[8]) const
    {
        const v4i u = up_raw[g];
        const __half2* h2 = reinterpret_cast<const __half2*>(&u);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float2 f = __half22float2(h2[i]);
            // hardware exp2 and reciprocal (about 1 ulp each): far inside the quantizer's tie tolerance
            v[2 * i] = v[2 * i] * __builtin_amdgcn_rcpf(1.0f + __expf(-v[2 * i])) * f.x;
            v[2 * i + 1] = v[2 * i + 1] * __builtin_amdgcn_rcpf(1.0f + __expf(-v[2 * i + 1])) * f.y;
        }
    }
};

template <int G, bool EXACT, int BITS = 4, typename DST, typename STEPS, typename XF = NoTransform>
__device__ __forceinline__ void rotate_quant_regs_with(const v4i (&raw)[G], const bool (&live)[G], int64_t chunk0,
                                                       int log2h, STEPS steps, DST dst_row, lds_f32_ptr xch,
                                                       int tid, bool active, XF xf = XF{})
{
    float mult, step;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    float v[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const v4i rg = live[g] ? raw[g] : (v4i){0, 0, 0, 0};
        const __half2* h2 = reinterpret_cast<const __half2*>(&rg);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float2 f = __half22float2(h2[i]);
            v[g][2 * i] = f.x;
            v[g][2 * i + 1] = f.y;
        }
        xf.apply(g, v[g]);
    }

    if constexpr (EXACT) {
        // no rotation: the unrotated value doubles as the exact tie-break operand
        steps.prepare(reinterpret_cast<float(&)[G * 8]>(v));
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (live[g]) {
                const int64_t e0 = chunk0 + (int64_t)g * kChunk + tid * 8;
                steps.get(e0, mult, step);
                store_codes<BITS, true>(v[g], mult, step, dst_row, e0, steps.zero_offset());
            }
        }
    } else {
#pragma unroll
        for (int g = 0; g < G; ++g) reg_stages8(v[g], log2h < 3 ? log2h : 3);
        float(&flat)[G * 8] = reinterpret_cast<float(&)[G * 8]>(v);
        if (log2h > 3) lane_stage<0>(flat, lane);
        if (log2h > 4) lane_stage<1>(flat, lane);
        if (log2h > 5) lane_stage<2>(flat, lane);
        if (log2h > 6) lane_stage<3>(flat, lane);
        if (log2h > 7) lane_stage<4>(flat, lane);
        if (log2h > 8) lane_stage<5>(flat, lane);
        if (log2h > 9) {
            // radix-4 (or radix-2 when h == 1024) exchange between the 4 wavefronts
            if (active) {
#pragma unroll
                for (int i = 0; i < G * 8; ++i) xch[(wave * G * 8 + i) * 64 + lane] = flat[i];
            }
            lds_sync();
            const bool two = log2h > 10;
            if (active) {
#pragma unroll
            for (int i = 0; i < G * 8; ++i) {
                const float a = xch[((wave ^ 1) * G * 8 + i) * 64 + lane];
                float r = (wave & 1) ? (a - flat[i]) : (a + flat[i]);
                if (two) {
                    const float b = xch[((wave ^ 2) * G * 8 + i) * 64 + lane];
                    const float c = xch[((wave ^ 3) * G * 8 + i) * 64 + lane];
                    const float rp = (wave & 1) ? (c - b) : (c + b);   // same stage-1 result in the partner pair
                    r = (wave & 2) ? (rp - r) : (rp + r);
                }
                flat[i] = r;
            }
            }
            lds_sync();   // the scratch may be reused by the next call
        }
        if constexpr (G > 1) {
            // d = 2048 * 2^j between groups
#pragma unroll
            for (int dg = 1; dg < G; dg <<= 1) {
                if (log2h > 11 + __builtin_ctz(dg)) {
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        if ((g & dg) == 0) {
#pragma unroll
                            for (int i = 0; i < 8; ++i) {
                                const float a = v[g][i], b = v[g + dg][i];
                                v[g][i] = a + b;
                                v[g + dg][i] = a - b;
                            }
                        }
                    }
                }
            }
        }
        steps.prepare(flat);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (live[g]) {
                const int64_t e0 = chunk0 + (int64_t)g * kChunk + tid * 8;
                steps.get(e0, mult, step);
                store_codes<BITS, false>(v[g], mult, step, dst_row, e0, steps.zero_offset());
            }
        }
    }
}

template <int G, bool EXACT, int BITS = 4, typename DST>
__device__ __forceinline__ void rotate_quant_regs(const v4i (&raw)[G], const bool (&live)[G], int64_t chunk0,
                                                  int log2h, float mult, float step, DST dst_row, lds_f32_ptr xch,
                                                  int tid, bool active)
{
    rotate_quant_regs_with<G, EXACT, BITS>(raw, live, chunk0, log2h, StaticStep{mult, step}, dst_row, xch, tid, active);
}

template <int G, bool EXACT, typename SRC, typename DST>
__device__ __forceinline__ void rotate_quant_chunk(SRC x_row, int64_t K, int64_t chunk0, int log2h, float mult,
                                                   float step, DST dst_row, lds_f32_ptr xch, int tid, bool active)
{
    v4i raw[G];
    bool live[G];
    load_chunk<G>(x_row, K, chunk0, tid, active, raw, live);
    rotate_quant_regs<G, EXACT>(raw, live, chunk0, log2h, mult, step, dst_row, xch, tid, active);
}

}  // namespace rq
}  // namespace pq
