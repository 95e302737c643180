/* pq.h — C ABI of the statically quantized W4A4 linear layer for AMD MI355X (gfx950).
 *
 * The layer is the inference hot path of PrefixQuant's static setting (Table 1, row O2:
 * weights per-channel, activations per-tensor static):
 *
 *   X fp16 [M,K] --online Hadamard rotation--> Y --static symmetric 4-bit quantization,
 *   two codes per byte--> Xq [M,K/2];  acc = Xq . Wq^T (int4 x int4, int32 accumulate);
 *   OUT fp16 [M,N] = acc * s_x * s_w[n].
 *
 * Conventions that hold for every entry point unless it says otherwise
 *   - every data pointer is a DEVICE pointer; the caller owns all buffers; the library
 *     allocates no device memory, never synchronises and never copies results back;
 *   - all work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream);
 *   - tensors are row-major and contiguous; base pointers must be 16-byte aligned;
 *   - 4-bit codes are two's-complement nibbles in [-8,7], two per byte, the even
 *     channel in the low nibble ("canonical" layout);
 *   - K % 32 == 0, N % 16 == 0, M >= 0 (M == 0 is a no-op that returns PQ_OK);
 *   - the return value is PQ_OK or a PQ_ERR_* code; on an error detected by argument
 *     checking nothing has been enqueued;
 *   - inputs must be finite.
 * State: the library keeps no handle and no per-call state; every entry point may be called from
 * several threads at once.  Process-wide are only (a) the three switches for sweeps and tests at the
 * end of this header (pq_set_gemm_variant, pq_set_gemm_tile, pq_set_gemm_f6_tile: atomic integers, read
 * by every product call; left alone, the automatic choice is a pure function of the shape), (b) a
 * per-kernel record that the runtime has been told about its LDS size (set once per device,
 * idempotent), and (c) the built-in scratch array of pq_linear_noalloc, which calls on one GPU share.
 */
#ifndef PQ_H
#define PQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    PQ_OK = 0,
    PQ_ERR_NULL = 1,        /* a required pointer is NULL                           */
    PQ_ERR_SHAPE = 2,       /* a size violates the conventions above                */
    PQ_ERR_ALIGN = 3,       /* a pointer is not 16-byte aligned                     */
    PQ_ERR_SCALE = 4,       /* a step size is not finite and positive               */
    PQ_ERR_WORKSPACE = 5,   /* workspace missing or too small                       */
    PQ_ERR_HIP = 6,         /* the HIP runtime reported an error at launch          */
    PQ_ERR_UNSUPPORTED = 7  /* valid request that this build has no kernel for      */
};

/* Library version as major*10000 + minor*100 + patch.  Host only. */
int pq_version(void);

/* Name of a status code; the string has static storage.  Host only. */
const char* pq_status_str(int status);

/* Online rotation + static quantization + packing (App. B "Online Rotation"; Eq. 1 in
 * its symmetric form; Sec. 3 "Dynamic and Static").
 * For every row m and every block b of had_block consecutive channels
 *     y[m, b*h + j] = sum_i x[m, b*h + i] * H_h[i][j] / sqrt(h),
 *     H_h[i][j] = (-1)^popcount(i & j)            (Sylvester order; fp32 sums: butterflies, or for blocks of
 *                                                  128 a product with H_128 on the matrix pipe),
 *     q = clamp(round_half_even(y / act_scale), -8, 7).
 * had_block: 0 or 1 = no rotation; otherwise a power of two in [2, 16384] that
 *            divides K.  With had_block <= 1 the codes are exactly
 *            round_half_even((double)x / (double)act_scale) clamped (no fp32 slip).
 * x_f16      in  [M,K] fp16.
 * xq_packed  out [M,K/2] uint8, canonical layout.
 */
int pq_rotate_quant(const void* x_f16, int64_t M, int64_t K, int32_t had_block,
                    float act_scale, void* xq_packed, void* stream);

/* Integer product + dequantisation (Sec. 3: low-bit matrix multiplication; Table 1 row
 * O2 for the two step sizes).
 *     acc[m,n] = sum_k xq[m,k] * wq[n,k]              (exact, int32)
 *     out[m,n] = fp16(acc[m,n] * (act_scale * w_scale[n]))   (fp32 multiply, RNE)
 * The kernel is chosen from M: weight-streaming kernels for M <= 16 (decode: 4-bit dot
 * products on packed nibbles for M <= 8, small matrix tiles up to 16 or 32), an INT8-MFMA tiled
 * kernel otherwise (prefill).  The tiled kernel carries 256 * acc in int32, which is exact for
 * K < 131072; longer rows with more than 8 tokens return PQ_ERR_UNSUPPORTED.
 * xq_packed in  [M,K/2] uint8 canonical.      wq_packed in [N,K/2] uint8 canonical.
 * w_scale   in  [N] fp32, 16-byte aligned.    act_scale: static step size of xq.
 * out_f16   out [M,N] fp16; may be NULL iff acc_i32 is not.
 * acc_i32   out [M,N] int32 raw accumulators, for verification; NULL in production.
 */
int pq_w4a4_gemm(const void* xq_packed, const void* wq_packed, const float* w_scale,
                 float act_scale, int64_t M, int64_t N, int64_t K,
                 void* out_f16, int32_t* acc_i32, void* stream);

/* The same product with scratch memory for the range between decode and prefill (Sec. 5.4 times
 * both ends; a serving batch of some dozens to some hundreds of tokens lies between): there the
 * output has far fewer tiles than the GPU has compute units, so the K dimension is split over
 * workgroups, each leaves an int32 plane of partial sums in `workspace`, and a second kernel adds
 * the planes and applies the epilogue.  Integer sums are exact in any order: accumulators and
 * outputs equal pq_w4a4_gemm's bit for bit.
 * pq_w4a4_gemm_workspace_bytes: what the cost model's choice needs for the shape, 0 where it would
 *   not split (one launch of a weight-streaming kernel serves, up to 16 tokens; or the output has
 *   enough tiles).  Host only.  With that much the split launch also takes over from two or more
 *   weight-streaming launches (17 to 32 tokens, very long rows) on matrices of 8 MB and more.
 * workspace: device memory, 256-byte aligned, or NULL; workspace_bytes may be smaller than asked
 *   for (fewer planes, or the unsplit kernel) or larger (the rest is untouched).  Its contents on
 *   return are unspecified.  Calls that share a workspace must be ordered on one stream.
 * Everything else as pq_w4a4_gemm, which is this call with workspace = NULL.
 */
size_t pq_w4a4_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
/* The same query for any of the products below: act_bits = 4 or 8 (else 0). */
size_t pq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int32_t act_bits);
int pq_w4a4_gemm_ws(const void* xq_packed, const void* wq_packed, const float* w_scale,
                    float act_scale, int64_t M, int64_t N, int64_t K,
                    void* out_f16, int32_t* acc_i32, void* workspace, size_t workspace_bytes,
                    void* stream);

/* Bytes of workspace pq_linear needs (holds Xq): M*K/2 rounded up to 256.  Host only.
 * pq_linear_workspace_bytes_split adds pq_w4a4_gemm_workspace_bytes(M,N,K): with that much,
 * pq_linear's product may split K as pq_w4a4_gemm_ws does (the codes come first, the planes after). */
size_t pq_linear_workspace_bytes(int64_t M, int64_t K);
size_t pq_linear_workspace_bytes_split(int64_t M, int64_t N, int64_t K);

/* The whole layer: pq_rotate_quant into `workspace`, then pq_w4a4_gemm (same stream).
 * For M <= 4 and M*K <= 8192 (16384 for a single token, 32768 without rotation) the two steps run in
 * one fused launch (every workgroup rotates and quantizes the few rows for itself while its first
 * weight loads are in flight).
 * workspace: device memory, 256-byte aligned, at least pq_linear_workspace_bytes(M,K);
 * its first M*K/2 bytes on return are the packed activation codes (canonical layout).
 */
int pq_linear(const void* x_f16, const void* wq_packed, const float* w_scale,
              float act_scale, int32_t had_block, int64_t M, int64_t N, int64_t K,
              void* out_f16, void* workspace, size_t workspace_bytes, void* stream);

/* Two layers that read the same tokens (gate_proj and up_proj of an MLP block, Sec. 3: one quantized input,
 * two low-bit products): X is rotated and quantized once, OUT_a = Xq . Wq_a^T and OUT_b = Xq . Wq_b^T with
 * their own channel steps and their own outputs [M, N_a] and [M, N_b].  Outputs equal those of two pq_linear
 * calls bit for bit.  Where pq_linear would take its fused launch (few tokens), one launch streams both
 * matrices, which saves the fixed cost of a launch (several microseconds where a matrix takes 4-8);
 * otherwise one pq_rotate_quant and two products.  N_a, N_b: multiples of 16; K, had_block, workspace
 * (pq_linear_workspace_bytes(M, K), or more for the split launch of the larger product) as for pq_linear.
 */
int pq_linear2(const void* x_f16, const void* wq_a, const float* w_scale_a, int64_t N_a, void* out_a_f16,
               const void* wq_b, const float* w_scale_b, int64_t N_b, void* out_b_f16, float act_scale,
               int32_t had_block, int64_t M, int64_t K, void* workspace, size_t workspace_bytes, void* stream);

/* pq_linear for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same layer, the same kernels and the same
 * outputs bit for bit, with pq_linear's workspace taken from an array built into the library
 * instead of from the caller.  The call allocates nothing, on the device or through any library.
 * Limit: the packed codes, M*K/2 bytes rounded up to 256, must fit pq_linear_noalloc_max_bytes()
 * (32 MiB: 2048 tokens of 28672 channels), else PQ_ERR_WORKSPACE and nothing is enqueued.  Every
 * GPU the library runs on holds one such array until the process ends, and every call on a GPU
 * uses that GPU's array: calls that overlap on one GPU (two streams, two threads) race; order
 * them on one stream.  The array's contents between calls are unspecified (nothing in it has to
 * start at zero: the quantizer writes every code before the product reads it).
 * Arguments and errors otherwise as pq_linear.
 */
size_t pq_linear_noalloc_max_bytes(void);
int pq_linear_noalloc(const void* x_f16, const void* wq_packed, const float* w_scale,
                      float act_scale, int32_t had_block, int64_t M, int64_t N, int64_t K,
                      void* out_f16, void* stream);

/* Plain, slow device kernel for the same product as pq_w4a4_gemm (one thread per
 * output, no tiling).  Kept as an on-device cross-check for the fast kernels.
 */
int pq_w4a4_gemm_simple(const void* xq_packed, const void* wq_packed, const float* w_scale,
                        float act_scale, int64_t M, int64_t N, int64_t K,
                        void* out_f16, int32_t* acc_i32, void* stream);

/* ---- measuring sticks for the rooflines (service calls, not part of the path) --------------
 * pq_probe_mfma_i8: `workgroups` workgroups of four wavefronts, each wavefront issues iters x 16
 *   independent 32x32x32 INT8 matrix instructions (2 * 32768 integer operations each) and nothing
 *   else; the operands are read once from `operands` (device, 16-byte aligned, operand_bytes a
 *   multiple of 16, at most 16 GiB), so their bit patterns are the caller's.  Operations of a launch:
 *   workgroups * 4 * iters * 16 * 65536.
 * pq_probe_stream_read: one launch of 256 workgroups reads `bytes` (multiple of 16) from `src`
 *   (device, 16-byte aligned) once and discards them.
 * sink: device int32, written practically never (keeps the work alive).  Errors as elsewhere.
 */
int pq_probe_mfma_i8(const void* operands, int64_t operand_bytes, int64_t iters, int32_t workgroups,
                     int32_t* sink, void* stream);
int pq_probe_stream_read(const void* src, int64_t bytes, int32_t* sink, void* stream);
/* The 6-bit floating-point matrix instruction of the same GPU (E3M2 operands, fp32 accumulate, twice
 * the nominal rate of INT8): every 4-bit code -8..7 (and +8) is exact in E3M2, products and sums
 * below 2^24 are exact in fp32, so it multiplies the codes of Eq. 1 exactly.
 * pq_probe_mfma_f6: as pq_probe_mfma_i8; operands are raw register images of 32 bytes (32 values of
 *   6 bits in the first 24 bytes), 32-byte aligned, operand_bytes a multiple of 32.  Operations of a
 *   launch: workgroups * 4 * iters * 16 * 131072.
 * pq_probe_f6_product: out[i][j] = sum_k a[i][k] b[j][k] for i, j < 32 through that instruction;
 *   a_codes, b_codes device int8 [32,K] with values in [-8, 8] (clamped), K % 64 == 0, K <= 262080,
 *   out_i32 device [32,32]; 16-byte aligned.  One wavefront; a check of exactness, not of speed.
 */
int pq_probe_mfma_f6(const void* operands, int64_t operand_bytes, int64_t iters, int32_t workgroups,
                     int32_t* sink, void* stream);
int pq_probe_f6_product(const int8_t* a_codes, const int8_t* b_codes, int64_t K, int32_t* out_i32,
                        void* stream);

/* ---- the same product on the 6-bit floating-point matrix instruction (prefill) ----------------
 * (Sec. 3, low-bit matrix multiplication.)  Every code of Eq. 1 is exact as a 6-bit float with 3
 * exponent and 2 mantissa bits, products and sums below 2^24 are exact in fp32: for K <= 262080 the
 * accumulators are the integer sums of pq_w4a4_gemm, bit for bit, and so are the outputs.  The
 * instruction has twice the nominal rate of the INT8 one.  Both operands are repacked first:
 * pq_repack_f6: codes_packed [rows,K/2] uint8 canonical -> `tiles`, pq_f6_tiles_bytes(rows,K) bytes:
 *   one block of 3072 bytes for every 32 rows and every 128 channels, blocks ordered [128-channel group
 *   kt][row block rb] (what a launch reads at one time, the same channels of many rows, lies side by
 *   side).  A block holds, for each of 64 lanes l and each of the instruction's two 64-channel steps
 *   s, a register image of 24 bytes: row 32 rb + l % 32, channels 128 kt + 64 s + 32 (l / 32) + 0..31 as a
 *   little-endian stream of 6-bit values (rows past the end are zero).  The images are stored as four
 *   planes, each lane after lane: bytes 0-15 of the first step's images (64 x 16 bytes), their bytes
 *   16-23 (64 x 8), bytes 0-7 of the second step's images (64 x 8), their bytes 8-23 (64 x 16): each plane
 *   is one load instruction of a wavefront.  K % 128 == 0, K <= 262080, the tiles under 4 GiB (else
 *   PQ_ERR_SHAPE / PQ_ERR_UNSUPPORTED).  Weights are repacked once, offline; activations are written in this
 *   form by pq_rotate_quant_f6 (pq_linear_f6 does it).
 * pq_w4a4_gemm_f6: x_tiles, w_tiles as written by pq_repack_f6 for [M,K] and [N,K]; everything else
 *   as pq_w4a4_gemm.
 * These calls are the optional prepacked layout of the boundary (a pure re-encoding of the canonical
 * nibbles, checked by a round trip against the layout's definition): pq_f6_tiles_bytes is its size
 * query, pq_repack_f6 the prepacking step, pq_w4a4_gemm_f6 and pq_linear_f6 the prepacked twins of
 * pq_w4a4_gemm and pq_linear; the canonical entry points work without them.
 */
size_t pq_f6_tiles_bytes(int64_t rows, int64_t K);
int pq_repack_f6(const void* codes_packed, int64_t rows, int64_t K, void* tiles, void* stream);
/* The same two calls under the names a caller who only wants "prepacked weights" looks for, and the layer on them:
 * pq_prepacked_bytes(N, K) = pq_f6_tiles_bytes(N, K); pq_prepack_weights = pq_repack_f6 on the [N,K] weight codes;
 * pq_linear_prepacked = pq_linear_f6 (declared below), with pq_linear_f6_workspace_bytes for its workspace. */
size_t pq_prepacked_bytes(int64_t N, int64_t K);
int pq_prepack_weights(const void* wq_packed, int64_t N, int64_t K, void* wq_tiled, void* stream);
int pq_w4a4_gemm_f6(const void* x_tiles, const void* w_tiles, const float* w_scale,
                    float act_scale, int64_t M, int64_t N, int64_t K,
                    void* out_f16, int32_t* acc_i32, void* stream);

/* pq_rotate_quant for the prepacked path: rotation + static quantization as pq_rotate_quant (the same
 * codes bit for bit), written as f6 tiles in one launch: x_tiles, pq_f6_tiles_bytes(M,K) bytes.
 * xq_packed: NULL, or where the canonical codes [M,K/2] go as well.  had_block: 0 or 1 = no rotation, else
 * a power of two up to 512 that divides K; larger blocks return PQ_ERR_UNSUPPORTED (pq_rotate_quant +
 * pq_repack_f6 serve those).  K % 128 == 0; limits as pq_repack_f6.
 */
int pq_rotate_quant_f6(const void* x_f16, int64_t M, int64_t K, int32_t had_block, float act_scale,
                       void* x_tiles, void* xq_packed, void* stream);

/* The whole layer on that instruction, for weights repacked beforehand (the prepacked twin of
 * pq_linear): pq_rotate_quant_f6, then pq_w4a4_gemm_f6, on one stream: two launches.  Rotation blocks
 * beyond 512 channels take pq_rotate_quant, pq_repack_f6 and pq_w4a4_gemm_f6: three.  The codes behind
 * the tiles are those of pq_rotate_quant bit for bit, the outputs those of pq_linear.
 * workspace: device memory, 256-byte aligned, pq_linear_f6_workspace_bytes(M,K,had_block) bytes; on
 * return it holds the activations' tiles (pq_f6_tiles_bytes(M,K)), and behind them, rounded up to 256,
 * the canonical packed codes [M,K/2] if had_block > 512.  K % 128 == 0; limits as pq_repack_f6 and
 * pq_rotate_quant.
 */
size_t pq_linear_f6_workspace_bytes(int64_t M, int64_t K, int32_t had_block);
int pq_linear_f6(const void* x_f16, const void* w_tiles, const float* w_scale,
                 float act_scale, int32_t had_block, int64_t M, int64_t N, int64_t K,
                 void* out_f16, void* workspace, size_t workspace_bytes, void* stream);

/* pq_linear2 on the prepacked path: two weight matrices as f6 tiles on the same tokens (gate_proj and up_proj),
 * X rotated, quantized and written as tiles once, two products.  Outputs equal those of two pq_linear_f6 calls
 * (and of pq_linear2 on the canonical weights) bit for bit.  Arguments as for pq_linear_f6; workspace of
 * pq_linear_f6_workspace_bytes(M, K, had_block). */
int pq_linear2_f6(const void* x_f16, const void* w_tiles_a, const float* w_scale_a, int64_t N_a, void* out_a_f16,
                  const void* w_tiles_b, const float* w_scale_b, int64_t N_b, void* out_b_f16, float act_scale,
                  int32_t had_block, int64_t M, int64_t K, void* workspace, size_t workspace_bytes, void* stream);
int pq_linear_prepacked(const void* x_f16, const void* wq_tiled, const float* w_scale, float act_scale, int32_t had_block,
                        int64_t M, int64_t N, int64_t K, void* out_f16, void* workspace, size_t workspace_bytes,
                        void* stream);

/* Force a kernel variant of pq_w4a4_gemm for sweeps and tests (host, process-wide, atomic;
 * see the end of this comment): 0 = automatic, 1 = weight-streaming matrix tiles (M <= 32, K % 256 == 0 and
 * the codes of 8 tokens fit in LDS; else PQ_ERR_UNSUPPORTED), 2 = MFMA tiled, 3 = simple,
 * 4 = weight-streaming 4-bit dot products (M <= 8 only), 5 = MFMA tiled with K split in up to 5
 * runs whenever the call has a workspace of two planes and K has 512 channels (else
 * PQ_ERR_UNSUPPORTED; the workspace queries then answer for 5 runs).  With 4 pq_linear uses its
 * fused single launch whenever the shape allows it; with 1, 2, 3 or 5 it always uses two launches.
 * pq_w4a8_gemm, pq_gemm_dynamic and pq_w4a4_gemm_zp use a weight-streaming kernel only with 0,
 * or with 1 or 4 where that kernel supports the shape, and the tiled kernel otherwise.  The
 * automatic choice for given codes: dot products up to 4 tokens (8 on matrices under 12 MB; with
 * int8 activations 2, 4 and 6 on matrices over 24 MB, over 12 MB and smaller), matrix tiles up to
 * 16 (up to 32 in two launches where a cost estimate puts that ahead of the tiled kernel: outputs
 * of few tiles), tiled beyond.  Every kernel gives the same accumulators and the same fp16 outputs
 * bit for bit.
 * Returns the previous value, or -1 if `variant` is unknown.  An atomic integer: safe to call from
 * any thread, but a product call running concurrently on another thread may see either value.
 */
int pq_set_gemm_variant(int variant);

/* Force the tiled kernel's tile (sweeps and tests; host, process-wide, atomic): -1 = by shape, 0 256x256,
 * 1 256x128, 2 128x128, 3 256x192, 4 64x128, 5-8 variants of these with more wavefronts or a deeper
 * ring; any forced tile also switches the mixed-width launch off.  Before the first call the value
 * is that of the environment variable PQ_GEMM_TILE, read once at the first product of the process.
 * pq_set_gemm_f6_tile: the same for pq_w4a4_gemm_f6 (tiles of 128 tokens): -1 = by shape, 2 = 256 channels per
 * tile, 3 = the mix of 512 and 384 in one launch where N allows it, else 384, 4 = 512 (environment variable
 * PQ_GEMM_F6_TILE).
 * Both return the previous value, or -2 if `tile` is unknown.
 */
int pq_set_gemm_tile(int tile);
int pq_set_gemm_f6_tile(int tile);

/* ---- 4-bit weights, 8-bit static activations (the W4A8 rows of Table 3) -------------------
 * Same layer with the activation quantizer at 8 bits: q = clamp(round_half_even(y/act_scale),
 * -128, 127), one int8 per code.  The three calls below mirror pq_rotate_quant, pq_w4a4_gemm and
 * pq_linear; they need K % 128 == 0, K <= 65536 and M*K < 2^32 (else PQ_ERR_UNSUPPORTED or
 * PQ_ERR_SHAPE as for the 4-bit calls); M <= 8 streams the weights once (decode kernel with 4-way
 * byte dot products), larger M uses the MFMA tiled kernel.
 *
 * "Grouped" int8 layout of xq8 [M,K]: inside every group of 32 consecutive channels the 16 even
 * channels are stored first, then the 16 odd ones: byte 32*g + 16*p + j holds channel
 * 32*g + 2*j + p (p = parity, j = 0..15).  It is the order in which the matrix kernel pairs them
 * with the even/odd nibbles of the packed weights, so no shuffle is needed at run time.
 */
int pq_rotate_quant8(const void* x_f16, int64_t M, int64_t K, int32_t had_block,
                     float act_scale, void* xq8_grouped, void* stream);

/* acc[m,n] = sum_k xq8[m,k] * wq[n,k] (exact, int32; |acc| <= 128*8*K fits for K <= 65536);
 * out = fp16(acc * (act_scale * w_scale[n])).  Arguments as pq_w4a4_gemm except xq8_grouped.
 */
int pq_w4a8_gemm(const void* xq8_grouped, const void* wq_packed, const float* w_scale,
                 float act_scale, int64_t M, int64_t N, int64_t K,
                 void* out_f16, int32_t* acc_i32, void* stream);

/* pq_w4a8_gemm with scratch memory for the split-K launch: workspace as for pq_w4a4_gemm_ws, sized by
 * pq_gemm_workspace_bytes(M,N,K,8); results equal pq_w4a8_gemm's bit for bit. */
int pq_w4a8_gemm_ws(const void* xq8_grouped, const void* wq_packed, const float* w_scale,
                    float act_scale, int64_t M, int64_t N, int64_t K,
                    void* out_f16, int32_t* acc_i32, void* workspace, size_t workspace_bytes,
                    void* stream);

/* Workspace of pq_linear_w4a8: M*K bytes rounded up to 256; _split adds the planes of
 * pq_gemm_workspace_bytes(M,N,K,8), which the layer's product then uses.  Host only. */
size_t pq_linear_w4a8_workspace_bytes(int64_t M, int64_t K);
size_t pq_linear_w4a8_workspace_bytes_split(int64_t M, int64_t N, int64_t K);

/* pq_rotate_quant8 into `workspace`, then pq_w4a8_gemm, on the same stream. */
int pq_linear_w4a8(const void* x_f16, const void* wq_packed, const float* w_scale,
                   float act_scale, int32_t had_block, int64_t M, int64_t N, int64_t K,
                   void* out_f16, void* workspace, size_t workspace_bytes, void* stream);

/* ---- per-token dynamic activation quantization (Table 1, row O1) ---------------------------
 * The step size is computed on the fly, one per token (row):
 *     y = rotation of x as in pq_rotate_quant;
 *     row_scale[m] = fp32(clip * max_k |y[m,k]| / qmax),  qmax = 7 (bits = 4) or 127 (bits = 8);
 *                    a row of zeros gets 1;
 *     q[m,k] = clamp(round_half_even(y[m,k] / row_scale[m]), -qmax - 1, qmax).
 * clip in (0, 1] is the tensor-wise clipping factor (Sec. 3 "Dynamic and Static"; 1 = none).
 * bits = 4: codes packed canonically [M,K/2]; bits = 8: grouped int8 layout [M,K].
 * Needs K % 128 == 0 and K <= 32768 (a workgroup holds a whole row), else PQ_ERR_SHAPE /
 * PQ_ERR_UNSUPPORTED.  row_scale: out [M] fp32, 4-byte aligned.
 * With had_block <= 1 codes and steps equal the definition evaluated in double precision.
 */
int pq_rotate_quant_dynamic(const void* x_f16, int64_t M, int64_t K, int32_t had_block,
                            float clip, int32_t bits, void* xq, float* row_scale, void* stream);

/* out[m,n] = fp16(acc[m,n] * (row_scale[m] * w_scale[n])), acc as in pq_w4a4_gemm (bits = 4) or
 * pq_w4a8_gemm (bits = 8).  K % 128 == 0, K <= 65536.  M <= 8 takes the weight-streaming decode
 * kernel (when the rows fit LDS), everything else the MFMA tiled kernel.
 */
int pq_gemm_dynamic(const void* xq, int32_t bits, const void* wq_packed, const float* w_scale,
                    const float* row_scale, int64_t M, int64_t N, int64_t K,
                    void* out_f16, int32_t* acc_i32, void* stream);

/* pq_gemm_dynamic with scratch memory for the split-K launch: workspace as for pq_w4a4_gemm_ws, sized
 * by pq_gemm_workspace_bytes(M,N,K,bits); results equal pq_gemm_dynamic's bit for bit. */
int pq_gemm_dynamic_ws(const void* xq, int32_t bits, const void* wq_packed, const float* w_scale,
                       const float* row_scale, int64_t M, int64_t N, int64_t K,
                       void* out_f16, int32_t* acc_i32, void* workspace, size_t workspace_bytes,
                       void* stream);

/* Workspace of pq_linear_dynamic: the codes (M*K/2 or M*K bytes, rounded up to 256) followed by
 * the M row steps (rounded up to 256); _split adds the planes of pq_gemm_workspace_bytes(M,N,K,bits)
 * behind them, which the layer's product then uses.  Host only.
 */
size_t pq_linear_dynamic_workspace_bytes(int64_t M, int64_t K, int32_t bits);
size_t pq_linear_dynamic_workspace_bytes_split(int64_t M, int64_t N, int64_t K, int32_t bits);

/* pq_rotate_quant_dynamic into `workspace`, then pq_gemm_dynamic, on the same stream.  On return
 * the workspace holds the codes at offset 0 and the fp32 row steps at offset
 * pq_linear_dynamic_workspace_bytes(M,K,bits) - roundup256(4*M).
 */
int pq_linear_dynamic(const void* x_f16, const void* wq_packed, const float* w_scale,
                      float clip, int32_t had_block, int32_t bits, int64_t M, int64_t N, int64_t K,
                      void* out_f16, void* workspace, size_t workspace_bytes, void* stream);

/* ---- attention side: online R3 and per-head static KV-cache quantization ------------------
 * (App. B "Online Rotation": queries and keys are rotated after RoPE, head by head; Table 1 row
 * O2: the KV cache is quantized per head with static steps.)
 *
 * x_f16 is [T, n_heads*head_dim] (a token's heads side by side); head_dim is a power of two in
 * [32, 2048].  rotate != 0 applies the head_dim-point Hadamard rotation of pq_rotate_quant to
 * every head (keys); rotate == 0 quantizes as is (values).  Codes are
 *     q[t, h*head_dim + j] = clamp(round_half_even(y[t, h*head_dim + j] / head_scale[h]), -8, 7),
 * packed canonically into xq_packed [T, n_heads*head_dim/2].  head_scale: device, [n_heads] fp32,
 * 4-byte aligned, every entry finite and positive (not checked: it lives on the device).
 * With rotate == 0 the codes equal the definition evaluated in double precision.
 */
int pq_rotate_quant_heads(const void* x_f16, int64_t T, int32_t n_heads, int32_t head_dim,
                          int32_t rotate, const float* head_scale, void* xq_packed, void* stream);

/* Group-wise dynamic variant (Table 1 row O1, "KV cache: group-wise dynamic"): every group of
 * `group` consecutive channels of a token (32, 64 or 128; a head or a part of one) gets its own step
 *     group_scale[t, c / group] = fp32(clip * max |y| over the group / 7)   (1 for a group of zeros),
 * codes as in pq_rotate_quant_heads with that step.  head_dim: rotation block when rotate != 0 (a power
 * of two in [32, 2048], a multiple of group); C = n_heads * head_dim channels per token.
 * group_scale: out, device, [T, C / group] fp32.  clip in (0, 1].
 */
int pq_rotate_quant_groups(const void* x_f16, int64_t T, int32_t n_heads, int32_t head_dim,
                           int32_t rotate, int32_t group, float clip, void* xq_packed,
                           float* group_scale, void* stream);

/* Rotation only (queries after RoPE): y = fp16(rotation of x) with blocks of had_block channels,
 * had_block a power of two in [2, 16384] dividing K; K % 32 == 0.  y_f16: out [M,K] fp16; may not
 * alias x_f16.  fp32 butterflies, one rounding to fp16.
 */
int pq_rotate_f16(const void* x_f16, int64_t M, int64_t K, int32_t had_block, void* y_f16,
                  void* stream);

/* ---- producer fusion (Sec. 3 "Dynamic and Static": static steps make operator fusion feasible) --
 * The elementwise producer of a linear's input is evaluated in the quantizer kernel, so the fp16
 * intermediate never exists in memory.
 *
 * down_proj: x = silu(gate) * up elementwise (silu(g) = g / (1 + exp(-g)), fp32, no intermediate
 * rounding to fp16), then rotation + static 4-bit quantization exactly as pq_rotate_quant.
 * gate_f16, up_f16: [M,K] fp16.
 */
int pq_silu_mul_rotate_quant(const void* gate_f16, const void* up_f16, int64_t M, int64_t K,
                             int32_t had_block, float act_scale, void* xq_packed, void* stream);

/* q/k/v/gate/up_proj: y[m,:] = x[m,:] / sqrt(mean_k x[m,k]^2 + eps) (RMS normalisation; its learned
 * weight is folded into the next linear, as the absorbed rotation requires), then static 4-bit
 * quantization of y with step act_scale, no rotation.  K % 32 == 0, K <= 32768 (a workgroup holds
 * a row); eps >= 0.
 */
int pq_rmsnorm_quant(const void* x_f16, int64_t M, int64_t K, float eps, float act_scale,
                     void* xq_packed, void* stream);

/* ---- static activation quantizer with a zero-point (Eq. 1 in its general form) ---------------
 *     X_INT = clamp(round_half_even(y / act_scale) + zero_point, 0, 15),   zero_point in [0, 15];
 * the stored nibble is the two's-complement code X_INT - 8, so zero_point = 8 is pq_rotate_quant.
 * The dequantised activation is (X_INT - zero_point) * act_scale, hence for output channel n
 *     sum_k (X_INT[k] - z) w[n,k] = acc[n] + (8 - z) * sum_k w[n,k]:
 * the matrix kernels are unchanged and a per-channel integer, prepared once per weight matrix,
 * joins the accumulator in the epilogue.
 */
int pq_rotate_quant_zp(const void* x_f16, int64_t M, int64_t K, int32_t had_block, float act_scale,
                       int32_t zero_point, void* xq_packed, void* stream);

/* zp_corr[n] = (8 - zero_point) * sum_k wq[n,k]   (device, [N] int32, 16-byte aligned). */
int pq_zero_point_correction(const void* wq_packed, int64_t N, int64_t K, int32_t zero_point,
                             int32_t* zp_corr, void* stream);

/* out[m,n] = fp16((acc[m,n] + zp_corr[n]) * (act_scale * w_scale[n])); acc_i32, if given, receives
 * the raw accumulators (without the correction).  K % 128 == 0, K <= 32768; M <= 8 takes the
 * weight-streaming kernel, larger M the MFMA tiled kernel.
 */
int pq_w4a4_gemm_zp(const void* xq_packed, const void* wq_packed, const float* w_scale,
                    float act_scale, const int32_t* zp_corr, int64_t M, int64_t N, int64_t K,
                    void* out_f16, int32_t* acc_i32, void* stream);
/* The same with scratch memory for the split-K launch (workspace as for pq_w4a4_gemm_ws, sized by
 * pq_gemm_workspace_bytes(M,N,K,4)); results equal pq_w4a4_gemm_zp's bit for bit. */
int pq_w4a4_gemm_zp_ws(const void* xq_packed, const void* wq_packed, const float* w_scale,
                       float act_scale, const int32_t* zp_corr, int64_t M, int64_t N, int64_t K,
                       void* out_f16, int32_t* acc_i32, void* workspace, size_t workspace_bytes,
                       void* stream);

/* ---- calibration of the static per-tensor step on the device --------------------------------
 * (Sec. 3 "Initialization of Quantization Parameters": max-min initialisation, and an MSE-based
 * grid search over the quantization parameter for per-tensor static quantization.  The paper
 * scores candidates by block outputs of the model; this library scores the tensor itself.)
 * With y = rotation of x_cal as in pq_rotate_quant, qmax = 2^(bits-1) - 1 and, for i = 0..n_grid-1,
 *     gamma_i = 1 - i (1 - gamma_min) / (n_grid - 1),   s_i = fp32(gamma_i * max|y| / qmax),
 *     err_i   = sum over the tensor of (y - s_i * clamp(round_half_even(y / s_i), -qmax-1, qmax))^2,
 * result (device, fp32, 4-byte aligned, 3 + n_grid entries) receives
 *     [0] s of the arg-min of err (lowest index on a tie), [1] s_0 = max|y| / qmax (max-min
 *     initialisation), [2] gamma of the arg-min, [3 + i] err_i.
 * x_cal_f16: [T,K] fp16, K % 32 == 0, K <= 32768; bits 4 or 8; 2 <= n_grid <= 128;
 * 0 < gamma_min < 1.  workspace: device, 256-byte aligned, pq_calibrate_workspace_bytes(T, n_grid).
 * Sums are taken in a fixed order (fp32 within a row, fp64 over rows): results are reproducible.
 * An all-zero tensor gives step 1.
 */
size_t pq_calibrate_workspace_bytes(int64_t T, int32_t n_grid);
int pq_calibrate_static(const void* x_cal_f16, int64_t T, int64_t K, int32_t had_block, int32_t bits,
                        int32_t n_grid, float gamma_min, float* result, void* workspace,
                        size_t workspace_bytes, void* stream);

/* The same search for Eq. 1 with a zero-point (4 bits): candidates are pairs of clipping factors,
 *     gamma_i = 1 - i (1 - gamma_min) / (n_gamma - 1) on hi = max(y, 0),
 *     beta_j  = 1 - j (1 - beta_min)  / (n_beta - 1)  on lo = min(y, 0)      (a single value: factor 1),
 *     s = fp32((gamma_i hi - beta_j lo) / 15),  z = clamp(-round(beta_j lo / s), 0, 15),
 *     err = sum (y - s (clamp(round(y / s) + z, 0, 15) - z))^2,   candidate index c = i * n_beta + j.
 * result (device, fp32, 6 + n_gamma * n_beta entries): [0] s and [1] z of the arg-min (lowest index on
 * a tie), [2] s and [3] z of candidate 0 (max-min initialisation), [4] i and [5] j of the arg-min,
 * [6 + c] err_c.  1 <= n_gamma, n_beta and n_gamma * n_beta in [2, 128]; other arguments as
 * pq_calibrate_static; workspace pq_calibrate_zp_workspace_bytes(T, n_gamma * n_beta).
 */
size_t pq_calibrate_zp_workspace_bytes(int64_t T, int32_t n_candidates);
int pq_calibrate_static_zp(const void* x_cal_f16, int64_t T, int64_t K, int32_t had_block,
                           int32_t n_gamma, int32_t n_beta, float gamma_min, float beta_min,
                           float* result, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PQ_H */
