// HIP kernels for gfx950 (MI355X): 4x1 structured-sparse INT8 SpMM with fused epilogue.
//
// What the paper's Algorithm 1 does with AVX-512 (broadcast the non-zero weight words,
// re-structure the input rows named by the weight's mask into the multiply instruction's
// operand format, multiply-accumulate u8 x s8 into s32, then "downconvert" with the fused
// post-operators) is mapped to CDNA4 as follows:
//
//  * multiply instruction: v_mfma_i32_16x16x64_i8.  A row tile of 16 output rows (four 4x1
//    block-rows) is multiplied against the union of its k positions, 64 listed k per
//    instruction (layout in spmm_internal.h).
//  * "re-structure the input by the mask" (the permute/shuffle sequence of Algorithm 1):
//    the activations of one token tile and one K segment sit in LDS row-major; the
//    gathered, k-contiguous operand is produced by ds_read_b64_tr_b8, whose lanes each
//    supply the address of an arbitrary activation row -- the gather by non-zero index and
//    the byte transpose happen in the LDS read itself, no VALU shuffles.
//  * u8 x s8: the matrix instruction multiplies signed bytes, so activations are stored in
//    LDS as x - 128 (one xor per dword while staging) and 128 * rowsum(W) is added back
//    by initialising the accumulators with it; exact in int32.
//  * post-operators (Section 3.3) are applied to the accumulators in registers; the
//    GELU->int8 chain is the 256-entry table of Algorithm 2, held in LDS.
//  * the two-dimensional blocking over output rows and tokens of Section 3.2 becomes the
//    workgroup decomposition: a workgroup owns a group of row tiles and walks over token
//    tiles, so the compressed weights it needs stay in registers.
//
// Four kernels share the layout and the inner step (two transposing LDS reads, one matrix
// instruction per 16 tokens); the host's plan (spmm_plan.hip) picks one by shape:
//   spmm_rowtile_mfma         persistent, software-pipelined: long batches
//   spmm_rowtile_mfma_simple  one workgroup per 128 rows x 16/32/64 tokens, segment by segment:
//                             small problems, and the independent cross-check of the others
//   spmm_rowtile_mfma_slab    the same decomposition with the whole K slab of activations in
//                             LDS and the weights streamed: short batches, 2048 < K <= 4096
//   spmm_rowtile_mfma_stream  segment staging with the streamed weights: short batches, longest K
//
// Lane roles of the matrix instruction (D = A.B, 64 lanes, g = lane / 16, c = lane % 16):
//   A operand (activations): row = token c, bytes t = k-list slots 16g .. 16g+15
//   B operand (weights)    : column = output row c, same k slots
//   D                      : D[token 4g + r][output row c], r = 0..3
//
// ds_read_b64_tr_b8 within a 16-lane group: the lane at position p supplies the address of
// 8 bytes; result lane p receives, as byte t, byte (p % 8) of the 8 bytes addressed by
// source position 2t + p / 8.  With source position 2t + h pointing at tokens 8h .. 8h+7
// of activation row k_t, result lane p holds token p of rows k_0 .. k_7.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "spmm_internal.h"

namespace spmm {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v2i* lds_v2i_ptr;

constexpr int FLIP = (int)0x80808080;   // x ^ 0x80 == x - 128 as a signed byte

// GELU in its erf form, y * Phi(y) = 0.5 * y * erfc(-y / sqrt(2)), in binary32, branch-free.
// With z = |y| / sqrt(2) and t = 2 / (2 + z), ln(erfc(z) exp(z^2) / t) is smooth on 0 < t <= 1
// (it tends to -ln(2 sqrt(pi)) as z grows), so erfc(z) = t * exp(P(t) - z^2) with P a degree-9
// polynomial: a least-squares fit of that function at 400 Chebyshev nodes, converted to powers
// of t.  The negative side is 0.5 * y * erfc(z) and keeps its relative accuracy in the tail; the
// positive side is y - 0.5 * y * erfc(z).  The rounding of z^2 and of the exponent grows with z^2,
// to about 2e-6 relative at |y| = 5; beyond |y| = 3 the result is below 4.1e-3 and the absolute
// part of the tolerance (1e-7) covers it.  Measured against the exact value on a dense sweep the
// error stays below a tenth of 1e-5 * |GELU| + 1e-7.
__device__ __forceinline__ float gelu_f32(float y)
{
    const float z = fabsf(y) * 0.70710678118654752440f;
    const float t = __builtin_amdgcn_rcpf(__fmaf_rn(0.5f, z, 1.0f));
    float p = 1.708727777e-01f;
    p = __fmaf_rn(p, t, -8.221522344e-01f);
    p = __fmaf_rn(p, t, 1.488515889e+00f);
    p = __fmaf_rn(p, t, -1.135204000e+00f);
    p = __fmaf_rn(p, t, 2.788680845e-01f);
    p = __fmaf_rn(p, t, -1.862880617e-01f);
    p = __fmaf_rn(p, t, 9.678418949e-02f);
    p = __fmaf_rn(p, t, 3.740919597e-01f);
    p = __fmaf_rn(p, t, 1.000023680e+00f);
    p = __fmaf_rn(p, t, -1.265512225e+00f);
    // exp(p - z^2) = 2^((p - z^2) * log2(e)); below 2^-126 the result flushes towards zero, where
    // |GELU| < 1e-30 anyway
    const float e = t * __builtin_amdgcn_exp2f((p - z * z) * 1.4426950408889634f);
    const float h = 0.5f * y * e;          // y < 0: the result; y >= 0: what is missing from y
    return y < 0.0f ? h : y - h;
}

// Where the table of Algorithm 2 is read from.
struct GlobalLut {
    const int8_t* p;
    __device__ __forceinline__ uint32_t operator()(uint32_t key) const { return (uint8_t)p[key]; }
};

// POST template parameters below are the SPMM_POST_* value, plus POST_SUM_BIT when the Sum
// post-operator (a second binary32 tensor added after BiasAdd / GeLU, before Quantize) is on.

// Output stores of the aligned paths go through a buffer resource that covers exactly the bytes
// the call may write (out_bytes, < 2 GiB on these paths): a store beyond it is dropped by the
// hardware.  Where one store instruction of a wave fills whole 128-byte lines (1-byte outputs in
// token-tile-major order: 16 rows x 32 bytes back to back) or the output is 4 bytes wide, the
// store goes out at agent scope (sc1), i.e. written through the XCD's L2 as it is issued: left at
// the default scope the lines stay dirty in that L2 and are written back when the kernel ends,
// behind all the compute, and that write-back is then the tail of every launch (measured inside
// the rotating benchmark step, outputs going to HBM: 4096 x 1024 at 90 %, 24.8 -> 23.1 us; binary32
// 3072 x 768, 18.4 -> 17.2 us).  Row-major 1-byte outputs leave in 64-byte runs, half a line per
// instruction; written through, those cost more at the memory than they save (25.0 -> 27.3 us),
// so they stay at the default scope and the L2 merges them.
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
constexpr int SCOPE_DEFAULT = 0, SCOPE_AGENT = 16;   // cache-policy operand of the buffer stores: none / sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t out_resource(const KernelArgs& a)
{
    // raw buffer (stride 0), 32-bit data format
    return __builtin_amdgcn_make_buffer_rsrc(a.out, 0, (int)a.out_bytes, 0x00020000);
}
// (byte_off: per lane; uniform_off: the same for the whole wave, held in a scalar register)
template <int SCOPE, typename V>
__device__ __forceinline__ void store16_out(const __amdgpu_buffer_rsrc_t rs, const uint32_t byte_off, const V v,
                                            const uint32_t uniform_off = 0)
{
    static_assert(sizeof(V) == 16, "16-byte store");
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, v), rs, (int)byte_off, (int)uniform_off, SCOPE);
}

// quantised code of one pre-activation y (Quantize post-operator / table look-up)
template <int OUT, int POST, typename Lut>
__device__ __forceinline__ uint32_t quantise(const KernelArgs& a, const float y, const Lut& lut)
{
    if constexpr ((POST & SPMM_POST_GELU) != 0) {
        // key = sat_s8(rint(y / mid_scale)) + 128; v_cvt_pk_u8_f32 converts with saturation to [0, 255]
        const float t = rintf(y * a.inv_mid) + 128.0f;
        return lut(__builtin_amdgcn_cvt_pk_u8_f32(t, 0u, 0u));
    } else {
        const float lo = (OUT == SPMM_OUT_U8) ? 0.0f : -128.0f;
        const float hi = (OUT == SPMM_OUT_U8) ? 255.0f : 127.0f;
        return (uint32_t)((int)fminf(hi, fmaxf(lo, rintf(y * a.inv_out) + a.out_zp_f))) & 0xffu;
    }
}

// Generic post-operators + store for 4 consecutive tokens m0..m0+3 of output row n: any
// alignment, any tail (the slow path of every kernel).
// WIDE: 1-byte outputs of an unaligned matrix are written in the widest pieces the address
// allows (dword, two halves, bytes) instead of bytes, and aligned 4-byte outputs go out at agent
// scope (see out_resource); costs registers the 16-wave pipelined kernels do not have (the
// host does not pick those for unaligned operands, and their full tiles take finish_tile_fast).
// OT: layout of a 1-byte output: 1 = token-tile-major, 0 = row-major, -1 = whichever the arguments say
template <int OUT, int POST, bool WIDE = false, int OT = -1, typename Lut>
__device__ __forceinline__ void finish4(const KernelArgs& a, const v4i acc, const float s, const float b,
                                        const int n, const int m0, const Lut& lut)
{
    const int valid = a.M - m0;   // > 0 guaranteed by caller
    if constexpr (OUT == SPMM_OUT_S32) {
        int32_t* o = (int32_t*)a.out + (int64_t)n * a.ldo + m0;
        if (a.out_vec_ok && valid >= 4) {
            if constexpr (WIDE) store16_out<SCOPE_AGENT>(out_resource(a), 4u * ((uint32_t)n * (uint32_t)a.ldo + (uint32_t)m0), acc);
            else *(v4i*)o = acc;
        } else {
            for (int r = 0; r < 4; ++r)
                if (r < valid) o[r] = acc[r];
        }
    } else {
        float y[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) y[r] = __fmaf_rn((float)acc[r], s, b);
        if constexpr (OUT == SPMM_OUT_F32 && (POST & SPMM_POST_GELU) != 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) y[r] = gelu_f32(y[r]);
        }
        if constexpr ((POST & POST_SUM_BIT) != 0) {
            const float* sp = a.sum + (int64_t)n * a.ld_sum + m0;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (r < valid) y[r] = y[r] + sp[r];
        }
        if constexpr (OUT == SPMM_OUT_F32) {
            float* o = (float*)a.out + (int64_t)n * a.ldo + m0;
            if (a.out_vec_ok && valid >= 4) {
                v4f v = {y[0], y[1], y[2], y[3]};
                if constexpr (WIDE) store16_out<SCOPE_AGENT>(out_resource(a), 4u * ((uint32_t)n * (uint32_t)a.ldo + (uint32_t)m0), v);
                else *(v4f*)o = v;
            } else {
                for (int r = 0; r < 4; ++r)
                    if (r < valid) o[r] = y[r];
            }
        } else {
            uint32_t q[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) q[r] = quantise<OUT, POST>(a, y[r], lut);
            // (token-tile-major output, [M / 32][N][32]: rows 32 bytes apart, a column's tile out_tile_stride
            // = 32 N bytes after the previous one; four consecutive tokens from a multiple of 4 share a tile)
            const bool ot = (OT == 1) || (OT == -1 && a.out_tile_stride != 0);
            uint8_t* o = (uint8_t*)a.out + (int64_t)n * a.ldo +
                         (ot ? (int64_t)(m0 >> 5) * a.out_tile_stride + (m0 & 31) : (int64_t)m0);
            if (valid >= 4 && (a.out_vec_ok || (WIDE && ((uintptr_t)o & 3) == 0))) {
                *(uint32_t*)o = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
            } else if (WIDE && valid >= 4 && ((uintptr_t)o & 1) == 0) {
                *(uint16_t*)o = (uint16_t)(q[0] | (q[1] << 8));
                *(uint16_t*)(o + 2) = (uint16_t)(q[2] | (q[3] << 8));
            } else {
                for (int r = 0; r < 4; ++r)
                    if (r < valid) o[r] = (uint8_t)q[r];
            }
        }
    }
}

// s_waitcnt vmcnt(0) only (expcnt / lgkmcnt fields left at their maxima).  Issued when the
// prefetches started at the beginning of a phase have long landed: it tells the compiler's
// wait-count bookkeeping that no global load is outstanding, so the next phase's multiply
// loop does not stall on the prefetches issued just before it.
__device__ __forceinline__ void wait_global_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Byte mask of a 16-byte piece of which the first nv bytes are wanted (nv <= 0: none).
__device__ __forceinline__ v4i piece_mask(const int nv)
{
    v4i m;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int keep = nv - 4 * w;
        m[w] = keep >= 4 ? -1 : (keep <= 0 ? 0 : (int)((1u << (8 * keep)) - 1u));
    }
    return m;
}

// Byte offset of token column `col` inside an activation row.  Row-major X: the column itself (rows
// are ldx apart).  Token-tile-major X, [ceil(M / 32)][K][32] (the re-structured input of Section 3.2:
// the rows of a 32-token tile lie back to back, so a workgroup's token tile is three or four
// contiguous regions of memory): rows are 32 bytes apart and a column's tile starts
// x_tile_stride = 32 K bytes after the previous one.  16-byte pieces start at multiples of 16 and
// never straddle two tiles; xcol(c1 + c2) = xcol(c1) + xcol(c2) when c1 is a multiple of 32.
// XT: 1 = token-tile-major, 0 = row-major, -1 = whichever the arguments say (a uniform run-time test).
// The pipelined kernel is instantiated for both layouts: its 16-wave forms have no register to spare
// for a choice at run time.
template <int XT = -1>
__device__ __forceinline__ int xcol(const KernelArgs& a, const int col)
{
    // (the whole X is smaller than 2 GiB in this layout, checked on the host: the offset fits an int)
    if constexpr (XT == 0) return col;
    else if constexpr (XT == 1) return (col >> 5) * a.x_tile_stride + (col & 31);
    else return a.x_tile_stride ? (col >> 5) * a.x_tile_stride + (col & 31) : col;
}

// 16 bytes of activation row `krow` starting at token `col`; tokens >= M read as 0.
// The general path (odd leading dimension or base, or the last, partial piece of a row) reads the
// aligned dwords that hold the wanted bytes and shifts them into place: every dword read holds
// at least one wanted byte, so nothing outside the pages of X is touched, and a piece costs at
// most five loads (byte loads of 64 different rows cost a cache-line look-up each: a 13-token
// tail made the whole launch three times longer).
template <int XT = -1>
__device__ __forceinline__ v4i load_x16(const KernelArgs& a, const int krow, const int col)
{
    const uint8_t* src = a.X + (int64_t)krow * a.ldx + xcol<XT>(a, col);
    const int nbytes = min(16, a.M - col);
    if (a.x_vec_ok && nbytes == 16) return *(const v4i*)src;
    v4i v = {0, 0, 0, 0};
    if (nbytes <= 0) return v;
    const uintptr_t p = (uintptr_t)src;
    const uint32_t sh = (uint32_t)(p & 3);
    const uint32_t* q = (const uint32_t*)(p - sh);
    const int span = (int)sh + nbytes;            // bytes from q[0] on that are wanted
    uint32_t d[5];
#pragma unroll
    for (int i = 0; i < 5; ++i) d[i] = (4 * i < span) ? q[i] : 0u;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t x = __builtin_amdgcn_alignbyte(d[w + 1], d[w], sh);
        const int keep = nbytes - 4 * w;          // wanted bytes of this dword
        const uint32_t mask = keep >= 4 ? 0xffffffffu : (keep <= 0 ? 0u : ((1u << (8 * keep)) - 1u));
        v[w] = (int)(x & mask);
    }
    return v;
}

// The same, byte by byte: few registers (the 16-wave pipelined kernels have 128 and none to
// spare for a path they take only with unaligned activations), slow.
template <int XT = -1>
__device__ __forceinline__ v4i load_x16_bytewise(const KernelArgs& a, const int krow, const int col)
{
    const uint8_t* src = a.X + (int64_t)krow * a.ldx + xcol<XT>(a, col);
    if (a.x_vec_ok && col + 16 <= a.M) return *(const v4i*)src;
    v4i v = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 16; ++j)
        if (col + j < a.M) v[j >> 2] |= (int)((uint32_t)src[j] << (8 * (j & 3)));
    return v;
}

// =======================================================================================
// Pipelined persistent kernel (the one spmm_run launches).
//
// Workgroup = NW waves.  Wave w owns row tile NW*rg + w (16 output rows) for the whole
// kernel; the workgroup walks over token tiles of TM tokens (stream, stream + S, ..) and,
// inside a token tile, over the K segments of 512 rows.  One (token tile, segment) pair is a
// "phase".  LDS holds two activation buffers [512 rows][TM + 16 bytes]; while phase p
// multiplies out of buffer p % 2, the global loads for phase p+1 are in flight in registers
// and are written to the other buffer afterwards; one barrier per phase.  The compressed
// weights of a phase (at most MAXS steps of 64 listed k) live in one of two register sets;
// with at most two segments they are loaded once per workgroup and reused for every token
// tile, otherwise they are prefetched one phase ahead.
//
// Two token-tile widths, both with one workgroup per CU, the table at LDS offset 0 and the
// buffers behind it:
//   TM = 128: the default.
//   TM =  96: chosen by the plan when it divides the tokens into a number of tiles that fills
//             the CUs more evenly (6144 tokens and 4 row groups: 256 workgroups instead of 192).
//             A row is 6 pieces of 16 bytes; 3/4 of the threads stage them.
// Every LDS row has 16 spare bytes behind its TM tokens (the pitch TM + 16 makes consecutive
// rows start 4 banks apart).  These spare chunks carry the output staging for 1-byte outputs:
// wave w transposes its 16 rows x 64 tokens through chunks 64w .. 64w+63 so that a row's
// tokens leave in 64-byte runs (32 for the last third of a 96-token tile) instead of 4-byte
// pieces.  Staging row r, 16-token piece j lives in chunk 4r + (j ^ (r >> 2)): with both
// pitches the 4-byte writes and the 16-byte reads then touch every LDS bank once.
// =======================================================================================
template <int TM>
struct Geo;

template <>
struct Geo<128> {
    static constexpr int STRIDE = 144, PIECES = 8, HALVES = 2;
    static constexpr int BUF = SEGMENT_ROWS * STRIDE;   // 73728
    static constexpr int X0 = 256;                      // table in [0, 256): the key is the address
    static constexpr int LDS = X0 + 2 * BUF;
    static __device__ __forceinline__ uint32_t lut_addr(uint32_t key) { return key; }
    // spare chunk n in [0, 1024): behind row n of the two back-to-back buffers
    static __device__ __forceinline__ uint32_t chunk(uint32_t n) { return X0 + n * STRIDE + 128; }
};

template <>
struct Geo<96> {
    static constexpr int STRIDE = 112, PIECES = 6, HALVES = 2;
    static constexpr int BUF = SEGMENT_ROWS * STRIDE;   // 57344
    static constexpr int X0 = 256;
    static constexpr int LDS = X0 + 2 * BUF;
    static __device__ __forceinline__ uint32_t lut_addr(uint32_t key) { return key; }
    static __device__ __forceinline__ uint32_t chunk(uint32_t n) { return X0 + n * STRIDE + 96; }
};

// TM = 64 (loader-wave kernel only): four pieces per row, twice as many tiles per stream; the output
// stores of a workgroup then start after half the time and the last tile's burst is half as long.
template <>
struct Geo<64> {
    static constexpr int STRIDE = 80, PIECES = 4, HALVES = 1;
    static constexpr int BUF = SEGMENT_ROWS * STRIDE;   // 40960
    static constexpr int X0 = 256;
    static constexpr int LDS = X0 + 2 * BUF;
    static __device__ __forceinline__ uint32_t lut_addr(uint32_t key) { return key; }
    static __device__ __forceinline__ uint32_t chunk(uint32_t n) { return X0 + n * STRIDE + 64; }
};

template <int TM>
struct LdsLut {
    const uint8_t* lds;
    __device__ __forceinline__ uint32_t operator()(uint32_t key) const { return lds[Geo<TM>::lut_addr(key)]; }
};

// Post-operators + store for one full token tile of one wave, everything in bounds and
// aligned: lane (g, c) holds tokens tok0 + 16 i + 4 g + {0..3} of output row 16 * tile + c.
// 4-byte outputs are stored straight from the accumulator layout (16 bytes per lane, 64-byte
// runs per row); 1-byte outputs go through the LDS staging chunks.
template <int TM, int OUT, int POST, int OT = -1>
__device__ __forceinline__ void finish_tile_fast(const KernelArgs& a, const v4i (&acc)[Geo<TM>::PIECES],
                                                 const float scale, const float bias, const int tile,
                                                 const int tok0, int lane, const int wave, uint8_t* lds)
{
    using G = Geo<TM>;
    // Keep the address arithmetic below local to the epilogue: without this the compiler hoists
    // it out of the phase loop and the long-lived results push the kernel into register spills.
    asm volatile("" : "+v"(lane));
    const int g = lane >> 4, c = lane & 15;
    if constexpr (OUT == SPMM_OUT_S32) {
        // fast path: the whole output is < 2 GiB (checked on the host), 32-bit offsets suffice
        const uint32_t off = (uint32_t)(tile * TILE_ROWS + c) * (uint32_t)a.ldo + (uint32_t)(tok0 + 4 * g);
        const __amdgpu_buffer_rsrc_t rs = out_resource(a);
        if (tile * TILE_ROWS + c < a.N) {
#pragma unroll
            for (int i = 0; i < G::PIECES; ++i) store16_out<SCOPE_AGENT>(rs, 4u * off + 64u * i, acc[i]);
        }
    } else if constexpr (OUT == SPMM_OUT_F32) {
        const uint32_t off = (uint32_t)(tile * TILE_ROWS + c) * (uint32_t)a.ldo + (uint32_t)(tok0 + 4 * g);
        const __amdgpu_buffer_rsrc_t rs = out_resource(a);
        // (Sum: the second operand is read in the accumulator layout, 16 bytes per lane)
        const float* sp = a.sum + ((uint32_t)(tile * TILE_ROWS + c) * (uint32_t)a.ld_sum + (uint32_t)(tok0 + 4 * g));
        if (tile * TILE_ROWS + c < a.N) {
#pragma unroll
            for (int i = 0; i < G::PIECES; ++i) {
                v4f y;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    y[r] = __fmaf_rn((float)acc[i][r], scale, bias);
                    if constexpr ((POST & SPMM_POST_GELU) != 0) y[r] = gelu_f32(y[r]);
                }
                if constexpr ((POST & POST_SUM_BIT) != 0) y = y + *(const v4f*)(sp + 16 * i);
                store16_out<SCOPE_AGENT>(rs, 4u * off + 64u * i, y);
            }
        }
    } else {
        const LdsLut<TM> lut{lds};
        // write side: this lane's quad of piece j goes to staging row c, piece j
        const uint32_t wbase = G::chunk(64 * wave + 4 * c) + 4 * g;
        const int wsw = c >> 2;
        // read side: this lane fetches 16 tokens of staging row lane / 4, piece lane % 4
        const int rr = lane >> 2, rj = lane & 3;
        const uint32_t raddr = G::chunk(64 * wave + 4 * rr + (rj ^ (rr >> 2)));
        const int orow = tile * TILE_ROWS + rr;
        // row-major: 64-byte steps between the halves; token-tile-major ([M / 32][N][32], tok0 a multiple of 32):
        // piece rj of half h lies in tile tok0 / 32 + rj / 2 + 2 h, at byte 16 (rj & 1) of the row
        const bool ot = (OT == 1) || (OT == -1 && a.out_tile_stride != 0);
        const uint32_t ots = (uint32_t)a.out_tile_stride;
        const uint32_t off = ot ? (uint32_t)((tok0 >> 5) + (rj >> 1)) * ots + (uint32_t)orow * 32u + (uint32_t)((rj & 1) * 16)
                                : (uint32_t)orow * (uint32_t)a.ldo + (uint32_t)(tok0 + 16 * rj);
        const uint32_t half_step = ot ? 2u * ots : 64u;
        const __amdgpu_buffer_rsrc_t rs = out_resource(a);
        // (Sum: read in the accumulator layout, row 16 * tile + c; rows past N are never stored)
        const bool sum_row_ok = tile * TILE_ROWS + c < a.N;
        const float* sp = a.sum + ((uint32_t)(tile * TILE_ROWS + c) * (uint32_t)a.ld_sum + (uint32_t)(tok0 + 4 * g));
#pragma unroll
        for (int h = 0; h < G::HALVES; ++h) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = 4 * h + j;
                if (i >= G::PIECES) continue;   // (a 96-token tile ends after piece 5)
                v4f y;
#pragma unroll
                for (int r = 0; r < 4; ++r) y[r] = __fmaf_rn((float)acc[i][r], scale, bias);
                if constexpr ((POST & POST_SUM_BIT) != 0) {
                    if (sum_row_ok) y = y + *(const v4f*)(sp + 16 * i);
                }
                uint32_t q[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) q[r] = quantise<OUT, POST>(a, y[r], lut);
                // (two shift-or pairs, then one more: three instructions)
                const uint32_t word = (q[0] | (q[1] << 8)) | ((q[2] | (q[3] << 8)) << 16);
                *(uint32_t*)(lds + wbase + (uint32_t)(j ^ wsw) * G::STRIDE) = word;
            }
            const v4i v = *(const v4i*)(lds + raddr);   // same wave: LDS operations complete in order
            if (orow < a.N && 4 * h + rj < G::PIECES) {
                if constexpr (OT == 1) {
                    store16_out<SCOPE_AGENT>(rs, off, v, half_step * h);
                } else if constexpr (OT == 0) {
                    *(v4i*)((uint8_t*)a.out + off + half_step * h) = v;
                } else {
                    if (ot) store16_out<SCOPE_AGENT>(rs, off, v, half_step * h);
                    else store16_out<SCOPE_DEFAULT>(rs, off, v, half_step * h);
                }
            }
        }
    }
}

template <int TM, int NW, int MAXS, int OUT, int POST, int LAYOUT = 0>
__global__ void __launch_bounds__(NW * 64) spmm_rowtile_mfma(const KernelArgs a)
{
    using G = Geo<TM>;
    // LAYOUT bit 0: activations token-tile-major; bit 1: (1-byte) outputs token-tile-major
    constexpr int XT = LAYOUT & 1, OTILED = (LAYOUT >> 1) & 1;
    constexpr int NTHREADS = NW * 64;
    constexpr int PIECES = G::PIECES;
    // activation rows one load pass covers: a power of two; with 6 pieces per row only
    // ROWS_PER_PASS * 6 threads (whole waves) stage
    constexpr int ROWS_PER_PASS = (NTHREADS / PIECES >= 128) ? 128 : 64;
    constexpr int STAGERS = ROWS_PER_PASS * PIECES;
    constexpr int XLOADS = SEGMENT_ROWS / ROWS_PER_PASS;            // 16-byte loads per staging thread and phase
    static_assert(STAGERS <= NTHREADS && STAGERS % 64 == 0, "staging threads must be whole waves of the workgroup");
    // The 16-wave kernels with 5 and 6 step slots use all 128 registers: the four mask registers of
    // the cut piece would spill in them, so there a token count that is not a multiple of 16 takes
    // the bytewise path for its last tile.
    constexpr bool MASKED_TAIL = !(NW == 16 && MAXS >= 5);
    __shared__ __attribute__((aligned(16))) uint8_t lds[G::LDS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;

    // workgroup -> (token-tile stream, row group) = (blockIdx.x, blockIdx.y).  Workgroups go to the
    // 8 XCDs round-robin in linear order (x fastest); the host makes gridDim.x a multiple of 8
    // whenever it can, so that all row groups of one stream run on the same XCD and share its L2.
    // With xcd_map 2 the two roles are swapped (all streams of a row group on one XCD): the host's
    // choice when the packed weight is the larger operand.
    const int S = a.n_streams;
    int stream = (a.xcd_map == 2) ? blockIdx.y : blockIdx.x;
    const int rg = (a.xcd_map == 2) ? blockIdx.x : blockIdx.y;
    // map 1 (S is then a multiple of 8): XCD x gets the S / 8 consecutive streams from x * S / 8 on, so
    // that token tiles next to each other in memory, which share cache lines when the tile width is
    // not a multiple of the line, mostly run on the same XCD
    if (a.xcd_map == 1) stream = (stream & 7) * (S >> 3) + (stream >> 3);
    const int n_my = a.tiles_per_stream + (stream < a.tiles_extra ? 1 : 0);   // token tiles of this stream (>= 1)
    const int total = n_my * a.nseg;                                          // phases

    const int tile = rg * NW + wave;
    const bool have_tile = tile < a.ntiles;
    const int n = tile * TILE_ROWS + c;                       // this lane's output row
    // per-lane constants of the post-operators: loaded in the start-up sequence below, behind
    // the activation and weight loads whose latency they would otherwise precede
    int init = 0;
    float scale = 0.0f, bias = 0.0f;

    v4i A0[MAXS], A1[MAXS];
    uint32_t I0[MAXS], I1[MAXS];
    int n0 = 0, n1 = 0;
    constexpr int XH = XLOADS / 2;   // the prefetch is issued and committed in two halves
    static_assert(XH * 2 == XLOADS, "even number of prefetch loads");
    v4i xr[XH];
    v4i acc[PIECES];

    // per-thread staging coordinates: XLOADS rows (ROWS_PER_PASS apart), one 16-byte piece
    const bool stager = (STAGERS == NTHREADS) || wave < STAGERS / 64;
    const int x_row0 = tid / PIECES, x_piece = tid % PIECES;
    const uint32_t x_lds0 = G::X0 + (uint32_t)x_row0 * G::STRIDE + x_piece * 16;

    // ---- global loads of half h of the activations of phase q into registers.  The common case
    // (16-byte aligned rows, full token tile) is branch-free so that all loads are in flight
    // together; rows past the end of K are redirected to the last valid row (never multiplied).
    // Two halves (first issued at the start of the previous phase, second half-way through its
    // multiply) keep only XH prefetch registers live.
    auto x_issue_to = [&](v4i (&xr)[XH], const int q, const int h) {
        const int j = q / a.nseg, seg = q - j * a.nseg;
        const int tok0 = (stream + j * S) * TM;
        const int k0 = seg * SEGMENT_ROWS;
        const int last = min(SEGMENT_ROWS, a.K - k0) - 1;
        if (!stager) return;
        if constexpr (XT == 0) {
            if (a.x_vec_ok && tok0 + TM <= a.M) {
                // fast path: K * ldx < 2 GiB (checked on the host), 32-bit offsets from a uniform base
                const uint8_t* src = a.X + (int64_t)k0 * a.ldx + tok0;
#pragma unroll
                for (int u = 0; u < XH; ++u) {
                    const int row = min(x_row0 + (h * XH + u) * ROWS_PER_PASS, last);
                    xr[u] = *(const v4i*)(src + ((uint32_t)row * (uint32_t)a.ldx + (uint32_t)(x_piece * 16)));
                }
            } else if (a.x_vec_ok && (MASKED_TAIL || (a.M & 15) == 0)) {
                // ragged last tile of an aligned matrix: a piece is whole, beyond the end, or cut by it.
                // The cut one is read whole as well (an aligned 16-byte chunk that holds a wanted byte
                // lies inside the row pitch) and masked: branch-free.  (Without MASKED_TAIL only token
                // counts that are multiples of 16 come here: no piece is cut.)
                const uint8_t* src = a.X + (int64_t)k0 * a.ldx;
                const int col = tok0 + x_piece * 16;
                const bool in = col < a.M;
#pragma unroll
                for (int u = 0; u < XH; ++u) {
                    const int row = min(x_row0 + (h * XH + u) * ROWS_PER_PASS, last);
                    const v4i v = *(const v4i*)(src + ((uint32_t)row * (uint32_t)a.ldx + (uint32_t)(in ? col : 0)));
                    if constexpr (MASKED_TAIL) xr[u] = v & piece_mask(a.M - col);
                    else xr[u] = in ? v : (v4i){0, 0, 0, 0};
                }
            } else {
#pragma unroll
                for (int u = 0; u < XH; ++u) {
                    const int row = min(x_row0 + (h * XH + u) * ROWS_PER_PASS, last);
                    if constexpr (NW == 16) xr[u] = load_x16_bytewise<0>(a, k0 + row, tok0 + x_piece * 16);
                    else xr[u] = load_x16<0>(a, k0 + row, tok0 + x_piece * 16);
                }
            }
        } else {
            // token-tile-major activations: the layout is 16-byte aligned and padded to whole 32-token tiles, so
            // a piece that starts before M is read whole and one that starts at or after M is not needed at
            // all (its columns are never stored): one branch-free form, no masks, no unaligned path
            // (the piece's offset is worked out again at every call, from a thread id the compiler cannot
            // see through: kept in a register across the phases it would be one register too many)
            int t = tid;
            asm volatile("" : "+v"(t));
            const int col = tok0 + (t % PIECES) * 16;
            const uint8_t* src = a.X + (int64_t)k0 * 32;
            const uint32_t off = col < a.M ? (uint32_t)xcol<1>(a, col) : 0u;
#pragma unroll
            for (int u = 0; u < XH; ++u) {
                const int row = min(x_row0 + (h * XH + u) * ROWS_PER_PASS, last);
                xr[u] = *(const v4i*)(src + ((uint32_t)row * 32u + off));
            }
        }
    };

    // ---- ... and from registers into LDS buffer q % 2, as x - 128
    auto x_commit_from = [&](const v4i (&xr)[XH], const int q, const int h) {
        if (!stager) return;
        uint8_t* buf = lds + (q & 1) * G::BUF + x_lds0 + h * XH * ROWS_PER_PASS * G::STRIDE;
#pragma unroll
        for (int u = 0; u < XH; ++u)
            *(v4i*)(buf + u * ROWS_PER_PASS * G::STRIDE) = xr[u] ^ (v4i){FLIP, FLIP, FLIP, FLIP};
    };
    auto x_issue = [&](const int q, const int h) { x_issue_to(xr, q, h); };
    auto x_commit = [&](const int q, const int h) { x_commit_from(xr, q, h); };
    // ---- compressed weights + activation-row indices of (tile, segment of phase q).  Loads are
    // unconditional (slots past the segment's step count re-read step 0 and are never used).
    auto w_issue_at = [&](const int s0, v4i (&A)[MAXS], uint32_t (&I)[MAXS], const int cnt) {
#pragma unroll
        for (int s = 0; s < MAXS; ++s) {
            const int step = (s < cnt) ? s0 + s : 0;
            A[s] = *(const v4i*)(a.vals + (int64_t)step * STEP_VAL_BYTES + lane * 16);
            I[s] = a.idx[(int64_t)step * STEP_IDX_DWORDS + 8 * g + (c >> 1)];
        }
    };
    auto w_issue = [&](const int q, v4i (&A)[MAXS], uint32_t (&I)[MAXS], int& cnt) {
        cnt = 0;
        int s0 = 0;
        if (have_tile) {
            const int seg = q % a.nseg;
            s0 = a.seg_ptr[tile * a.nseg + seg];
            cnt = a.seg_ptr[tile * a.nseg + seg + 1] - s0;
        }
        w_issue_at(s0, A, I, cnt);
    };
    // ---- multiply phase q: gather + transpose out of LDS, PIECES matrix instructions per step.
    // Half-way (after step slot MAXS/2 - 1, executed or not) the first half of the next phase's
    // activations is committed and the second half's loads are issued.
    auto multiply = [&](const int q, const bool nxt, const v4i (&A)[MAXS], const uint32_t (&I)[MAXS], const int cnt) {
        const uint32_t base = G::X0 + (uint32_t)(q & 1) * G::BUF + (c & 1) * 8;
#pragma unroll
        for (int s = 0; s < MAXS; ++s) {
            if (s < cnt) {
                // this lane supplies the address of list slot 16g + c/2 (and + 8), token half c & 1
                const uint32_t a0 = (I[s] & 0xffffu) * G::STRIDE + base;
                const uint32_t a1 = (I[s] >> 16) * G::STRIDE + base;
#pragma unroll
                for (int i = 0; i < PIECES; ++i) {
                    const v2i x0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a0 + 16 * i));
                    const v2i x1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a1 + 16 * i));
                    const v4i xa = {x0[0], x0[1], x1[0], x1[1]};
                    acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa, A[s], acc[i], 0, 0, 0);
                }
            }
            if (s == MAXS / 2 - 1 && nxt) {
                x_commit(q + 1, 0);
                x_issue(q + 1, 1);
            }
        }
    };
    // ---- after the last segment of a token tile: post-operators, store, reset accumulators
    auto finish = [&](const int q) {
        const int j = q / a.nseg;
        if (q - j * a.nseg != a.nseg - 1) return;
        const int tok0 = (stream + j * S) * TM;
        if (have_tile) {
            if (a.out_vec_ok && tok0 + TM <= a.M) {
                finish_tile_fast<TM, OUT, POST, OTILED>(a, acc, scale, bias, tile, tok0, lane, wave, lds);
            } else if (n < a.N) {
                const LdsLut<TM> lut{lds};
#pragma unroll
                for (int i = 0; i < PIECES; ++i) {
                    const int m0 = tok0 + 16 * i + 4 * g;
                    if (m0 < a.M) finish4<OUT, POST, NW != 16, OTILED>(a, acc[i], scale, bias, n, m0, lut);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < PIECES; ++i) acc[i] = (v4i){init, init, init, init};
    };
    const bool reload = a.nseg > 2;   // otherwise set q % 2 always holds segment q % nseg

    {   // ---- start-up: every load of the first phase is issued before anything waits -- both
        // halves of the activations (the second in registers that are not live yet), the weights,
        // then the per-lane constants and the table -- and consumed in that order
        v4i x2[XH];
        // (the step range of the first weights: a scalar load whose latency the address arithmetic
        // of the activation loads covers)
        int w_s0 = 0;
        if (have_tile) {
            w_s0 = a.seg_ptr[tile * a.nseg];
            n0 = a.seg_ptr[tile * a.nseg + 1] - w_s0;
        }
        x_issue_to(xr, 0, 0);
        x_issue_to(x2, 0, 1);
        w_issue_at(w_s0, A0, I0, n0);
        if (have_tile) init = a.rowsum[n] * a.corr_mul;
        if constexpr (OUT != SPMM_OUT_S32) {
            if (have_tile && n < a.N) {
                scale = a.w_scale[n] * a.x_scale;
                if (a.bias) bias = a.bias[n];
            }
        }
        constexpr bool TABLE = (POST & SPMM_POST_GELU) != 0 && (OUT == SPMM_OUT_S8 || OUT == SPMM_OUT_U8);
        int table_byte = 0;
        if constexpr (TABLE) {
            if (tid < 256) table_byte = a.lut[tid];
        }
        x_commit_from(xr, 0, 0);
        x_commit_from(x2, 0, 1);
        if constexpr (TABLE) {
            if (tid < 256) lds[G::lut_addr(tid)] = (uint8_t)table_byte;
        }
    }
#pragma unroll
    for (int i = 0; i < PIECES; ++i) acc[i] = (v4i){init, init, init, init};
    wait_global_loads();
    __syncthreads();
    for (int p = 0; p < total; p += 2) {
        {   // even phase: register set 0, LDS buffer 0
            const bool nxt = p + 1 < total;
            if (nxt) {
                x_issue(p + 1, 0);
                if (reload || p + 1 < 2) w_issue(p + 1, A1, I1, n1);
            }
            multiply(p, nxt, A0, I0, n0);
            if (nxt) x_commit(p + 1, 1);
            wait_global_loads();   // before the output stores: they must not be waited for
            finish(p);
            __syncthreads();
        }
        if (p + 1 >= total) break;
        {   // odd phase: register set 1, LDS buffer 1
            const bool nxt = p + 2 < total;
            if (nxt) {
                x_issue(p + 2, 0);
                if (reload) w_issue(p + 2, A0, I0, n0);
            }
            multiply(p + 1, nxt, A1, I1, n1);
            if (nxt) x_commit(p + 2, 1);
            wait_global_loads();
            finish(p + 1);
            __syncthreads();
        }
    }
}

// =======================================================================================
// Pipelined persistent kernel with loader waves: the same decomposition, LDS geometry and
// phases as spmm_rowtile_mfma, but the workgroup is NW compute waves (one row tile each)
// plus LW = 4 waves that do nothing but stage the activations.
//
// Why: on this architecture loads and stores of a wave share one completion counter and may
// complete out of order with each other, so a wave that has stored a tile's outputs cannot
// wait for its next activation loads without also waiting until the stores have reached
// memory.  In spmm_rowtile_mfma every wave does both, and for 4-byte outputs (the downconvert
// of Section 3.3 left out: 4 N M bytes) the whole workgroup then stands still at the next
// commit until the burst of stores has drained.  Here the waves that store never load
// activations (with at most two K segments they load nothing at all after start-up), and the
// waves that load never store: the stores of tile j drain while tile j + 1 is multiplied.
//
// Loader wave: at the start of phase p its registers hold the activations of phase p + 1
// (requested a whole phase earlier); it writes them to buffer (p + 1) % 2, whose readers
// finished before the last barrier, requests phase p + 2 and goes to the barrier.
// Compute wave: multiply out of buffer p % 2, post-operators after the last segment, barrier.
// Both kinds pass exactly 1 + phases barriers.
// =======================================================================================
template <int TM, int NW, int LW, int MAXS, int OUT, int POST>
__global__ void __launch_bounds__((NW + LW) * 64) spmm_rowtile_mfma_fed(const KernelArgs a)
{
    using G = Geo<TM>;
    constexpr int PIECES = G::PIECES;
    constexpr int LTHREADS = LW * 64;
    constexpr int ROWS_PER_PASS = 32;
    constexpr int STAGERS = ROWS_PER_PASS * PIECES;              // 256 (128 tokens) or 192 (96 tokens)
    constexpr int XLOADS = SEGMENT_ROWS / ROWS_PER_PASS;         // 16-byte loads per staging thread and phase
    static_assert(STAGERS <= LTHREADS, "the loader waves must cover one pass of rows");
    __shared__ __attribute__((aligned(16))) uint8_t lds[G::LDS];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;

    // workgroup -> (token-tile stream, row group): as in spmm_rowtile_mfma
    const int S = a.n_streams;
    int stream = (a.xcd_map == 2) ? blockIdx.y : blockIdx.x;
    const int rg = (a.xcd_map == 2) ? blockIdx.x : blockIdx.y;
    if (a.xcd_map == 1) stream = (stream & 7) * (S >> 3) + (stream >> 3);
    const int n_my = a.tiles_per_stream + (stream < a.tiles_extra ? 1 : 0);
    const int total = n_my * a.nseg;                                          // phases
    constexpr bool TABLE = (POST & SPMM_POST_GELU) != 0 && (OUT == SPMM_OUT_S8 || OUT == SPMM_OUT_U8);

    if (wave >= NW) {
        // ------------------------------------------------------------------ loader wave
        const int ltid = tid - NW * 64;
        const bool stager = ltid < STAGERS;
        const int x_row0 = ltid / PIECES, x_piece = ltid % PIECES;
        const uint32_t x_lds0 = G::X0 + (uint32_t)x_row0 * G::STRIDE + x_piece * 16;
        const uint32_t x_off = (uint32_t)xcol(a, x_piece * 16);
        v4i xr[XLOADS];
        auto x_issue = [&](const int q) {
            const int j = q / a.nseg, seg = q - j * a.nseg;
            const int tok0 = (stream + j * S) * TM;
            const int k0 = seg * SEGMENT_ROWS;
            const int last = min(SEGMENT_ROWS, a.K - k0) - 1;   // rows past K repeat the last one (never multiplied)
            if (!stager) return;
            if (a.x_vec_ok && tok0 + TM <= a.M) {
                const uint8_t* src = a.X + (int64_t)k0 * a.ldx + xcol(a, tok0);
#pragma unroll
                for (int u = 0; u < XLOADS; ++u) {
                    const int row = min(x_row0 + u * ROWS_PER_PASS, last);
                    xr[u] = *(const v4i*)(src + ((uint32_t)row * (uint32_t)a.ldx + x_off));
                }
            } else if (a.x_vec_ok) {
                // ragged last tile of an aligned matrix: a piece is whole, beyond the end, or cut by it;
                // the cut one is read whole (it lies inside the row pitch) and masked
                const uint8_t* src = a.X + (int64_t)k0 * a.ldx;
                const int col = tok0 + x_piece * 16;
                const bool in = col < a.M;
                const v4i mask = piece_mask(a.M - col);
#pragma unroll
                for (int u = 0; u < XLOADS; ++u) {
                    const int row = min(x_row0 + u * ROWS_PER_PASS, last);
                    xr[u] = *(const v4i*)(src + ((uint32_t)row * (uint32_t)a.ldx + (uint32_t)xcol(a, in ? col : 0))) & mask;
                }
            } else {
#pragma unroll
                for (int u = 0; u < XLOADS; ++u) {
                    const int row = min(x_row0 + u * ROWS_PER_PASS, last);
                    xr[u] = load_x16(a, k0 + row, tok0 + x_piece * 16);
                }
            }
        };
        auto x_commit = [&](const int q) {
            if (!stager) return;
            uint8_t* buf = lds + (q & 1) * G::BUF + x_lds0;
#pragma unroll
            for (int u = 0; u < XLOADS; ++u)
                *(v4i*)(buf + u * ROWS_PER_PASS * G::STRIDE) = xr[u] ^ (v4i){FLIP, FLIP, FLIP, FLIP};
        };
        x_issue(0);
        int table_byte = 0;
        if constexpr (TABLE) table_byte = a.lut[ltid];          // LTHREADS == 256 entries
        x_commit(0);
        if constexpr (TABLE) lds[G::lut_addr(ltid)] = (uint8_t)table_byte;
        if (1 < total) x_issue(1);
        __syncthreads();
        for (int p = 0; p < total; ++p) {
            if (p + 1 < total) x_commit(p + 1);
            if (p + 2 < total) x_issue(p + 2);
            __syncthreads();
        }
        return;
    }

    // ---------------------------------------------------------------------- compute wave
    const int tile = rg * NW + wave;
    const bool have_tile = tile < a.ntiles;
    const int n = tile * TILE_ROWS + c;                       // this lane's output row
    int init = 0;
    float scale = 0.0f, bias = 0.0f;
    v4i A0[MAXS], A1[MAXS];
    uint32_t I0[MAXS], I1[MAXS];
    int n0 = 0, n1 = 0;
    v4i acc[PIECES];

    auto w_issue = [&](const int q, v4i (&A)[MAXS], uint32_t (&I)[MAXS], int& cnt) {
        cnt = 0;
        int s0 = 0;
        if (have_tile) {
            const int seg = q % a.nseg;
            s0 = a.seg_ptr[tile * a.nseg + seg];
            cnt = a.seg_ptr[tile * a.nseg + seg + 1] - s0;
        }
#pragma unroll
        for (int s = 0; s < MAXS; ++s) {
            const int step = (s < cnt) ? s0 + s : 0;           // unused slots re-read step 0
            A[s] = *(const v4i*)(a.vals + (int64_t)step * STEP_VAL_BYTES + lane * 16);
            I[s] = a.idx[(int64_t)step * STEP_IDX_DWORDS + 8 * g + (c >> 1)];
        }
    };
    auto multiply = [&](const int q, const v4i (&A)[MAXS], const uint32_t (&I)[MAXS], const int cnt) {
        const uint32_t base = G::X0 + (uint32_t)(q & 1) * G::BUF + (c & 1) * 8;
#pragma unroll
        for (int s = 0; s < MAXS; ++s) {
            if (s < cnt) {
                const uint32_t a0 = (I[s] & 0xffffu) * G::STRIDE + base;
                const uint32_t a1 = (I[s] >> 16) * G::STRIDE + base;
#pragma unroll
                for (int i = 0; i < PIECES; ++i) {
                    const v2i x0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a0 + 16 * i));
                    const v2i x1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a1 + 16 * i));
                    const v4i xa = {x0[0], x0[1], x1[0], x1[1]};
                    acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa, A[s], acc[i], 0, 0, 0);
                }
            }
        }
    };
    auto finish = [&](const int q) {
        const int j = q / a.nseg;
        if (q - j * a.nseg != a.nseg - 1) return;
        const int tok0 = (stream + j * S) * TM;
        if (have_tile) {
            if (a.out_vec_ok && tok0 + TM <= a.M) {
                finish_tile_fast<TM, OUT, POST>(a, acc, scale, bias, tile, tok0, lane, wave, lds);
            } else if (n < a.N) {
                const LdsLut<TM> lut{lds};
#pragma unroll
                for (int i = 0; i < PIECES; ++i) {
                    const int m0 = tok0 + 16 * i + 4 * g;
                    if (m0 < a.M) finish4<OUT, POST, false>(a, acc[i], scale, bias, n, m0, lut);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < PIECES; ++i) acc[i] = (v4i){init, init, init, init};
    };
    const bool reload = a.nseg > 2;   // otherwise register set q % 2 always holds segment q % nseg

    w_issue(0, A0, I0, n0);
    if (have_tile) init = a.rowsum[n] * a.corr_mul;
    if constexpr (OUT != SPMM_OUT_S32) {
        if (have_tile && n < a.N) {
            scale = a.w_scale[n] * a.x_scale;
            if (a.bias) bias = a.bias[n];
        }
    }
#pragma unroll
    for (int i = 0; i < PIECES; ++i) acc[i] = (v4i){init, init, init, init};
    __syncthreads();
    for (int p = 0; p < total; p += 2) {
        {   // even phase: register set 0, LDS buffer 0
            if (p + 1 < total && (reload || p + 1 < 2)) w_issue(p + 1, A1, I1, n1);
            multiply(p, A0, I0, n0);
            finish(p);
            __syncthreads();
        }
        if (p + 1 >= total) break;
        {   // odd phase: register set 1, LDS buffer 1
            if (p + 2 < total && reload) w_issue(p + 2, A0, I0, n0);
            multiply(p + 1, A1, I1, n1);
            finish(p + 1);
            __syncthreads();
        }
    }
}

// Workgroup id -> (token tile, row group) of the simple and short-batch kernels.  Ids go round the
// 8 XCDs; map 1 keeps the workgroups of a token tile on one XCD, map 2 those of a row group (the
// host picks the one that slices the larger operand over the L2s).  False: a padding workgroup.
__device__ __forceinline__ bool decode_workgroup(const KernelArgs& a, const int b, int& tt, int& rg)
{
    const int xcd = b & 7, local = b >> 3;
    if (a.xcd_map == 2) {
        rg = xcd + 8 * (local / a.n_tok_tiles);
        tt = local % a.n_tok_tiles;
        return rg < a.n_row_groups;
    }
    // (an XCD takes consecutive token tiles: tiles narrower than a cache line share their lines)
    tt = xcd * ((a.n_tok_tiles + 7) >> 3) + local / a.n_row_groups;
    rg = local % a.n_row_groups;
    return tt < a.n_tok_tiles;
}

// =======================================================================================
// Simple kernel (token tile 64, 32 or 16, one K segment in LDS, no software pipelining, table
// read from global memory): an independent second implementation of the same layout, selected
// with spmm_set_tuning(h, 64 / 32 / 16, 101 or 102) and, automatically, for problems too small
// to fill the chip (there the narrowest token tile that still fits one workgroup per CU: a
// workgroup's time is bound by its CU's LDS, so narrower tiles on more CUs finish sooner).
// Different tilings must agree bit for bit because int32 accumulation is order-free.
// =======================================================================================
template <int TM, int NW, int R, int OUT, int POST>
__global__ void __launch_bounds__(NW * 64) spmm_rowtile_mfma_simple(const KernelArgs a)
{
    // row pitch in LDS: 80 / 48 / 48 bytes = 20 / 12 / 12 banks, so that 16 rows whose indices
    // differ mod 16 (the packer's order) start in 16 different groups of four banks
    constexpr int STRIDE = (TM == 16) ? 48 : TM + 16;
    constexpr int PIECES = TM / 16;
    static_assert(TM == 64 || TM == 32 || TM == 16, "token tile of the simple kernel");
    __shared__ __attribute__((aligned(16))) uint8_t lds[SEGMENT_ROWS * STRIDE];

    int tt, rg;
    if (!decode_workgroup(a, blockIdx.x, tt, rg)) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const int tok0 = tt * TM;

    v4i acc[R][PIECES];
    int row_of[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int tile = (rg * NW + wave) * R + r;
        row_of[r] = tile * TILE_ROWS + c;
        int init = 0;
        if (tile < a.ntiles) init = a.rowsum[row_of[r]] * a.corr_mul;
#pragma unroll
        for (int i = 0; i < PIECES; ++i) acc[r][i] = (v4i){init, init, init, init};
    }

    // Staging: XL 16-byte pieces per thread and segment.  The pieces of segment seg + 1 are
    // requested before segment seg is multiplied and written to the (single) LDS buffer after it,
    // so their latency hides behind the multiply.
    constexpr int XL = SEGMENT_ROWS * PIECES / (NW * 64);
    static_assert(XL * NW * 64 == SEGMENT_ROWS * PIECES, "threads must tile a segment");
    v4i xs[XL];
    auto x_load = [&](const int seg) __attribute__((always_inline)) {
        const int k0 = seg * SEGMENT_ROWS;
        const int last = min(SEGMENT_ROWS, a.K - k0) - 1;      // rows past K repeat the last one (never multiplied)
        if (a.x_vec_ok && tok0 + TM <= a.M) {
            const uint8_t* src = a.X + (int64_t)k0 * a.ldx;
#pragma unroll
            for (int u = 0; u < XL; ++u) {
                const int p = tid + u * NW * 64;
                const int row = min(p / PIECES, last), piece = p % PIECES;
                xs[u] = *(const v4i*)(src + ((uint32_t)row * (uint32_t)a.ldx + (uint32_t)xcol(a, tok0 + piece * 16)));
            }
        } else if (a.x_vec_ok) {
            // ragged last tile of an aligned matrix: whole pieces, none, or the cut one read whole
            // and masked; branch-free
            const uint8_t* src = a.X + (int64_t)k0 * a.ldx;
#pragma unroll
            for (int u = 0; u < XL; ++u) {
                const int p = tid + u * NW * 64;
                const int row = min(p / PIECES, last), col = tok0 + (p % PIECES) * 16;
                const bool in = col < a.M;
                const v4i v = *(const v4i*)(src + ((uint32_t)row * (uint32_t)a.ldx + (uint32_t)xcol(a, in ? col : 0)));
                xs[u] = v & piece_mask(a.M - col);
            }
        } else {
#pragma unroll
            for (int u = 0; u < XL; ++u) {
                const int p = tid + u * NW * 64;
                const int row = min(p / PIECES, last), piece = p % PIECES;
                xs[u] = load_x16(a, k0 + row, tok0 + piece * 16);
            }
        }
    };
    auto x_store = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < XL; ++u) {
            const int p = tid + u * NW * 64;
            *(v4i*)(lds + (p / PIECES) * STRIDE + (p % PIECES) * 16) = xs[u] ^ (v4i){FLIP, FLIP, FLIP, FLIP};
        }
    };
    x_load(0);
    x_store();
    __syncthreads();
    for (int seg = 0; seg < a.nseg; ++seg) {
        if (seg + 1 < a.nseg) x_load(seg + 1);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int tile = (rg * NW + wave) * R + r;
            if (tile >= a.ntiles) continue;
            const int s0 = a.seg_ptr[tile * a.nseg + seg];
            const int s1 = a.seg_ptr[tile * a.nseg + seg + 1];
            for (int s = s0; s < s1; ++s) {
                const v4i w = *(const v4i*)(a.vals + (int64_t)s * STEP_VAL_BYTES + lane * 16);
                const uint32_t ix = a.idx[(int64_t)s * STEP_IDX_DWORDS + 8 * g + (c >> 1)];
                const uint32_t a0 = (ix & 0xffffu) * STRIDE + (c & 1) * 8;
                const uint32_t a1 = (ix >> 16) * STRIDE + (c & 1) * 8;
#pragma unroll
                for (int i = 0; i < PIECES; ++i) {
                    const v2i x0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a0 + 16 * i));
                    const v2i x1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a1 + 16 * i));
                    const v4i xa = {x0[0], x0[1], x1[0], x1[1]};
                    acc[r][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa, w, acc[r][i], 0, 0, 0);
                }
            }
        }
        if (seg + 1 < a.nseg) {
            __syncthreads();   // everyone has finished reading this segment
            x_store();
            __syncthreads();
        }
    }

    const GlobalLut lut{a.lut};
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int n = row_of[r];
        if (n >= a.N) continue;
        float s = 0.0f, bias = 0.0f;
        if constexpr (OUT != SPMM_OUT_S32) {
            s = a.w_scale[n] * a.x_scale;
            if (a.bias) bias = a.bias[n];
        }
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int m0 = tok0 + 16 * i + 4 * g;
            if (m0 < a.M) finish4<OUT, POST, true>(a, acc[r][i], s, bias, n, m0, lut);
        }
    }
}

// =======================================================================================
// Short-batch kernel (token tile 16 with K <= 4096, or 32 with K <= 3072): the paper's own regime of 32 to 384 tokens,
// where a launch is a few microseconds long and its time is memory latency, not throughput.
// A workgroup (NW row tiles x TM tokens) requests its whole [K x TM] slab of activations at
// once and keeps it in LDS (TM = 16: 16 bytes per row, no padding: rows whose indices differ mod
// 16, the packer's order, start in different groups of four banks), so there is one barrier in
// the kernel and no per-segment round trip to memory.  Each wave then walks all steps of its
// row tile in one flat loop, its weights arriving through three rotating register sets of
// CH steps each (the first three sets are requested before the slab is stored).  The segment a
// step belongs to, which gives the LDS base of its segment-local indices, is tracked with the
// row tile's segment boundaries held one per lane.
// =======================================================================================
// TM = 16: 16 bytes per row, up to SLAB_SEGMENTS segments (64 KB).  TM = 32: 48 bytes per row (the
// pitch of the simple kernel's 32-token tile), up to SLAB_SEGMENTS_32 segments (144 KB).
template <int TM, int NW, int OUT, int POST>
__global__ void __launch_bounds__(NW * 64) spmm_rowtile_mfma_slab(const KernelArgs a)
{
    static_assert(TM == 16 || TM == 32, "token tile of the short-batch kernel");
    constexpr int STRIDE = (TM == 16) ? 16 : 48, PIECES = TM / 16, CH = 8;
    constexpr int SEGS = (TM == 16) ? SLAB_SEGMENTS : SLAB_SEGMENTS_32;
    static_assert(NW * 64 == SEGMENT_ROWS, "one thread per activation row of a segment");
    __shared__ __attribute__((aligned(16))) uint8_t lds[SEGS * SEGMENT_ROWS * STRIDE];

    int tt, rg;
    if (!decode_workgroup(a, blockIdx.x, tt, rg)) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const int tok0 = tt * TM;
    const int tile = rg * NW + wave;
    const bool have_tile = tile < a.ntiles;
    const int n = tile * TILE_ROWS + c;

    // lane q holds the first step of segment q of this row tile (q = nseg: one past the last step)
    int bounds = 0;
    if (have_tile && lane <= a.nseg) bounds = a.seg_ptr[tile * a.nseg + lane];

    // the slab: PIECES 16-byte pieces per thread and segment (rows past K repeat the last one; no
    // step refers to them)
    v4i xr[SEGS][PIECES];
    const bool fast = a.x_vec_ok && tok0 + TM <= a.M;
#pragma unroll
    for (int seg = 0; seg < SEGS; ++seg) {
        if (seg < a.nseg) {
#pragma unroll
            for (int u = 0; u < PIECES; ++u) {
                const int p = tid + u * NW * 64;
                const int row = min(seg * SEGMENT_ROWS + p / PIECES, a.K - 1), col = tok0 + (p % PIECES) * 16;
                if (fast) {
                    xr[seg][u] = *(const v4i*)(a.X + ((uint32_t)row * (uint32_t)a.ldx + (uint32_t)xcol(a, col)));
                } else if (a.x_vec_ok) {      // ragged last tile of an aligned matrix: whole chunks, masked
                    const v4i v = *(const v4i*)(a.X + ((uint32_t)row * (uint32_t)a.ldx + (uint32_t)xcol(a, col < a.M ? col : 0)));
                    xr[seg][u] = v & piece_mask(a.M - col);
                } else {
                    xr[seg][u] = load_x16(a, row, col);
                }
            }
        }
    }

    int init = 0;
    if (have_tile) init = a.rowsum[n] * a.corr_mul;
    v4i acc[PIECES];
#pragma unroll
    for (int i = 0; i < PIECES; ++i) acc[i] = (v4i){init, init, init, init};
    float scale = 0.0f, bias = 0.0f;
    if constexpr (OUT != SPMM_OUT_S32) {
        if (have_tile && n < a.N) {
            scale = a.w_scale[n] * a.x_scale;
            if (a.bias) bias = a.bias[n];
        }
    }

    const int s_begin = __builtin_amdgcn_readlane(bounds, 0);
    const int s_end = __builtin_amdgcn_readlane(bounds, a.nseg);
    const int nchunks = (s_end - s_begin + CH - 1) / CH;

    v4i A0[CH], A1[CH], A2[CH];
    uint32_t I0[CH], I1[CH], I2[CH];
    auto w_load = [&](const int chunk, v4i (&A)[CH], uint32_t (&I)[CH]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            int step = s_begin + chunk * CH + j;
            step = (step < s_end) ? step : 0;          // step 0 is always readable
            A[j] = *(const v4i*)(a.vals + (int64_t)step * STEP_VAL_BYTES + lane * 16);
            I[j] = a.idx[(int64_t)step * STEP_IDX_DWORDS + 8 * g + (c >> 1)];
        }
    };
    w_load(0, A0, I0);
    if (nchunks > 1) w_load(1, A1, I1);
    if (nchunks > 2) w_load(2, A2, I2);

#pragma unroll
    for (int seg = 0; seg < SEGS; ++seg) {
        if (seg < a.nseg) {
#pragma unroll
            for (int u = 0; u < PIECES; ++u) {
                const int p = tid + u * NW * 64;
                *(v4i*)(lds + (seg * SEGMENT_ROWS + p / PIECES) * STRIDE + (p % PIECES) * 16) =
                    xr[seg][u] ^ (v4i){FLIP, FLIP, FLIP, FLIP};
            }
        }
    }
    __syncthreads();

    int seg = 0;
    int seg_end = __builtin_amdgcn_readlane(bounds, 1);
    auto multiply = [&](const int chunk, const v4i (&A)[CH], const uint32_t (&I)[CH]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int step = s_begin + chunk * CH + j;
            if (step < s_end) {
                while (step >= seg_end && seg + 1 < a.nseg) {      // (empty segments are skipped here)
                    ++seg;
                    seg_end = __builtin_amdgcn_readlane(bounds, seg + 1);
                }
                const uint32_t base = (uint32_t)seg * (SEGMENT_ROWS * STRIDE) + (c & 1) * 8;
                const uint32_t a0 = (I[j] & 0xffffu) * STRIDE + base;
                const uint32_t a1 = (I[j] >> 16) * STRIDE + base;
#pragma unroll
                for (int i = 0; i < PIECES; ++i) {
                    const v2i x0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a0 + 16 * i));
                    const v2i x1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a1 + 16 * i));
                    const v4i xa = {x0[0], x0[1], x1[0], x1[1]};
                    acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa, A[j], acc[i], 0, 0, 0);
                }
            }
        }
    };
    for (int ch = 0; ch < nchunks; ch += 3) {
        multiply(ch, A0, I0);
        if (ch + 3 < nchunks) w_load(ch + 3, A0, I0);
        if (ch + 1 < nchunks) {
            multiply(ch + 1, A1, I1);
            if (ch + 4 < nchunks) w_load(ch + 4, A1, I1);
        }
        if (ch + 2 < nchunks) {
            multiply(ch + 2, A2, I2);
            if (ch + 5 < nchunks) w_load(ch + 5, A2, I2);
        }
    }

    if (have_tile && n < a.N) {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int m0 = tok0 + 16 * i + 4 * g;
            if (m0 < a.M) finish4<OUT, POST, true>(a, acc[i], scale, bias, n, m0, GlobalLut{a.lut});
        }
    }
}

// =======================================================================================
// Streamed kernel (token tile 64, 32 or 16, any K): the segment-by-segment staging of the simple
// kernel (one segment of activations in LDS, the next one prefetched into registers) with the
// weight stream of the short-batch kernel: each wave walks all steps of its row tile in one flat
// loop through three rotating register sets of CH steps, so a step's weights were requested two
// sets earlier instead of when it is multiplied (the simple kernel exposes that latency at every
// step, which is what it costs at 70-80 % sparsity).  A wave crosses into the next segment where
// its own step list does, wherever that falls in the unrolled loop: advance() is the only place
// with barriers, and every wave of the workgroup runs it exactly nseg - 1 times, in the loop or
// in the drain after it (waves without a row tile, or with fewer steps, only in the drain).
// =======================================================================================
template <int TM, int NW, int OUT, int POST>
__global__ void __launch_bounds__(NW * 64) spmm_rowtile_mfma_stream(const KernelArgs a)
{
    static_assert(TM == 64 || TM == 32 || TM == 16, "token tile of the streamed kernel");
    constexpr int STRIDE = (TM == 16) ? 16 : TM + 16, PIECES = TM / 16, CH = 8;
    constexpr int XL = SEGMENT_ROWS * PIECES / (NW * 64);
    static_assert(XL * NW * 64 == SEGMENT_ROWS * PIECES, "threads must tile a segment");
    __shared__ __attribute__((aligned(16))) uint8_t lds[SEGMENT_ROWS * STRIDE];

    int tt, rg;
    if (!decode_workgroup(a, blockIdx.x, tt, rg)) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const int tok0 = tt * TM;
    const int tile = rg * NW + wave;
    const bool have_tile = tile < a.ntiles;
    const int n = tile * TILE_ROWS + c;
    const int nseg = a.nseg;

    // first step of every segment of this row tile, and one past the last: in LDS-free form only
    // the current boundary is kept (a scalar), fetched when a segment is entered
    const int32_t* const bounds = a.seg_ptr + (have_tile ? tile * nseg : 0);
    const int s_begin = have_tile ? bounds[0] : 0;
    const int s_end = have_tile ? bounds[nseg] : 0;
    const int nchunks = (s_end - s_begin + CH - 1) / CH;

    v4i xs[XL];
    const bool fast = a.x_vec_ok && tok0 + TM <= a.M;
    auto x_load = [&](const int seg) __attribute__((always_inline)) {
        const int k0 = seg * SEGMENT_ROWS;
        const int last = min(SEGMENT_ROWS, a.K - k0) - 1;      // rows past K repeat the last one (never multiplied)
#pragma unroll
        for (int u = 0; u < XL; ++u) {
            const int p = tid + u * NW * 64;
            const int row = k0 + min(p / PIECES, last), col = tok0 + (p % PIECES) * 16;
            if (fast) {
                xs[u] = *(const v4i*)(a.X + ((uint32_t)row * (uint32_t)a.ldx + (uint32_t)xcol(a, col)));
            } else if (a.x_vec_ok) {          // ragged last tile of an aligned matrix: whole chunks, masked
                const v4i v = *(const v4i*)(a.X + ((uint32_t)row * (uint32_t)a.ldx + (uint32_t)xcol(a, col < a.M ? col : 0)));
                xs[u] = v & piece_mask(a.M - col);
            } else {
                xs[u] = load_x16(a, row, col);
            }
        }
    };
    auto x_store = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < XL; ++u) {
            const int p = tid + u * NW * 64;
            *(v4i*)(lds + (p / PIECES) * STRIDE + (p % PIECES) * 16) = xs[u] ^ (v4i){FLIP, FLIP, FLIP, FLIP};
        }
    };
    x_load(0);

    v4i A0[CH], A1[CH], A2[CH];
    uint32_t I0[CH], I1[CH], I2[CH];
    auto w_load = [&](const int chunk, v4i (&A)[CH], uint32_t (&I)[CH]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            int step = s_begin + chunk * CH + j;
            step = (step < s_end) ? step : 0;          // step 0 is always readable
            A[j] = *(const v4i*)(a.vals + (int64_t)step * STEP_VAL_BYTES + lane * 16);
            I[j] = a.idx[(int64_t)step * STEP_IDX_DWORDS + 8 * g + (c >> 1)];
        }
    };
    w_load(0, A0, I0);
    if (nchunks > 1) w_load(1, A1, I1);
    if (nchunks > 2) w_load(2, A2, I2);

    int init = 0;
    if (have_tile) init = a.rowsum[n] * a.corr_mul;
    v4i acc[PIECES];
#pragma unroll
    for (int i = 0; i < PIECES; ++i) acc[i] = (v4i){init, init, init, init};
    float scale = 0.0f, bias = 0.0f;
    if constexpr (OUT != SPMM_OUT_S32) {
        if (have_tile && n < a.N) {
            scale = a.w_scale[n] * a.x_scale;
            if (a.bias) bias = a.bias[n];
        }
    }

    x_store();
    __syncthreads();
    int seg = 0;                                   // the segment in LDS
    if (nseg > 1) x_load(1);
    int seg_end = have_tile ? bounds[1] : 0;       // first step past segment `seg` (only compared when have_tile)
    // every wave: exactly nseg - 1 calls in total
    auto advance = [&]() __attribute__((always_inline)) {
        __syncthreads();                           // everyone has finished reading segment seg
        x_store();                                 // segment seg + 1, requested when seg was entered
        __syncthreads();
        ++seg;
        if (seg + 1 < nseg) x_load(seg + 1);
        if (have_tile) seg_end = bounds[seg + 1];
    };
    auto multiply = [&](const int chunk, const v4i (&A)[CH], const uint32_t (&I)[CH]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int step = s_begin + chunk * CH + j;
            if (step < s_end) {
                while (step >= seg_end && seg + 1 < nseg) advance();     // (also skips empty segments)
                const uint32_t a0 = (I[j] & 0xffffu) * STRIDE + (c & 1) * 8;
                const uint32_t a1 = (I[j] >> 16) * STRIDE + (c & 1) * 8;
#pragma unroll
                for (int i = 0; i < PIECES; ++i) {
                    const v2i x0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a0 + 16 * i));
                    const v2i x1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a1 + 16 * i));
                    const v4i xa = {x0[0], x0[1], x1[0], x1[1]};
                    acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa, A[j], acc[i], 0, 0, 0);
                }
            }
        }
    };
    for (int ch = 0; ch < nchunks; ch += 3) {
        multiply(ch, A0, I0);
        if (ch + 3 < nchunks) w_load(ch + 3, A0, I0);
        if (ch + 1 < nchunks) {
            multiply(ch + 1, A1, I1);
            if (ch + 4 < nchunks) w_load(ch + 4, A1, I1);
        }
        if (ch + 2 < nchunks) {
            multiply(ch + 2, A2, I2);
            if (ch + 5 < nchunks) w_load(ch + 5, A2, I2);
        }
    }
    while (seg + 1 < nseg) advance();              // drain: the segments after this wave's last step

    if (have_tile && n < a.N) {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int m0 = tok0 + 16 * i + 4 * g;
            if (m0 < a.M) finish4<OUT, POST, true>(a, acc[i], scale, bias, n, m0, GlobalLut{a.lut});
        }
    }
}

}  // namespace spmm
