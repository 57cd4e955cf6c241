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
//  * post-operators (Section 3.3) are applied to the accumulators in registers.
//
// Lane roles of the matrix instruction (D = A.B, 64 lanes, g = lane / 16, c = lane % 16):
//   A operand (activations): row = token c, bytes t = k-list slots 16g .. 16g+15
//   B operand (weights)    : column = output row c, same k slots
//   D                      : D[token 4g + r][output row c], r = 0..3
#include <hip/hip_runtime.h>

#include <cstdint>

#include "spmm_internal.h"

namespace spmm {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v2i* lds_v2i_ptr;

template <int TM>
struct TileCfg {
    static constexpr int STRIDE = TM + 16;   // LDS row pitch in bytes: rows k, k+1, .. start 4 banks apart
    static constexpr int LDS_BYTES = SEGMENT_ROWS * STRIDE;
    static constexpr int PIECES = TM / 16;   // 16-byte pieces per activation row
};

// Exact GELU evaluated in double on the binary32 pre-activation, rounded once to binary32.
__device__ __forceinline__ float gelu_f32(float y)
{
    const double x = (double)y;
    return (float)(0.5 * x * erfc(-x * 0.70710678118654752440));
}

template <int OUT, int POST>
__device__ __forceinline__ void finish4(const KernelArgs& a, const v4i acc, const float s, const float b,
                                        const int n, const int m0)
{
    // acc: 4 consecutive tokens m0..m0+3 of output row n.
    const int valid = a.M - m0;   // > 0 guaranteed by caller
    if constexpr (OUT == SPMM_OUT_S32) {
        int32_t* o = (int32_t*)a.out + (int64_t)n * a.ldo + m0;
        if (a.out_vec_ok && valid >= 4) {
            *(v4i*)o = acc;
        } else {
            for (int r = 0; r < 4; ++r)
                if (r < valid) o[r] = acc[r];
        }
    } else {
        float y[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) y[r] = __fmaf_rn((float)acc[r], s, b);
        if constexpr (OUT == SPMM_OUT_F32) {
            if constexpr (POST == SPMM_POST_GELU) {
#pragma unroll
                for (int r = 0; r < 4; ++r) y[r] = gelu_f32(y[r]);
            }
            float* o = (float*)a.out + (int64_t)n * a.ldo + m0;
            if (a.out_vec_ok && valid >= 4) {
                v4f v = {y[0], y[1], y[2], y[3]};
                *(v4f*)o = v;
            } else {
                for (int r = 0; r < 4; ++r)
                    if (r < valid) o[r] = y[r];
            }
        } else {
            uint32_t q[4];
            if constexpr (POST == SPMM_POST_GELU) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    // key = sat_s8(rint(y / mid_scale)); looked up as key + 128 in [0, 255]
                    const float t = rintf(y[r] * a.inv_mid) + 128.0f;
                    const uint32_t key = __builtin_amdgcn_cvt_pk_u8_f32(t, 0u, 0u);
                    q[r] = (uint32_t)(uint8_t)a.lut[key];
                }
            } else {
                const float lo = (OUT == SPMM_OUT_U8) ? 0.0f : -128.0f;
                const float hi = (OUT == SPMM_OUT_U8) ? 255.0f : 127.0f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float t = fminf(hi, fmaxf(lo, rintf(y[r] * a.inv_out) + a.out_zp_f));
                    q[r] = (uint32_t)((int)t) & 0xffu;
                }
            }
            uint8_t* o = (uint8_t*)a.out + (int64_t)n * a.ldo + m0;
            if (a.out_vec_ok && valid >= 4) {
                *(uint32_t*)o = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
            } else {
                for (int r = 0; r < 4; ++r)
                    if (r < valid) o[r] = (uint8_t)q[r];
            }
        }
    }
}

// One workgroup = NW waves; wave w owns R row tiles; the workgroup covers NW*R*16 output rows
// and TM tokens, and walks over the K segments with the activations of one segment in LDS.
template <int TM, int NW, int R, int OUT, int POST>
__global__ void __launch_bounds__(NW * 64) spmm_rowtile_mfma(const KernelArgs a)
{
    using C = TileCfg<TM>;
    __shared__ __attribute__((aligned(16))) uint8_t lds[C::LDS_BYTES];

    // XCD-aware decomposition: workgroups are handed to the 8 XCDs round-robin, so the
    // workgroups that share a token tile (and therefore its activations) get ids that are
    // congruent mod 8 and meet in the same L2.
    const int b = blockIdx.x;
    const int xcd = b & 7, local = b >> 3;
    const int tt = xcd + 8 * (local / a.n_row_groups);
    const int rg = local % a.n_row_groups;
    if (tt >= a.n_tok_tiles) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const int tok0 = tt * TM;

    // accumulators start at 128 * rowsum(W) of this lane's output row (activations are x - 128)
    v4i acc[R][C::PIECES];
    int row_of[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int tile = (rg * NW + wave) * R + r;
        row_of[r] = tile * TILE_ROWS + c;
        int init = 0;
        if (tile < a.ntiles) init = a.rowsum[row_of[r]] * a.corr_mul;
#pragma unroll
        for (int i = 0; i < C::PIECES; ++i) acc[r][i] = (v4i){init, init, init, init};
    }

    for (int seg = 0; seg < a.nseg; ++seg) {
        // ---- stage activations X[seg*kc .. +rows][tok0 .. tok0+TM) into LDS as (x - 128)
        const int k0 = seg * a.kc;
        const int rows = min(a.kc, a.K - k0);
        if (seg > 0) __syncthreads();
        for (int p = tid; p < rows * C::PIECES; p += NW * 64) {
            const int row = p / C::PIECES, piece = p % C::PIECES;
            const int col = tok0 + piece * 16;
            const uint8_t* src = a.X + (int64_t)(k0 + row) * a.ldx + col;
            v4i v;
            if (a.x_vec_ok && col + 16 <= a.M) {
                v = *(const v4i*)src;
            } else {
                uint32_t w[4] = {0, 0, 0, 0};
                for (int j = 0; j < 16; ++j)
                    if (col + j < a.M) w[j >> 2] |= (uint32_t)src[j] << (8 * (j & 3));
                v = (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
            }
            v ^= (v4i){(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
            *(v4i*)(lds + row * C::STRIDE + piece * 16) = v;
        }
        __syncthreads();

        // ---- multiply: every wave streams the steps of its row tiles for this segment
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int tile = (rg * NW + wave) * R + r;
            if (tile >= a.ntiles) continue;
            const int s0 = a.seg_ptr[tile * a.nseg + seg];
            const int s1 = a.seg_ptr[tile * a.nseg + seg + 1];
            if (s0 >= s1) continue;
            v4i w = *(const v4i*)(a.vals + (int64_t)s0 * STEP_VAL_BYTES + lane * 16);
            uint32_t ix = a.idx[(int64_t)s0 * STEP_IDX_DWORDS + 8 * g + (c >> 1)];
            for (int s = s0; s < s1; ++s) {
                const v4i w_cur = w;
                const uint32_t ix_cur = ix;
                if (s + 1 < s1) {   // prefetch the next step's weights and indices
                    w = *(const v4i*)(a.vals + (int64_t)(s + 1) * STEP_VAL_BYTES + lane * 16);
                    ix = a.idx[(int64_t)(s + 1) * STEP_IDX_DWORDS + 8 * g + (c >> 1)];
                }
                // this lane supplies the address of list slot 16g + c/2 (and + 8), half c & 1
                const uint32_t a0 = (ix_cur & 0xffffu) * C::STRIDE + (c & 1) * 8;
                const uint32_t a1 = (ix_cur >> 16) * C::STRIDE + (c & 1) * 8;
#pragma unroll
                for (int i = 0; i < C::PIECES; ++i) {
                    const v2i x0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a0 + 16 * i));
                    const v2i x1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + a1 + 16 * i));
                    const v4i xa = {x0[0], x0[1], x1[0], x1[1]};
                    acc[r][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xa, w_cur, acc[r][i], 0, 0, 0);
                }
            }
        }
    }

    // ---- post-operators on the accumulators (registers), then store
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
        for (int i = 0; i < C::PIECES; ++i) {
            const int m0 = tok0 + 16 * i + 4 * g;
            if (m0 < a.M) finish4<OUT, POST>(a, acc[r][i], s, bias, n, m0);
        }
    }
}

// ---------------------------------------------------------------------------------------
// host side: plan + dispatch
// ---------------------------------------------------------------------------------------
bool plan_supported(int token_tile, int row_tiles_per_wave)
{
    return (token_tile == 64) && (row_tiles_per_wave == 1 || row_tiles_per_wave == 2);
}

Plan make_plan(int64_t N, int64_t K, int64_t M, int ntiles, spmm_out_t out_type, int force_tm, int force_r)
{
    (void)N; (void)K; (void)out_type;
    Plan p;
    p.token_tile = force_tm ? force_tm : 64;
    p.waves = 8;
    p.row_tiles_per_wave = force_r ? force_r : ((ntiles >= 64) ? 2 : 1);
    const int64_t n_tok = (M + p.token_tile - 1) / p.token_tile;
    const int64_t n_rg = (ntiles + p.waves * p.row_tiles_per_wave - 1) / (p.waves * p.row_tiles_per_wave);
    p.workgroups = 8 * n_rg * ((n_tok + 7) / 8);
    return p;
}

template <int TM, int NW, int R>
static int launch_tmr(const Plan& plan, const KernelArgs& a, spmm_out_t out_type, spmm_postop_t postop, hipStream_t st)
{
    const dim3 grid((unsigned)plan.workgroups), block(NW * 64);
#define SPMM_LAUNCH(OUT, POST) \
    hipLaunchKernelGGL((spmm_rowtile_mfma<TM, NW, R, OUT, POST>), grid, block, 0, st, a)
    const bool gelu = (postop == SPMM_POST_GELU);
    switch (out_type) {
    case SPMM_OUT_S32: SPMM_LAUNCH(SPMM_OUT_S32, SPMM_POST_NONE); break;
    case SPMM_OUT_F32:
        if (gelu) SPMM_LAUNCH(SPMM_OUT_F32, SPMM_POST_GELU); else SPMM_LAUNCH(SPMM_OUT_F32, SPMM_POST_NONE);
        break;
    case SPMM_OUT_S8:
        if (gelu) SPMM_LAUNCH(SPMM_OUT_S8, SPMM_POST_GELU); else SPMM_LAUNCH(SPMM_OUT_S8, SPMM_POST_NONE);
        break;
    case SPMM_OUT_U8:
        if (gelu) SPMM_LAUNCH(SPMM_OUT_U8, SPMM_POST_GELU); else SPMM_LAUNCH(SPMM_OUT_U8, SPMM_POST_NONE);
        break;
    }
#undef SPMM_LAUNCH
    return (int)hipGetLastError();
}

int launch_spmm(const Plan& plan, KernelArgs& a, spmm_out_t out_type, spmm_postop_t postop, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    const int rows_per_wg = plan.waves * plan.row_tiles_per_wave;
    a.n_tok_tiles = (int)((a.M + plan.token_tile - 1) / plan.token_tile);
    a.n_row_groups = (a.ntiles + rows_per_wg - 1) / rows_per_wg;
    if (plan.token_tile == 64 && plan.waves == 8) {
        if (plan.row_tiles_per_wave == 1) return launch_tmr<64, 8, 1>(plan, a, out_type, postop, st);
        if (plan.row_tiles_per_wave == 2) return launch_tmr<64, 8, 2>(plan, a, out_type, postop, st);
    }
    return (int)hipErrorInvalidValue;
}

}  // namespace spmm
