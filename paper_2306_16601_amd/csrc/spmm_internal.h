// Internal declarations shared by the host packer, the C ABI glue and the HIP kernels.
// Not part of the public interface (see include/spmm.h).
#pragma once

#include <cstdint>
#include <vector>

#include "spmm.h"

namespace spmm {

// ---------------------------------------------------------------------------------------
// Device layout: "row-tile union" format.
//
// The weight is cut into row tiles of TILE_ROWS = 16 output rows (four 4x1 block-rows in
// the paper's orientation).  For each row tile and each K segment of `kc` consecutive k,
// the k positions at which ANY of the 16 rows is non-zero are listed; the list is padded
// to a multiple of STEP_K = 64 and cut into steps.  One step is exactly one
// v_mfma_i32_16x16x64_i8: 16 rows x 64 listed k, stored dense (zero where a row has no
// block at that k) in the register layout of the weight operand:
//     vals[step][lane][t] = W[16*tile + (lane % 16)][ k_list[16*(lane / 16) + t] ],  t < 16
// so a wave fetches a step with one coalesced 16-byte load per lane.  The matching
// activation rows are named by segment-local indices, stored pairwise so that the lane that
// supplies the LDS address of list slot 16g+t (first transposing read) and 16g+8+t (second)
// finds both in one dword:
//     idx[step][8*g + t] = k_local[16g + t] | k_local[16g + 8 + t] << 16,   g < 4, t < 8
// Padding slots carry zero weights and the index of some resident row, so they add nothing.
// Inside a step the listed k are ordered for conflict-free LDS banks, not ascending (pack.cpp).
// ---------------------------------------------------------------------------------------
constexpr int TILE_ROWS = 16;
constexpr int STEP_K = 64;
constexpr int STEP_VAL_BYTES = TILE_ROWS * STEP_K;   // 1024
constexpr int STEP_IDX_DWORDS = STEP_K / 2;          // 32
constexpr int SEGMENT_ROWS = 512;                    // kc: activation rows of one K segment (one LDS buffer)

struct HostLayout {
    int kc = 0, nseg = 0, ntiles = 0;
    int64_t nsteps = 0;
    int max_steps_per_tile = 0;
    int max_steps_per_segment = 0;  // largest step count of any (tile, segment)
    std::vector<uint8_t> vals;      // nsteps * 1024
    std::vector<uint32_t> idx;      // nsteps * 32
    std::vector<int32_t> seg_ptr;   // ntiles * nseg + 1
    std::vector<int32_t> rowsum;    // ntiles * 16
};

// Canonical 4x1 block-sparse-row form (host): what spmm_unpack and spmm_info read.
struct Bsr {
    int64_t N = 0, K = 0;
    spmm_block_t block = SPMM_BLOCK_N4K1;
    int64_t block_rows = 0;             // ceil(N/4) (N4K1) or N (N1K4)
    std::vector<int64_t> row_ptr;       // block_rows + 1
    std::vector<int32_t> index;         // k (N4K1) or K-block c (N1K4), ascending per block-row
    std::vector<int8_t> vals;           // 4 per block
};

void bsr_from_dense(const int8_t* W, int64_t N, int64_t K, int64_t ldw, spmm_block_t block, Bsr& out);
void bsr_to_dense(const Bsr& b, int8_t* W, int64_t ldw);
void layout_from_bsr(const Bsr& b, int kc, HostLayout& out);
// row_order[i] = row of the weight that becomes row i (a permutation of 0..N-1 that moves whole
// block-rows), chosen so that rows with overlapping k lists share a row tile
void order_rows_by_k_overlap(const Bsr& b, int kc, std::vector<int32_t>& row_order);
void bsr_permute_rows(const Bsr& b, const std::vector<int32_t>& row_order, Bsr& out);

// ---------------------------------------------------------------------------------------
// Kernel launch interface (plan and dispatch in spmm_plan.hip, kernels in spmm_kernels.h).
// ---------------------------------------------------------------------------------------
struct KernelArgs {
    const uint8_t* vals;
    const uint32_t* idx;
    const int32_t* seg_ptr;
    const int32_t* rowsum;
    const uint8_t* X;
    void* out;
    const float* w_scale;
    const float* bias;
    const int8_t* lut;
    const float* sum;    // Sum post-operator: [N][ld_sum] or nullptr
    int64_t ldx, ldo, ld_sum;
    int N, K, M;
    int kc, nseg, ntiles;
    int n_tok_tiles, n_row_groups;
    int n_streams;       // persistent kernel: workgroups per row group, each walking token tiles j*n_streams + stream
    int tiles_per_stream, tiles_extra;   // n_tok_tiles = tiles_per_stream * n_streams + tiles_extra
    int xcd_map;         // simple / short-batch kernels: how a workgroup id decodes, see decode_workgroup()
    int corr_mul;        // 128 - x_zero_point: the activations are multiplied as (x - 128)
    float x_scale, inv_out, inv_mid, out_zp_f;
    int x_vec_ok;        // X base 16-byte aligned, ldx % 16 == 0 and K * ldx < 2^31 (tile-major: the whole X < 2^31 bytes)
    int out_vec_ok;      // out base 16-byte aligned, row pitch a multiple of 16 bytes, whole output < 2^31 bytes
                         // (and, with Sum, the same for the second operand)
    int out_tile_stride; // 0: out row-major [N][ldo]; else 1-byte out token-tile-major [ceil(M/32)][N][32], ldo = 32 and this = 32 N
    int x_tile_stride;   // 0: X row-major [K][ldx]; else X token-tile-major [ceil(M/32)][K][32], ldx = 32 and this = 32 K
    uint32_t out_bytes;  // with out_vec_ok: bytes from out to the end of the last element the call may write (< 2^31)
};

struct Plan {
    int token_tile;          // TM of the pipelined kernel (128 or 96), or 64 for the simple kernel
    int row_tiles_per_wave;  // 1 (pipelined) or 1 / 2 (simple kernel)
    int waves;               // NW: waves that own a row tile
    int loaders;             // pipelined kernel: extra waves that only stage activations (0 or 4)
    int simple;              // 1: simple kernel
    int slab;                // 1: the short-batch kernel (token tile 16 or 32, whole K resident in LDS) in its place
    int stream;              // 1: the streamed kernel (segment staging, flat weight stream) in its place
    int max_steps;           // unroll bound of the per-segment step loop (pipelined kernel)
    int n_row_groups, n_tok_tiles, n_streams, xcd_map;
    int64_t workgroups;
};

// variant: 0 = automatic, 8 / 16 = waves per workgroup (pipelined, token tile 128 or 96),
// 108 / 112 = pipelined with 8 / 12 compute waves and 4 loader waves (token tile 128; 112 also 96),
// 101 / 102 = simple kernel with 1 / 2 row tiles per wave (token tile 64; 101 also 32 and 16),
// 103 = short-batch kernel (token tile 16 or 32), 104 = streamed kernel (token tile 64, 32 or 16)
constexpr int SLAB_SEGMENTS = 8;      // K segments the short-batch kernel keeps in LDS, token tile 16
constexpr int SLAB_SEGMENTS_32 = 6;   // and token tile 32
// what the plan needs to know of a packed weight
struct WeightDims {
    int ntiles, nseg, K;
    int64_t nsteps;
    int max_steps_per_segment, max_steps_per_tile;
};
bool plan_supported(int token_tile, int variant);
// aligned: X and out take the 16-byte paths (base and row pitch aligned); if not, the automatic choice
// avoids the 16-wave pipelined kernels, whose general paths are the slow bytewise ones
// out_bytes: size of an output element (the plan gives 4-byte outputs workgroups with loader waves)
Plan make_plan(int64_t M, const WeightDims& w, int num_cus, int force_tm, int variant, bool aligned = true,
               int out_bytes = 1);
// Launches the SpMM kernel; returns a hipError_t value as int (0 = success).
// postop: SPMM_POST_* value, plus POST_SUM_BIT when a.sum is to be added
constexpr int POST_SUM_BIT = 4;   // (a bit no SPMM_POST_* value uses)
int launch_spmm(const Plan& plan, KernelArgs& a, spmm_out_t out_type, int postop, void* stream);

}  // namespace spmm
