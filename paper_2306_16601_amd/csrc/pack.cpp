// Host-side packer: dense-with-zeros int8 weight -> canonical 4x1 block-sparse rows ->
// the device's row-tile union layout (see spmm_internal.h).  Pure C++, no GPU calls.
//
// Paper Section 3.1 / Figure 1: blocks of 4x1 with the sparsity dimension on the output
// channels.  Section 3.2: the kernel is specialised on the sparse weight and its indices,
// and the block count is padded to what the multiply instruction accumulates over (note
// after Algorithm 1).  Here that instruction is the 16x16x64 int8 matrix op, so the unit
// of padding is 64 listed k positions per 16-row tile.
#include <algorithm>
#include <cstring>

#include "spmm_internal.h"

namespace spmm {

void bsr_from_dense(const int8_t* W, int64_t N, int64_t K, int64_t ldw, spmm_block_t block, Bsr& out)
{
    out.N = N;
    out.K = K;
    out.block = block;
    out.row_ptr.clear();
    out.index.clear();
    out.vals.clear();
    if (block == SPMM_BLOCK_N4K1) {
        out.block_rows = (N + 3) / 4;
        out.row_ptr.reserve(out.block_rows + 1);
        out.row_ptr.push_back(0);
        for (int64_t br = 0; br < out.block_rows; ++br) {
            const int64_t n0 = br * 4;
            const int rows = (int)std::min<int64_t>(4, N - n0);
            for (int64_t k = 0; k < K; ++k) {
                int8_t v[4] = {0, 0, 0, 0};
                bool any = false;
                for (int i = 0; i < rows; ++i) {
                    v[i] = W[(n0 + i) * ldw + k];
                    any |= (v[i] != 0);
                }
                if (any) {
                    out.index.push_back((int32_t)k);
                    out.vals.insert(out.vals.end(), v, v + 4);
                }
            }
            out.row_ptr.push_back((int64_t)out.index.size());
        }
    } else {
        out.block_rows = N;
        const int64_t kblocks = (K + 3) / 4;
        out.row_ptr.reserve(N + 1);
        out.row_ptr.push_back(0);
        for (int64_t n = 0; n < N; ++n) {
            for (int64_t c = 0; c < kblocks; ++c) {
                const int cols = (int)std::min<int64_t>(4, K - 4 * c);
                int8_t v[4] = {0, 0, 0, 0};
                bool any = false;
                for (int j = 0; j < cols; ++j) {
                    v[j] = W[n * ldw + 4 * c + j];
                    any |= (v[j] != 0);
                }
                if (any) {
                    out.index.push_back((int32_t)c);
                    out.vals.insert(out.vals.end(), v, v + 4);
                }
            }
            out.row_ptr.push_back((int64_t)out.index.size());
        }
    }
}

void bsr_to_dense(const Bsr& b, int8_t* W, int64_t ldw)
{
    for (int64_t n = 0; n < b.N; ++n) std::memset(W + n * ldw, 0, (size_t)b.K);
    for (int64_t br = 0; br < b.block_rows; ++br) {
        for (int64_t e = b.row_ptr[br]; e < b.row_ptr[br + 1]; ++e) {
            const int8_t* v = &b.vals[(size_t)e * 4];
            if (b.block == SPMM_BLOCK_N4K1) {
                const int64_t k = b.index[e];
                for (int i = 0; i < 4 && br * 4 + i < b.N; ++i) W[(br * 4 + i) * ldw + k] = v[i];
            } else {
                const int64_t k0 = (int64_t)b.index[e] * 4;
                for (int j = 0; j < 4 && k0 + j < b.K; ++j) W[br * ldw + k0 + j] = v[j];
            }
        }
    }
}

// Expand the block-rows that intersect row tile `tile` into a dense 16 x K scratch.
static void expand_tile(const Bsr& b, int64_t tile, std::vector<int8_t>& buf)
{
    std::fill(buf.begin(), buf.end(), (int8_t)0);
    const int64_t K = b.K;
    const int64_t n0 = tile * TILE_ROWS;
    if (b.block == SPMM_BLOCK_N4K1) {
        for (int q = 0; q < TILE_ROWS / 4; ++q) {
            const int64_t br = n0 / 4 + q;
            if (br >= b.block_rows) break;
            for (int64_t e = b.row_ptr[br]; e < b.row_ptr[br + 1]; ++e) {
                const int64_t k = b.index[e];
                for (int i = 0; i < 4; ++i) buf[(size_t)(q * 4 + i) * K + k] = b.vals[(size_t)e * 4 + i];
            }
        }
    } else {
        for (int r = 0; r < TILE_ROWS; ++r) {
            const int64_t n = n0 + r;
            if (n >= b.N) break;
            for (int64_t e = b.row_ptr[n]; e < b.row_ptr[n + 1]; ++e) {
                const int64_t k0 = (int64_t)b.index[e] * 4;
                for (int j = 0; j < 4 && k0 + j < K; ++j) buf[(size_t)r * K + k0 + j] = b.vals[(size_t)e * 4 + j];
            }
        }
    }
}

void layout_from_bsr(const Bsr& b, int kc, HostLayout& out)
{
    const int64_t N = b.N, K = b.K;
    out.kc = kc;
    out.nseg = (int)((K + kc - 1) / kc);
    out.ntiles = (int)((N + TILE_ROWS - 1) / TILE_ROWS);
    out.vals.clear();
    out.idx.clear();
    out.seg_ptr.assign(1, 0);
    out.rowsum.assign((size_t)out.ntiles * TILE_ROWS, 0);
    out.max_steps_per_tile = 0;
    out.max_steps_per_segment = 0;

    std::vector<int8_t> buf((size_t)TILE_ROWS * K);
    std::vector<int32_t> list;
    for (int64_t tile = 0; tile < out.ntiles; ++tile) {
        expand_tile(b, tile, buf);
        for (int r = 0; r < TILE_ROWS; ++r) {
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += buf[(size_t)r * K + k];
            out.rowsum[(size_t)tile * TILE_ROWS + r] = s;
        }
        int steps_this_tile = 0;
        for (int seg = 0; seg < out.nseg; ++seg) {
            const int64_t k_lo = (int64_t)seg * kc, k_hi = std::min<int64_t>(K, k_lo + kc);
            list.clear();
            for (int64_t k = k_lo; k < k_hi; ++k) {
                bool any = false;
                for (int r = 0; r < TILE_ROWS; ++r) any |= (buf[(size_t)r * K + k] != 0);
                if (any) list.push_back((int32_t)(k - k_lo));
            }
            const int nsteps = (int)((list.size() + STEP_K - 1) / STEP_K);
            for (int s = 0; s < nsteps; ++s) {
                const size_t vbase = out.vals.size(), ibase = out.idx.size();
                out.vals.resize(vbase + STEP_VAL_BYTES, 0);
                out.idx.resize(ibase + STEP_IDX_DWORDS, 0);
                auto slot_k = [&](int slot) -> int32_t {   // segment-local k of list slot, -1 = padding
                    const size_t e = (size_t)s * STEP_K + slot;
                    return e < list.size() ? list[e] : -1;
                };
                for (int lane = 0; lane < 64; ++lane) {
                    const int g = lane / 16, r = lane % 16;
                    for (int t = 0; t < 16; ++t) {
                        const int32_t kl = slot_k(16 * g + t);
                        if (kl >= 0) out.vals[vbase + (size_t)lane * 16 + t] = (uint8_t)buf[(size_t)r * K + k_lo + kl];
                    }
                }
                for (int g = 0; g < 4; ++g)
                    for (int t = 0; t < 8; ++t) {
                        const int32_t ka = std::max(0, slot_k(16 * g + t));
                        const int32_t kb = std::max(0, slot_k(16 * g + 8 + t));
                        out.idx[ibase + 8 * g + t] = (uint32_t)ka | ((uint32_t)kb << 16);
                    }
            }
            steps_this_tile += nsteps;
            out.max_steps_per_segment = std::max(out.max_steps_per_segment, nsteps);
            out.seg_ptr.push_back(out.seg_ptr.back() + nsteps);
        }
        out.max_steps_per_tile = std::max(out.max_steps_per_tile, steps_this_tile);
    }
    out.nsteps = out.seg_ptr.back();
}

}  // namespace spmm
