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

// Order the listed k of one (row tile, segment) inside its steps so that the transposing
// LDS reads hit distinct banks.
//
// One ds_read_b64_tr_b8 of a wave touches 32 activation rows (4 lane groups x 8 rows), 16 bytes
// each; with the row pitch used by the kernels (token tile + 16 bytes) a row starts at LDS
// bank 4 * ((9 * row) % 16), so two rows collide exactly when their indices are congruent
// mod 16.  The 64 slots of a step are read by two instructions (slots t < 8 and t >= 8 of
// every group), each in two half-waves (groups {0,1} and {2,3}): four "half-reads" of 16 rows.
// The entries are dealt out so that a half-read holds every residue mod 16 at most once
// whenever the counts allow it; padding slots (zero weights) are pointed at a row of a
// residue the half-read still lacks instead of all hitting row 0.
// slot_k[s*64 + 16*g + t] = segment-local k or -1 (padding); slot_row = row actually read.
static void arrange_for_lds_banks(const std::vector<int32_t>& list, int rows_in_segment, int nsteps,
                                  std::vector<int32_t>& slot_k, std::vector<int32_t>& slot_row)
{
    const int H = 4 * nsteps;   // half-reads
    slot_k.assign((size_t)nsteps * STEP_K, -1);
    slot_row.assign((size_t)nsteps * STEP_K, 0);
    if (nsteps == 0) return;
    std::vector<std::vector<int32_t>> by_res(16);
    for (int32_t k : list) by_res[k & 15].push_back(k);
    int order[16];
    for (int r = 0; r < 16; ++r) order[r] = r;
    std::stable_sort(order, order + 16, [&](int x, int y) { return by_res[x].size() > by_res[y].size(); });

    // Largest residue class first; each class is spread over the least-filled half-reads, one
    // entry per half-read, so that no half-read runs out of room while others still have
    // holes.  Only a class with more than H entries is forced to double up somewhere.
    std::vector<std::vector<int32_t>> hr((size_t)H);
    std::vector<uint32_t> mask((size_t)H, 0);
    std::vector<int> by_load((size_t)H);
    for (int oi = 0; oi < 16; ++oi) {
        const int r = order[oi];
        size_t next = 0;
        while (next < by_res[r].size()) {
            for (int h = 0; h < H; ++h) by_load[h] = h;
            std::stable_sort(by_load.begin(), by_load.end(),
                             [&](int x, int y) { return hr[x].size() < hr[y].size(); });
            bool placed = false;
            for (int i = 0; i < H && next < by_res[r].size(); ++i) {
                const int h = by_load[i];
                if (hr[h].size() >= 16) break;
                hr[h].push_back(by_res[r][next++]);
                mask[h] |= 1u << r;
                placed = true;
            }
            if (!placed) break;   // cannot happen: 16 * H slots >= list.size()
        }
    }
    for (int h = 0; h < H; ++h) {
        const int s = h / 4, instr = (h / 2) % 2, pair = h % 2;
        int next_res = 0;
        for (int j = 0; j < 16; ++j) {
            const int g = 2 * pair + j / 8, t = 8 * instr + j % 8;
            const size_t slot = (size_t)s * STEP_K + 16 * g + t;
            if (j < (int)hr[h].size()) {
                slot_k[slot] = hr[h][j];
                slot_row[slot] = hr[h][j];
            } else {
                while (next_res < 16 && (mask[h] & (1u << next_res))) ++next_res;
                int row = 0;
                if (next_res < 16) {
                    if (next_res < rows_in_segment) row = next_res;
                    mask[h] |= 1u << next_res;
                }
                slot_row[slot] = row;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Offline ordering of the output rows (Section 3.2: what can be tuned offline for a given
// sparse weight).  A row tile multiplies the UNION of the k lists of its rows, padded to
// whole steps, so rows with similar lists belong in one tile.  The movable unit is what
// keeps the block structure: a 4x1 block-row (four consecutive rows) in the paper's
// orientation, a single row for 1x4 blocks; a trailing partial block-row stays last, so the
// first N rows of the new order are exactly the N rows of the weight.
//
// Greedy clustering: units are taken heaviest first; a tile is opened with the heaviest
// unit left and filled with the units (among the next `window` in that order) that add the
// fewest steps, then the fewest listed k, to the tile's per-segment unions.  Heaviest-first
// also puts rows of similar length next to each other, which is what the waves of one
// workgroup (one row tile each, in lock-step per segment) want.
// ---------------------------------------------------------------------------------------
namespace {

struct KSet {
    std::vector<uint64_t> w;   // one bit per k
};

inline int popcount64(uint64_t x) { return __builtin_popcountll(x); }

// steps of a union, per segment of kc (a multiple of 64) positions
int64_t steps_of(const std::vector<uint64_t>& u, int words_per_seg, int64_t* listed)
{
    int64_t steps = 0, total = 0;
    for (size_t w0 = 0; w0 < u.size(); w0 += (size_t)words_per_seg) {
        int cnt = 0;
        for (size_t w = w0; w < std::min(u.size(), w0 + (size_t)words_per_seg); ++w) cnt += popcount64(u[w]);
        steps += (cnt + STEP_K - 1) / STEP_K;
        total += cnt;
    }
    if (listed) *listed = total;
    return steps;
}

}  // namespace

void order_rows_by_k_overlap(const Bsr& b, int kc, std::vector<int32_t>& row_order)
{
    const bool n4 = (b.block == SPMM_BLOCK_N4K1);
    const int unit_rows = n4 ? 4 : 1;
    const int group = TILE_ROWS / unit_rows;             // units per row tile
    const int64_t full_units = n4 ? b.N / 4 : b.N;       // a trailing partial block-row is not moved
    const int words = (int)((b.K + 63) / 64), words_per_seg = kc / 64;

    std::vector<KSet> ks((size_t)full_units);
    std::vector<int64_t> weight((size_t)full_units);
    for (int64_t u = 0; u < full_units; ++u) {
        ks[(size_t)u].w.assign((size_t)words, 0);
        weight[(size_t)u] = b.row_ptr[u + 1] - b.row_ptr[u];
        for (int64_t e = b.row_ptr[u]; e < b.row_ptr[u + 1]; ++e) {
            if (n4) {
                const int64_t k = b.index[e];
                ks[(size_t)u].w[(size_t)(k >> 6)] |= (uint64_t)1 << (k & 63);
            } else {
                for (int j = 0; j < 4; ++j) {
                    const int64_t k = (int64_t)b.index[e] * 4 + j;
                    if (k < b.K) ks[(size_t)u].w[(size_t)(k >> 6)] |= (uint64_t)1 << (k & 63);
                }
            }
        }
    }
    std::vector<int64_t> by_weight((size_t)full_units);
    for (int64_t u = 0; u < full_units; ++u) by_weight[(size_t)u] = u;
    std::stable_sort(by_weight.begin(), by_weight.end(),
                     [&](int64_t x, int64_t y) { return weight[(size_t)x] > weight[(size_t)y]; });

    const int64_t window = 512;
    std::vector<char> used((size_t)full_units, 0);
    std::vector<int64_t> unit_order;
    unit_order.reserve((size_t)full_units);
    std::vector<uint64_t> uni((size_t)words), trial((size_t)words);
    int64_t first_free = 0;   // position in by_weight of the heaviest unit not yet placed
    while ((int64_t)unit_order.size() < full_units) {
        while (used[(size_t)by_weight[(size_t)first_free]]) ++first_free;
        const int64_t seed = by_weight[(size_t)first_free];
        used[(size_t)seed] = 1;
        unit_order.push_back(seed);
        uni = ks[(size_t)seed].w;
        for (int slot = 1; slot < group && (int64_t)unit_order.size() < full_units; ++slot) {
            int64_t best = -1, best_steps = 0, best_listed = 0, seen = 0;
            for (int64_t p = first_free; p < full_units && seen < window; ++p) {
                const int64_t u = by_weight[(size_t)p];
                if (used[(size_t)u]) continue;
                ++seen;
                for (int w = 0; w < words; ++w) trial[(size_t)w] = uni[(size_t)w] | ks[(size_t)u].w[(size_t)w];
                int64_t listed = 0;
                const int64_t st = steps_of(trial, words_per_seg, &listed);
                if (best < 0 || st < best_steps || (st == best_steps && listed < best_listed)) {
                    best = u; best_steps = st; best_listed = listed;
                }
            }
            used[(size_t)best] = 1;
            unit_order.push_back(best);
            for (int w = 0; w < words; ++w) uni[(size_t)w] |= ks[(size_t)best].w[(size_t)w];
        }
    }
    row_order.clear();
    row_order.reserve((size_t)b.N);
    for (const int64_t u : unit_order)
        for (int i = 0; i < unit_rows; ++i) row_order.push_back((int32_t)(u * unit_rows + i));
    for (int64_t n = full_units * unit_rows; n < b.N; ++n) row_order.push_back((int32_t)n);   // the partial block-row
}

// The weight with its rows in the given order (whole units, see above), as a canonical form of its own.
void bsr_permute_rows(const Bsr& b, const std::vector<int32_t>& row_order, Bsr& out)
{
    const int unit_rows = (b.block == SPMM_BLOCK_N4K1) ? 4 : 1;
    out.N = b.N; out.K = b.K; out.block = b.block; out.block_rows = b.block_rows;
    out.row_ptr.assign(1, 0);
    out.index.clear(); out.vals.clear();
    out.index.reserve(b.index.size()); out.vals.reserve(b.vals.size());
    for (int64_t br = 0; br < b.block_rows; ++br) {
        const int64_t src = row_order[(size_t)(br * unit_rows)] / unit_rows;
        out.index.insert(out.index.end(), b.index.begin() + b.row_ptr[src], b.index.begin() + b.row_ptr[src + 1]);
        out.vals.insert(out.vals.end(), b.vals.begin() + 4 * b.row_ptr[src], b.vals.begin() + 4 * b.row_ptr[src + 1]);
        out.row_ptr.push_back((int64_t)out.index.size());
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
    std::vector<int32_t> list, slot_k, slot_row;
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
            arrange_for_lds_banks(list, (int)(k_hi - k_lo), nsteps, slot_k, slot_row);
            for (int s = 0; s < nsteps; ++s) {
                const size_t vbase = out.vals.size(), ibase = out.idx.size();
                out.vals.resize(vbase + STEP_VAL_BYTES, 0);
                out.idx.resize(ibase + STEP_IDX_DWORDS, 0);
                const int32_t* sk = &slot_k[(size_t)s * STEP_K];     // segment-local k, -1 = padding
                const int32_t* sr = &slot_row[(size_t)s * STEP_K];   // activation row the slot reads
                for (int lane = 0; lane < 64; ++lane) {
                    const int g = lane / 16, r = lane % 16;
                    for (int t = 0; t < 16; ++t) {
                        const int32_t kl = sk[16 * g + t];
                        if (kl >= 0) out.vals[vbase + (size_t)lane * 16 + t] = (uint8_t)buf[(size_t)r * K + k_lo + kl];
                    }
                }
                for (int g = 0; g < 4; ++g)
                    for (int t = 0; t < 8; ++t)
                        out.idx[ibase + 8 * g + t] = (uint32_t)sr[16 * g + t] | ((uint32_t)sr[16 * g + 8 + t] << 16);
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
