// C ABI of the library (declared in include/spmm.h): argument checking, handle
// ownership, device upload of the packed weight and kernel dispatch.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "spmm_internal.h"

struct spmm_handle {
    spmm::Bsr bsr;                 // canonical host copy (unpack / info), rows in the caller's order
    std::vector<int32_t> row_order;   // empty: identity; else row i of the packed weight = row row_order[i]
    int64_t nnz_blocks = 0;
    int device = 0;
    spmm::HostLayout hl;           // host copy of the row-tile union layout
    // device copy of the same
    bool on_device = false;
    int kc = 0, nseg = 0, ntiles = 0, max_steps_per_tile = 0, max_steps_per_segment = 0;
    int num_cus = 256;
    int64_t nsteps = 0;
    uint8_t* d_vals = nullptr;
    uint32_t* d_idx = nullptr;
    int32_t* d_seg_ptr = nullptr;
    int32_t* d_rowsum = nullptr;
    int64_t device_bytes = 0;
    int force_tm = 0, force_r = 0;
};

namespace {

template <typename T>
hipError_t upload(T*& dst, const std::vector<T>& src, int64_t& total)
{
    // at least one zero step's worth, so that step index 0 is always readable
    const size_t bytes = std::max<size_t>(src.size() * sizeof(T), spmm::STEP_VAL_BYTES);
    hipError_t e = hipMalloc((void**)&dst, bytes);
    if (e != hipSuccess) return e;
    total += (int64_t)bytes;
    if (src.size() * sizeof(T) < bytes) e = hipMemset(dst, 0, bytes);
    if (e != hipSuccess) return e;
    if (!src.empty()) e = hipMemcpy(dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice);
    return e;
}

void free_device(spmm_handle* h)
{
    if (h->d_vals) (void)hipFree(h->d_vals);
    if (h->d_idx) (void)hipFree(h->d_idx);
    if (h->d_seg_ptr) (void)hipFree(h->d_seg_ptr);
    if (h->d_rowsum) (void)hipFree(h->d_rowsum);
    h->d_vals = nullptr; h->d_idx = nullptr; h->d_seg_ptr = nullptr; h->d_rowsum = nullptr;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

spmm::Plan plan_for(const spmm_handle* h, int64_t M, bool aligned = true, int out_bytes = 1)
{
    const spmm::WeightDims w{h->ntiles, h->nseg, (int)h->bsr.K, h->nsteps, h->max_steps_per_segment,
                             h->max_steps_per_tile};
    return spmm::make_plan(M, w, h->num_cus, h->force_tm, h->force_r, aligned, out_bytes);
}

}  // namespace

extern "C" {

static spmm_status_t pack_common(const int8_t* W_host, int64_t N, int64_t K, int64_t ldw, spmm_block_t block,
                                 bool to_device, bool reorder, spmm_handle_t** out_handle)
{
    if (!W_host || !out_handle) return SPMM_E_ARG;
    if (N <= 0 || K <= 0 || ldw < K) return SPMM_E_ARG;
    if (block != SPMM_BLOCK_N4K1 && block != SPMM_BLOCK_N1K4) return SPMM_E_ARG;
    if (K > 65536 || N > (int64_t)1 << 24) return SPMM_E_UNSUPPORTED;

    spmm_handle* h = nullptr;
    try {
        h = new spmm_handle();
        spmm::bsr_from_dense(W_host, N, K, ldw, block, h->bsr);
        h->nnz_blocks = (int64_t)h->bsr.index.size();
        if (reorder) {
            spmm::order_rows_by_k_overlap(h->bsr, spmm::SEGMENT_ROWS, h->row_order);
            spmm::Bsr ordered;
            spmm::bsr_permute_rows(h->bsr, h->row_order, ordered);
            spmm::layout_from_bsr(ordered, spmm::SEGMENT_ROWS, h->hl);
        } else {
            spmm::layout_from_bsr(h->bsr, spmm::SEGMENT_ROWS, h->hl);
        }
    } catch (...) {   // bad_alloc, length_error, ...: nothing crosses the C boundary
        delete h;
        return SPMM_E_ALLOC;
    }
    const spmm::HostLayout& hl = h->hl;
    h->kc = hl.kc; h->nseg = hl.nseg; h->ntiles = hl.ntiles; h->nsteps = hl.nsteps;
    h->max_steps_per_tile = hl.max_steps_per_tile;
    h->max_steps_per_segment = hl.max_steps_per_segment;

    if (to_device) {
        hipError_t e = hipGetDevice(&h->device);
        if (e == hipSuccess) {
            int cus = 0;
            if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->device) == hipSuccess && cus > 0)
                h->num_cus = cus;
        }
        if (e == hipSuccess) e = upload(h->d_vals, hl.vals, h->device_bytes);
        if (e == hipSuccess) e = upload(h->d_idx, hl.idx, h->device_bytes);
        if (e == hipSuccess) e = upload(h->d_seg_ptr, hl.seg_ptr, h->device_bytes);
        if (e == hipSuccess) e = upload(h->d_rowsum, hl.rowsum, h->device_bytes);
        if (e != hipSuccess) {
            free_device(h);
            delete h;
            return (e == hipErrorOutOfMemory) ? SPMM_E_ALLOC : SPMM_E_DEVICE;
        }
        h->on_device = true;
    }
    *out_handle = h;
    return SPMM_OK;
}

spmm_status_t spmm_pack(const int8_t* W_host, int64_t N, int64_t K, int64_t ldw, spmm_block_t block,
                        spmm_handle_t** out_handle)
{
    return pack_common(W_host, N, K, ldw, block, true, false, out_handle);
}

spmm_status_t spmm_pack_host(const int8_t* W_host, int64_t N, int64_t K, int64_t ldw, spmm_block_t block,
                             spmm_handle_t** out_handle)
{
    return pack_common(W_host, N, K, ldw, block, false, false, out_handle);
}

spmm_status_t spmm_pack_ex(const int8_t* W_host, int64_t N, int64_t K, int64_t ldw, spmm_block_t block,
                           uint32_t flags, spmm_handle_t** out_handle)
{
    if (flags & ~(uint32_t)(SPMM_PACK_HOST_ONLY | SPMM_PACK_REORDER_ROWS)) return SPMM_E_ARG;
    return pack_common(W_host, N, K, ldw, block, (flags & SPMM_PACK_HOST_ONLY) == 0,
                       (flags & SPMM_PACK_REORDER_ROWS) != 0, out_handle);
}

spmm_status_t spmm_row_order(const spmm_handle_t* h, int32_t* order_host)
{
    if (!h || !order_host) return SPMM_E_ARG;
    for (int64_t i = 0; i < h->bsr.N; ++i) order_host[i] = h->row_order.empty() ? (int32_t)i : h->row_order[(size_t)i];
    return SPMM_OK;
}

spmm_status_t spmm_layout_dims(const spmm_handle_t* h, int32_t* tile_rows, int32_t* step_k,
                               int32_t* segment_rows, int64_t* n_tiles, int64_t* n_segments, int64_t* n_steps)
{
    if (!h) return SPMM_E_ARG;
    if (tile_rows) *tile_rows = spmm::TILE_ROWS;
    if (step_k) *step_k = spmm::STEP_K;
    if (segment_rows) *segment_rows = h->kc;
    if (n_tiles) *n_tiles = h->ntiles;
    if (n_segments) *n_segments = h->nseg;
    if (n_steps) *n_steps = h->nsteps;
    return SPMM_OK;
}

spmm_status_t spmm_layout_export(const spmm_handle_t* h, uint8_t* vals_host, uint32_t* idx_host,
                                 int32_t* seg_ptr_host, int32_t* rowsum_host)
{
    if (!h) return SPMM_E_ARG;
    const spmm::HostLayout& hl = h->hl;
    if (vals_host && !hl.vals.empty()) std::memcpy(vals_host, hl.vals.data(), hl.vals.size());
    if (idx_host && !hl.idx.empty()) std::memcpy(idx_host, hl.idx.data(), hl.idx.size() * sizeof(uint32_t));
    if (seg_ptr_host) std::memcpy(seg_ptr_host, hl.seg_ptr.data(), hl.seg_ptr.size() * sizeof(int32_t));
    if (rowsum_host) std::memcpy(rowsum_host, hl.rowsum.data(), hl.rowsum.size() * sizeof(int32_t));
    return SPMM_OK;
}

spmm_status_t spmm_unpack(const spmm_handle_t* h, int8_t* W_host_out, int64_t ldw)
{
    if (!h || !W_host_out || ldw < h->bsr.K) return SPMM_E_ARG;
    spmm::bsr_to_dense(h->bsr, W_host_out, ldw);
    return SPMM_OK;
}

spmm_status_t spmm_info(const spmm_handle_t* h, int64_t* N, int64_t* K, int64_t* nnz_blocks,
                        int64_t* padded_blocks, int64_t* device_bytes)
{
    if (!h) return SPMM_E_ARG;
    if (N) *N = h->bsr.N;
    if (K) *K = h->bsr.K;
    if (nnz_blocks) *nnz_blocks = h->nnz_blocks;
    // every step multiplies 16 rows x 64 listed k = 256 block slots of 4 elements
    if (padded_blocks) *padded_blocks = h->nsteps * (spmm::TILE_ROWS * spmm::STEP_K / 4);
    if (device_bytes) *device_bytes = h->device_bytes;
    return SPMM_OK;
}

spmm_status_t spmm_plan(const spmm_handle_t* h, int64_t M, spmm_out_t out_type, int32_t* token_tile,
                        int32_t* rows_per_workgroup, int64_t* workgroups)
{
    if (!h || M <= 0) return SPMM_E_ARG;
    const spmm::Plan p = plan_for(h, M, true, (out_type == SPMM_OUT_S32 || out_type == SPMM_OUT_F32) ? 4 : 1);
    if (token_tile) *token_tile = p.token_tile;
    if (rows_per_workgroup) *rows_per_workgroup = p.waves * p.row_tiles_per_wave * spmm::TILE_ROWS;
    if (workgroups) *workgroups = p.workgroups;
    return SPMM_OK;
}

spmm_status_t spmm_set_tuning(spmm_handle_t* h, int32_t token_tile, int32_t variant)
{
    if (!h || token_tile < 0 || variant < 0) return SPMM_E_ARG;
    if (token_tile == 0 && variant != 0) return SPMM_E_ARG;
    if (token_tile != 0 && !spmm::plan_supported(token_tile, variant)) return SPMM_E_UNSUPPORTED;
    h->force_tm = token_tile;
    h->force_r = variant;
    return SPMM_OK;
}

static spmm_status_t run_common(const spmm_handle_t* h, const uint8_t* X_dev, int64_t M, int64_t ldx, bool x_tiled,
                                const spmm_epilogue_t* ep, void* out_dev, int64_t ldo, bool out_tiled, void* hip_stream);

spmm_status_t spmm_run(const spmm_handle_t* h, const uint8_t* X_dev, int64_t M, int64_t ldx,
                       const spmm_epilogue_t* ep, void* out_dev, int64_t ldo, void* hip_stream)
{
    return run_common(h, X_dev, M, ldx, false, ep, out_dev, ldo, false, hip_stream);
}

spmm_status_t spmm_run_tiled(const spmm_handle_t* h, const uint8_t* X_dev, int64_t M, int64_t ldx,
                             const spmm_epilogue_t* ep, void* out_dev, int64_t ldo, uint32_t tiled, void* hip_stream)
{
    if (tiled & ~(uint32_t)(SPMM_TILED_X | SPMM_TILED_OUT)) return SPMM_E_ARG;
    const bool xt = (tiled & SPMM_TILED_X) != 0, ot = (tiled & SPMM_TILED_OUT) != 0;
    // (a tile-major operand has no leading dimension: any value passes the range checks below)
    return run_common(h, X_dev, M, xt ? M : ldx, xt, ep, out_dev, ot ? M : ldo, ot, hip_stream);
}

static spmm_status_t run_common(const spmm_handle_t* h, const uint8_t* X_dev, int64_t M, int64_t ldx, bool x_tiled,
                                const spmm_epilogue_t* ep, void* out_dev, int64_t ldo, bool out_tiled, void* hip_stream)
{
    if (!h || !X_dev || !ep || !out_dev) return SPMM_E_ARG;
    if (!h->on_device) return SPMM_E_ARG;   // packed with spmm_pack_host: nothing to run on
    {   // the handle's buffers live on the device it was packed on
        int dev_now = -1;
        if (hipGetDevice(&dev_now) != hipSuccess || dev_now != h->device) return SPMM_E_ARG;
    }
    if (M <= 0 || ldx < M || ldo < M) return SPMM_E_ARG;
    if (M > (int64_t)1 << 30 || ldx > (int64_t)1 << 40 || ldo > (int64_t)1 << 40) return SPMM_E_UNSUPPORTED;
    const spmm_out_t ot = ep->out_type;
    const spmm_postop_t po = ep->postop;
    if (ot != SPMM_OUT_S32 && ot != SPMM_OUT_F32 && ot != SPMM_OUT_S8 && ot != SPMM_OUT_U8) return SPMM_E_ARG;
    if (po != SPMM_POST_NONE && po != SPMM_POST_GELU && po != SPMM_POST_TABLE) return SPMM_E_ARG;
    if (ep->x_zero_point < 0 || ep->x_zero_point > 255) return SPMM_E_ARG;
    const bool quant = (ot == SPMM_OUT_S8 || ot == SPMM_OUT_U8);
    if (po == SPMM_POST_TABLE && !quant) return SPMM_E_UNSUPPORTED;
    // with a 1-byte output GELU is itself a table look-up: TABLE runs the same kernels
    const bool gelu = (po == SPMM_POST_GELU || po == SPMM_POST_TABLE);
    if (ot != SPMM_OUT_S32) {
        if (!ep->w_scale) return SPMM_E_ARG;
        if (!(ep->x_scale == ep->x_scale)) return SPMM_E_ARG;   // NaN
    }
    if (ep->sum) {
        if (ep->ld_sum < M || ep->ld_sum > (int64_t)1 << 40) return SPMM_E_ARG;
        if (ot == SPMM_OUT_S32 || (quant && gelu)) return SPMM_E_UNSUPPORTED;
    }
    spmm::KernelArgs a;
    std::memset(&a, 0, sizeof(a));
    if (quant && gelu) {
        if (!ep->lut || !(ep->mid_scale > 0.0f)) return SPMM_E_ARG;
        a.inv_mid = 1.0f / ep->mid_scale;
    } else if (quant) {
        if (!(ep->out_scale > 0.0f)) return SPMM_E_ARG;
        const int lo = (ot == SPMM_OUT_U8) ? 0 : -128, hi = (ot == SPMM_OUT_U8) ? 255 : 127;
        if (ep->out_zero_point < lo || ep->out_zero_point > hi) return SPMM_E_ARG;
        a.inv_out = 1.0f / ep->out_scale;
        a.out_zp_f = (float)ep->out_zero_point;
    }

    a.vals = h->d_vals; a.idx = h->d_idx; a.seg_ptr = h->d_seg_ptr; a.rowsum = h->d_rowsum;
    a.X = X_dev; a.out = out_dev;
    a.w_scale = ep->w_scale; a.bias = ep->bias; a.lut = ep->lut;
    a.ldx = ldx; a.ldo = ldo;
    a.N = (int)h->bsr.N; a.K = (int)h->bsr.K; a.M = (int)M;
    a.kc = h->kc; a.nseg = h->nseg; a.ntiles = h->ntiles;
    a.corr_mul = 128 - ep->x_zero_point;
    a.x_scale = ep->x_scale;
    // fast paths use 16-byte accesses and 32-bit offsets
    a.x_vec_ok = aligned(X_dev, 16) && (ldx % 16 == 0) && (h->bsr.K * ldx < ((int64_t)1 << 31));
    if (x_tiled) {
        // token-tile-major activations: [ceil(M / 32)][K][32] bytes, 16-byte aligned
        if (!aligned(X_dev, 16)) return SPMM_E_ARG;
        const int64_t tiles = (M + SPMM_X_TILE - 1) / SPMM_X_TILE;
        if (tiles * h->bsr.K * SPMM_X_TILE >= ((int64_t)1 << 31)) return SPMM_E_UNSUPPORTED;
        a.ldx = SPMM_X_TILE;
        a.x_tile_stride = (int)(h->bsr.K * SPMM_X_TILE);
        a.x_vec_ok = 1;
    }
    const int64_t esz = quant ? 1 : 4;
    a.out_vec_ok = aligned(out_dev, 16) && ((ldo * esz) % 16 == 0) && (h->bsr.N * ldo * esz < ((int64_t)1 << 31));
    if (out_tiled) {
        // token-tile-major 1-byte output: [ceil(M / 32)][N][32] bytes, 16-byte aligned
        if (!quant) return SPMM_E_UNSUPPORTED;
        if (!aligned(out_dev, 16)) return SPMM_E_ARG;
        const int64_t tiles = (M + SPMM_X_TILE - 1) / SPMM_X_TILE;
        if (tiles * h->bsr.N * SPMM_X_TILE >= ((int64_t)1 << 31)) return SPMM_E_UNSUPPORTED;
        a.ldo = SPMM_X_TILE;
        a.out_tile_stride = (int)(h->bsr.N * SPMM_X_TILE);
        a.out_vec_ok = 1;
    }
    if (ep->sum) {
        a.sum = ep->sum;
        a.ld_sum = ep->ld_sum;
        a.out_vec_ok = a.out_vec_ok && aligned(ep->sum, 16) && (ep->ld_sum % 4 == 0) &&
                       (h->bsr.N * ep->ld_sum * 4 < ((int64_t)1 << 31));
    }

    if (a.out_vec_ok) {
        // extent of the output (the fast paths store through a buffer resource of this size: the
        // hardware drops a store that would leave it)
        const int64_t tiles = (M + SPMM_X_TILE - 1) / SPMM_X_TILE;
        const int64_t extent = out_tiled ? tiles * h->bsr.N * SPMM_X_TILE : ((h->bsr.N - 1) * ldo + M) * esz;
        a.out_bytes = (uint32_t)extent;
    }

    const spmm::Plan p = plan_for(h, M, a.x_vec_ok && a.out_vec_ok, (int)esz);
    const int rc = spmm::launch_spmm(p, a, ot, (gelu ? SPMM_POST_GELU : SPMM_POST_NONE) | (ep->sum ? spmm::POST_SUM_BIT : 0),
                                     hip_stream);
    return rc == 0 ? SPMM_OK : SPMM_E_DEVICE;
}

spmm_status_t spmm_make_gelu_lut(float mid_scale, float out_scale, int32_t out_zero_point,
                                 spmm_out_t out_type, int8_t lut_host[256])
{
    if (!lut_host || !(mid_scale > 0.0f) || !(out_scale > 0.0f)) return SPMM_E_ARG;
    if (out_type != SPMM_OUT_S8 && out_type != SPMM_OUT_U8) return SPMM_E_ARG;
    const double lo = (out_type == SPMM_OUT_U8) ? 0.0 : -128.0;
    const double hi = (out_type == SPMM_OUT_U8) ? 255.0 : 127.0;
    if (out_zero_point < (int)lo || out_zero_point > (int)hi) return SPMM_E_ARG;
    for (int key = -128; key <= 127; ++key) {
        const double x = (double)key * (double)mid_scale;            // dequantised pre-activation
        const double gelu = 0.5 * x * std::erfc(-x / std::sqrt(2.0));  // x * Phi(x)
        double q = std::nearbyint(gelu / (double)out_scale) + (double)out_zero_point;
        q = std::fmin(hi, std::fmax(lo, q));
        lut_host[key + 128] = (int8_t)(uint8_t)((int)q & 0xff);
    }
    return SPMM_OK;
}

const char* spmm_kernel_name(void) { return "spmm_rowtile_mfma"; }

spmm_status_t spmm_kernel_variant(const spmm_handle_t* h, int64_t M, spmm_out_t out_type, spmm_postop_t postop,
                                  char* buf, int64_t buflen)
{
    return spmm_kernel_variant_tiled(h, M, out_type, postop, 0, buf, buflen);
}

spmm_status_t spmm_kernel_variant_tiled(const spmm_handle_t* h, int64_t M, spmm_out_t out_type, spmm_postop_t postop,
                                        uint32_t tiled, char* buf, int64_t buflen)
{
    if (!h || M <= 0 || !buf || buflen <= 0) return SPMM_E_ARG;
    if (tiled & ~(uint32_t)(SPMM_TILED_X | SPMM_TILED_OUT)) return SPMM_E_ARG;
    const bool quant_out = (out_type == SPMM_OUT_S8 || out_type == SPMM_OUT_U8);
    if ((tiled & SPMM_TILED_OUT) && !quant_out) return SPMM_E_UNSUPPORTED;
    if (out_type < SPMM_OUT_S32 || out_type > SPMM_OUT_U8) return SPMM_E_ARG;
    if (postop != SPMM_POST_NONE && postop != SPMM_POST_GELU && postop != SPMM_POST_TABLE) return SPMM_E_ARG;
    if (postop == SPMM_POST_TABLE) postop = SPMM_POST_GELU;   // same kernels
    const spmm::Plan p = plan_for(h, M, true, (out_type == SPMM_OUT_S32 || out_type == SPMM_OUT_F32) ? 4 : 1);
    const int post = (out_type == SPMM_OUT_S32) ? 0 : (int)postop;   // S32 output ignores the post-operator
    if (p.stream)
        std::snprintf(buf, (size_t)buflen, "void spmm::spmm_rowtile_mfma_stream<%d, %d, %d, %d>(spmm::KernelArgs)",
                      p.token_tile, p.waves, (int)out_type, post);
    else if (p.slab)
        std::snprintf(buf, (size_t)buflen, "void spmm::spmm_rowtile_mfma_slab<%d, %d, %d, %d>(spmm::KernelArgs)",
                      p.token_tile, p.waves, (int)out_type, post);
    else if (p.simple)
        std::snprintf(buf, (size_t)buflen, "void spmm::spmm_rowtile_mfma_simple<%d, %d, %d, %d, %d>(spmm::KernelArgs)",
                      p.token_tile, p.waves, p.row_tiles_per_wave, (int)out_type, post);
    else if (p.loaders)
        std::snprintf(buf, (size_t)buflen, "void spmm::spmm_rowtile_mfma_fed<%d, %d, %d, %d, %d, %d>(spmm::KernelArgs)",
                      p.token_tile, p.waves, p.loaders, p.max_steps, (int)out_type, post);
    else
        // (8-wave configurations run 5-step weights with the 6-step instantiation)
        // (last parameter: the layout instantiation, bit 0 activations, bit 1 outputs tile-major)
        std::snprintf(buf, (size_t)buflen, "void spmm::spmm_rowtile_mfma<%d, %d, %d, %d, %d, %d>(spmm::KernelArgs)",
                      p.token_tile, p.waves, (p.waves == 8 && p.max_steps == 5) ? 6 : p.max_steps, (int)out_type, post,
                      (int)tiled);
    return SPMM_OK;
}

void spmm_destroy(spmm_handle_t* h)
{
    if (!h) return;
    free_device(h);
    delete h;
}

const char* spmm_status_string(spmm_status_t s)
{
    switch (s) {
    case SPMM_OK: return "ok";
    case SPMM_E_ARG: return "invalid argument";
    case SPMM_E_UNSUPPORTED: return "unsupported size or configuration";
    case SPMM_E_ALLOC: return "allocation failed";
    case SPMM_E_DEVICE: return "device error";
    }
    return "unknown status";
}

}  // extern "C"
