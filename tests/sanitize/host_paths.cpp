// Host-only driver run under AddressSanitizer + UndefinedBehaviorSanitizer by tests/test_sanitizers.py:
// the packer (dense -> 4x1 BSR -> device layout -> dense) and the CPU oracle on shapes chosen to
// hit the edges (N not a multiple of 4 or 16, K not a multiple of 4, 64 or 512, empty block-rows,
// dense rows, both block orientations, value -128).  Exit status 0 = every round trip exact and no
// sanitizer report (a report aborts the process).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "spmm_internal.h"

extern "C" {
void oracle_acc_s32(const int8_t* W, int64_t ldw, const uint8_t* X, int64_t ldx, int64_t N, int64_t K, int64_t M,
                    int32_t x_zp, int32_t* acc);
int oracle_gelu_lut(float mid_scale, float out_scale, int32_t out_zp, int out_type, int8_t* lut);
int oracle_epilogue_sum(const int32_t* acc, int64_t N, int64_t M, const float* w_scale, float x_scale, const float* bias,
                        int postop, const float* sum, int64_t ld_sum, int out_type, float out_scale, int32_t out_zp,
                        float mid_scale, const int8_t* lut, void* out, int64_t ldo);
}

static uint32_t rng_state = 12345u;
static uint32_t rnd() { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }

static int round_trip(int64_t N, int64_t K, int pct_dense, spmm_block_t block)
{
    const int64_t ldw = K + (rnd() % 3);
    std::vector<int8_t> W((size_t)(N * ldw), 0);
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            if ((int)(rnd() % 100) < pct_dense) W[(size_t)(n * ldw + k)] = (int8_t)((int)(rnd() % 256) - 128);
    if (N > 20)   // an empty stretch of rows and a fully dense row
        for (int64_t k = 0; k < K; ++k) { W[(size_t)(17 * ldw + k)] = 0; W[(size_t)(18 * ldw + k)] = 0; W[(size_t)(19 * ldw + k)] = -128; }
    spmm::Bsr b;
    spmm::bsr_from_dense(W.data(), N, K, ldw, block, b);
    spmm::HostLayout hl;
    spmm::layout_from_bsr(b, spmm::SEGMENT_ROWS, hl);
    if ((int64_t)hl.vals.size() != hl.nsteps * spmm::STEP_VAL_BYTES) return 1;
    if ((int64_t)hl.idx.size() != hl.nsteps * spmm::STEP_IDX_DWORDS) return 2;
    if (hl.seg_ptr.empty() || hl.seg_ptr.back() != hl.nsteps) return 3;
    std::vector<int8_t> back((size_t)(N * ldw), 0x55);
    spmm::bsr_to_dense(b, back.data(), ldw);
    for (int64_t n = 0; n < N; ++n)
        if (std::memcmp(&back[(size_t)(n * ldw)], &W[(size_t)(n * ldw)], (size_t)K) != 0) return 4;
    // every listed index names a row of its segment
    for (int t = 0; t < hl.ntiles; ++t)
        for (int sg = 0; sg < hl.nseg; ++sg) {
            const int64_t rows = std::min<int64_t>(hl.kc, K - (int64_t)sg * hl.kc);
            for (int s = hl.seg_ptr[(size_t)(t * hl.nseg + sg)]; s < hl.seg_ptr[(size_t)(t * hl.nseg + sg + 1)]; ++s)
                for (int i = 0; i < spmm::STEP_IDX_DWORDS; ++i) {
                    const uint32_t v = hl.idx[(size_t)s * spmm::STEP_IDX_DWORDS + i];
                    if ((int64_t)(v & 0xffffu) >= rows || (int64_t)(v >> 16) >= rows) return 5;
                }
        }
    return 0;
}

static int oracle_paths()
{
    const int64_t N = 7, K = 13, M = 5;
    std::vector<int8_t> W((size_t)(N * K));
    std::vector<uint8_t> X((size_t)(K * M));
    for (auto& w : W) w = (int8_t)((int)(rnd() % 256) - 128);
    for (auto& x : X) x = (uint8_t)(rnd() % 256);
    std::vector<int32_t> acc((size_t)(N * M));
    oracle_acc_s32(W.data(), K, X.data(), M, N, K, M, 3, acc.data());
    std::vector<float> ws((size_t)N, 0.01f), bias((size_t)N, -0.5f), sum((size_t)(N * M), 0.25f);
    int8_t lut[256];
    if (oracle_gelu_lut(0.05f, 0.04f, 0, 2, lut) != 0) return 10;
    std::vector<float> of((size_t)(N * M));
    std::vector<int8_t> o8((size_t)(N * M));
    for (int post = 0; post < 2; ++post) {
        if (oracle_epilogue_sum(acc.data(), N, M, ws.data(), 0.02f, bias.data(), post, sum.data(), M, 1, 1.0f, 0, 1.0f, nullptr, of.data(), M)) return 11;
        if (oracle_epilogue_sum(acc.data(), N, M, ws.data(), 0.02f, nullptr, post, nullptr, 0, 2, 0.04f, 0, 0.05f, lut, o8.data(), M)) return 12;
    }
    return 0;
}

int main()
{
    const int64_t shapes[][2] = {{1, 1}, {3, 5}, {4, 4}, {17, 33}, {50, 70}, {130, 1025}, {16, 2049}, {260, 100}, {5, 3000}, {64, 512}, {33, 640}};
    for (const auto& sh : shapes)
        for (int dense : {0, 3, 10, 35, 100})
            for (spmm_block_t bl : {SPMM_BLOCK_N4K1, SPMM_BLOCK_N1K4}) {
                const int rc = round_trip(sh[0], sh[1], dense, bl);
                if (rc) { std::fprintf(stderr, "round trip failed: N %lld K %lld dense %d block %d rc %d\n", (long long)sh[0], (long long)sh[1], dense, (int)bl, rc); return 1; }
            }
    const int rc = oracle_paths();
    if (rc) { std::fprintf(stderr, "oracle path failed: %d\n", rc); return 1; }
    std::puts("ok");
    return 0;
}
