// One kernel configuration of the SpMM kernels: this file is compiled once per configuration
// (see build.py), so that the instantiations build in parallel.
//   pipelined kernel : -DSPMM_CFG_TM=<128|96> -DSPMM_CFG_NW=<16|8> -DSPMM_CFG_MAXS=<4|5|6|8>
//   simple kernel    : -DSPMM_CFG_SIMPLE=<1|2>      (row tiles per wave; token tile 64)
//                      -DSPMM_CFG_SIMPLE=1 -DSPMM_CFG_SIMPLE_TM=<32|16>
//   short-batch kernel: -DSPMM_CFG_SLAB=<16|32>      (token tile)
//   streamed kernel  : -DSPMM_CFG_STREAM=<64|32|16>  (token tile)
//   loader-fed pipelined kernel: -DSPMM_CFG_FED_TM=<128|96> -DSPMM_CFG_NW=<12|8> -DSPMM_CFG_MAXS=<4|6|8>
// Each defines one function launch_cfg_<...>() that picks the epilogue instantiation and
// launches it; spmm_plan.hip calls them.
#include "spmm_kernels.h"

namespace spmm {

// postop: SPMM_POST_NONE / SPMM_POST_GELU, plus POST_SUM_BIT (combinations the host has
// checked: no Sum with S32 output or with the table chain)
template <class L>
static void dispatch_epilogue(spmm_out_t out_type, int postop, dim3 grid, dim3 block, hipStream_t st,
                              const KernelArgs& a)
{
    const bool gelu = (postop & SPMM_POST_GELU) != 0, sum = (postop & POST_SUM_BIT) != 0;
    constexpr int NONE = SPMM_POST_NONE, GELU = SPMM_POST_GELU, SUM = POST_SUM_BIT;
    switch (out_type) {
    case SPMM_OUT_S32: L::template go<SPMM_OUT_S32, NONE>(grid, block, st, a); break;
    case SPMM_OUT_F32:
        if (gelu && sum) L::template go<SPMM_OUT_F32, GELU | SUM>(grid, block, st, a);
        else if (gelu) L::template go<SPMM_OUT_F32, GELU>(grid, block, st, a);
        else if (sum) L::template go<SPMM_OUT_F32, NONE | SUM>(grid, block, st, a);
        else L::template go<SPMM_OUT_F32, NONE>(grid, block, st, a);
        break;
    case SPMM_OUT_S8:
        if (gelu) L::template go<SPMM_OUT_S8, GELU>(grid, block, st, a);
        else if (sum) L::template go<SPMM_OUT_S8, NONE | SUM>(grid, block, st, a);
        else L::template go<SPMM_OUT_S8, NONE>(grid, block, st, a);
        break;
    case SPMM_OUT_U8:
        if (gelu) L::template go<SPMM_OUT_U8, GELU>(grid, block, st, a);
        else if (sum) L::template go<SPMM_OUT_U8, NONE | SUM>(grid, block, st, a);
        else L::template go<SPMM_OUT_U8, NONE>(grid, block, st, a);
        break;
    }
}

#define SPMM_CAT_(a, b) a##b
#define SPMM_CAT(a, b) SPMM_CAT_(a, b)

// The launcher structs below have the same name in every configuration's object file but launch
// different instantiations: internal linkage keeps the linker from folding their member functions
// into one (which would launch the wrong kernel for every configuration but the one it kept).

#if defined(SPMM_CFG_FED_TM)
namespace {
template <int TM, int NW, int MAXS>
struct FedLaunch {
    template <int OUT, int POST>
    static void go(dim3 grid, dim3 block, hipStream_t st, const KernelArgs& a)
    {
        hipLaunchKernelGGL((spmm_rowtile_mfma_fed<TM, NW, 4, MAXS, OUT, POST>), grid, block, 0, st, a);
    }
};
}  // namespace

void SPMM_CAT(SPMM_CAT(SPMM_CAT(SPMM_CAT(SPMM_CAT(launch_cfg_fed_, SPMM_CFG_FED_TM), _), SPMM_CFG_NW), _), SPMM_CFG_MAXS)(
    spmm_out_t out_type, int postop, unsigned grid_x, unsigned grid_y, unsigned block, void* stream, const KernelArgs& a)
{
    dispatch_epilogue<FedLaunch<SPMM_CFG_FED_TM, SPMM_CFG_NW, SPMM_CFG_MAXS>>(out_type, postop, dim3(grid_x, grid_y),
                                                                               dim3(block), (hipStream_t)stream, a);
}
#elif defined(SPMM_CFG_STREAM)
namespace {
struct StreamLaunch {
    template <int OUT, int POST>
    static void go(dim3 grid, dim3 block, hipStream_t st, const KernelArgs& a)
    {
        hipLaunchKernelGGL((spmm_rowtile_mfma_stream<SPMM_CFG_STREAM, 8, OUT, POST>), grid, block, 0, st, a);
    }
};
}  // namespace

void SPMM_CAT(launch_cfg_stream, SPMM_CFG_STREAM)(spmm_out_t out_type, int postop, unsigned grid_x, unsigned grid_y,
                                                  unsigned block, void* stream, const KernelArgs& a)
{
    dispatch_epilogue<StreamLaunch>(out_type, postop, dim3(grid_x, grid_y), dim3(block), (hipStream_t)stream, a);
}
#elif defined(SPMM_CFG_SLAB)
namespace {
struct SlabLaunch {
    template <int OUT, int POST>
    static void go(dim3 grid, dim3 block, hipStream_t st, const KernelArgs& a)
    {
        hipLaunchKernelGGL((spmm_rowtile_mfma_slab<SPMM_CFG_SLAB, 8, OUT, POST>), grid, block, 0, st, a);
    }
};
}  // namespace

void SPMM_CAT(launch_cfg_slab, SPMM_CFG_SLAB)(spmm_out_t out_type, int postop, unsigned grid_x, unsigned grid_y, unsigned block, void* stream,
                     const KernelArgs& a)
{
    dispatch_epilogue<SlabLaunch>(out_type, postop, dim3(grid_x, grid_y), dim3(block), (hipStream_t)stream, a);
}
#elif defined(SPMM_CFG_SIMPLE)
#ifdef SPMM_CFG_SIMPLE_TM
#define SPMM_SIMPLE_NAME SPMM_CAT(SPMM_CAT(launch_cfg_simple, SPMM_CFG_SIMPLE_TM), _)
#else
#define SPMM_CFG_SIMPLE_TM 64
#define SPMM_SIMPLE_NAME launch_cfg_simple_
#endif

namespace {
template <int R>
struct SimpleLaunch {
    template <int OUT, int POST>
    static void go(dim3 grid, dim3 block, hipStream_t st, const KernelArgs& a)
    {
        hipLaunchKernelGGL((spmm_rowtile_mfma_simple<SPMM_CFG_SIMPLE_TM, 8, R, OUT, POST>), grid, block, 0, st, a);
    }
};
}  // namespace

void SPMM_CAT(SPMM_SIMPLE_NAME, SPMM_CFG_SIMPLE)(spmm_out_t out_type, int postop, unsigned grid_x,
                                                   unsigned grid_y, unsigned block, void* stream,
                                                   const KernelArgs& a)
{
    dispatch_epilogue<SimpleLaunch<SPMM_CFG_SIMPLE>>(out_type, postop, dim3(grid_x, grid_y), dim3(block),
                                                     (hipStream_t)stream, a);
}
#else
namespace {
template <int TM, int NW, int MAXS>
struct PipeLaunch {
    template <int OUT, int POST>
    static void go(dim3 grid, dim3 block, hipStream_t st, const KernelArgs& a)
    {
        // one instantiation per layout of the activations and of 1-byte outputs (row-major / token-tile-major):
        // the 16-wave forms have no register to spare for a choice at run time
        const int layout = (a.x_tile_stride ? 1 : 0) | (a.out_tile_stride ? 2 : 0);
        if constexpr (OUT == SPMM_OUT_S8 || OUT == SPMM_OUT_U8) {
            if (layout == 3) { hipLaunchKernelGGL((spmm_rowtile_mfma<TM, NW, MAXS, OUT, POST, 3>), grid, block, 0, st, a); return; }
            if (layout == 2) { hipLaunchKernelGGL((spmm_rowtile_mfma<TM, NW, MAXS, OUT, POST, 2>), grid, block, 0, st, a); return; }
        }
        if (layout & 1) hipLaunchKernelGGL((spmm_rowtile_mfma<TM, NW, MAXS, OUT, POST, 1>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((spmm_rowtile_mfma<TM, NW, MAXS, OUT, POST, 0>), grid, block, 0, st, a);
    }
};
}  // namespace

void SPMM_CAT(SPMM_CAT(SPMM_CAT(SPMM_CAT(SPMM_CAT(launch_cfg_, SPMM_CFG_TM), _), SPMM_CFG_NW), _), SPMM_CFG_MAXS)(
    spmm_out_t out_type, int postop, unsigned grid_x, unsigned grid_y, unsigned block, void* stream, const KernelArgs& a)
{
    dispatch_epilogue<PipeLaunch<SPMM_CFG_TM, SPMM_CFG_NW, SPMM_CFG_MAXS>>(out_type, postop, dim3(grid_x, grid_y),
                                                                            dim3(block), (hipStream_t)stream, a);
}
#endif

}  // namespace spmm
