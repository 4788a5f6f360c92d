// One ping-pong tile shape of the LDS-tiled matrix-core kernel (gemm_tile.h), selected by ECLIP_PP_ID at compile time:
// both 16-bit types and the three addressing forms.  One translation unit per shape keeps the build parallel; the
// build script compiles this file once for every id listed in ECLIP_PP_TILES.
#include "gemm_tile.h"

#ifndef ECLIP_PP_ID
#error "compile with -DECLIP_PP_ID=<variant id>"
#endif

namespace eclip {

namespace {

constexpr PPTile kTile = pp_tile(ECLIP_PP_ID);
static_assert(kTile.id == ECLIP_PP_ID, "ECLIP_PP_ID is not in ECLIP_PP_TILES");

template <typename T, int AMODE>
hipError_t launch_one(const GemmDev &d, dim3 grid, hipStream_t s)
{
    hipLaunchKernelGGL((conv_gemm_kernel<T, kTile.bm, kTile.bn, kTile.bk, 2, 4, kTile.rs, kTile.loop, AMODE>), grid, dim3(512),
                       lds_bytes(kTile.bm, kTile.bn, kTile.bk, 16, kTile.loop != LOOP_PP_BDIRECT), s, d);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_mode(const GemmDev &d, dim3 grid, hipStream_t s)
{
    switch (gemm_amode(d, kTile.bk)) {
    case A_MATRIX: return launch_one<T, A_MATRIX>(d, grid, s);
    case A_UNIFORM: return launch_one<T, A_UNIFORM>(d, grid, s);
    default: return launch_one<T, A_GENERAL>(d, grid, s);
    }
}

template <typename T, int AMODE>
hipError_t init_one()
{
    return hipFuncSetAttribute((const void *)conv_gemm_kernel<T, kTile.bm, kTile.bn, kTile.bk, 2, 4, kTile.rs, kTile.loop, AMODE>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes(kTile.bm, kTile.bn, kTile.bk, 16, kTile.loop != LOOP_PP_BDIRECT));
}

}  // namespace

template <> hipError_t launch_pp<ECLIP_PP_ID>(const GemmDev &d, int dtype, dim3 grid, hipStream_t s)
{
    return dtype == DT_BF16 ? launch_mode<bf16_t>(d, grid, s) : launch_mode<f16_t>(d, grid, s);
}

template <> hipError_t init_pp<ECLIP_PP_ID>()
{
    hipError_t e;
    if ((e = init_one<bf16_t, A_GENERAL>()) != hipSuccess || (e = init_one<bf16_t, A_UNIFORM>()) != hipSuccess ||
        (e = init_one<bf16_t, A_MATRIX>()) != hipSuccess || (e = init_one<f16_t, A_GENERAL>()) != hipSuccess ||
        (e = init_one<f16_t, A_UNIFORM>()) != hipSuccess || (e = init_one<f16_t, A_MATRIX>()) != hipSuccess)
        return e;
    return hipSuccess;
}

}  // namespace eclip
