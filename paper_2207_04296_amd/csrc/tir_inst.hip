// One translation unit of kernel instantiations; compiled once per TIR_UNIT value so the units
// build in parallel.  Each line of tir_variants.def owned by this unit becomes an explicit
// instantiation of launch_cfg<Cfg<...>>, which the dispatcher references by address.
#include "tir_kernel.h"
#include "tir_launch.h"

#ifndef TIR_UNIT
#error "compile with -DTIR_UNIT=<n>"
#endif

namespace tir {

template <class C> hipError_t launch_cfg(const Params& p, hipStream_t stream) {
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)p.batch, 1);
    if constexpr (C::AMODE == A_CONV_PATCH) {
        grid.x = (unsigned)(p.batch_imgs * p.tiles_m * p.tiles_n);
        hipLaunchKernelGGL((conv_patch_kernel<C::DT, C::OUT>), grid, dim3(512), 0, stream, p);
    } else if constexpr (C::AMODE == A_GENERIC || C::AMODE == A_CONV_GENERIC)
        hipLaunchKernelGGL(contract_staged_kernel<C>, grid, dim3(C::THREADS), 0, stream, p);
    else {
        grid.z = (unsigned)p.ksplit;
        hipLaunchKernelGGL(contract_direct_kernel<C>, grid, dim3(C::THREADS), 0, stream, p);
    }
    return hipGetLastError();
}

#define TIR_DEFINE(name, DT, OUT, BM, BN, WM, WN, AM, BMO, RB, NS, KW, CW) \
    template hipError_t launch_cfg<Cfg<DT, OUT, BM, BN, WM, WN, AM, BMO, RB, NS, KW, CW>>(const Params&, hipStream_t);
#define TIR_SKIP(...)

#if TIR_UNIT == 0
#define V0 TIR_DEFINE
#else
#define V0 TIR_SKIP
#endif
#if TIR_UNIT == 1
#define V1 TIR_DEFINE
#else
#define V1 TIR_SKIP
#endif
#if TIR_UNIT == 2
#define V2 TIR_DEFINE
#else
#define V2 TIR_SKIP
#endif
#if TIR_UNIT == 3
#define V3 TIR_DEFINE
#else
#define V3 TIR_SKIP
#endif
#if TIR_UNIT == 4
#define V4 TIR_DEFINE
#else
#define V4 TIR_SKIP
#endif
#if TIR_UNIT == 5
#define V5 TIR_DEFINE
#else
#define V5 TIR_SKIP
#endif
#include "tir_variants.def"

}  // namespace tir
