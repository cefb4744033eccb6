// Instantiations of the kernels outside the tile-variant table (fused attention, depth-wise
// convolution) and the tables the dispatcher picks from.
#include "tir_attention.h"
#include "tir_depthwise.h"

namespace tir {

template <int DT, int OUT, int DH> static hipError_t launch_attn(const AttnParams& p, hipStream_t stream) {
    hipLaunchKernelGGL((attention_kernel<DT, OUT, DH>), dim3((unsigned)(p.batch * p.tiles_m)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

attn_launch_fn attention_launcher(int dt, int out, int dh) {
#define TIR_ATTN(DT, OUT, DH) \
    if (dt == DT && out == OUT && dh == DH) return &launch_attn<DT, OUT, DH>;
    TIR_ATTN(DT_F16, DT_F16, 64) TIR_ATTN(DT_F16, DT_F32, 64) TIR_ATTN(DT_F16, DT_F16, 128) TIR_ATTN(DT_F16, DT_F32, 128)
    TIR_ATTN(DT_BF16, DT_BF16, 64) TIR_ATTN(DT_BF16, DT_F32, 64) TIR_ATTN(DT_BF16, DT_BF16, 128) TIR_ATTN(DT_BF16, DT_F32, 128)
#undef TIR_ATTN
    return nullptr;
}

template <int DT, int OUT, bool STREAM> static void launch_dw_as(const Params& p, hipStream_t stream) {
    constexpr int VEC = 16 / elem_size(DT);
    constexpr int PP = 256 / (kDwChannels / VEC);
    dim3 grid((unsigned)((p.M + kDwPixPerThread * PP - 1) / (kDwPixPerThread * PP)), (unsigned)((p.Cin + kDwChannels - 1) / kDwChannels));
    if (p.R == 3 && p.S == 3 && p.dil_w == 1 && (p.stride_w == 1 || p.stride_w == 2) && p.Q >= kDwBlockPix) {
        // four adjacent pixels per thread
        const long long groups = (long long)p.batch_imgs * p.P * ((p.Q + kDwBlockPix - 1) / kDwBlockPix);
        grid.x = (unsigned)((groups + PP - 1) / PP);
        if (p.stride_w == 1) hipLaunchKernelGGL((depthwise3x3_blocked_kernel<DT, OUT, 1, STREAM>), grid, dim3(256), 0, stream, p);
        else hipLaunchKernelGGL((depthwise3x3_blocked_kernel<DT, OUT, 2, STREAM>), grid, dim3(256), 0, stream, p);
    } else if (p.R == 3 && p.S == 3) hipLaunchKernelGGL((depthwise_kernel<DT, OUT, true, STREAM>), grid, dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((depthwise_kernel<DT, OUT, false, STREAM>), grid, dim3(256), 0, stream, p);
}

template <int DT, int OUT> static hipError_t launch_dw(const Params& p, hipStream_t stream) {
    if (p.store_nt) launch_dw_as<DT, OUT, true>(p, stream);
    else launch_dw_as<DT, OUT, false>(p, stream);
    return hipGetLastError();
}

dw_launch_fn depthwise_launcher(int dt, int out) {
#define TIR_DW(DT, OUT) \
    if (dt == DT && out == OUT) return &launch_dw<DT, OUT>;
    TIR_DW(DT_F16, DT_F16) TIR_DW(DT_F16, DT_F32) TIR_DW(DT_BF16, DT_BF16) TIR_DW(DT_BF16, DT_F32) TIR_DW(DT_I8, DT_I32) TIR_DW(DT_I8, DT_I8)
#undef TIR_DW
    return nullptr;
}

}  // namespace tir
