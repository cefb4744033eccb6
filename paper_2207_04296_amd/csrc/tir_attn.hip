// Instantiations of the fused attention kernel and the table the dispatcher picks from.
#include "tir_attention.h"

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

}  // namespace tir
