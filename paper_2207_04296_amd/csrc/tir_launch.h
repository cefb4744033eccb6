// Launcher declarations shared by the instantiation units and the dispatcher.
#pragma once
#include <hip/hip_runtime.h>
#include "tir_params.h"

namespace tir {

// Defined (explicitly instantiated) in tir_inst.hip for every line of tir_variants.def.
template <class C> hipError_t launch_cfg(const Params& p, hipStream_t stream);

typedef hipError_t (*launch_fn)(const Params&, hipStream_t);

struct Variant {
    const char* name;
    int dt, out, bm, bn, wm, wn, amode, bmode, rowb, nstage, kw, cw;
    launch_fn fn;
};

}  // namespace tir
