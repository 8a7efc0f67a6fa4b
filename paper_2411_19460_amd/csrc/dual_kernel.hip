// Launchers of the dual-form passes (see dual_body.h) as kernels of their own.
#include "dual_body.h"

namespace ssdk {
namespace {

using namespace dualk;

template <int Q, int EPI>
__global__ __launch_bounds__(DualCfg<Q>::NTHR) void mk_dual(SegParams sp) {
    __shared__ __attribute__((aligned(16))) DualLds<Q> L;
    dual_body<Q, EPI>(sp, L, blockIdx.x, gridDim.x);
}

template <int Q, int EPI>
hipError_t launch_dual_q(const SegParams& sp0, int kid, hipStream_t st) {
    SegParams sp = sp0;
    // as few head slices as still give every compute unit a workgroup: the persistent operands are then
    // shared by as many heads as possible
    sp.dual_split = pick_split(sp.hpg, (int64_t)sp.Bt * sp.nc * sp.G, sp.wg_target);
    SSDK_LAUNCH(kid, st, (mk_dual<Q, EPI>), dim3(sp.Bt * sp.nc * sp.G * sp.dual_split), dim3(DualCfg<Q>::NTHR), sp);
    return hipSuccess;
}

template <int EPI>
hipError_t launch_dual_epi(const SegParams& sp, int kid, hipStream_t st) {
    switch (sp.Q) {
        case 64: return launch_dual_q<64, EPI>(sp, kid, st);
        case 128: return launch_dual_q<128, EPI>(sp, kid, st);
        case 256: return launch_dual_q<256, EPI>(sp, kid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t mfma_launch_dual(const SegParams& sp, int epi, hipStream_t st) {
    switch (epi) {
        case 0: return launch_dual_epi<0>(sp, K_MFMA_CHUNK_OUT, st);
        case 2: return launch_dual_epi<2>(sp, K_MFMA_BWD_MAIN, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ssdk
