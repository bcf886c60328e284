// Large-tile kernel, results that leave as codes for the next quantized layer: instantiations for the hardware
// activation format (E4M3-class codes) with 8-bit and 4-bit hardware weight formats, both accumulate modes.  Other
// operand pairings with codes out take the register-staged kernels.
#include "gemm_dma_kernel.h"

namespace fpq {

template <int XKIND, int WKIND, int ACC>
static int launch_dma_q_shape(const GemmArgs& a, hipStream_t st)
{
    if (a.tile == TILE_128x160_S2)
        return a.conv_out ? launch_dma_one<128, 160, 2, XKIND, WKIND, ACC, true, true>(a, st)
                          : launch_dma_one<128, 160, 2, XKIND, WKIND, ACC, false, true>(a, st);
    return a.conv_out ? launch_dma_one<256, 160, 3, XKIND, WKIND, ACC, true, true>(a, st)
                      : launch_dma_one<256, 160, 3, XKIND, WKIND, ACC, false, true>(a, st);
}

int launch_gemm_dma_q(const GemmArgs& a, hipStream_t st)
{
    if (a.xkind != OPK_FP8 || !a.yq) return FPQ_ERR_UNSUPPORTED;
    if (a.acc_mode == FPQ_ACC_FP8_MFMA) {
        if (a.wkind == OPK_FP8) return launch_dma_q_shape<OPK_FP8, OPK_FP8, FPQ_ACC_FP8_MFMA>(a, st);
        if (a.wkind == OPK_FP4) return launch_dma_q_shape<OPK_FP8, OPK_FP4, FPQ_ACC_FP8_MFMA>(a, st);
        return FPQ_ERR_UNSUPPORTED;
    }
    if (a.wkind == OPK_FP8) return launch_dma_q_shape<OPK_FP8, OPK_FP8, FPQ_ACC_FP32>(a, st);
    if (a.wkind == OPK_FP4) return launch_dma_q_shape<OPK_FP8, OPK_FP4, FPQ_ACC_FP32>(a, st);
    return FPQ_ERR_UNSUPPORTED;
}

}  // namespace fpq
