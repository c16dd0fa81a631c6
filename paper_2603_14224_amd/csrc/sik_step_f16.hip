// The one-launch decode step for f16 K, V and q: instantiates the kernel of sik_step_kernel.h.
#define SIK_STEP_TL_SETTER sik_dbg_tl_step_f16
#include "sik_step_kernel.h"

namespace sik {

hipError_t launch_step_f16(const Dims& d, int T, int nchunk, size_t dyn, const void* q, const float* codebook,
                            const uint8_t* codes, int32_t* seq_len, const void* K, const void* V, const StepArgs& a,
                            bool out_f32, hipStream_t s) {
    return out_f32 ? launch_step_t<kF16, kF32>(d, T, nchunk, dyn, q, codebook, codes, seq_len, K, V, a, s)
                   : launch_step_t<kF16, kF16>(d, T, nchunk, dyn, q, codebook, codes, seq_len, K, V, a, s);
}

}  // namespace sik
