// naut_attn_inst.hip -- the kernel instantiations of one (input type, output type) pair.
//
// Compiled once per pair with -DNAUT_INST_IN=<naut_dtype> -DNAUT_INST_OUT=<naut_dtype> (bf16/bf16,
// bf16/f32, f16/f16, f16/f32), so that the pairs build in parallel; naut_attn.hip declares these
// launchers extern and holds none of the kernels.
#include "naut_attn_kernels.h"

#if !defined(NAUT_INST_IN) || !defined(NAUT_INST_OUT)  // a bare compile of this file gives the bf16 -> bf16 pair
#undef NAUT_INST_IN
#undef NAUT_INST_OUT
#define NAUT_INST_IN NAUT_BF16
#define NAUT_INST_OUT NAUT_BF16
#endif

namespace naut_k {

template int launch<64, NAUT_INST_IN, NAUT_INST_OUT>(const Params&, int, hipStream_t);
template int launch<128, NAUT_INST_IN, NAUT_INST_OUT>(const Params&, int, hipStream_t);
template int launch<256, NAUT_INST_IN, NAUT_INST_OUT>(const Params&, int, hipStream_t);

}  // namespace naut_k
