// attn_vsa_pp_kernel (Alg. 2 on the ping-pong structure) in a translation unit of its own, because it is compiled with
// one code-generation option more than the rest of the library (build.py: VSA_EXTRA_FLAGS).  The kernel lives at 233
// of 256 vector registers; with the default register-pressure tracking of the scheduler the allocator spills an
// accumulator inside the steady loops of this formulation, with the option it does not.  The option changes
// scheduling decisions only; the results are the same either way.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "attn_vsa.hpp"
#include "vsa_pp.hpp"

int vfa_detail_vsa_pp_raise_lds(void) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_vsa_pp_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               VSA_LDS_BYTES) == hipSuccess ? 0 : -1;
}

int vfa_detail_vsa_pp_launch(const void* params, unsigned long params_bytes, unsigned n_wg, void* stream) {
    if (params_bytes != sizeof(Params)) return -1;  // the two translation units disagree about the parameter block
    Params q;
    memcpy(&q, params, sizeof(Params));
    attn_vsa_pp_kernel<<<dim3(n_wg), 512, VSA_LDS_BYTES, static_cast<hipStream_t>(stream)>>>(q);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
