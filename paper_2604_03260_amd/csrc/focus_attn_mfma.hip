// placeholder until the matrix-core kernel lands: route bf16 through the vector kernel
#include "focus_internal.h"
namespace focus {
hipError_t launch_attn_mfma(const Layout& L, const HeadMap& hm, const void* q, const void* k, const void* v,
                            char* ws, void* out, float* lse, int32_t* row_pairs, hipStream_t st)
{
    return launch_attn_simple(L, hm, q, k, v, ws, out, lse, row_pairs, st);
}
}  // namespace focus
