// Dense attention baseline (Eq. 6) -- placeholder until the kernel lands.
#include "psa_internal.h"

extern "C" {
size_t dense_attn_workspace_bytes(const psa_shape_t*) { return 0; }
int dense_attn_fwd(const void*, const void*, const void*, const int32_t*, void*, const psa_shape_t*, void*, size_t, void*)
{
    return PSA_ERR_ARG;
}
}
