#include "dfa_internal.h"
namespace dfa {
int launch_fwd_bf16(const dfa_shape&, const void*, const void*, const void*, void*, float*, hipStream_t) { return DFA_ERR_DTYPE; }
int launch_bwd_bf16(const dfa_shape&, const void*, const void*, const void*, const float*, const float*, const void*,
                    float*, float*, float*, int, hipStream_t) { return DFA_ERR_DTYPE; }
}
