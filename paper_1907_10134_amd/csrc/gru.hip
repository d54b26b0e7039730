// GRU variants of the builder and of the parameter-gradient reduction.
#include "bppsa_internal.h"

bppsa_status bppsa_build_jacobians_gru(int, int, int, int, const float*, const float*,
                                       const float*, const float*, const float*, const float*,
                                       float*, hipStream_t) {
  return BPPSA_EUNSUPPORTED;
}

size_t bppsa_param_grads_gru_ws(int, int, int, int) { return 0; }

bppsa_status bppsa_param_grads_gru(int, int, int, int, const float*, const float*, const float*,
                                   const float*, const float*, const float*, const float*,
                                   float*, float*, float*, float*, void*, size_t, hipStream_t) {
  return BPPSA_EUNSUPPORTED;
}
