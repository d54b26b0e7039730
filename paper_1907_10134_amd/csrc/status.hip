#include "bppsa_internal.h"

extern "C" const char* bppsa_strerror(int status) {
  switch (status) {
    case BPPSA_OK: return "BPPSA_OK";
    case BPPSA_EINVAL: return "BPPSA_EINVAL: null pointer or non-positive size";
    case BPPSA_ESHAPE: return "BPPSA_ESHAPE: size not accepted by the kernels";
    case BPPSA_EWORKSPACE: return "BPPSA_EWORKSPACE: workspace missing or too small";
    case BPPSA_EOVERFLOW: return "BPPSA_EOVERFLOW: index does not fit its integer type";
    case BPPSA_EHIP: return "BPPSA_EHIP: HIP runtime or launch failure";
    case BPPSA_EUNSUPPORTED: return "BPPSA_EUNSUPPORTED: no kernel for this cell or size";
    default: return "BPPSA: unknown status";
  }
}
