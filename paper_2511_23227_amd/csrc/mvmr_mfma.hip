// Matrix-core (MFMA) MVMR kernels for the tuned channel shapes.
#include "pcpp_internal.h"

namespace pcpp {

int mvmr_rows_mfma(const MvmrArgs &a, hipStream_t stream, bool *handled)
{
    (void)a; (void)stream;
    *handled = false;
    return PCPP_OK;
}

}  // namespace pcpp
