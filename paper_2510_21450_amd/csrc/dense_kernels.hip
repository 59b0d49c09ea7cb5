// Dense-Jacobian path: placeholder until the MFMA scan lands.
#include "dense.h"
#include "../../include/pararnn.h"

namespace pararnn {

size_t dense_workspace_bytes(int, int, int, int, int) { return 0; }

int dense_forward(int, const float *, const void *, const void *, int, int, int, float, int, void *, int *, float *,
                  void *, size_t, hipStream_t)
{
    return PARARNN_UNSUPPORTED;
}

}  // namespace pararnn
