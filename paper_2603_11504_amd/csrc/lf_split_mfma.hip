// Matrix-core split kernel (bf16, head_dim 128): placeholder until the MFMA path lands.
#include "lf_host.h"
namespace lf {
hipError_t launch_split_mfma(const Plan &p, const void *q, int n, hipStream_t s)
{
    return launch_split_valu(p, q, n, s);
}
} // namespace lf
