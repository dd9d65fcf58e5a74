// Encryption of the weight rows (Algorithm 1 step 1): the instances of the product kernel that
// assemble c0 = Delta w + e - a s behind the product, in a translation unit of their own (see
// rlwe_kernels.hpp).
#include "rlwe_kernels.hpp"

namespace nimbus {

hipError_t launch_encrypt_rows(const PolyArgs &a, int logN, size_t polys, hipStream_t stream)
{
    return launch_poly<true>(a, logN, polys, stream);
}

}  // namespace nimbus
