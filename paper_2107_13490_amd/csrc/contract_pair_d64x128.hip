// Paired gradient kernels whose data-gradient tile is 64 x 128
#include "contract_pair.hpp"

namespace adapt {
hipError_t launch_pair_d64x128(adapt_ctx *ctx, const ContractPlan &d, const ContractPlan &w, bool *done)
{
    return launch_pair_for<64, 128>(ctx, d, w, done);
}
}  // namespace adapt
