// Paired launch of a layer's two gradient contractions (see contract_pair_kernel).  The kernels are
// instantiated in one translation unit per data-gradient tile to keep build times parallel.
#pragma once
#include "contract_kernel.hpp"

namespace adapt {

template <int LM, int BKT, int DBM, int DBN, int WBM, int WBN>
static hipError_t launch_pair(adapt_ctx *ctx, const ContractPlan &d, const ContractPlan &w)
{
    typedef typename LoaderSelect<OP_DGRAD, true, LOAD_VEC, DBM, LM, BKT>::type DA;
    typedef typename LoaderSelect<OP_DGRAD, false, LOAD_ROWS, DBN, LM, BKT>::type DB;
    typedef typename LoaderSelect<OP_WGRAD, true, LOAD_ROWS, WBM, LM, BKT>::type WA;
    typedef typename LoaderSelect<OP_WGRAD, false, LOAD_ROWS, WBN, LM, BKT>::type WB;
    const size_t lds = std::max<size_t>(DA::TILE_BYTES + DB::TILE_BYTES, WA::TILE_BYTES + WB::TILE_BYTES) * limbs_of(LM);
    void (*kern)(const ContractArgs, const ContractArgs, const unsigned, const unsigned, const unsigned) =
        contract_pair_kernel<LM, BKT, OP_DGRAD, LOAD_VEC, LOAD_ROWS, DBM, DBN, OP_WGRAD, LOAD_ROWS, LOAD_ROWS, WBM, WBN>;
    if (d.kern.amax_part != nullptr || w.kern.amax_part != nullptr)
        kern = contract_pair_kernel<LM, BKT, OP_DGRAD, LOAD_VEC, LOAD_ROWS, DBM, DBN, OP_WGRAD, LOAD_ROWS, LOAD_ROWS, WBM, WBN, true>;
    if (hipError_t e = allow_big_lds(ctx, reinterpret_cast<const void *>(kern), lds); e != hipSuccess) return e;
    const unsigned tiles_d = (unsigned)(((d.kern.M + DBM - 1) / DBM) * ((d.kern.N + DBN - 1) / DBN));
    const unsigned tiles_w = (unsigned)(((w.kern.M + WBM - 1) / WBM) * ((w.kern.N + WBN - 1) / WBN));
    const unsigned n_d = tiles_d * (unsigned)d.splits, n_w = tiles_w * (unsigned)w.splits;
    hipLaunchKernelGGL(kern, dim3(n_d + n_w), dim3(kThreads), lds, ctx->stream, d.kern, w.kern, n_d, tiles_d, tiles_w);
    note_amax_blocks(ctx, d.kern, n_d);
    note_amax_blocks(ctx, w.kern, n_w);
    return hipGetLastError();
}

// dispatch on the weight-gradient tile; *done stays false when the tile has no paired kernel.  Two-limb
// pairs exist for equal square tiles only (a 128-wide two-limb tile allows one block per CU, which
// would also hold back a 64-wide partner).
template <int DBM, int DBN>
static hipError_t launch_pair_for(adapt_ctx *ctx, const ContractPlan &d, const ContractPlan &w, bool *done)
{
    *done = true;
    if (d.limbs == 2) {
        if constexpr (DBM == DBN)
            if (w.tile.bm == DBM && w.tile.bn == DBN) {
                // one limb mode for the launch: balanced only when both contractions can take it
                if (d.kern.balanced && w.kern.balanced) return launch_pair<3, 64, DBM, DBN, DBM, DBN>(ctx, d, w);
                return launch_pair<2, 64, DBM, DBN, DBM, DBN>(ctx, d, w);
            }
        *done = false;
        return hipSuccess;
    }
    if (w.tile.bm == 64 && w.tile.bn == 64) return launch_pair<1, 192, DBM, DBN, 64, 64>(ctx, d, w);
    if (w.tile.bm == 128 && w.tile.bn == 64) return launch_pair<1, 192, DBM, DBN, 128, 64>(ctx, d, w);
    if (w.tile.bm == 64 && w.tile.bn == 128) return launch_pair<1, 192, DBM, DBN, 64, 128>(ctx, d, w);
    if (w.tile.bm == 128 && w.tile.bn == 128) return launch_pair<1, 192, DBM, DBN, 128, 128>(ctx, d, w);
    *done = false;
    return hipSuccess;
}

hipError_t launch_pair_d64x64(adapt_ctx *ctx, const ContractPlan &d, const ContractPlan &w, bool *done);
hipError_t launch_pair_d128x64(adapt_ctx *ctx, const ContractPlan &d, const ContractPlan &w, bool *done);
hipError_t launch_pair_d64x128(adapt_ctx *ctx, const ContractPlan &d, const ContractPlan &w, bool *done);
hipError_t launch_pair_d128x128(adapt_ctx *ctx, const ContractPlan &d, const ContractPlan &w, bool *done);

}  // namespace adapt
