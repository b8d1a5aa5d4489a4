// placeholder until the matrix-core engine lands
#include "engines.hpp"
namespace lc {
void mfma_fill_plan(Plan& pl)
{
    pl.order.ndig = 0;
    if (pl.log2R) pl.order.bits[pl.order.ndig++] = (unsigned char)pl.log2R;
    for (int i = 0; i < pl.log2L2; ++i) pl.order.bits[pl.order.ndig++] = 1;
    pl.kscale = 1.0f / (float)(int64_t(1) << pl.log2L);
    pl.dkscale = pl.kscale;
}
hipError_t mfma_conv(const void*, const float2*, void*, __half2*, bool, const Problem&, const Plan&, const float2*, hipStream_t) { return hipErrorNotSupported; }
hipError_t mfma_dk(const void*, const void*, float*, float*, const __half2*, const __half2*, __half2*, const Problem&, const Plan&, const float2*, hipStream_t) { return hipErrorNotSupported; }
}
