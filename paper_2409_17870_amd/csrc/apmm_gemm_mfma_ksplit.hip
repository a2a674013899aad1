// Matrix-unit GEMM kernels whose four waves split K (apmm_gemm_mfma_ksplit.h): instantiations and launch rule.
#include "apmm_gemm_mfma_ksplit.h"

namespace apmm {

namespace {

template <int P, int Q>
hipError_t launch_ksplit_tiles(const GemmArgs &g, hipStream_t stream, int wn)
{
    switch (wn) {
    case 4: return mfma::launch_ksplit_variant<P, Q, 2, 4>(g, stream);
    case 5: return mfma::launch_ksplit_variant<P, Q, 2, 5>(g, stream);
    default: return mfma::launch_ksplit_variant<P, Q, 2, 6>(g, stream);
    }
}

template <int P>
hipError_t launch_ksplit_p(const GemmArgs &g, hipStream_t stream, int wn)
{
    switch (g.q) {
    case 1: return launch_ksplit_tiles<P, 1>(g, stream, wn);
    case 2: return launch_ksplit_tiles<P, 2>(g, stream, wn);
    case 3: return launch_ksplit_tiles<P, 3>(g, stream, wn);
    case 4: return launch_ksplit_tiles<P, 4>(g, stream, wn);
    }
    return hipErrorInvalidValue;
}

// Tile width (column blocks of 32; the tile has two row blocks): the one that fills most of the 256 compute
// units in a single round of tiles, or 0 when every width needs more than one round.
int one_round_width(const GemmArgs &g)
{
    int best = 0;
    int64_t best_tiles = 0;
    for (int wn = 4; wn <= 6; ++wn) {
        const int64_t tiles = ((g.M + 63) / 64) * ((g.N + 32 * wn - 1) / (32 * wn));
        if (tiles <= 256 && tiles > best_tiles) {
            best = wn;
            best_tiles = tiles;
        }
    }
    return best;
}

}  // namespace

bool gemm_mfma_ksplit_supported(const GemmArgs &g)
{
    return gemm_mfma_fp4_supported(g) && activation_field_form(g.p);
}

// Measured against the large-tile kernel (W2A4 and W1A4, 512 x 5120 outputs, fp16 output, inside a graph): equal at
// K = 5120 and 8192 (14.5 / 21.6 us), 15 % faster at K = 13824 and 16384 (28.2 against 33.1 us): the exchange
// through LDS and the colder start of waves that each begin at another place of K cost about 2 us per tile, the k
// loop gains 0.5 us per 1024 elements of K.  With more than one round of tiles the large tiles win (their
// fixed costs are paid once per larger tile).
bool gemm_mfma_ksplit_pays(const GemmArgs &g)
{
    return gemm_mfma_ksplit_supported(g) && g.nkb >= 80 && one_round_width(g) != 0;
}

hipError_t launch_gemm_mfma_ksplit(const GemmArgs &g, hipStream_t stream)
{
    int wn = one_round_width(g);
    if (wn == 0) wn = 5;  // explicit request for a shape of several rounds
    switch (g.p) {
    case 3: return launch_ksplit_p<3>(g, stream, wn);
    case 4: return launch_ksplit_p<4>(g, stream, wn);
    }
    return hipErrorInvalidValue;
}

}  // namespace apmm
