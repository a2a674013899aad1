// E2M1 (fp4) MFMA GEMM kernels for 1-, 2- and (activations only) 4-bit operands: the register-direct kernel of
// apmm_gemm_mfma_direct.h in four tile shapes.
#include "apmm_gemm_mfma_direct.h"

namespace apmm {
namespace {

// Tile choice: estimate each candidate as (rounds of 256 tiles) x (tile area) x (measured relative
// cost per MFMA of that tile shape) and take the cheapest.  APMM_MFMA_TILE=0..3 forces one (debugging).
template <int P, int Q>
hipError_t launch_tiles(const GemmArgs &g, hipStream_t stream)
{
    struct Cand { int bm, bn; double cost; };
    const Cand cands[4] = {{256, 256, 1.0}, {256, 128, 1.2}, {128, 256, 1.2}, {128, 128, 1.2}};
    int best = 0;
    double best_t = 0;
    static const char *forced = std::getenv("APMM_MFMA_TILE");
    if (forced && forced[0] >= '0' && forced[0] <= '3') {
        best = forced[0] - '0';
    } else {
        for (int c = 0; c < 4; ++c) {
            const int64_t tiles = ((g.M + cands[c].bm - 1) / cands[c].bm) * ((g.N + cands[c].bn - 1) / cands[c].bn);
            const double t = (double)((tiles + 255) / 256) * cands[c].bm * cands[c].bn * cands[c].cost;
            if (c == 0 || t < best_t) {
                best = c;
                best_t = t;
            }
        }
    }
    switch (best) {
    case 0: return mfma::launch_direct_variant<P, Q, 4, 4>(g, stream);
    case 1: return mfma::launch_direct_variant<P, Q, 4, 2>(g, stream);
    case 2: return mfma::launch_direct_variant<P, Q, 2, 4>(g, stream);
    default: return mfma::launch_direct_variant<P, Q, 2, 2>(g, stream);
    }
}

}  // namespace

hipError_t launch_gemm_mfma_fp4_impl(const GemmArgs &g, hipStream_t stream)
{
    if (g.p == 1 && g.q == 1) return launch_tiles<1, 1>(g, stream);
    if (g.p == 1 && g.q == 2) return launch_tiles<1, 2>(g, stream);
    if (g.p == 2 && g.q == 1) return launch_tiles<2, 1>(g, stream);
    if (g.p == 2 && g.q == 2) return launch_tiles<2, 2>(g, stream);
    if (g.p == 4 && g.q == 1) return launch_tiles<4, 1>(g, stream);
    if (g.p == 4 && g.q == 2) return launch_tiles<4, 2>(g, stream);
    return hipErrorInvalidValue;
}

}  // namespace apmm
