// Matrix-unit GEMM kernels whose four waves split K (apmm_gemm_mfma_ksplit.h): launch rule.  The kernels are
// instantiated in apmm_gemm_mfma_ksplit_p<P>.hip, one translation unit per activation width.
#include "apmm_kernels.h"

namespace apmm {

hipError_t launch_gemm_mfma_ksplit_p1(const GemmArgs &g, hipStream_t stream, int wn);
hipError_t launch_gemm_mfma_ksplit_p2(const GemmArgs &g, hipStream_t stream, int wn);
hipError_t launch_gemm_mfma_ksplit_p3(const GemmArgs &g, hipStream_t stream, int wn);
hipError_t launch_gemm_mfma_ksplit_p4(const GemmArgs &g, hipStream_t stream, int wn);

namespace {

// Tile width (column blocks of 32: 2, 4, 5 or 6; the tile has two row blocks): the one that fills most of the 256
// compute units in a single round of tiles, i.e. the narrowest with at most 256 tiles, or 0 when every width needs
// more than one round.  Activations in the group form (1 and 2 bits) have the 64 x 64 and 64 x 128 tiles only.
int one_round_width(const GemmArgs &g)
{
    int best = 0;
    int64_t best_tiles = 0;
    for (int wn = 2; wn <= (activation_field_form(g.p) ? 6 : 4); ++wn) {
        if (wn == 3) continue;
        const int64_t tiles = ((g.M + 63) / 64) * ((g.N + 32 * wn - 1) / (32 * wn));
        if (tiles <= 256 && tiles > best_tiles) {
            best = wn;
            best_tiles = tiles;
        }
    }
    return best;
}

}  // namespace

bool gemm_mfma_ksplit_supported(const GemmArgs &g) { return gemm_mfma_fp4_supported(g); }

// Launch rule, measured against the large-tile kernel inside a graph; with more than one round of tiles the large
// tiles win by 30 - 70 % (their fixed costs are paid once per larger tile), so one round is a condition throughout.
//   Field form (3, 4 bits; W2A4 and W1A4, 512 x 5120 outputs, fp16 output): slower below K = 4096 (the exchange
//   through LDS and the colder start of waves that each begin at another place of K cost about 2 us per tile),
//   equal to 10 % faster at K = 5120 (14.2 against 14.5 us on one box, 12.1 against 13.4 us on another), 15 - 26 %
//   faster at K = 13824 (28.2 against 33.1, 22.5 against 30.4 us): the k loop gains 0.5 us per 1024 elements of K.
//   Taken from K = 5120 on; with the 64 x 128 tile (outputs of up to 256 of them, e.g. up to 512 tokens at 4096
//   channels or 128 at 11008) already from K = 3072 on: 1 - 256 tokens at 4096 x 4096 9.4 - 9.8 against 11.2 - 12.6 us,
//   at 4096 x 11008 15.5 - 16.2 against 22.7 - 24.1 us, equal at K = 1024.
//   Group form (1, 2 bits; W2A2 and W1A2, fp16 or int32 output), where the large-tile kernel has 128 x 128 tiles for
//   these outputs: 512 x 4096 outputs 5.9 / 7.3 / 9.9 / 16.6 us against 6.7 / 7.5 / 8.6 / 11.6 us here at K = 1024 / 2048 /
//   4096 / 8192; 512 x 4096 x 11008 22.0 against 13.8 us; 65 x 4096 and 96 x 11008 outputs faster at every K (10.7
//   against 7.9 us at K = 4096).  Taken from K = 3072 on, and at every K up to 128 tokens.
//   The 64 x 64 tile (outputs of up to 256 of them: up to 256 tokens at 4096 channels, 128 at 8192), every width:
//   65 - 256 tokens at 4096 x 4096 5.3 - 5.9 us (W1A1, W2A2), 6.9 - 7.4 us (W2A4) against 7.5 - 8.5 and 9.6 - 9.9 us with the
//   64 x 128 tile and 9.3 - 11.5 us on the large tiles; at 4096 x 11008 7.4 - 8.5 and 10.7 - 11.9 against 11.0 - 12.1 and
//   15.8 - 16.5 us; at K = 1024 4.4 - 5.0 against 5.5 - 6.6 us on the large tiles.  Taken at every K.
bool gemm_mfma_ksplit_pays(const GemmArgs &g)
{
    if (!gemm_mfma_ksplit_supported(g) || one_round_width(g) == 0) return false;
    if (one_round_width(g) == 2) return true;
    if (activation_field_form(g.p)) return g.nkb >= 40 || (one_round_width(g) == 4 && g.nkb >= 24);
    return g.nkb >= 24 || g.M <= 128;
}

hipError_t launch_gemm_mfma_ksplit(const GemmArgs &g, hipStream_t stream)
{
    int wn = one_round_width(g);
    if (wn == 0) wn = activation_field_form(g.p) ? 5 : 4;  // explicit request for a shape of several rounds
    switch (g.p) {
    case 1: return launch_gemm_mfma_ksplit_p1(g, stream, wn);
    case 2: return launch_gemm_mfma_ksplit_p2(g, stream, wn);
    case 3: return launch_gemm_mfma_ksplit_p3(g, stream, wn);
    case 4: return launch_gemm_mfma_ksplit_p4(g, stream, wn);
    }
    return hipErrorInvalidValue;
}

}  // namespace apmm
