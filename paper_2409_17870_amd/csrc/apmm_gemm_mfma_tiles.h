// Tile choice and width dispatch of the E2M1 MFMA GEMM (apmm_gemm_mfma_direct.h).  One translation
// unit per activation width instantiates the kernels, so that they compile in parallel.
#pragma once
#include "apmm_gemm_mfma_direct.h"

namespace apmm {
namespace mfma {

// Switches for A/B measurements of the launch rule exist only in builds with -DAPMM_DEBUG_SWITCHES; the
// product build reads no environment variable.
inline const char *debug_switch(const char *name)
{
#ifdef APMM_DEBUG_SWITCHES
    return std::getenv(name);
#else
    (void)name;
    return nullptr;
#endif
}

// Tile choice: estimate each candidate as (rounds of 256 tiles) x (tile area) x (measured relative
// cost per MFMA of that tile shape) and take the cheapest.  (Debug builds: APMM_MFMA_TILE=0..3 forces one.)
template <int P, int Q>
hipError_t launch_tiles(const GemmArgs &g, hipStream_t stream)
{
    struct Cand { int bm, bn; double cost; };
    // activations in the field form need 24 raw registers per row block: only the tiles with two row blocks
    // per wave are built for them (the others are given a cost no choice survives)
    constexpr bool AF = activation_field_form(P);
    const Cand cands[4] = {{256, 256, AF ? 1e9 : 1.0}, {256, 128, AF ? 1e9 : 1.2}, {128, 256, AF ? 1.0 : 1.2},
                           {128, 128, AF ? 1.15 : 1.2}};
    int best = 0;
    double best_t = 0;
    static const char *forced = debug_switch("APMM_MFMA_TILE");
    static const char *no_split = debug_switch("APMM_MFMA_SPLIT");
    if (forced && forced[0] >= '0' && forced[0] <= '3' && !(AF && forced[0] < '2')) {
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
    if constexpr (AF) {
        (void)no_split;
        static const char *square = debug_switch("APMM_MFMA_AF_2X2");
        const bool old_arrangement = square && square[0] == '1';
        if (best == 2) {
            // 1-bit weights: four wave tiles of 32 x 256 need 3.5 instead of 4 KB per wave and k step (with wider
            // weights the 2 x 2 arrangement of 64 x 128 wave tiles is the lighter one).  Measured at M = 2048 with both
            // outputs: 8 % faster at K = 11008, 2 - 5 % slower at K = 4096, where the store of the tile weighs more
            // than the k loop: taken from K = 8192 on.
            if constexpr (Q == 1) {
                if (!old_arrangement && g.nkb >= 64) return launch_direct_variant<P, Q, 1, 8>(g, stream);
            }
            return launch_direct_variant<P, Q, 2, 4>(g, stream);
        }
        // The 128 x 128 tile as four wave tiles of 32 x 128 one above the other: every activation row block (6 bits per
        // element, three quarters of the bytes) is loaded by one wave only, 14 instead of 16 KB through L1 per k step,
        // and these tiles are bound by L1: measured 12 % faster than 2 x 2 wave tiles of 64 x 64
        // (APMM_MFMA_AF_2X2=1 brings those back, for comparison).
        if (old_arrangement) return launch_direct_variant<P, Q, 2, 2>(g, stream);
        return launch_direct_variant<P, Q, 1, 4>(g, stream);
    } else {
        switch (best) {
        case 0: {
            // Two-phase kernels (part of the store under the k loop).  APMM_MFMA_SPLIT=0, 2, 3 forces the one-phase,
            // the even or the uneven one where usable (debugging); otherwise the measured rule.  A split pays when
            // the store is exposed and the memory system is the limit: one round of tiles on most of the chip
            // (with more rounds the next tile's k loop already covers the store, with few tiles the store is
            // fast), one sweep, K of at most 16 stages (beyond, the slower k loop costs what the store saves).
            // The uneven cut wins over the even one when the weight group is a single plane (cheapest expansion,
            // which the short second phase repeats per row block).
            constexpr int sweeps = ((P + 1) / 2) * ((Q + 1) / 2);
            const int64_t nst = g.nkb / 2;
            const int64_t tiles = ((g.M + 255) / 256) * ((g.N + 255) / 256);
            const bool pays = sweeps * nst <= 16 && tiles > 128 && tiles <= 256;
            const char want = no_split ? no_split[0] : 0;
            if constexpr (Q == 1) {
                const bool ok3 = direct_split_usable<P, Q, 4, 4, 3>(g);
                if (ok3 && (want == '3' || (want == 0 && pays))) return launch_direct_variant<P, Q, 4, 4, 3>(g, stream);
            }
            const bool ok2 = direct_split_usable<P, Q, 4, 4, 2>(g);
            if (ok2 && (want == '2' || (want == 0 && pays))) return launch_direct_variant<P, Q, 4, 4, 2>(g, stream);
            return launch_direct_variant<P, Q, 4, 4>(g, stream);
        }
        case 1: return launch_direct_variant<P, Q, 4, 2>(g, stream);
        case 2: return launch_direct_variant<P, Q, 2, 4>(g, stream);
        default: return launch_direct_variant<P, Q, 2, 2>(g, stream);
        }
    }
}

template <int P>
hipError_t launch_fp4_p(const GemmArgs &g, hipStream_t stream)
{
    switch (g.q) {
    case 1: return launch_tiles<P, 1>(g, stream);
    case 2: return launch_tiles<P, 2>(g, stream);
    case 3: return launch_tiles<P, 3>(g, stream);
    case 4: return launch_tiles<P, 4>(g, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace mfma
}  // namespace apmm
