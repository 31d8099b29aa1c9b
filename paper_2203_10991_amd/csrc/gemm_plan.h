// Host-side planning shared by the 16-bit and the 8-bit sparse-MFMA update GEMMs: how the rows of dW are split between
// the 384 x 256 and the 256 x 256 tile kernels, where a launch writes (dW itself, or split-K partial sums in the
// workspace), the shift table of a convolution's row-shifted views.  Pure functions of the problem size: the two
// paths differ only in the constants they pass (tokens per stage, measured cost of a round of tall tiles).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "smfmac_common.h"        // ShiftArg

namespace nm {

constexpr int NM_CUS = 256;       // compute units of the device the plans are tuned for

// Rows [0, tall_rows) of dW go to the 384 x 256 kernel (tall_tiles_m tile rows), the rest to the 256 x 256 kernel.
// The taller tile moves fewer operand bytes per product and is faster per product, but a GPU-wide round of its tiles
// takes `tall_round` times as long as a round of 256 x 256 tiles, and a partly filled last round costs a full one:
// the split minimises the summed cost of whole rounds (tall_tiles_m = 0: no tall launch).
struct RowSplit { int64_t tall_rows; int tall_tiles_m; };
inline RowSplit split_rows_tall(int64_t O, int64_t I, double tall_round, bool allow_tall)
{
    const int64_t tn = (I + 255) / 256;
    double best = 1e300;
    int64_t best_mt = 0;
    for (int64_t mt = 0; allow_tall && mt <= (O + 383) / 384; ++mt) {
        const int64_t left = O - std::min<int64_t>(O, mt * 384), m256 = (left + 255) / 256;
        const double cost = tall_round * (double)((mt * tn + NM_CUS - 1) / NM_CUS) + (double)((m256 * tn + NM_CUS - 1) / NM_CUS);
        if (cost < best - 1e-9) { best = cost; best_mt = mt; }
    }
    return RowSplit{std::min<int64_t>(O, best_mt * 384), (int)best_mt};
}

// Split-K: with more than one slab the kernels write binary32 partial sums [slabs][O][I] into the workspace (row
// stride I, never accumulating) and launch_splitk_reduce sums them into dW in slab order; with one slab they write
// (or accumulate into) dW directly.
struct OutTarget { float *out; int64_t ldo, slab_stride; int accumulate; };
inline OutTarget splitk_target(int slabs, float *dW, int64_t lddw, void *workspace, int64_t O, int64_t I, int accumulate)
{
    if (slabs > 1) return OutTarget{(float *)workspace, I, O * I, 0};
    return OutTarget{dW, lddw, 0, accumulate};
}
inline size_t splitk_workspace_bytes(int slabs, int64_t O, int64_t I)
{
    return slabs > 1 ? (size_t)slabs * (size_t)O * (size_t)I * sizeof(float) : 0;
}

// slabs of the reduction axis as whole trips of the kernels' LDS stage ring: `groups` token groups, `per_trip` groups
// per trip of the ring; returns groups per slab and corrects the slab count to what that gives
inline int64_t slab_groups(int64_t groups, int &slabs, int64_t per_trip)
{
    int64_t gps = (groups + slabs - 1) / std::max(slabs, 1);
    gps = (gps + per_trip - 1) / per_trip * per_trip;
    if (gps < per_trip) gps = per_trip;
    slabs = groups > 0 ? (int)((groups + gps - 1) / gps) : 1;
    return gps;
}

// the dense operand as n row-shifted views of one [rows x cb] matrix
inline ShiftArg make_shift_arg(int64_t cb, const int64_t *rows, int n)
{
    ShiftArg sh{};
    sh.cb = (int)cb; sh.n = n; sh.margin = 0;
    for (int j = 0; j < n; ++j) {
        sh.rows[j] = (int)rows[j];
        sh.margin = std::max(sh.margin, (int)(rows[j] < 0 ? -rows[j] : rows[j]));
    }
    return sh;
}

}  // namespace nm
