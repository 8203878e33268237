// Work-item decoding of the LDS-patch convolution kernels: plain integer logic, shared by the
// kernels (device) and by a host-side check that walks every grid size.
#pragma once

#if defined(__HIPCC__)
#define SGPRS_HD __host__ __device__ __forceinline__
#else
#define SGPRS_HD inline
#endif

namespace sgprs {

// Work-item index -> (split, channel block, row tile).  Workgroup b of a launch
// runs on die b % 8 and keeps that die for all its items (the grid is a
// multiple of 8).  With up to kRowTilePerDieMaxBlocks channel blocks, row tile
// 8g + die and all its channel blocks run on one die at about the same time:
// the input rows they share come from HBM once and hit in that die's L2, and
// the weights of all channel blocks fit there as well (measured 5-7% faster on
// the 128- and 256-channel layers).  With more channel blocks the weights would
// not fit, so each die keeps one channel block (xcd_groups = 8 / n_ntiles) and
// the input patches stream through.
constexpr int kRowTilePerDieMaxBlocks = 4;
struct PatchItem { int split, ntile, mtile; bool valid; };
template <class Args> SGPRS_HD PatchItem decode_item(const Args& a, int item)
{
    PatchItem r;
    if (a.xcd_groups > 0) {
        const int x = item & 7, s = item >> 3;
        r.split = 0;
        if (a.n_ntiles <= kRowTilePerDieMaxBlocks) {
            r.ntile = s % a.n_ntiles;
            r.mtile = (s / a.n_ntiles) * 8 + x;
            r.valid = r.mtile < a.n_mtiles;
        } else {
            r.ntile = x % a.n_ntiles;
            r.mtile = s * a.xcd_groups + x / a.n_ntiles;
            r.valid = item < a.n_slots && r.mtile < a.n_mtiles;
        }
    } else {
        r.split = item % a.splits;
        const int t2 = item / a.splits;
        r.ntile = t2 % a.n_ntiles;
        r.mtile = t2 / a.n_ntiles;
        r.valid = item < a.n_slots;
    }
    return r;
}

// Host side: the index space of a launch of n_mtiles x n_ntiles tiles (x splits split-K slices).
// xcd_groups > 0 selects the die-keyed layouts above (unsplit launches of 1, 2, 4 or 8 channel
// blocks); n_slots is the size of the padded index space that decode_item understands.
inline void patch_index_space(int n_mtiles, int n_ntiles, int splits, int* xcd_groups, int* n_slots)
{
    *xcd_groups = (splits == 1 && n_ntiles <= 8 && 8 % n_ntiles == 0) ? 8 / n_ntiles : 0;
    *n_slots = !*xcd_groups ? n_mtiles * n_ntiles * splits
               : n_ntiles <= kRowTilePerDieMaxBlocks ? (n_mtiles + 7) / 8 * 8 * n_ntiles
                                                      : 8 * ((n_mtiles + *xcd_groups - 1) / *xcd_groups);
}

// The first valid work item among item, item + stride, item + 2 * stride, ... (item is advanced to
// it), or an invalid one when none is left.  The die-keyed index spaces are padded, and with a
// grid that is not a multiple of 8 (a partition of fewer than 8 CUs) valid items follow invalid
// ones, so a workgroup skips over holes instead of stopping at the first.
template <class Args> SGPRS_HD PatchItem next_item(const Args& a, int& item, int stride)
{
    PatchItem r = decode_item(a, item);
    while (!r.valid && item + stride < a.n_slots) {
        item += stride;
        r = decode_item(a, item);
    }
    return r;
}

}  // namespace sgprs
