// How the 128-row tiles of a launch that runs both tile heights are dealt to the workgroups of an XCD.
// Plain C++ (compiles on the host as well, where a test checks that every tile is dealt exactly once).
#pragma once

#if defined(__HIPCC__)
#define BM_HOST_DEVICE __host__ __device__ __forceinline__
#else
#define BM_HOST_DEVICE inline
#endif

namespace bm {

// Deals an XCD's 128-row tiles (ids 0 .. n_small - 1) to its `stride` workgroups after the 256-row tiles:
// the first R workgroups (the "heavy" ones) hold one 256-row tile more than the other L = stride - R.  The
// tiles go out in batches, each batch to the class with the smaller load so far, one tile per workgroup of
// the class; a 256-row tile counts 20, a 128-row tile 13 (measured tile times 53 and 35 us).  Every
// workgroup replays the same sequence and picks out its own tiles, so no memory is shared.
struct SmallTileDealer {
    int base, load_l, load_h, R, L, n_small, slot;
    BM_HOST_DEVICE void init(int n_big, int n_small_, int stride, int slot_) {
        R = n_big % stride; L = stride - R; n_small = n_small_; slot = slot_; base = 0;
        load_l = 20 * (n_big / stride);
        load_h = load_l + 20;
    }
    // the next tile of this workgroup; false when it has none left
    BM_HOST_DEVICE bool next(int &tile) {
        while (base < n_small) {
            const bool to_light = R == 0 || load_l <= load_h;
            const int cnt = to_light ? L : R;
            const int mine = to_light ? slot - R : (slot < R ? slot : -1);
            const int id = base + mine;
            base += cnt;
            if (to_light) load_l += 13; else load_h += 13;
            if (mine >= 0 && id < n_small) { tile = id; return true; }
        }
        return false;
    }
};

}  // namespace bm
