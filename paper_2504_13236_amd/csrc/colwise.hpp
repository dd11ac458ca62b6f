// Column walker for the kernels that reduce along the first axis of a tiled
// tensor (layer norm over the embedding axis, softmax over the key axis).
//
// A "column" is one index combination of the axes 1..3; along axis 0 it crosses
// grid[0] tiles, and inside each of them its elements are contiguous.  One
// wavefront owns one column: its 64 lanes read 64 * V consecutive elements per
// step, so every access is a full-width coalesced vector access.
#pragma once
#include "device_util.hpp"

namespace nnt {

struct Column {
    int tile0;        // tile number of (0, t1, t2, t3)
    int colidx;       // position of the column among the tile's columns
    int c1, c2, c3;   // logical coordinates
    int stat_tile;    // tile number in a companion tensor whose axis 0 is not tiled
    int ncol_tile;    // number of columns in this tile (= ext1 * ext2 * ext3)
};

// (callers keep the number of columns below 2^31, so the index arithmetic is 32-bit: a 64-bit division
// costs some hundred instructions on this hardware)
__device__ __forceinline__ Column column_of(const TiledView& v, int64_t col64) {
    Column c;
    unsigned col = (unsigned)col64;
    const unsigned s1 = (unsigned)v.shape[1], s2 = (unsigned)v.shape[2];
    unsigned q = col / s1;
    c.c1 = (int)(col - q * s1);
    col = q;
    q = col / s2;
    c.c2 = (int)(col - q * s2);
    c.c3 = (int)q;
    const int t1 = (int)((unsigned)c.c1 / (unsigned)v.base[1]), t2 = (int)((unsigned)c.c2 / (unsigned)v.base[2]);
    const int t3 = (int)((unsigned)c.c3 / (unsigned)v.base[3]);
    const int l1 = t1 * v.base[1], l2 = t2 * v.base[2], l3 = t3 * v.base[3];
    const int e1 = min(v.base[1], v.shape[1] - l1), e2 = min(v.base[2], v.shape[2] - l2);
    const int e3 = min(v.base[3], v.shape[3] - l3);
    c.stat_tile = t1 + v.grid[1] * (t2 + v.grid[2] * t3);
    c.tile0 = v.grid[0] * c.stat_tile;
    c.colidx = (c.c1 - l1) + e1 * ((c.c2 - l2) + e2 * (c.c3 - l3));
    c.ncol_tile = e1 * e2 * e3;
    return c;
}

__device__ __forceinline__ int ext0_of(const TiledView& v, int l) { return min(v.base[0], v.shape[0] - l * v.base[0]); }

template <typename T>
__device__ __forceinline__ T* col_ptr(const TiledView& v, const Column& c, int l, int ext0) {
    T* base = static_cast<T*>(v.tiles[c.tile0 + l]);
    return base ? base + (int64_t)c.colidx * ext0 : nullptr;
}

inline int64_t n_columns(const nnt_tensor* t) {
    int64_t n = 1;
    for (int a = 1; a < t->ndim; a++) n *= t->shape[a];
    return n;
}

}  // namespace nnt
