// Wave-level classification of a (32-query patch, 32-key block) pair.  Used by the bf16 kernels
// (device) and by the host-side count of executed pairs, so that the reported "executed" work is
// exactly what the kernels feed to the matrix pipeline.
#pragma once
#include <hip/hip_runtime.h>

namespace clear {

enum BlockClass : int { kBlockSkip = 0, kBlockPartial = 1, kBlockFull = 2 };

__host__ __device__ inline int imin(int a, int b) { return a < b ? a : b; }
__host__ __device__ inline int imax(int a, int b) { return a > b ? a : b; }

// Image keys.  Query patch: rows [qy0, qy0+qh), cols [qx0, qx0+qw).  Key block: rows [ky0, ky0+kh),
// cols [kx0, kx0+kw).  Both may hang over the grid border.  The mask of Eq. 3 (Sec. 3.2) admits
// a pair iff dx^2 + dy^2 < r2.
//   skip    : no in-grid pair is admitted (smallest distance between the clipped rectangles >= r)
//   full    : the key block lies inside the grid and even the largest distance is admitted
//   partial : everything else; the element mask must be applied
__host__ __device__ inline int classify_image_block(int qy0, int qx0, int qh, int qw, int ky0, int kx0,
                                                    int kh, int kw, int gridH, int gridW, int r2)
{
    if (qy0 >= gridH || qx0 >= gridW || ky0 >= gridH || kx0 >= gridW) return kBlockSkip;
    const int qy1 = imin(qy0 + qh, gridH) - 1, qx1 = imin(qx0 + qw, gridW) - 1;
    const int ky1 = imin(ky0 + kh, gridH) - 1, kx1 = imin(kx0 + kw, gridW) - 1;
    const int dy_min = imax(0, imax(ky0 - qy1, qy0 - ky1));
    const int dx_min = imax(0, imax(kx0 - qx1, qx0 - kx1));
    if (dy_min * dy_min + dx_min * dx_min >= r2) return kBlockSkip;
    const bool inside = (ky0 + kh <= gridH) && (kx0 + kw <= gridW);
    const int dy_max = imax(qy0 + qh - 1 - ky0, ky0 + kh - 1 - qy0);
    const int dx_max = imax(qx0 + qw - 1 - kx0, kx0 + kw - 1 - qx0);
    return (inside && dy_max * dy_max + dx_max * dx_max < r2) ? kBlockFull : kBlockPartial;
}

// Keys taken from a contiguous token range [.., limit): block = tokens [base, base + n).
__host__ __device__ inline int classify_linear_block(long long base, int n, long long limit)
{
    if (base >= limit) return kBlockSkip;
    return (base + n <= limit) ? kBlockFull : kBlockPartial;
}

}  // namespace clear
