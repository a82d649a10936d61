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

// Other local masks through the same machinery (the attention variants the paper compares with, Sec. 4.2 and
// the appendix on efficient-attention baselines; all keep the text rule of Eq. 3):
//   kMaskDisc    dx^2 + dy^2 < r^2                                   (Eq. 3, CLEAR)
//   kMaskSquare  |dx| < r and |dy| < r                               (neighbourhood-style square window, cut off at the border)
//   kMaskSwin    both tokens in the same r x r window of the partition whose origin is moved up and left by `shift`
//                (shift 0: windows start at the grid origin; the paper alternates shift 0 and r / 2 between layers)
//   strided      the key's offset from the query, modulo r on each axis (non-negative remainder), equals
//                (shift % r, (shift / r) % r); shift carries the layer index.  The bf16 kernels do not test
//                this predicate: they run one dense problem per residue class of (y % r, x % r) with strided
//                token addresses, inside which every pair is admitted (kMaskFull).
enum MaskKind : int { kMaskDisc = 0, kMaskSquare = 1, kMaskSwin = 2, kMaskStrided = 3, kMaskFull = 4 };

struct MaskSpec {
    int kind;
    int r;      // radius (disc, square) or window size (Swin)
    int shift;  // Swin only, 0 <= shift < r
};

// The mask between two image tokens.
__host__ __device__ inline bool mask_admits(const MaskSpec& m, int qy, int qx, int ky, int kx)
{
    const int dy = qy - ky, dx = qx - kx;
    if (m.kind == kMaskSquare) return dy < m.r && -dy < m.r && dx < m.r && -dx < m.r;
    if (m.kind == kMaskSwin) return (qy + m.shift) / m.r == (ky + m.shift) / m.r && (qx + m.shift) / m.r == (kx + m.shift) / m.r;
    if (m.kind == kMaskStrided) return ((-dx % m.r) + m.r) % m.r == m.shift % m.r && ((-dy % m.r) + m.r) % m.r == (m.shift / m.r) % m.r;
    if (m.kind == kMaskFull) return true;
    return dx * dx + dy * dy < m.r * m.r;
}

// Square and Swin windows factor into one condition per axis: mask_admits = axis_admits(rows) && axis_admits(columns).
__host__ __device__ inline bool axis_admits(int kind, int r, int shift, int q, int k)
{
    if (kind == kMaskSwin) return (q + shift) / r == (k + shift) / r;
    return q - k < r && k - q < r;  // square window
}

// classify_image_block for any mask kind (same meaning of skip / full / partial).
__host__ __device__ inline int classify_image_block_spec(const MaskSpec& m, int qy0, int qx0, int qh, int qw, int ky0, int kx0,
                                                         int kh, int kw, int gridH, int gridW)
{
    if (m.kind == kMaskDisc) return classify_image_block(qy0, qx0, qh, qw, ky0, kx0, kh, kw, gridH, gridW, m.r * m.r);
    if (qy0 >= gridH || qx0 >= gridW || ky0 >= gridH || kx0 >= gridW) return kBlockSkip;
    const int qy1 = imin(qy0 + qh, gridH) - 1, qx1 = imin(qx0 + qw, gridW) - 1;
    const int ky1 = imin(ky0 + kh, gridH) - 1, kx1 = imin(kx0 + kw, gridW) - 1;
    const bool inside = (ky0 + kh <= gridH) && (kx0 + kw <= gridW);
    if (m.kind == kMaskSquare) {
        const int dy_min = imax(0, imax(ky0 - qy1, qy0 - ky1)), dx_min = imax(0, imax(kx0 - qx1, qx0 - kx1));
        if (dy_min >= m.r || dx_min >= m.r) return kBlockSkip;
        const int dy_max = imax(qy0 + qh - 1 - ky0, ky0 + kh - 1 - qy0), dx_max = imax(qx0 + qw - 1 - kx0, kx0 + kw - 1 - qx0);
        return (inside && dy_max < m.r && dx_max < m.r) ? kBlockFull : kBlockPartial;
    }
    // Swin: ranges of window indices covered by the (clipped) patch and block, per axis
    const int wqy0 = (qy0 + m.shift) / m.r, wqy1 = (qy1 + m.shift) / m.r, wky0 = (ky0 + m.shift) / m.r, wky1 = (ky1 + m.shift) / m.r;
    const int wqx0 = (qx0 + m.shift) / m.r, wqx1 = (qx1 + m.shift) / m.r, wkx0 = (kx0 + m.shift) / m.r, wkx1 = (kx1 + m.shift) / m.r;
    if (wqy1 < wky0 || wky1 < wqy0 || wqx1 < wkx0 || wkx1 < wqx0) return kBlockSkip;
    // full: the unclipped patch and the block each lie in one window, the same one
    const int uqy1 = (qy0 + qh - 1 + m.shift) / m.r, uqx1 = (qx0 + qw - 1 + m.shift) / m.r;
    const bool one = wqy0 == uqy1 && wky0 == wky1 && wqy0 == wky0 && wqx0 == uqx1 && wkx0 == wkx1 && wqx0 == wkx0;
    return (inside && one) ? kBlockFull : kBlockPartial;
}

// Every pair admitted (one residue class of the strided mask): the query patch lives on a qH x qW grid, the key
// block on a kH x kW grid of its own.
__host__ __device__ inline int classify_full_block(int qy0, int qx0, int qH, int qW, int ky0, int kx0, int kh, int kw, int kH, int kW)
{
    if (qy0 >= qH || qx0 >= qW || ky0 >= kH || kx0 >= kW) return kBlockSkip;
    return (ky0 + kh <= kH && kx0 + kw <= kW) ? kBlockFull : kBlockPartial;
}

// Keys taken from a contiguous token range [.., limit): block = tokens [base, base + n).
__host__ __device__ inline int classify_linear_block(long long base, int n, long long limit)
{
    if (base >= limit) return kBlockSkip;
    return (base + n <= limit) ? kBlockFull : kBlockPartial;
}

}  // namespace clear
