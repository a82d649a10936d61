// Host-side integer geometry of the CLEAR mask (Eq. 3, Sec. 3.2): tile schedule, sum(M), and the
// count of pairs the kernels execute.  No device code here.
#include "block_class.h"
#include "clear_internal.h"

namespace clear {

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline long long imin_ll(long long a, long long b) { return a < b ? a : b; }

// Smallest |a - b| for a in [a0, a1], b in [b0, b1].
static inline int interval_gap(int a0, int a1, int b0, int b1)
{
    if (b0 > a1) return b0 - a1;
    if (a0 > b1) return a0 - b1;
    return 0;
}

long long schedule_pair_bound(int gridH, int gridW, int r, int qth, int qtw, int kth, int ktw)
{
    // per query tile: the rectangle of key tiles that come within r - 1 on each axis (what build_schedule scans)
    const int n_qty = ceil_div(gridH, qth), n_qtx = ceil_div(gridW, qtw), n_kty = ceil_div(gridH, kth), n_ktx = ceil_div(gridW, ktw);
    long long rows = 0, cols = 0;  // the count factorises over the two axes
    for (int ty = 0; ty < n_qty; ++ty) {
        const int qy0 = ty * qth, qy1 = imin(qy0 + qth, gridH) - 1;
        const long long lo = imax(0, (int)(((long long)qy0 - (r - 1)) / kth) - 1), hi = imin(n_kty - 1, (int)imin_ll(((long long)qy1 + r - 1) / kth, n_kty));
        rows += hi >= lo ? hi - lo + 1 : 0;
    }
    for (int tx = 0; tx < n_qtx; ++tx) {
        const int qx0 = tx * qtw, qx1 = imin(qx0 + qtw, gridW) - 1;
        const long long lo = imax(0, (int)(((long long)qx0 - (r - 1)) / ktw) - 1), hi = imin(n_ktx - 1, (int)imin_ll(((long long)qx1 + r - 1) / ktw, n_ktx));
        cols += hi >= lo ? hi - lo + 1 : 0;
    }
    return rows * cols;
}

void build_schedule(int gridH, int gridW, int r, int qth, int qtw, int kth, int ktw, Schedule* s, int mask_kind, int mask_shift)
{
    s->gridH = gridH; s->gridW = gridW; s->r = r;
    s->mask_kind = mask_kind; s->mask_shift = mask_shift;
    s->qth = qth; s->qtw = qtw; s->kth = kth; s->ktw = ktw;
    s->n_qty = ceil_div(gridH, qth); s->n_qtx = ceil_div(gridW, qtw);
    s->n_kty = ceil_div(gridH, kth); s->n_ktx = ceil_div(gridW, ktw);
    s->row_ptr.assign(1, 0);
    s->col_idx.clear();
    s->flags.clear();
    const long long r2 = (long long)r * r;
    for (int ty = 0; ty < s->n_qty; ++ty)
        for (int tx = 0; tx < s->n_qtx; ++tx) {
            // extent of the query tile inside the grid
            const int qy0 = ty * qth, qy1 = imin(qy0 + qth, gridH) - 1;
            const int qx0 = tx * qtw, qx1 = imin(qx0 + qtw, gridW) - 1;
            const bool q_inside = (qy0 + qth <= gridH) && (qx0 + qtw <= gridW);
            // key tiles that can come within distance r-1 on each axis
            const int kty_lo = imax(0, (qy0 - (r - 1)) / kth - 1), kty_hi = imin(s->n_kty - 1, (qy1 + r - 1) / kth);
            const int ktx_lo = imax(0, (qx0 - (r - 1)) / ktw - 1), ktx_hi = imin(s->n_ktx - 1, (qx1 + r - 1) / ktw);
            for (int ky = kty_lo; ky <= kty_hi; ++ky)
                for (int kx = ktx_lo; kx <= ktx_hi; ++kx) {
                    const int ky0 = ky * kth, ky1 = imin(ky0 + kth, gridH) - 1;
                    const int kx0 = kx * ktw, kx1 = imin(kx0 + ktw, gridW) - 1;
                    const long long dy = interval_gap(qy0, qy1, ky0, ky1), dx = interval_gap(qx0, qx1, kx0, kx1);
                    const bool k_inside = (ky0 + kth <= gridH) && (kx0 + ktw <= gridW);
                    const long long fy = imax(qy1 - ky0, ky1 - qy0), fx = imax(qx1 - kx0, kx1 - qx0);
                    bool full;
                    if (mask_kind == kMaskSquare) {
                        if (dy >= r || dx >= r) continue;  // no pair inside the square window: not listed
                        full = q_inside && k_inside && fy < r && fx < r;
                    } else if (mask_kind == kMaskSwin) {
                        // windows (per axis) that the two tiles touch: listed iff they share one
                        const int wq0 = (qy0 + mask_shift) / r, wq1 = (qy1 + mask_shift) / r, wk0 = (ky0 + mask_shift) / r, wk1 = (ky1 + mask_shift) / r;
                        const int vq0 = (qx0 + mask_shift) / r, vq1 = (qx1 + mask_shift) / r, vk0 = (kx0 + mask_shift) / r, vk1 = (kx1 + mask_shift) / r;
                        if (wq1 < wk0 || wk1 < wq0 || vq1 < vk0 || vk1 < vq0) continue;
                        full = q_inside && k_inside && wq0 == wq1 && wk0 == wk1 && wq0 == wk0 && vq0 == vq1 && vk0 == vk1 && vq0 == vk0;
                    } else {
                        if (dy * dy + dx * dx >= r2) continue;  // no pair closer than r: not listed
                        full = q_inside && k_inside && fy * fy + fx * fx < r2;
                    }
                    s->col_idx.push_back(ky * s->n_ktx + kx);
                    s->flags.push_back(full ? 1 : 0);
                }
            s->row_ptr.push_back((int)s->col_idx.size());
        }
}

unsigned long long mask_count(int n_text, int gridH, int gridW, int r, int mask_kind, int mask_shift)
{
    if (mask_kind == kMaskStrided) {
        // a query in column residue a sees the columns of residue (a + r_x) % r; rows likewise; the two axes factorise
        const unsigned long long n_img = (unsigned long long)gridH * gridW, N = n_img + n_text;
        const int rx = mask_shift % r, ry = (mask_shift / r) % r;
        auto count = [&](int n, int a) -> unsigned long long { return a < n ? (unsigned long long)((n - a + r - 1) / r) : 0ull; };
        unsigned long long sx = 0, sy = 0;
        for (int a = 0; a < r; ++a) sx += count(gridW, a) * count(gridW, (a + rx) % r);
        for (int b = 0; b < r; ++b) sy += count(gridH, b) * count(gridH, (b + ry) % r);
        return (unsigned long long)n_text * N + n_img * n_text + sx * sy;
    }
    if (mask_kind == kMaskSwin) {
        // every window of h x w tokens contributes (h w)^2 pairs; windows are the cells of the shifted partition
        const unsigned long long n_img = (unsigned long long)gridH * gridW, N = n_img + n_text;
        unsigned long long sy = 0, sx = 0, img = 0;
        // sum over window rows of h^2 ... the count factorises: sum_{wy, wx} (h_wy w_wx)^2 = (sum h^2)(sum w^2)
        for (int y = 0; y < gridH;) {
            const int end = imin(gridH, ((y + mask_shift) / r + 1) * r - mask_shift);
            sy += (unsigned long long)(end - y) * (end - y);
            y = end;
        }
        for (int x = 0; x < gridW;) {
            const int end = imin(gridW, ((x + mask_shift) / r + 1) * r - mask_shift);
            sx += (unsigned long long)(end - x) * (end - x);
            x = end;
        }
        img = sy * sx;
        return (unsigned long long)n_text * N + n_img * n_text + img;
    }
    // Each offset (dy, dx) of the open disc occurs (gridH - |dy|)(gridW - |dx|) times on the raster.
    const unsigned long long n_img = (unsigned long long)gridH * gridW, N = n_img + n_text;
    unsigned long long img = 0;
    const long long r2 = (long long)r * r;
    for (long long dy = -(r - 1); dy <= r - 1; ++dy) {
        const long long ady = dy < 0 ? -dy : dy;
        if (ady >= gridH) continue;
        for (long long dx = -(r - 1); dx <= r - 1; ++dx) {
            const long long adx = dx < 0 ? -dx : dx;
            if (adx >= gridW || (mask_kind == kMaskDisc && dx * dx + dy * dy >= r2)) continue;  // (square: every |dx|, |dy| < r)
            img += (unsigned long long)(gridH - ady) * (unsigned long long)(gridW - adx);
        }
    }
    return (unsigned long long)n_text * N + n_img * n_text + img;
}

// Lane masks of the bf16 kernels for a (4 x 8 query patch, 4 x 8 key block) pair whose origins differ by
// (4 dby, 8 dbx), |dby| <= ry, |dbx| <= rx: entry (dby + ry) * (2 rx + 1) + dbx + rx holds 16 words, one per
// score register r; bit l is set iff lane l (query l % 32 of the patch, key slot 8 (r/4) + 4 (l/32) + r % 4
// of the block) is admitted by the mask: Eq. 3, dx^2 + dy^2 < r^2, or the square window |dx| < r and |dy| < r
// (the two kinds that depend on the offset alone).  Two more entries follow: all ones, all zeros.
void build_bf16_mask_table(int r, int ry, int rx, int mask_kind, std::vector<unsigned long long>* tbl)
{
    const MaskSpec spec = {mask_kind, r, 0};
    const long long r2 = (long long)r * r;
    const int ncol = 2 * rx + 1;
    tbl->assign((size_t)((2 * ry + 1) * ncol + 2) * 16, 0ull);
    for (int dby = -ry; dby <= ry; ++dby)
        for (int dbx = -rx; dbx <= rx; ++dbx) {
            unsigned long long* e = tbl->data() + (size_t)((dby + ry) * ncol + dbx + rx) * 16;
            for (int reg = 0; reg < 16; ++reg)
                for (int l = 0; l < 64; ++l) {
                    const int qi = l & 31, hh = l >> 5;
                    const long long dy = 4 * dby + (reg >> 2) - (qi >> 3);
                    const long long dx = 8 * dbx + 4 * hh + (reg & 3) - (qi & 7);
                    const bool in_reach = dx > -r && dx < r && dy > -r && dy < r;  // (also keeps the products below in range)
                    if (in_reach && (mask_kind == kMaskDisc ? dx * dx + dy * dy < r2 : mask_admits(spec, 0, 0, (int)dy, (int)dx))) e[reg] |= 1ull << l;
                }
        }
    unsigned long long* ones = tbl->data() + tbl->size() - 32;
    for (int reg = 0; reg < 16; ++reg) ones[reg] = ~0ull;
}

void build_wave_descriptors(const Schedule& s, const std::vector<int>& k_col, const std::vector<int>& n_plain, int mask_ry, int mask_rx,
                            std::vector<int>* desc)
{
    const int nwy = s.qth / kWaveQH, nwx = s.qtw / kWaveQW, waves = nwy * nwx;
    const MaskSpec spec = {s.mask_kind, s.r, s.mask_shift};
    const int ncol = 2 * mask_rx + 1;
    const int ones = (2 * mask_ry + 1) * ncol, zeros = ones + 1;
    desc->assign(k_col.size() * (size_t)waves, kWaveSkipsTile);
    for (size_t qt = 0; qt + 1 < s.row_ptr.size(); ++qt) {
        const int qy0 = (int)(qt / s.n_qtx) * s.qth, qx0 = (int)(qt % s.n_qtx) * s.qtw;
        for (int e = s.row_ptr[qt]; e < s.row_ptr[qt] + n_plain[qt]; ++e) {
            const int ta = k_col[e] >> 16, tb = k_col[e] & 0xffff;
            for (int w = 0; w < waves; ++w) {
                const int wy0 = qy0 + (w / nwx) * kWaveQH, wx0 = qx0 + (w % nwx) * kWaveQW;
                int idx[2];
                bool any = false;
                for (int kb = 0; kb < 2; ++kb) {
                    const int cls = classify_image_block_spec(spec, wy0, wx0, kWaveQH, kWaveQW, ta + kKeyBlockH * kb, tb, kKeyBlockH, kKeyBlockW,
                                                              s.gridH, s.gridW);
                    any |= cls != kBlockSkip;
                    const int dby = ((ta - wy0) >> 2) + kb, dbx = (tb - wx0) >> 3;  // relative block offset in blocks (exact: both are aligned)
                    idx[kb] = cls == kBlockPartial ? (dby + mask_ry) * ncol + dbx + mask_rx : (cls == kBlockFull ? ones : zeros);
                }
                if (any) (*desc)[(size_t)e * waves + w] = idx[0] | (idx[1] << 16);
            }
        }
    }
}

unsigned long long executed_pairs_bf16(const Schedule& s, int n_text, int text_split_keys)
{
    (void)text_split_keys;  // splits are multiples of the 64-key stage: the block count does not depend on them
    const long long N = (long long)n_text + (long long)s.gridH * s.gridW;
    unsigned long long blocks = 0;  // executed (32 query x 32 key) blocks
    const int n_text_tiles = ceil_div(n_text, kKeyTileKeys);
    const int nwy = s.qth / kWaveQH, nwx = s.qtw / kWaveQW;
    const MaskSpec spec = {s.mask_kind, s.r, s.mask_shift};
    for (int ty = 0; ty < s.n_qty; ++ty)
        for (int tx = 0; tx < s.n_qtx; ++tx) {
            const int qt = ty * s.n_qtx + tx;
            for (int wy = 0; wy < nwy; ++wy)
                for (int wx = 0; wx < nwx; ++wx) {
                    const int y0 = ty * s.qth + wy * kWaveQH, x0 = tx * s.qtw + wx * kWaveQW;
                    if (y0 >= s.gridH || x0 >= s.gridW) continue;  // wave has no query: it computes nothing
                    // a wave runs both 32-key blocks of a staged tile, or skips the tile when neither is reachable
                    for (int t = 0; t < n_text_tiles; ++t)
                        blocks += 2 * (classify_linear_block((long long)t * kKeyTileKeys, 32, n_text) != kBlockSkip);
                    for (int e = s.row_ptr[qt]; e < s.row_ptr[qt + 1]; ++e) {
                        const int ky0 = (s.col_idx[e] / s.n_ktx) * s.kth, kx0 = (s.col_idx[e] % s.n_ktx) * s.ktw;
                        bool any = false;
                        for (int kb = 0; kb < 2; ++kb)
                            any |= classify_image_block_spec(spec, y0, x0, kWaveQH, kWaveQW, ky0 + kKeyBlockH * kb, kx0, kKeyBlockH,
                                                             kKeyBlockW, s.gridH, s.gridW) != kBlockSkip;
                        blocks += 2 * any;
                    }
                }
        }
    // text-query pass: every wave that holds at least one text query visits every 32-key block of [0, N)
    const unsigned long long text_waves = (unsigned long long)ceil_div(n_text, kTextQueriesPerWave);
    blocks += text_waves * 2ull * (unsigned long long)((N + kKeyTileKeys - 1) / kKeyTileKeys);
    return blocks * 1024ull;
}

unsigned long long executed_pairs_bf16_strided(const Schedule& s, int n_text, int gridH, int gridW, int stride, int layer)
{
    const long long N = (long long)n_text + (long long)gridH * gridW;
    const int rx = layer % stride, ry = (layer / stride) % stride;
    const int n_text_tiles = ceil_div(n_text, kKeyTileKeys);
    const int nwy = s.qth / kWaveQH, nwx = s.qtw / kWaveQW;
    auto extent = [&](int n, int a) { return a < n ? (n - a + stride - 1) / stride : 0; };
    unsigned long long blocks = 0;
    for (int b = 0; b < stride; ++b)
        for (int a = 0; a < stride; ++a) {
            const int qH = extent(gridH, b), qW = extent(gridW, a);
            const int kH = extent(gridH, (b + ry) % stride), kW = extent(gridW, (a + rx) % stride);
            for (int ty = 0; ty < s.n_qty; ++ty)
                for (int tx = 0; tx < s.n_qtx; ++tx) {
                    const int qt = ty * s.n_qtx + tx;
                    for (int wy = 0; wy < nwy; ++wy)
                        for (int wx = 0; wx < nwx; ++wx) {
                            const int y0 = ty * s.qth + wy * kWaveQH, x0 = tx * s.qtw + wx * kWaveQW;
                            if (y0 >= qH || x0 >= qW) continue;
                            for (int t = 0; t < n_text_tiles; ++t)
                                blocks += 2 * (classify_linear_block((long long)t * kKeyTileKeys, 32, n_text) != kBlockSkip);
                            for (int e = s.row_ptr[qt]; e < s.row_ptr[qt + 1]; ++e) {
                                const int ky0 = (s.col_idx[e] / s.n_ktx) * s.kth, kx0 = (s.col_idx[e] % s.n_ktx) * s.ktw;
                                bool any = false;
                                for (int kb = 0; kb < 2; ++kb)
                                    any |= classify_full_block(y0, x0, qH, qW, ky0 + kKeyBlockH * kb, kx0, kKeyBlockH, kKeyBlockW, kH, kW) != kBlockSkip;
                                blocks += 2 * any;
                            }
                        }
                }
        }
    const unsigned long long text_waves = (unsigned long long)ceil_div(n_text, kTextQueriesPerWave);
    blocks += text_waves * 2ull * (unsigned long long)((N + kKeyTileKeys - 1) / kKeyTileKeys);
    return blocks * 1024ull;
}

unsigned long long executed_pairs_f32(const Schedule& s, int n_text)
{
    const long long N = (long long)n_text + (long long)s.gridH * s.gridW;
    const unsigned long long n_text_tiles = (unsigned long long)ceil_div(n_text, kKeyTileKeys);
    unsigned long long pairs = 0;
    for (size_t qt = 0; qt + 1 < s.row_ptr.size(); ++qt)
        pairs += (n_text_tiles + (unsigned long long)(s.row_ptr[qt + 1] - s.row_ptr[qt])) * kKeyTileKeys * (unsigned long long)(s.qth * s.qtw);
    pairs += (unsigned long long)n_text * (unsigned long long)(((N + kKeyTileKeys - 1) / kKeyTileKeys) * kKeyTileKeys);
    return pairs;
}

}  // namespace clear
