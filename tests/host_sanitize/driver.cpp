// Host-side entry points of the library run under the host sanitizers (AddressSanitizer + UndefinedBehaviorSanitizer),
// on a machine without a GPU: the schedule builder on ragged, thin, tiny and large shapes and every mask kind, the
// lattice counts, the lane-mask tables, the per-wave tile descriptors, the band layout, and the argument checks of the calls that need a device
// (each must return an error code before any launch).  Results are cross-checked where a second way to get them
// exists; the point of the run is that no sanitizer report appears.  Exit code 0 = clean.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/clear_attn.h"
#include "../../paper_2412_16112_amd/csrc/block_class.h"
#include "../../paper_2412_16112_amd/csrc/clear_internal.h"

static int failures = 0;
#define EXPECT(cond)                                                       \
    do {                                                                   \
        if (!(cond)) {                                                     \
            std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); \
            ++failures;                                                    \
        }                                                                  \
    } while (0)

static void schedules()
{
    const int shapes[][3] = {{16, 16, 4},   {20, 28, 4}, {64, 64, 16}, {33, 17, 9}, {24, 40, 16}, {7, 5, 1},
                             {9, 70, 32},   {1, 1, 3},   {1, 200, 5},  {200, 1, 5}, {128, 128, 8}, {192, 320, 32},
                             {40, 40, 1000}, {17, 3, 2}};
    const int tiles[][4] = {{16, 16, 8, 8}, {4, 8, 4, 8}, {2, 2, 1, 2}, {8, 16, 8, 8}, {3, 5, 7, 2}};
    const int kinds[][2] = {{CLEAR_MASK_DISC, 0}, {CLEAR_MASK_SQUARE, 0}, {CLEAR_MASK_SWIN, 0}, {CLEAR_MASK_SWIN, 1}};
    for (const auto& sh : shapes)
        for (const auto& tl : tiles)
            for (const auto& kd : kinds) {
                const int r = sh[2], shift = kd[1] < r ? kd[1] : 0;
                int nq = 0;
                long long np = 0;
                int rc = clear_attn_schedule_host_masked(sh[0], sh[1], r, kd[0], shift, tl[0], tl[1], tl[2], tl[3], &nq, &np, nullptr, nullptr, nullptr);
                EXPECT(rc == CLEAR_OK);
                std::vector<int> row_ptr((size_t)nq + 1), col((size_t)np + 1);
                std::vector<unsigned char> flags((size_t)np + 1);
                rc = clear_attn_schedule_host_masked(sh[0], sh[1], r, kd[0], shift, tl[0], tl[1], tl[2], tl[3], &nq, &np, row_ptr.data(), col.data(),
                                                     flags.data());
                EXPECT(rc == CLEAR_OK);
                EXPECT(row_ptr[0] == 0 && row_ptr[(size_t)nq] == np);
                const int n_kt = ((sh[0] + tl[2] - 1) / tl[2]) * ((sh[1] + tl[3] - 1) / tl[3]);
                for (long long e = 0; e < np; ++e) EXPECT(col[(size_t)e] >= 0 && col[(size_t)e] < n_kt && flags[(size_t)e] <= 1);
                for (int q = 0; q < nq; ++q)
                    for (int e = row_ptr[(size_t)q] + 1; e < row_ptr[(size_t)q + 1]; ++e) EXPECT(col[(size_t)e - 1] < col[(size_t)e]);
            }
    // the pair bound is an upper bound, and refuses what would not fit int indices
    EXPECT(clear::schedule_pair_bound(64, 64, 16, 16, 16, 8, 8) >= 4 * 4 * 36 - 200);
    int nq = 0;
    long long np = 0;
    EXPECT(clear_attn_schedule_host(32767, 32767, 32768, 16, 16, 8, 8, &nq, &np, nullptr, nullptr, nullptr) == CLEAR_ERR_UNSUPPORTED);
    EXPECT(clear_attn_schedule_host(0, 4, 1, 16, 16, 8, 8, &nq, &np, nullptr, nullptr, nullptr) == CLEAR_ERR_INVALID_ARG);
    EXPECT(clear_attn_schedule_host(4, 4, 1, 16, 16, 8, 0, &nq, &np, nullptr, nullptr, nullptr) == CLEAR_ERR_INVALID_ARG);
    EXPECT(clear_attn_schedule_host(4, 4, 1, 16, 16, 8, 8, nullptr, &np, nullptr, nullptr, nullptr) == CLEAR_ERR_INVALID_ARG);
    EXPECT(clear_attn_schedule_host_masked(32, 32, 4, CLEAR_MASK_STRIDED, 0, 16, 16, 8, 8, &nq, &np, nullptr, nullptr, nullptr) == CLEAR_ERR_UNSUPPORTED);
}

static void counts()
{
    // sum(M) against a visit of every pair, on shapes small enough for that
    const int shapes[][4] = {{8, 16, 16, 4}, {0, 9, 13, 3}, {5, 7, 5, 1}, {3, 12, 10, 40}, {2, 20, 28, 6}};
    for (const auto& sh : shapes) {
        const int n_text = sh[0], gh = sh[1], gw = sh[2], r = sh[3];
        for (int kind = 0; kind < 4; ++kind) {
            const int shift = kind == CLEAR_MASK_SWIN ? r / 2 : (kind == CLEAR_MASK_STRIDED ? r + 1 : 0);
            if (kind == CLEAR_MASK_SWIN && shift >= r) continue;
            unsigned long long got = 0;
            EXPECT(clear_attn_mask_count_masked(n_text, gh, gw, r, kind, shift, &got) == CLEAR_OK);
            const clear::MaskSpec spec = {kind, r, shift};
            const long long N = n_text + (long long)gh * gw;
            unsigned long long want = (unsigned long long)n_text * N + (unsigned long long)gh * gw * n_text;
            for (int qy = 0; qy < gh; ++qy)
                for (int qx = 0; qx < gw; ++qx)
                    for (int ky = 0; ky < gh; ++ky)
                        for (int kx = 0; kx < gw; ++kx) want += clear::mask_admits(spec, qy, qx, ky, kx) ? 1 : 0;
            EXPECT(got == want);
        }
    }
    unsigned long long v = 0;
    EXPECT(clear_attn_mask_count(512, 512, 512, 16, &v) == CLEAR_OK && v == 471125568ull);
    EXPECT(clear_attn_mask_count(512, 32767, 32767, 32768, &v) == CLEAR_OK);
    EXPECT(clear_attn_mask_count(-1, 4, 4, 1, &v) == CLEAR_ERR_INVALID_ARG);
    EXPECT(clear_attn_mask_count(1, 4, 4, 1, nullptr) == CLEAR_ERR_INVALID_ARG);
}

static void mask_tables()
{
    for (int r : {1, 2, 5, 8, 16, 33})
        for (int kind : {CLEAR_MASK_DISC, CLEAR_MASK_SQUARE}) {
            const int ry = (r + 2) / 4, rx = (r + 6) / 8;
            std::vector<unsigned long long> tbl;
            clear::build_bf16_mask_table(r, ry, rx, kind, &tbl);
            EXPECT(tbl.size() == (size_t)((2 * ry + 1) * (2 * rx + 1) + 2) * 16);
            // entry (0, 0), register 0: lane l keeps key slot 4 (l / 32) of the block against query l % 32
            const unsigned long long w = tbl[(size_t)(ry * (2 * rx + 1) + rx) * 16];
            for (int l = 0; l < 64; ++l) {
                const int dy = -((l & 31) >> 3), dx = 4 * (l >> 5) - (l & 7);
                const bool want = kind == CLEAR_MASK_DISC ? dx * dx + dy * dy < r * r : (dx < r && -dx < r && -dy < r);
                EXPECT(((w >> l) & 1) == (want ? 1u : 0u));
            }
            EXPECT(tbl[tbl.size() - 32] == ~0ull && tbl[tbl.size() - 1] == 0ull);
        }
}

// The per-wave tile descriptors the kernels follow against the classification they replace and against the count of
// executed pairs the library reports: every wave that runs a tile runs both of its 32-key blocks.
static void wave_descriptors()
{
    using namespace clear;
    const int shapes[][4] = {{64, 64, 16, 512}, {40, 56, 8, 300}, {33, 17, 9, 0}, {128, 128, 16, 70}, {24, 40, 100, 5}, {7, 5, 1, 8}, {96, 96, 32, 512}};
    for (const auto& sh : shapes)
        for (int kind : {CLEAR_MASK_DISC, CLEAR_MASK_SQUARE}) {
            const int gh = sh[0], gw = sh[1], r = sh[2], n_text = sh[3];
            Schedule sc;
            build_schedule(gh, gw, r, kBf16QTileH, kBf16QTileW, kKeyTileH, kKeyTileW, &sc, kind, 0);
            // kernel order of the tile lists: tiles inside the grid first (any order will do here), then the cut ones
            std::vector<int> k_col(sc.col_idx.size()), n_plain(sc.row_ptr.size() - 1, 0);
            auto cut = [&](int id) { return (id / sc.n_ktx + 1) * sc.kth > gh || (id % sc.n_ktx + 1) * sc.ktw > gw; };
            auto origin = [&](int id) { return ((id / sc.n_ktx) * sc.kth) << 16 | ((id % sc.n_ktx) * sc.ktw); };
            for (size_t qt = 0; qt + 1 < sc.row_ptr.size(); ++qt) {
                int w = sc.row_ptr[qt];
                for (int e = sc.row_ptr[qt]; e < sc.row_ptr[qt + 1]; ++e)
                    if (!cut(sc.col_idx[e])) k_col[(size_t)w++] = origin(sc.col_idx[e]);
                n_plain[qt] = w - sc.row_ptr[qt];
                for (int e = sc.row_ptr[qt]; e < sc.row_ptr[qt + 1]; ++e)
                    if (cut(sc.col_idx[e])) k_col[(size_t)w++] = origin(sc.col_idx[e]);
            }
            const int ry = std::min((r + 2) / 4, (gh + 3) / 4), rx = std::min((r + 6) / 8, (gw + 7) / 8);
            const int ncol = 2 * rx + 1, ones = (2 * ry + 1) * ncol, zeros = ones + 1;
            std::vector<int> desc;
            build_wave_descriptors(sc, k_col, n_plain, ry, rx, &desc);
            const int waves = kBf16NWY * kBf16NWX;
            EXPECT(desc.size() == k_col.size() * (size_t)waves);
            const MaskSpec spec = {kind, r, 0};
            unsigned long long run_tiles = 0;  // (wave, tile) pairs that are run: plain tiles from the descriptors, cut tiles classified here
            for (size_t qt = 0; qt + 1 < sc.row_ptr.size(); ++qt)
                for (int e = sc.row_ptr[qt]; e < sc.row_ptr[qt + 1]; ++e)
                    for (int w = 0; w < waves; ++w) {
                        const int wy0 = (int)(qt / sc.n_qtx) * sc.qth + (w / kBf16NWX) * kWaveQH, wx0 = (int)(qt % sc.n_qtx) * sc.qtw + (w % kBf16NWX) * kWaveQW;
                        const int ta = k_col[(size_t)e] >> 16, tb = k_col[(size_t)e] & 0xffff;
                        const int c0 = classify_image_block_spec(spec, wy0, wx0, kWaveQH, kWaveQW, ta, tb, kKeyBlockH, kKeyBlockW, gh, gw);
                        const int c1 = classify_image_block_spec(spec, wy0, wx0, kWaveQH, kWaveQW, ta + kKeyBlockH, tb, kKeyBlockH, kKeyBlockW, gh, gw);
                        const bool any = c0 != kBlockSkip || c1 != kBlockSkip;
                        const int d = desc[(size_t)e * waves + w];
                        if (e < sc.row_ptr[qt] + n_plain[qt]) {
                            EXPECT((d != kWaveSkipsTile) == any);
                            if (d != kWaveSkipsTile) {
                                const int i0 = d & 0xffff, i1 = (int)((unsigned)d >> 16);
                                EXPECT((i0 == zeros) == (c0 == kBlockSkip) && (i0 == ones) == (c0 == kBlockFull));
                                EXPECT((i1 == zeros) == (c1 == kBlockSkip) && (i1 == ones) == (c1 == kBlockFull));
                                EXPECT(i0 >= 0 && i0 <= zeros && i1 >= 0 && i1 <= zeros);
                                if (c0 == kBlockPartial) EXPECT(i0 == (((ta - wy0) >> 2) + ry) * ncol + ((tb - wx0) >> 3) + rx);
                            }
                        } else {
                            EXPECT(d == kWaveSkipsTile);  // cut tiles are classified in the kernel
                        }
                        if (wy0 < gh && wx0 < gw) run_tiles += any;
                    }
            // executed pairs of the library: 2 blocks x 1024 pairs per run tile, the text tiles of every wave with queries, the text-query pass
            sc.mask_kind = kind;
            unsigned long long text_tile_runs = 0;
            for (size_t qt = 0; qt + 1 < sc.row_ptr.size(); ++qt)
                for (int w = 0; w < waves; ++w) {
                    const int wy0 = (int)(qt / sc.n_qtx) * sc.qth + (w / kBf16NWX) * kWaveQH, wx0 = (int)(qt % sc.n_qtx) * sc.qtw + (w % kBf16NWX) * kWaveQW;
                    if (wy0 < gh && wx0 < gw) text_tile_runs += (unsigned long long)((n_text + 63) / 64);
                }
            const long long N = n_text + (long long)gh * gw;
            const unsigned long long text_query = (unsigned long long)((n_text + 31) / 32) * 2ull * (unsigned long long)((N + 63) / 64);
            EXPECT(executed_pairs_bf16(sc, n_text, 0) == (2ull * (run_tiles + text_tile_runs) + text_query) * 1024ull);
        }
}

static void bands_and_argument_checks()
{
    int y0, y1, ht, hb;
    int covered = 0;
    for (int b = 0; b < 8; ++b) {
        EXPECT(clear_attn_band_layout(512, 16, 8, b, &y0, &y1, &ht, &hb) == CLEAR_OK);
        EXPECT(y0 == covered && y1 - y0 == 64);
        covered = y1;
    }
    EXPECT(clear_attn_band_layout(64, 16, 8, 0, &y0, &y1, &ht, &hb) == CLEAR_ERR_UNSUPPORTED);
    EXPECT(clear_attn_band_layout(8, 4, 2, 2, &y0, &y1, &ht, &hb) == CLEAR_ERR_INVALID_ARG);
    int a, b2, c, d;
    EXPECT(clear_attn_tile_shape(128, CLEAR_BF16, &a, &b2, &c, &d) == CLEAR_OK && a == 16 && b2 == 16 && c == 8 && d == 8);
    EXPECT(clear_attn_tile_shape(128, CLEAR_F32, &a, &b2, &c, &d) == CLEAR_ERR_UNSUPPORTED);
    // calls that need a device: every argument error is found first
    clear_attn_ctx* ctx = nullptr;
    EXPECT(clear_attn_create(nullptr, 8, 16, 16, 128, 4, CLEAR_BF16) == CLEAR_ERR_INVALID_ARG);
    EXPECT(clear_attn_create(&ctx, 8, 0, 16, 128, 4, CLEAR_BF16) == CLEAR_ERR_INVALID_ARG);
    EXPECT(clear_attn_create(&ctx, 8, 16, 16, 96, 4, CLEAR_BF16) == CLEAR_ERR_UNSUPPORTED);
    EXPECT(clear_attn_create(&ctx, 8, 16, 16, 128, 0, CLEAR_BF16) == CLEAR_ERR_INVALID_ARG);
    EXPECT(clear_attn_create(&ctx, 512, 8192, 8192, 128, 16, CLEAR_BF16) == CLEAR_ERR_UNSUPPORTED);  // N >= 2^24
    EXPECT(clear_attn_create_masked(&ctx, 8, 16, 16, 128, 4, CLEAR_BF16, 9, 0) == CLEAR_ERR_INVALID_ARG);
    EXPECT(clear_attn_create_masked(&ctx, 8, 16, 16, 128, 4, CLEAR_BF16, CLEAR_MASK_SWIN, 4) == CLEAR_ERR_INVALID_ARG);
    EXPECT(ctx == nullptr);
    EXPECT(clear_attn_last_error(nullptr) != nullptr);
    float dummy[4] = {0};
    EXPECT(clear_attn_forward(nullptr, dummy, dummy, dummy, dummy, 1, 1, 8, 16, 16, 128, 4, nullptr) == CLEAR_ERR_INVALID_ARG);
    EXPECT(clear_attn_forward_noalloc(nullptr, dummy, dummy, dummy, dummy, 1, 1, 8, 16, 16, 128, 4, nullptr) == CLEAR_ERR_INVALID_ARG);
    EXPECT(clear_attn_reserve(nullptr, 1) == CLEAR_ERR_INVALID_ARG);
    const float* parts[1] = {dummy};
    EXPECT(clear_attn_merge_text(0, parts, parts, 1, 1, 8, 264, 128, CLEAR_MERGE_EXACT, dummy, CLEAR_BF16, nullptr) == CLEAR_ERR_INVALID_ARG);
    EXPECT(clear_attn_merge_text(1, parts, parts, 1, 1, 8, 4, 128, CLEAR_MERGE_EXACT, dummy, CLEAR_BF16, nullptr) == CLEAR_ERR_INVALID_ARG);
    clear_attn_destroy(nullptr);
}

int main()
{
    schedules();
    counts();
    mask_tables();
    wave_descriptors();
    bands_and_argument_checks();
    if (failures) {
        std::printf("%d check(s) failed\n", failures);
        return 1;
    }
    std::printf("host entry points clean under the sanitizers\n");
    return 0;
}
