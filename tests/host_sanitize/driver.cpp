// Host-side entry points of the library run under the host sanitizers (AddressSanitizer + UndefinedBehaviorSanitizer),
// on a machine without a GPU: the schedule builder on ragged, thin, tiny and large shapes and every mask kind, the
// lattice counts, the lane-mask tables, the band layout, and the argument checks of the calls that need a device
// (each must return an error code before any launch).  Results are cross-checked where a second way to get them
// exists; the point of the run is that no sanitizer report appears.  Exit code 0 = clean.
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
    bands_and_argument_checks();
    if (failures) {
        std::printf("%d check(s) failed\n", failures);
        return 1;
    }
    std::printf("host entry points clean under the sanitizers\n");
    return 0;
}
