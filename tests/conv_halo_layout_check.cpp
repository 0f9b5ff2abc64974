// Host-side model of the halo-staged convolution kernel's LDS data path and tile plan, compiled from the
// header the kernel uses (csrc/conv_halo_layout.h): the slot map of the direct-to-LDS loads against the
// layout function, every fragment of every tap against the definition of the convolution's gather, the
// bank groups a fragment read touches, the division by multiplication, and the plan's cuts and model time
// against a simulation of the CUs.
#include <cstdio>
#include <cstdlib>
#include <queue>
#include <vector>

#include "../paper_2604_01489_amd/csrc/conv_halo_layout.h"

using namespace ge_halo;

static int fails = 0;
#define CHECK(c, ...) do { if (!(c)) { if (fails < 20) { printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } ++fails; } } while (0)

// one 16-byte chunk of the input: (input row, input column, chunk of 8 channels), or "zero" for padding
struct Chunk { int ih, iw, c; bool zero; bool written; };

static void check_tile(int H, int W, int ph, int pw, int oh0, int R)
{
    const int OW = W + 2 * pw - 2, OH = H + 2 * ph - 2;
    if (OW < 1 || OW > MAX_OW || oh0 + R > OH) return;
    std::vector<Chunk> lds(HALO_BUF_BYTES / 16, Chunk{0, 0, 0, false, false});
    // the loads: halo row j by the four waves; a row outside the image or beyond R + 2 is not read (zeros land)
    for (int j = 0; j < HALO_ROWS; ++j)
        for (int w = 0; w < 4; ++w)
            for (int lane = 0; lane < 64; ++lane) {
                const int at = j * HALO_ROW_BYTES + w * 1024 + 16 * lane;
                const int col = halo_slot_col(w, lane), c = halo_slot_chunk(w, lane);
                CHECK(at == halo_offset(j * HALO_PITCH + col, c), "slot map row %d wave %d lane %d", j, w, lane);
                const int ih = oh0 - ph + j, iw = col - pw;
                const bool live = j < R + 2 && ih >= 0 && ih < H && iw >= 0 && iw < W;
                CHECK(!lds[at / 16].written, "two lanes land on one chunk");
                lds[at / 16] = Chunk{ih, iw, c, !live, true};
            }
    // the fragments: output position pos of the tile, tap (dh, dw), lane group c
    const int posMul = 65536 / OW + 1;
    for (int pos = 0; pos < R * OW; ++pos) {
        CHECK(((pos * posMul) >> 16) == pos / OW, "division by multiplication pos %d OW %d", pos, OW);
        for (int dh = 0; dh < 3; ++dh)
            for (int dw = 0; dw < 3; ++dw)
                for (int c = 0; c < 4; ++c) {
                    const int at = halo_offset(halo_pos(pos, OW, dw), c) + dh * HALO_ROW_BYTES;
                    CHECK(at >= 0 && at + 16 <= HALO_ROWS * HALO_ROW_BYTES, "fragment read outside the halo");
                    const Chunk &g = lds[at / 16];
                    const int ih = oh0 + pos / OW - ph + dh, iw = pos % OW - pw + dw;
                    const bool inside = ih >= 0 && ih < H && iw >= 0 && iw < W;
                    CHECK(g.written, "fragment reads a chunk no load wrote");
                    if (inside) CHECK(!g.zero && g.ih == ih && g.iw == iw && g.c == c, "pos %d tap %d,%d chunk %d: got (%d,%d,%d)", pos, dh, dw, c, g.ih, g.iw, g.c);
                    else CHECK(g.zero, "pos %d tap %d,%d: padding must read zeros", pos, dh, dw);
                }
    }
}

// 8 positions in a row of the halo, same chunk: 8 different 16-byte bank groups (128 bytes = all 32 banks once)
static void check_banks()
{
    for (int h0 = 0; h0 + 8 <= HALO_PITCH * HALO_ROWS; ++h0)
        for (int c = 0; c < 4; ++c) {
            unsigned seen = 0;
            for (int l = 0; l < 8; ++l) seen |= 1u << ((halo_offset(h0 + l, c) / 16) % 8);
            CHECK(seen == 0xffu, "bank groups of positions %d.. chunk %d: %02x", h0, c, seen);
        }
}

// the launch as the device runs it: tiles taken in order by whichever CU is free first
static long long simulate(long long n1, int c1, long long n2, int c2, int cus)
{
    std::priority_queue<long long, std::vector<long long>, std::greater<long long>> free_at;
    for (int i = 0; i < cus; ++i) free_at.push(0);
    long long end = 0;
    for (long long t = 0; t < n1 + n2; ++t) {
        long long at = free_at.top();
        free_at.pop();
        at += t < n1 ? c1 : c2;
        if (at > end) end = at;
        free_at.push(at);
    }
    return end;
}

static void check_plan()
{
    // the 56 x 56 workload: 32 images, one tile column, 256 CUs -> 8 groups of 4 rows and 8 of 3 per image
    const HaloPlan p = halo_plan(32, 56, 56, 1, 256, 2, 14, 11);
    CHECK(p.R1 == 4 && p.g1 == 8 && p.R2 == 3 && p.g2 == 8, "56 x 56: %d x %d + %d x %d", p.g1, p.R1, p.g2, p.R2);
    CHECK(p.cost == 16 + 13, "56 x 56 model time %lld", p.cost);
    srand(7);
    for (int it = 0; it < 3000; ++it) {
        const int images = 1 + rand() % 64, OH = 1 + rand() % 80, OW = 1 + rand() % MAX_OW, tilesN = 1 + rand() % 3;
        const int tmb1 = 8 + rand() % 9, tmb2 = 4 + rand() % (tmb1 - 3), ovh = rand() % 4;
        const HaloPlan q = halo_plan(images, OH, OW, tilesN, 256, ovh, tmb1, tmb2);
        if (q.cost < 0) {
            CHECK(OW > tmb1 * 16, "a single row of %d fits %d blocks, yet no plan", OW, tmb1);
            continue;
        }
        CHECK(q.R1 * q.g1 + q.R2 * q.g2 == OH, "cut does not cover the rows");
        CHECK(q.R1 >= 1 && q.R1 <= MAX_R && q.R2 >= 1 && q.R2 <= q.R1, "rows per tile");
        CHECK(q.R1 * OW <= tmb1 * 16 && (q.g2 == 0 || q.R2 * OW <= tmb2 * 16), "tile larger than the variant's loop");
        const long long n1 = (long long)images * q.g1 * tilesN, n2 = (long long)images * q.g2 * tilesN;
        const long long sim = simulate(n1, tmb1 + ovh, n2, tmb2 + ovh, 256);
        // the closed form bounds the simulated time from above and stays within one short tile of it
        CHECK(q.cost >= sim && q.cost <= sim + tmb2 + ovh, "model %lld, simulated %lld (n1 %lld n2 %lld c %d %d)", q.cost, sim, n1, n2,
              tmb1 + ovh, tmb2 + ovh);
    }
}

int main()
{
    check_banks();
    for (int W = 1; W <= MAX_OW; W += (W < 8 ? 1 : 5))
        for (int pw = 0; pw <= 2; ++pw)
            for (int ph = 0; ph <= 2; ++ph)
                for (int R = 1; R <= MAX_R; ++R)
                    for (int oh0 = 0; oh0 < 7; oh0 += 3) check_tile(8, W, ph, pw, oh0, R);
    check_tile(56, 56, 1, 1, 0, 4);
    check_tile(56, 56, 1, 1, 53, 3);
    check_tile(56, 56, 1, 1, 32, 3);
    check_tile(62, 62, 1, 1, 57, 5);
    check_tile(60, 60, 2, 2, 0, 4);
    check_plan();
    if (fails) { printf("%d checks failed\n", fails); return 1; }
    printf("conv halo layout checks passed\n");
    return 0;
}
