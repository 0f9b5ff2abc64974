// Host-side model of the few-channel convolution kernel's data path, built from the kernel's own index
// header: input rows -> staged images -> five aligned dwords per lane, shifted and masked -> operands
// of the 16 x 16 x 32 matrix instruction -> accumulator lanes -> output channels.  Compared with the
// convolution's definition on small integers (exact).
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#include <vector>

#include "../paper_2604_01489_amd/csrc/conv_rows_layout.h"

using namespace ge_conv_rows;

static int failures = 0;
#define CHECK(c, ...) do { if (!(c)) { if (failures < 20) { std::printf("FAIL %s:%d: ", __FILE__, __LINE__); std::printf(__VA_ARGS__); std::printf("\n"); } ++failures; } } while (0)

// ({hi, lo} >> 8 * shift), low 32 bits: the byte-align instruction
static uint32_t alignbyte(uint32_t hi, uint32_t lo, unsigned shift)
{
    const uint64_t v = ((uint64_t)hi << 32) | lo;
    return (uint32_t)(v >> (8 * (shift & 3)));
}

struct Geo { int H, W, Cin, KH, KW, sh, sw, ph, pw, dh, Cout; };

static void run(const Geo &g, unsigned seed)
{
    const int OH = (g.H + 2 * g.ph - g.dh * (g.KH - 1) - 1) / g.sh + 1;
    const int OW = (g.W + 2 * g.pw - (g.KW - 1) - 1) / g.sw + 1;
    const int kwcin = g.KW * g.Cin, rowElems = g.W * g.Cin, NT = g.Cout / 16;
    CHECK(kwcin <= KSTEP && g.KH <= KH_MAX && OH > 0 && OW > 0, "geometry");
    std::srand(seed);
    // values as small integers kept in 16 bits (the model moves 16-bit patterns; the product is done on them as integers)
    std::vector<int16_t> X((size_t)g.H * rowElems), Wt((size_t)g.Cout * g.KH * kwcin);
    for (auto &v : X) v = (int16_t)(std::rand() % 7 - 3);
    for (auto &v : Wt) v = (int16_t)(std::rand() % 5 - 2);

    // the filter bank as the kernel keeps it in LDS: its dwords, then BANK_PAD dwords (zeros in the kernel;
    // a pattern here, to show that the mask hides whatever lies behind a filter row)
    std::vector<uint32_t> bank(Wt.size() / 2 + BANK_PAD, 0x7fc07fc0u);
    for (size_t d = 0; d < Wt.size() / 2; ++d) bank[d] = (uint32_t)(uint16_t)Wt[2 * d] | ((uint32_t)(uint16_t)Wt[2 * d + 1] << 16);
    {
        const int pd = pitch_dwords(g.W, g.Cin, OW, g.sw, g.pw), front = front_dwords(g.KH, pd, g.Cout);
        CHECK(pd % 64 == 0, "a row is filled by whole wave-wide loads");
        CHECK(front >= 2 * g.KH * pd && front >= g.KH * (g.Cout / 16) * 64 * 4, "row images and fragment table fit in front of the bank");
        CHECK(lds_dwords(g.KH, pd, g.Cout, kwcin) == front + (int)(Wt.size() / 2) + BANK_PAD, "LDS size");
        // a wave-wide load lands lane l's dword at image dword d = l + 64 i, from byte 4 d - 2 left_pad of the row
        for (int d = 0; d < pd; ++d)
            CHECK(4 * d - 2 * left_pad(g.pw, g.Cin) == 2 * source_element(d, 0, g.pw, g.Cin), "byte offset of image dword %d", d);
    }
    const int pitch = pitch_dwords(g.W, g.Cin, OW, g.sw, g.pw);
    const int tilesW = (OW + PIX - 1) / PIX;
    CHECK(left_pad(g.pw, g.Cin) % 2 == 0 && left_pad(g.pw, g.Cin) >= g.pw * g.Cin, "left pad");

    for (int oh = 0; oh < OH; ++oh) {
        // stage the KH rows
        std::vector<uint32_t> img((size_t)g.KH * pitch, 0xdeadbeefu);
        for (int kh = 0; kh < g.KH; ++kh) {
            const int ih = oh * g.sh - g.ph + kh * g.dh;
            const bool rowOk = ih >= 0 && ih < g.H;
            for (int d = 0; d < pitch; ++d) {
                uint32_t v = 0;
                for (int half = 0; half < 2; ++half) {
                    const int j = source_element(d, half, g.pw, g.Cin);
                    if (rowOk && j >= 0 && j < rowElems) v |= (uint32_t)(uint16_t)X[(size_t)ih * rowElems + j] << (16 * half);
                }
                img[(size_t)kh * pitch + d] = v;
            }
        }
        for (int tile = 0; tile < tilesW; ++tile) {
            // accumulators of the 64 lanes: acc[t][lane][r]
            std::vector<long long> acc((size_t)NT * 64 * 4, 0);
            for (int kh = 0; kh < g.KH; ++kh) {
                // operands of every lane
                int16_t xf[64][8], wf[4][64][8];
                for (int lane = 0; lane < 64; ++lane) {
                    const int m = lane & 15, grp = lane >> 4;
                    const int ow = tile * PIX + m;
                    const int e0 = window_start(ow, g.sw, g.Cin, g.pw) + 8 * grp;
                    const unsigned sh = (unsigned)(e0 & 1) * 2u;
                    const size_t first = (size_t)kh * pitch + (e0 >> 1);
                    CHECK((e0 >> 1) + 4 < pitch, "read beyond the image row: e0 %d pitch %d", e0, pitch);
                    uint32_t q[5];
                    for (int j = 0; j < 5; ++j) q[j] = img[first + j];
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t f = alignbyte(q[j + 1], q[j], sh) & k_mask(grp, j, kwcin);
                        xf[lane][2 * j] = (int16_t)(f & 0xffffu);
                        xf[lane][2 * j + 1] = (int16_t)(f >> 16);
                    }
                    // the filters' fragments are cut from the bank's copy the same way
                    for (int t = 0; t < NT; ++t) {
                        const int w0 = (channel_of(t, m) * g.KH + kh) * kwcin + 8 * grp;
                        CHECK((w0 >> 1) + 4 < (int)bank.size(), "read beyond the bank: %d of %d", (w0 >> 1) + 4, (int)bank.size());
                        for (int j = 0; j < 4; ++j) {
                            const uint32_t f = alignbyte(bank[(w0 >> 1) + j + 1], bank[(w0 >> 1) + j], (unsigned)(w0 & 1) * 2u) & k_mask(grp, j, kwcin);
                            wf[t][lane][2 * j] = (int16_t)(f & 0xffffu);
                            wf[t][lane][2 * j + 1] = (int16_t)(f >> 16);
                        }
                    }
                }
                // D[i][j] += sum_k A[i][k] B[k][j]: lane l supplies A[l % 16][8 (l / 16) + e] and B[8 (l / 16) + e][l % 16],
                // and holds D[4 (l / 16) + r][l % 16]
                for (int t = 0; t < NT; ++t)
                    for (int lane = 0; lane < 64; ++lane)
                        for (int r = 0; r < 4; ++r) {
                            const int i = 4 * (lane >> 4) + r, j = lane & 15;
                            long long s = 0;
                            for (int k = 0; k < 32; ++k) s += (long long)wf[t][(k >> 3) * 16 + i][k & 7] * xf[(k >> 3) * 16 + j][k & 7];
                            acc[((size_t)t * 64 + lane) * 4 + r] += s;
                        }
            }
            // compare with the definition
            for (int lane = 0; lane < 64; ++lane) {
                const int m = lane & 15, grp = lane >> 4, ow = tile * PIX + m;
                if (ow >= OW) continue;
                for (int h = 0; h < NT / 2; ++h)
                    for (int e = 0; e < 8; ++e) {
                        const int co = 32 * h + 8 * grp + e;                 // what the kernel stores at (position, co)
                        const int t = 2 * h + (e >> 2), r = e & 3;
                        CHECK(channel_of(t, 4 * grp + r) == co, "channel map t %d g %d r %d", t, grp, r);
                        long long ref = 0;
                        for (int kh = 0; kh < g.KH; ++kh)
                            for (int kw = 0; kw < g.KW; ++kw)
                                for (int c = 0; c < g.Cin; ++c) {
                                    const int ih = oh * g.sh - g.ph + kh * g.dh, iw = ow * g.sw - g.pw + kw;
                                    if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) continue;
                                    ref += (long long)X[((size_t)ih * g.W + iw) * g.Cin + c] * Wt[(((size_t)co * g.KH + kh) * g.KW + kw) * g.Cin + c];
                                }
                        CHECK(acc[((size_t)t * 64 + lane) * 4 + r] == ref, "oh %d ow %d co %d: %lld != %lld", oh, ow, co,
                              acc[((size_t)t * 64 + lane) * 4 + r], ref);
                    }
            }
        }
    }
    // every channel is produced exactly once per position
    std::vector<int> seen(g.Cout, 0);
    for (int t = 0; t < NT; ++t) for (int i = 0; i < 16; ++i) { const int c = channel_of(t, i); CHECK(c >= 0 && c < g.Cout, "channel range"); if (c >= 0 && c < g.Cout) ++seen[c]; }
    for (int c = 0; c < g.Cout; ++c) CHECK(seen[c] == 1, "channel %d seen %d times", c, seen[c]);
}

int main()
{
    const Geo cases[] = {
        {12, 40, 3, 7, 7, 2, 2, 3, 3, 1, 64},    // the first layer's geometry, small
        {9, 37, 3, 7, 7, 2, 2, 3, 3, 1, 32},     // odd row length: windows begin at odd and even elements
        {7, 21, 3, 3, 3, 1, 1, 1, 1, 1, 64},     // stride 1: a lane's window starts at any element
        {8, 33, 1, 7, 7, 2, 2, 3, 3, 1, 32},     // one channel
        {8, 19, 4, 5, 7, 2, 3, 2, 2, 2, 64},     // four channels, stride 3, dilated rows
        {6, 50, 2, 1, 16, 1, 1, 0, 0, 1, 32},    // the widest filter row: all 32 elements of the step, no padding
        {5, 16, 3, 2, 2, 1, 2, 0, 1, 1, 64},     // even filter, padding on one side in effect
        {8, 20, 1, 3, 3, 1, 1, 1, 1, 1, 32},     // three elements to a filter row: the last filters' fragments reach farthest past the bank
        {4, 9, 1, 1, 1, 1, 1, 0, 0, 1, 32},      // one element to a filter row
    };
    unsigned seed = 1;
    for (const Geo &g : cases) run(g, seed++);
    if (failures) { std::printf("%d failures\n", failures); return 1; }
    std::printf("conv rows layout checks passed\n");
    return 0;
}
