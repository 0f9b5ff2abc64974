// Index functions and the tile plan of the halo-staged 3 x 3 convolution kernel (conv_halo.h), as plain
// constexpr functions (no HIP types) so that the same code is compiled into the kernel, into the host
// code that plans a launch and into the host-side layout test.
//
// A tile is R whole output rows of one image.  For 32 input channels at a time the input rows the
// tile needs (R + 2 of them, with one column of padding left and right) are staged once as a
// "halo": HALO_PITCH = 64 positions per input row, 64 bytes (32 channels) per position, so one
// wave-wide direct-to-LDS load of 1 KB is 16 positions and the four waves of the block fetch one
// input row per load.  The nine taps are then nine fragment reads of the same halo at shifted
// positions: a filter row further down is +64 positions (an immediate of 4096 bytes), a filter
// column further right +1 position (a lane base of its own per column, since the swizzle follows
// the position).
#pragma once

#if defined(__HIPCC__)
#define GE_HALO_HD __host__ __device__
#else
#define GE_HALO_HD
#endif

namespace ge_halo {

constexpr int HALO_PITCH = 64;      // halo positions per staged input row
constexpr int HALO_ROWS = 7;        // staged input rows at most: R + 2 <= 7
constexpr int POS_BYTES = 64;       // 32 channels of bf16
constexpr int HALO_ROW_BYTES = HALO_PITCH * POS_BYTES;       // 4 KB: one load of each of the four waves
constexpr int HALO_BUF_BYTES = HALO_ROWS * HALO_ROW_BYTES;   // 28 KB; the kernel keeps two
constexpr int MAX_OW = HALO_PITCH - 2;
constexpr int MAX_R = HALO_ROWS - 2;

// LDS byte offset, within a halo buffer, of 16-byte chunk c (8 channels, c < 4) of halo position
// hpos = row * 64 + column.  The chunk is XORed with bits 1-2 of the position: a 16-byte-per-lane read is
// served eight lanes at a time, and eight consecutive positions reading the same chunk then cover all
// 32 banks (128 bytes) once, whatever the first position is (a tap shift moves it by one or two).
// (XORed with bits 2-3, which spreads sixteen positions over 256 bytes instead, every such read took two
// turns: the kernel ran no faster than the gathering one.)
GE_HALO_HD constexpr int halo_offset(int hpos, int c) { return hpos * POS_BYTES + ((c ^ ((hpos >> 1) & 3)) * 16); }

// Halo column and channel chunk fetched by lane `lane` of wave `w` in the load of one input row
// (the load lands at row * 4096 + w * 1024 + 16 * lane).
GE_HALO_HD constexpr int halo_slot_col(int w, int lane) { return w * 16 + (lane >> 2); }
GE_HALO_HD constexpr int halo_slot_chunk(int w, int lane) { return (lane & 3) ^ ((halo_slot_col(w, lane) >> 1) & 3); }

// Halo position of output position pos (row-major within the tile, OW columns) for the tap in
// filter column dw of filter row 0: halo column = output column + dw (the halo starts one column
// left of the image for a padding of one), halo row = output row.
GE_HALO_HD constexpr int halo_pos(int pos, int OW, int dw) { return (pos / OW) * HALO_PITCH + pos % OW + dw; }

// ---- tile plan -------------------------------------------------------------------------------
// The OH output rows of every image are cut into g1 groups of R1 rows followed by g2 groups of R2 <= R1
// rows.  All tiles of the first kind are launched ahead of those of the second, so that with one block
// per CU the short tiles fill in behind the long ones: 56 rows as 8 x 4 + 8 x 3 give each of 256 CUs
// one tile of 4 and one of 3 rows for 32 images, where 14 x 4 would be two rounds of 4.
struct HaloPlan {
    int R1, g1, R2, g2;
    int blocks16a, blocks16b;    // row blocks of 16 positions the kernel multiplies for a tile of either kind
    long long cost;              // model time of the launch, in row blocks
};

// Time of a launch on `cus` CUs that run one tile at a time, tiles taken in launch order: n1 tiles of
// cost c1, then n2 of cost c2 <= c1.
GE_HALO_HD constexpr long long halo_makespan(long long n1, int c1, long long n2, int c2, int cus)
{
    // the first kind in whole rounds; the CUs left idle by its last round start on the second kind
    const long long full1 = n1 / cus, rem1 = n1 % cus;
    long long t = full1 * c1;
    if (n2 == 0) return t + (rem1 ? c1 : 0);
    if (rem1 == 0) {
        return t + ((n2 + cus - 1) / cus) * c2;
    }
    // rem1 CUs are busy until t + c1, cus - rem1 are free from t on
    const long long early = cus - rem1;
    // second-kind tiles the early CUs finish before the late ones become free
    const long long lead = (long long)(c1 / c2) * early;
    if (n2 <= lead) return t + c1 > t + ((n2 + early - 1) / early) * c2 ? t + c1 : t + ((n2 + early - 1) / early) * c2;
    // afterwards all CUs take tiles, the early ones offset by c1 % c2: bound it by whole rounds of all
    const long long rest = n2 - lead;
    return t + c1 + ((rest + cus - 1) / cus) * c2;
}

// The best cut for a kernel variant that multiplies tmb1 row blocks for a tile of the first kind and tmb2
// for one of the second.  overhead: cost of a tile beyond its row blocks (prologue, epilogue), in row blocks.
// cost < 0: the variant has no cut for this shape.
GE_HALO_HD constexpr HaloPlan halo_plan(int images, int OH, int OW, int tilesN, int cus, int overhead, int tmb1, int tmb2)
{
    HaloPlan best{0, 0, 0, 0, tmb1, tmb2, -1};
    for (int R1 = 1; R1 <= MAX_R && R1 <= OH && R1 * OW <= tmb1 * 16; ++R1) {
        for (int R2 = 1; R2 <= R1 && R2 * OW <= tmb2 * 16; ++R2) {
            for (int g1 = 1; g1 * R1 <= OH; ++g1) {
                const int left = OH - g1 * R1;
                if (left % R2 != 0) continue;
                const int g2 = left / R2;
                if (R2 == R1 && g2 != 0) continue;           // the same cut is found with g2 = 0
                const long long n1 = (long long)images * g1 * tilesN, n2 = (long long)images * g2 * tilesN;
                const long long cost = halo_makespan(n1, tmb1 + overhead, n2, tmb2 + overhead, cus);
                if (best.cost < 0 || cost < best.cost || (cost == best.cost && g1 + g2 < best.g1 + best.g2))
                    best = HaloPlan{R1, g1, g2 ? R2 : R1, g2, tmb1, tmb2, cost};
            }
        }
    }
    return best;
}

}  // namespace ge_halo
