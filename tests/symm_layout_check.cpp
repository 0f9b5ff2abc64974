// Host-side functional model of the symmetric-operand kernel's LDS data path (no GPU), compiled from
// the very header the kernel uses (csrc/symm_layout.h): global sub-tile -> direct-to-LDS slabs ->
// image -> the two kinds of fragment reads -> MFMA operand registers.  Checks that the slab map is a
// bijection onto the stage, that every lane and element of a fragment holds the matrix entry the
// 16x16x32 MFMA expects there (along the rows for T * B, across them for T^T * B), that the small
// operand's fragments do, that all addresses stay inside their buffers, and the enumeration of the
// super-tiles with the bookkeeping of the terms: every (row block, term) pair is produced exactly once.
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "../paper_2604_01489_amd/csrc/symm_layout.h"
using namespace ge_symm;

static int fails = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (fails < 20) { printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } ++fails; } } while (0)

// The transposing 64-bit read as the hardware performs it for 16-bit elements: within a group of 16
// lanes, lane j supplies the address of 4 consecutive elements; the 16 addresses form a block of 4 rows
// (row = j / 4) by 16 columns (4 (j % 4) .. +3), and lane i receives column i of it, rows 0..3.
static void tr_read(const std::vector<int> &mem, const int (&addr)[64], int (&out)[64][4])
{
    for (int lane = 0; lane < 64; ++lane) {
        const int g = lane >> 4, i = lane & 15;
        for (int e = 0; e < 4; ++e) {
            const int src = g * 16 + 4 * e + (i >> 2);          // the lane that supplied row e, columns 4 (i/4) ..
            out[lane][e] = mem[addr[src] / 2 + (i & 3)];
        }
    }
}

int main()
{
    // ---- sub-tile image: element id (row << 8) | col
    std::vector<int> lds(STAGE_BYTES / 2, -1);
    for (int slab = 0; slab < SLABS; ++slab)
        for (int lane = 0; lane < 64; ++lane) {
            const int row = slab_row(slab, lane), ch = slab_chunk(slab, lane);
            CHECK(row >= 0 && row < SUB && ch >= 0 && ch < 16, "slab lane outside the sub-tile");
            const int at = slab * 1024 + lane * 16;             // where the hardware puts this lane's 16 bytes
            CHECK(at == image_offset(row, ch), "slab %d lane %d lands at %d, image says %d", slab, lane, at, image_offset(row, ch));
            for (int e = 0; e < 8; ++e) {
                CHECK(lds[at / 2 + e] == -1, "image written twice");
                lds[at / 2 + e] = (row << 8) | (ch * 8 + e);
            }
        }
    for (int v : lds) CHECK(v != -1, "image not fully covered");

    // ---- fragments along the rows (operand of T * B)
    for (int rowBase = 0; rowBase < SUB; rowBase += 16)
        for (int ks = 0; ks < SUB / 32; ++ks)
            for (int lane = 0; lane < 64; ++lane) {
                const int off = row_frag_offset(rowBase, ks, lane);
                CHECK(off >= 0 && off % 16 == 0 && off + 16 <= STAGE_BYTES, "row fragment address");
                for (int e = 0; e < 8; ++e) {
                    const int want = ((rowBase + (lane & 15)) << 8) | (32 * ks + 8 * (lane >> 4) + e);
                    CHECK(lds[off / 2 + e] == want, "row fragment lane %d elem %d", lane, e);
                }
            }

    // ---- fragments across the rows (operand of T^T * B): index = column, k = row
    for (int colBase = 0; colBase < SUB; colBase += 16)
        for (int ks = 0; ks < SUB / 32; ++ks)
            for (int h = 0; h < 2; ++h) {
                int addr[64], out[64][4];
                for (int lane = 0; lane < 64; ++lane) {
                    addr[lane] = col_frag_offset(colBase, ks, lane, h);
                    CHECK(addr[lane] >= 0 && addr[lane] % 8 == 0 && addr[lane] + 8 <= STAGE_BYTES, "column fragment address");
                }
                tr_read(lds, addr, out);
                for (int lane = 0; lane < 64; ++lane)
                    for (int e = 0; e < 4; ++e) {
                        const int want = ((32 * ks + 8 * (lane >> 4) + 4 * h + e) << 8) | (colBase + (lane & 15));
                        CHECK(out[lane][e] == want, "column fragment lane %d h %d elem %d holds %x want %x", lane, h, e, out[lane][e], want);
                    }
            }

    // ---- the small operand's image [k][NP] and its fragments: index = column n, k = row
    for (int np : {16, 32})
        for (int st : {256, 512}) {
            std::vector<int> img(st * np, -1);
            for (int k = 0; k < st; ++k)
                for (int n = 0; n < np; ++n) {
                    const int off = small_offset(np, k, n);
                    CHECK(off >= 0 && off + 2 <= st * np * 2 && img[off / 2] == -1, "small image offset");
                    img[off / 2] = (k << 8) | n;
                }
            for (int kBase = 0; kBase < st; kBase += 32)
                for (int j = 0; j < np / 16; ++j)
                    for (int h = 0; h < 2; ++h) {
                        int addr[64], out[64][4];
                        for (int lane = 0; lane < 64; ++lane) {
                            addr[lane] = small_frag_offset(np, kBase, j, lane, h);
                            CHECK(addr[lane] >= 0 && addr[lane] % 8 == 0 && addr[lane] + 8 <= st * np * 2, "small fragment address");
                        }
                        tr_read(img, addr, out);
                        for (int lane = 0; lane < 64; ++lane)
                            for (int e = 0; e < 4; ++e) {
                                const int want = ((kBase + 8 * (lane >> 4) + 4 * h + e) << 8) | (16 * j + (lane & 15));
                                CHECK(out[lane][e] == want, "small fragment np %d lane %d", np, lane);
                            }
                    }
        }

    // ---- super-tile enumeration and the terms: for T rows of super-tiles, workgroup x owns (a, b), a >= b;
    // with the lower triangle stored (I, J) = (a, b): P1 is term J of row block I, P2 term I of row block J,
    // on the diagonal one term I of row block I; with the upper one stored (I, J) = (b, a), same rule.
    for (int T : {1, 2, 5, 32, 64})
        for (int upper = 0; upper < 2; ++upper) {
            std::vector<int> produced(T * T, 0);
            const unsigned count = (unsigned)(T * (T + 1) / 2);
            for (unsigned x = 0; x < count; ++x) {
                unsigned a, b;
                pair_of_index(x, &a, &b);
                CHECK(a < (unsigned)T && b <= a && a * (a + 1) / 2 + b == x, "pair of index %u", x);
                const int I = upper ? (int)b : (int)a, J = upper ? (int)a : (int)b;
                if (I == J) produced[I * T + I] += 1;
                else { produced[I * T + J] += 1; produced[J * T + I] += 1; }
            }
            for (int v : produced) CHECK(v == 1, "a (row block, term) pair produced %d times", v);
        }

    if (fails == 0) printf("symmetric layout checks passed\n");
    return fails == 0 ? 0 : 1;
}
