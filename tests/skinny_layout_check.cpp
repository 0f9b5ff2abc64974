// Host-side functional model of the tall-skinny kernel's LDS data path (no GPU), compiled from the very
// header the kernel uses (csrc/skinny_layout.h): slab maps onto the two images, fragment reads, MFMA
// operand registers.
#include <cstdio>
#include <vector>
#include "../paper_2604_01489_amd/csrc/skinny_layout.h"
using namespace ge_skinny;

static int fails = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (fails < 20) { printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } ++fails; } } while (0)

// the transposing 64-bit read for 16-bit elements: in a group of 16 lanes, lane j supplies the address of 4
// consecutive elements (block row j / 4, columns 4 (j % 4) .. +3); lane i receives column i, rows 0..3
static void tr_read(const std::vector<int> &mem, const int (&addr)[64], int (&out)[64][4])
{
    for (int lane = 0; lane < 64; ++lane) {
        const int g = lane >> 4, i = lane & 15;
        for (int e = 0; e < 4; ++e) out[lane][e] = mem[addr[g * 16 + 4 * e + (i >> 2)] / 2 + (i & 3)];
    }
}

int main()
{
    // ---- A image: element id (row << 12) | k
    std::vector<int> a(A_BYTES / 2, -1);
    for (int slab = 0; slab < A_SLABS; ++slab)
        for (int lane = 0; lane < 64; ++lane) {
            const int row = a_slab_row(slab, lane), ch = a_slab_chunk(slab, lane);
            CHECK(row >= 0 && row < BM && ch >= 0 && ch < A_CHUNKS, "A slab lane outside the stage");
            const int at = slab * 1024 + lane * 16;
            CHECK(at == a_offset(row, ch), "A slab %d lane %d lands at %d, image says %d", slab, lane, at, a_offset(row, ch));
            for (int e = 0; e < 8; ++e) {
                CHECK(a[at / 2 + e] == -1, "A image written twice");
                a[at / 2 + e] = (row << 12) | (ch * 8 + e);
            }
        }
    for (int v : a) CHECK(v != -1, "A image not covered");
    for (int rowBase = 0; rowBase < BM; rowBase += 16)
        for (int kk = 0; kk < KS; kk += 32)
            for (int lane = 0; lane < 64; ++lane) {
                const int off = a_frag_offset(rowBase, kk, lane);
                CHECK(off >= 0 && off % 16 == 0 && off + 16 <= A_BYTES, "A fragment address");
                for (int e = 0; e < 8; ++e)
                    CHECK(a[off / 2 + e] == (((rowBase + (lane & 15)) << 12) | (kk + 8 * (lane >> 4) + e)), "A fragment lane %d elem %d", lane, e);
            }
    // 16 lanes reading one chunk of 16 consecutive rows hit 16 different 16-byte bank groups of the 256-byte bank span
    for (int kk = 0; kk < KS; kk += 32)
        for (int g = 0; g < 4; ++g) {
            int seen = 0;
            for (int i = 0; i < 16; ++i) seen |= 1 << ((a_frag_offset(0, kk, g * 16 + i) % 256) / 16);
            CHECK(seen == 0xFFFF, "A fragment read: bank conflict");
        }

    // ---- B image [k][np]: element id (k << 12) | n
    for (int np : {16, 32}) {
        std::vector<int> b(b_bytes(np) / 2, -1);
        for (int slab = 0; slab < b_slabs(np); ++slab)
            for (int lane = 0; lane < 64; ++lane) {
                const int k = b_slab_k(np, slab, lane), ch = b_slab_chunk(np, lane);
                CHECK(k >= 0 && k < KS && ch >= 0 && ch < np / 8, "B slab lane outside the stage");
                const int at = slab * 1024 + lane * 16;
                CHECK(at == b_offset(np, k, ch * 8), "B slab %d lane %d lands at %d, image says %d", slab, lane, at, b_offset(np, k, ch * 8));
                for (int e = 0; e < 8; ++e) {
                    CHECK(b[at / 2 + e] == -1, "B image written twice");
                    b[at / 2 + e] = (k << 12) | (ch * 8 + e);
                }
            }
        for (int v : b) CHECK(v != -1, "B image not covered");
        for (int kk = 0; kk < KS; kk += 32)
            for (int j = 0; j < np / 16; ++j)
                for (int h = 0; h < 2; ++h) {
                    int addr[64], out[64][4];
                    for (int lane = 0; lane < 64; ++lane) {
                        addr[lane] = b_frag_offset(np, kk, j, lane, h);
                        CHECK(addr[lane] >= 0 && addr[lane] % 8 == 0 && addr[lane] + 8 <= b_bytes(np), "B fragment address");
                    }
                    tr_read(b, addr, out);
                    for (int lane = 0; lane < 64; ++lane)
                        for (int e = 0; e < 4; ++e)
                            CHECK(out[lane][e] == (((kk + 8 * (lane >> 4) + 4 * h + e) << 12) | (16 * j + (lane & 15))), "B fragment np %d lane %d", np, lane);
                }
    }
    if (fails == 0) printf("skinny layout checks passed\n");
    return fails == 0 ? 0 : 1;
}
