// Host-side functional model of the bf16 kernel's LDS data path (no GPU): global tile ->
// direct-to-LDS slots -> fragment reads -> MFMA operand registers.  Checks that every lane and
// element ends up holding the matrix entry the 16x16x32 MFMA expects there, that the slot maps
// are bijections onto the stage, and that fragment reads are bank-conflict free under a
// 64-bank x 4-byte model in which a 128-bit read serves 16 lanes per pass and a 64-bit
// (transposing) read 32 lanes per pass (the hardware counter is the final judge).
#include <cstdio>
#include <cstdlib>
#include <set>
#include <vector>
#include "../paper_2604_01489_amd/csrc/bf16_layout.h"
using namespace ge;

static int fails = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (fails < 20) { printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } ++fails; } } while (0)

template <int BM> void check_a()
{
    // element id stored in the model LDS: (row << 8) | k
    std::vector<int> lds(BM * 32, -1);           // one int per bf16 element
    for (int wl = 0; wl < BM / 16; ++wl)
        for (int lane = 0; lane < 64; ++lane) {
            const int row = a_slot_row(wl, lane), c = a_slot_chunk(lane);
            CHECK(row >= 0 && row < BM && c >= 0 && c < 4, "A slot out of tile wl=%d lane=%d", wl, lane);
            const int slot = wl * 1024 + lane * 16;      // where the hardware puts this lane's 16 bytes
            CHECK(slot == lds_a_offset(row, c), "A slot/offset mismatch wl=%d lane=%d", wl, lane);
            for (int e = 0; e < 8; ++e) {
                CHECK(lds[slot / 2 + e] == -1, "A slot written twice");
                lds[slot / 2 + e] = (row << 8) | (c * 8 + e);
            }
        }
    for (int v : lds) CHECK(v != -1, "A stage not fully covered");
    for (int rowBase = 0; rowBase < BM; rowBase += 16) {
        std::set<int> banks[4];
        for (int lane = 0; lane < 64; ++lane) {
            const int off = a_frag_offset(rowBase, lane);
            CHECK(off % 16 == 0 && off >= 0 && off + 16 <= BM * 64, "A fragment address");
            for (int e = 0; e < 8; ++e) {
                const int want = ((rowBase + (lane & 15)) << 8) | (8 * (lane >> 4) + e);
                CHECK(lds[off / 2 + e] == want, "A fragment lane %d elem %d holds %x want %x", lane, e, lds[off / 2 + e], want);
            }
            CHECK(banks[lane >> 4].insert((off % 256) / 16).second, "A fragment bank conflict rowBase=%d lane=%d", rowBase, lane);
        }
    }
}

// the 64-k stage of a k-contiguous operand: slot map, both fragment halves, banks
template <int BM> void check_a64()
{
    std::vector<int> lds(BM * 64, -1);
    for (int wl = 0; wl < BM / 8; ++wl)
        for (int lane = 0; lane < 64; ++lane) {
            const int row = a64_slot_row(wl, lane), c = a64_slot_chunk(wl, lane);
            CHECK(row >= 0 && row < BM && c >= 0 && c < 8, "A64 slot out of tile wl=%d lane=%d", wl, lane);
            const int slot = wl * 1024 + lane * 16;
            CHECK(slot == lds_a64_offset(row, c), "A64 slot/offset mismatch wl=%d lane=%d", wl, lane);
            // eight neighbouring lanes cover one row: one 128-byte line of the operand
            CHECK(row == a64_slot_row(wl, lane & ~7), "A64 lanes of a line");
            for (int e = 0; e < 8; ++e) {
                CHECK(lds[slot / 2 + e] == -1, "A64 slot written twice");
                lds[slot / 2 + e] = (row << 8) | (c * 8 + e);
            }
        }
    for (int v : lds) CHECK(v != -1, "A64 stage not fully covered");
    for (int rowBase = 0; rowBase < BM; rowBase += 16)
        for (int h = 0; h < 2; ++h) {
            std::set<int> banks[4];
            for (int lane = 0; lane < 64; ++lane) {
                const int off = a64_frag_offset(rowBase, lane, h);
                CHECK(off % 16 == 0 && off >= 0 && off + 16 <= BM * 128, "A64 fragment address");
                // what the kernel relies on: the row block and the lane part separate, the k half is
                // carried by the lane part alone
                CHECK(off == rowBase * 128 + a64_frag_offset(0, lane, h), "A64 fragment base + immediate");
                for (int e = 0; e < 8; ++e) {
                    const int want = ((rowBase + (lane & 15)) << 8) | (32 * h + 8 * (lane >> 4) + e);
                    CHECK(lds[off / 2 + e] == want, "A64 fragment lane %d elem %d holds %x want %x", lane, e, lds[off / 2 + e], want);
                }
                CHECK(banks[lane >> 4].insert((off % 256) / 16).second, "A64 fragment bank conflict rowBase=%d lane=%d", rowBase, lane);
            }
        }
}

template <int BN> void check_b()
{
    std::vector<int> lds(32 * BN, -1);
    for (int wl = 0; wl < 32 * BN * 2 / 1024; ++wl)
        for (int lane = 0; lane < 64; ++lane) {
            const int k = b_slot_k<BN>(wl, lane), c = b_slot_chunk<BN>(wl, lane);
            CHECK(k >= 0 && k < 32 && c >= 0 && c < BN / 8, "B slot out of tile");
            const int slot = wl * 1024 + lane * 16;
            CHECK(slot == lds_b_offset<BN>(k, c), "B slot/offset mismatch wl=%d lane=%d", wl, lane);
            for (int e = 0; e < 8; ++e) {
                CHECK(lds[slot / 2 + e] == -1, "B slot written twice");
                lds[slot / 2 + e] = (k << 12) | (c * 8 + e);
            }
        }
    for (int v : lds) CHECK(v != -1, "B stage not fully covered");
    for (int colBase = 0; colBase < BN; colBase += 16)
        for (int r = 0; r < 2; ++r) {
            // the transposing read: within each 16-lane group, lane i receives, as element e, the
            // (i%4)-th 16-bit word ... of the 64 bits addressed by lane 4*e + i/4 of the group
            int addr[64];
            for (int lane = 0; lane < 64; ++lane) {
                addr[lane] = b_frag_offset<BN>(colBase, lane, r);
                CHECK(addr[lane] % 8 == 0 && addr[lane] >= 0 && addr[lane] + 8 <= 32 * BN * 2, "B fragment address");
            }
            for (int half = 0; half < 2; ++half) {       // 32 lanes x 8 bytes = one pass over the 64 banks
                std::multiset<int> banks;
                for (int lane = half * 32; lane < half * 32 + 32; ++lane) {
                    banks.insert((addr[lane] % 256) / 4);
                    banks.insert((addr[lane] % 256) / 4 + 1);
                }
                for (int b : banks) CHECK(banks.count(b) == 1, "B fragment bank conflict BN=%d col=%d r=%d", BN, colBase, r);
            }
            for (int lane = 0; lane < 64; ++lane) {
                const int g = lane >> 4, i = lane & 15;
                for (int e = 0; e < 4; ++e) {
                    const int src = g * 16 + 4 * e + (i >> 2);      // supplier lane of element e
                    const int got = lds[addr[src] / 2 + (i & 3)];
                    const int want = ((8 * g + 4 * r + e) << 12) | (colBase + i);
                    CHECK(got == want, "B fragment col=%d r=%d lane %d elem %d holds %x want %x", colBase, r, lane, e, got, want);
                }
            }
        }
}

// the kernel steps through fragments with immediates and an XOR instead of recomputing offsets
template <int BN> void check_steps()
{
    for (int lane = 0; lane < 64; ++lane) {
        for (int rowBase = 0; rowBase < 256; rowBase += 64)
            for (int i = 0; i < 8 && rowBase + 16 * i < 256; ++i)
                CHECK(a_frag_offset(rowBase + 16 * i, lane) == a_frag_offset(rowBase, lane) + i * 1024, "A step");
        for (int wtn = 64; wtn <= 128; wtn += 64)
            for (int colBase = 0; colBase < BN; colBase += wtn)
                for (int j = 0; j < wtn / 16; ++j)
                    for (int r = 0; r < 2; ++r) {
                        const int stepped = (b_frag_offset<BN>(colBase, lane, 0) ^ (j * 32)) + r * 4 * BN * 2;
                        CHECK(b_frag_offset<BN>(colBase + 16 * j, lane, r) == stepped, "B step BN=%d col=%d j=%d r=%d lane=%d", BN, colBase, j, r, lane);
                    }
    }
}

// fp32 kernel: same byte geometry, a 16-byte chunk holds 4 floats; BNB = 2 * BN
template <int BM, int BN> void check_f32()
{
    constexpr int BNB = 2 * BN;
    std::vector<int> ldsA(BM * 16, -1), ldsB(16 * BN, -1);      // one int per float
    for (int wl = 0; wl < BM * 64 / 1024; ++wl)
        for (int lane = 0; lane < 64; ++lane) {
            const int row = a_slot_row(wl, lane), c = a_slot_chunk(lane), slot = wl * 1024 + lane * 16;
            CHECK(row < BM && slot == lds_a_offset(row, c), "f32 A slot");
            for (int e = 0; e < 4; ++e) ldsA[slot / 4 + e] = (row << 8) | (4 * c + e);
        }
    for (int wl = 0; wl < 16 * BN * 4 / 1024; ++wl)
        for (int lane = 0; lane < 64; ++lane) {
            const int k = b_slot_k<BNB>(wl, lane), c = b_slot_chunk<BNB>(wl, lane), slot = wl * 1024 + lane * 16;
            CHECK(k < 16 && c < BN / 4 && slot == lds_b_offset<BNB>(k, c), "f32 B slot");
            for (int e = 0; e < 4; ++e) ldsB[slot / 4 + e] = (k << 12) | (4 * c + e);
        }
    for (int v : ldsA) CHECK(v != -1, "f32 A stage not covered");
    for (int v : ldsB) CHECK(v != -1, "f32 B stage not covered");
    for (int lane = 0; lane < 64; ++lane) {
        const int g = lane >> 5, l32 = lane & 31;
        for (int rowBase = 0; rowBase < BM; rowBase += 32)
            for (int rho = 0; rho < 2; ++rho) {
                const int off = lds_a_offset(rowBase % 64 == 0 ? rowBase + l32 : rowBase + l32, 2 * rho + g);
                CHECK(off == lds_a_offset((rowBase / 64) * 64 + l32, 2 * rho + g) + ((rowBase % 64) / 32) * 2048, "f32 A step");
                for (int e = 0; e < 4; ++e)
                    CHECK(ldsA[off / 4 + e] == (((rowBase + l32) << 8) | (8 * rho + 4 * g + e)), "f32 A fragment");
            }
        for (int colBase = 0; colBase < BN; colBase += 32)
            for (int rho = 0; rho < 2; ++rho)
                for (int e = 0; e < 4; ++e) {
                    const int k = 8 * rho + 4 * g + e, n = colBase + l32;
                    const int off = lds_b_offset<BNB>(k, n >> 2) + (n & 3) * 4;
                    CHECK(off % 4 == 0 && off + 4 <= 16 * BN * 4, "f32 B address");
                    CHECK(ldsB[off / 4] == ((k << 12) | n), "f32 B fragment");
                }
    }
}

int main()
{
    check_f32<128, 128>();
    check_f32<64, 64>();
    check_steps<256>();
    check_steps<128>();
    check_a<256>();
    check_a<128>();
    check_b<256>();
    check_b<128>();
    check_a64<256>();
    check_a64<128>();
    if (fails) { printf("%d checks failed\n", fails); return 1; }
    printf("layout checks passed\n");
    return 0;
}
