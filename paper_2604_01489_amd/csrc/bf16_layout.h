// LDS layouts of the bf16 GEMM kernel, as plain constexpr index functions (no HIP types) so
// that the same code is compiled into the kernel and into the host-side layout test.
//
// A stage: BM rows x 32 k (64 bytes per row, four 16-byte chunks).  B stage: 32 k rows x BN
// columns (2*BN bytes per row).  A wave-wide direct-to-LDS load fills 1 KB: lane l lands at
// slot base + 16*l, so each layout is defined by the map slot -> (row, chunk) the lanes use to
// pick their global chunk, and fragment reads use the inverse.
#pragma once

#if defined(__HIPCC__)
#define GE_HD __host__ __device__
#else
#define GE_HD
#endif

namespace ge {

// LDS byte offset of 16-byte chunk c (8 bf16 along k, c < 4) of row r in an A stage.  Address
// bits 4-5: chunk ^ r[2:1]; bit 6: r[0]; bit 7: r[3]; 256-byte line: (r/16)*4 + r[2:1].  Any 8
// or 16 consecutive rows reading the same chunk fall in distinct banks.
GE_HD constexpr int lds_a_offset(int r, int c)
{
    return (((r >> 4) * 4 + ((r >> 1) & 3)) * 256) + (((r >> 3) & 1) * 128) + ((r & 1) * 64) +
           ((c ^ ((r >> 1) & 3)) * 16);
}

// row and chunk fetched by lane `lane` of the wave-wide load that fills 1 KB slab `wl` of an A stage
GE_HD constexpr int a_slot_row(int wl, int lane)
{
    return wl * 16 + ((lane >> 3) & 1) * 8 + ((lane >> 4) & 3) * 2 + ((lane >> 2) & 1);
}
GE_HD constexpr int a_slot_chunk(int lane) { return (lane & 3) ^ ((lane >> 4) & 3); }

// B stage swizzle.  One transposing read serves, per half wave, the k rows {k0..k0+3, k0+8..k0+11}
// with 32 bytes each: the 64-byte column segments are rotated by a 3-bit hash of the row
// (k[1:0] | k[3] << 2) and the two 32-byte halves of a segment are swapped for rows with k[3] set,
// so those 8 x 32 bytes fall in 8 different 32-byte bank groups (measured: the version without
// the half swap spent a quarter of its LDS cycles on bank conflicts).
GE_HD constexpr int lds_b_hash(int k) { return (k & 3) | ((k >> 1) & 4); }
GE_HD constexpr int lds_b_half(int k) { return ((k >> 3) & 1) << 1; }

// LDS byte offset of 16-byte chunk c (8 bf16 along n) of k row k in a B stage of width BN
template <int BN>
GE_HD constexpr int lds_b_offset(int k, int c)
{
    return k * (BN * 2) + ((((c >> 2) ^ lds_b_hash(k)) & (BN / 32 - 1)) * 64) + (((c & 3) ^ lds_b_half(k)) * 16);
}

// k row and column chunk fetched by lane `lane` of the load that fills slab `wl` of a B stage
template <int BN>
GE_HD constexpr int b_slot_k(int wl, int lane) { return (wl * 64 + lane) / (BN / 8); }
template <int BN>
GE_HD constexpr int b_slot_chunk(int wl, int lane)
{
    const int q = wl * 64 + lane, k = q / (BN / 8), pc = q % (BN / 8);
    return ((((pc >> 2) ^ lds_b_hash(k)) & (BN / 32 - 1)) * 4) + ((pc & 3) ^ lds_b_half(k));
}

// A fragment of the 16x16x32 MFMA: lane l reads the 16 bytes of row rowBase + l%16, chunk l/16
// (k = 8*(l/16) + e for element e).
GE_HD constexpr int a_frag_offset(int rowBase, int lane) { return lds_a_offset(rowBase + (lane & 15), lane >> 4); }

// B fragment: two transposing 64-bit reads r = 0, 1.  The 16-lane group g = l/16 covers
// k = 8g + 4r .. +3 of columns colBase .. +15; lane i of the group addresses k row i/4 and the
// 4 columns from 4*(i%4), and receives column i of that 4 x 16 block (element e <-> k + e).
template <int BN>
GE_HD constexpr int b_frag_offset(int colBase, int lane, int r)
{
    const int i = lane & 15, k = 8 * (lane >> 4) + 4 * r + (i >> 2), n = colBase + (i & 3) * 4;
    return lds_b_offset<BN>(k, n >> 3) + (n & 7) * 2;
}

// ---- k-contiguous stage of 64 k (rows of 128 bytes, eight 16-byte chunks) -----------------------
// For an operand whose memory rows run along k a stage that spans 64 k lets eight neighbouring
// lanes of a direct-to-LDS load fetch one whole 128-byte line (two requests of 64 bytes to the
// same line, K steps apart, otherwise).  Chunk c of row r sits at r*128 + (c ^ r[3:1])*16: the 16
// rows a fragment read touches (same chunk) fall in 16 different 16-byte bank groups.
GE_HD constexpr int lds_a64_offset(int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) * 16); }

// row and chunk fetched by lane `lane` of the load that fills 1 KB slab `wl` (8 rows) of such a stage
GE_HD constexpr int a64_slot_row(int wl, int lane) { return wl * 8 + (lane >> 3); }
GE_HD constexpr int a64_slot_chunk(int wl, int lane) { return (lane & 7) ^ ((a64_slot_row(wl, lane) >> 1) & 7); }

// Fragment of the 16x16x32 MFMA for the k half h (k = 32 h + 8*(l/16) + e): lane l reads row
// rowBase + l%16, chunk 4 h + l/16.  rowBase is a multiple of 16.
GE_HD constexpr int a64_frag_offset(int rowBase, int lane, int h)
{
    return lds_a64_offset(rowBase + (lane & 15), 4 * h + (lane >> 4));
}

}  // namespace ge
