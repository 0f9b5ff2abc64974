// Index functions of the symmetric-operand kernel (gemm_symm.h), as plain constexpr code with no HIP
// types, so that the same functions are compiled into the kernel and into the host-side model test.
//
// A 128 x 128 bf16 sub-tile of the stored triangle is staged in LDS as a row-major image, 256 bytes
// per row, its sixteen 16-byte chunks XOR-swizzled by the row.  Direct-to-LDS loads fill it 1 KB
// (4 rows) per wave instruction: lane l lands at slab base + 16 l, so the swizzle is applied by
// choosing which chunk of the row each lane fetches.  The image is read two ways: along its rows
// (16 bytes per lane: the operand of T * B) and across them by transposing reads (the operand of
// T^T * B).
#pragma once

#if defined(__HIPCC__)
#define GE_SYMM_HD __host__ __device__
#else
#define GE_SYMM_HD
#endif

namespace ge_symm {

constexpr int SUB = 128;                 // side of a sub-tile
constexpr int ROW_BYTES = SUB * 2;       // 256
constexpr int STAGE_BYTES = SUB * ROW_BYTES;   // 32 KB
constexpr int SLABS = STAGE_BYTES / 1024;      // 32 wave-wide loads fill a stage

// byte offset of 16-byte chunk c (8 columns from 8 c) of row r in the image
GE_SYMM_HD constexpr int image_offset(int r, int c) { return r * ROW_BYTES + ((c ^ (r & 15)) << 4); }

// row and (logical) chunk that lane `lane` of the load filling slab `slab` fetches
GE_SYMM_HD constexpr int slab_row(int slab, int lane) { return slab * 4 + (lane >> 4); }
GE_SYMM_HD constexpr int slab_chunk(int slab, int lane) { return (lane & 15) ^ (slab_row(slab, lane) & 15); }

// Operand of T * B for the 16 rows from rowBase and the 32 columns of k step ks: lane l reads 16 bytes,
// row rowBase + l%16, columns 32 ks + 8 (l/16) .. +7 (element e <-> column + e).
GE_SYMM_HD constexpr int row_frag_offset(int rowBase, int ks, int lane)
{
    return image_offset(rowBase + (lane & 15), 4 * ks + (lane >> 4));
}

// Operand of T^T * B for the 16 columns from colBase and the 32 rows of k step ks, as two transposing
// 64-bit reads h = 0, 1: the 16-lane group g = l/16 covers rows 32 ks + 8 g + 4 h .. +3; lane i of the
// group addresses row (that) + i/4 and the 4 columns from colBase + 4 (i%4), and receives column
// colBase + i of the 4 x 16 block (element e <-> row 32 ks + 8 g + 4 h + e).
GE_SYMM_HD constexpr int col_frag_offset(int colBase, int ks, int lane, int h)
{
    const int i = lane & 15, g = lane >> 4;
    const int row = 32 * ks + 8 * g + 4 * h + (i >> 2), col = colBase + 4 * (i & 3);
    return image_offset(row, col >> 3) + (col & 7) * 2;
}

// The small operand's block: an image [k][NP] of bf16, NP = 16 or 32 columns, k < ST rows.  Fragment
// for the 32 k from kBase and the 16 columns from 16 j, two transposing reads h = 0, 1 as above.
GE_SYMM_HD constexpr int small_offset(int np, int k, int n) { return (k * np + n) * 2; }
GE_SYMM_HD constexpr int small_frag_offset(int np, int kBase, int j, int lane, int h)
{
    const int i = lane & 15, g = lane >> 4;
    return small_offset(np, kBase + 8 * g + 4 * h + (i >> 2), 16 * j + 4 * (i & 3));
}

// Super-tile (a, b), a >= b, of linear index x = a (a + 1) / 2 + b.
GE_SYMM_HD inline void pair_of_index(unsigned x, unsigned *a, unsigned *b)
{
    unsigned t = 0;
    // integer square root of 8 x + 1 by Newton steps from a float estimate would do; the count of
    // super-tile rows is small (at most a few hundred), so walk
    while ((unsigned long long)(t + 1) * (t + 2) / 2 <= x) ++t;
    *a = t;
    *b = x - t * (t + 1) / 2;
}

}  // namespace ge_symm
