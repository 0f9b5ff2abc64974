// Index functions of the tall-skinny kernel (gemm_skinny.h), plain constexpr code with no HIP types:
// compiled into the kernel and into the host-side model test.
//
// A stage holds 32 rows x KS k of A as a row-major image of 2 KS-byte rows, the 16-byte chunks of a
// row XOR-swizzled by the row's low four bits, and the matching KS k rows of B as an image [k][NP]
// (NP = 16 or 32 columns, 32 or 64 bytes per row, not swizzled).  Direct-to-LDS loads fill both 1 KB
// per wave instruction (lane l lands at slab base + 16 l): whole rows of the A image (four with
// KS = 128), 32 or 16 rows of the B image.
#pragma once

#if defined(__HIPCC__)
#define GE_SKINNY_HD __host__ __device__
#else
#define GE_SKINNY_HD
#endif

namespace ge_skinny {

constexpr int BM = 32;                       // rows of A (and C) per workgroup
constexpr int KS = 128;                      // k per stage (a multiple of 128: the swizzle needs 16 chunks per row or more)
constexpr int A_ROW_BYTES = KS * 2;
constexpr int A_CHUNKS = A_ROW_BYTES / 16;   // 16-byte chunks per row
constexpr int A_BYTES = BM * A_ROW_BYTES;
constexpr int A_SLABS = A_BYTES / 1024;

GE_SKINNY_HD constexpr int a_offset(int r, int c) { return r * A_ROW_BYTES + ((c ^ (r & 15)) << 4); }
GE_SKINNY_HD constexpr int a_slab_row(int slab, int lane) { return slab * (64 / A_CHUNKS) + lane / A_CHUNKS; }
GE_SKINNY_HD constexpr int a_slab_chunk(int slab, int lane) { return (lane % A_CHUNKS) ^ (a_slab_row(slab, lane) & 15); }
// fragment of the 16x16x32 MFMA for the 16 rows from rowBase and the 32 k from kk (a multiple of 32):
// lane l reads 16 bytes, row rowBase + l%16, k = kk + 8 (l/16) + e
GE_SKINNY_HD constexpr int a_frag_offset(int rowBase, int kk, int lane) { return a_offset(rowBase + (lane & 15), kk / 8 + (lane >> 4)); }

// B image [k][np]: chunks per row np / 8; lane l of the load filling slab `slab` fetches chunk l % cpr of k row ...
GE_SKINNY_HD constexpr int b_bytes(int np) { return KS * np * 2; }
GE_SKINNY_HD constexpr int b_slabs(int np) { return b_bytes(np) / 1024; }
GE_SKINNY_HD constexpr int b_slab_k(int np, int slab, int lane) { return slab * (64 / (np / 8)) + lane / (np / 8); }
GE_SKINNY_HD constexpr int b_slab_chunk(int np, int lane) { return lane % (np / 8); }
GE_SKINNY_HD constexpr int b_offset(int np, int k, int n) { return (k * np + n) * 2; }
// fragment for the 32 k from kk and the 16 columns from 16 j, as two transposing 64-bit reads h = 0, 1: the
// 16-lane group g = l/16 covers k = kk + 8 g + 4 h .. +3; lane i of the group addresses k row (that) + i/4 and
// the 4 columns from 16 j + 4 (i%4), and receives column 16 j + i (element e <-> k + e)
GE_SKINNY_HD constexpr int b_frag_offset(int np, int kk, int j, int lane, int h)
{
    const int i = lane & 15, g = lane >> 4;
    return b_offset(np, kk + 8 * g + 4 * h + (i >> 2), 16 * j + 4 * (i & 3));
}

}  // namespace ge_skinny
