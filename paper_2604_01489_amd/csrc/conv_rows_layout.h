// Index functions of the few-channel convolution kernel (conv_rows.h), as plain constexpr code with
// no HIP types, so that the same functions are compiled into the kernel and into the host-side
// model test.
//
// A layer with few input channels (a first layer: 3 of them) has no 32 channels of one tap to make
// a K step of.  But in channels-last storage the KW * Cin elements that one output position needs
// from one input row are contiguous, so a K step here is one whole filter ROW: k = kw * Cin + c,
// KW * Cin <= 32 elements, padded with zeros to the 32 of the matrix instruction.  The input rows an
// output row needs are staged in LDS once, each as an image with the horizontal padding written out
// as zeros, and a lane's 8 consecutive k are then 16 consecutive bytes of such an image.
#pragma once

#if defined(__HIPCC__)
#define GE_ROWS_HD __host__ __device__
#else
#define GE_ROWS_HD
#endif

namespace ge_conv_rows {

constexpr int KSTEP = 32;        // elements of one K step: one filter row, KW * Cin <= KSTEP
constexpr int KH_MAX = 7;        // filter rows whose fragments a lane keeps in registers
constexpr int PIX = 16;          // output positions of one matrix-instruction tile
constexpr int BANK_PAD = 16;     // dwords of zeros behind the filter bank's copy in LDS: the last filters' fragments read up to
                                 // (24 - KW * Cin) / 2 + 4 dwords past its end

// Elements of zero padding written at the left of a staged row: the layer's own, made even so that an
// element pair of the input (one dword of a 4-byte aligned row) stays a pair in the image.
GE_ROWS_HD constexpr int left_pad(int pw, int cin) { return pw * cin + ((pw * cin) & 1); }

// Element of the image at which the window of output column ow begins.
GE_ROWS_HD constexpr int window_start(int ow, int sw, int cin, int pw)
{
    return ow * sw * cin + (left_pad(pw, cin) - pw * cin);
}

// Dwords per staged row, a multiple of 64 (a row is filled by wave-wide loads of 64 dwords): the image
// holds the left padding and the W * Cin elements of the row, and every fragment read stays inside it: lane group g of the last tile of a row (whose positions at or
// beyond OW are computed and dropped) reads the five dwords from element (start + 8 g) / 2 * 2.
GE_ROWS_HD constexpr int pitch_dwords(int W, int cin, int OW, int sw, int pw)
{
    const int tilesW = (OW + PIX - 1) / PIX;
    const int lastRead = window_start(tilesW * PIX - 1, sw, cin, pw) + 24 + 10;   // one past the last element read
    const int data = left_pad(pw, cin) + W * cin;
    const int elems = lastRead > data ? lastRead : data;
    return ((elems + 1) / 2 + 63) / 64 * 64;        // whole wave-wide loads of 64 dwords
}

// Staged rows of one output row: input rows oh * sh - ph + [0, rows_in).
GE_ROWS_HD constexpr int rows_in(int KH, int dh) { return (KH - 1) * dh + 1; }

// Input element (index into the W * Cin elements of the row, or out of range: zero) that lands in
// half `half` of dword d of the image.
GE_ROWS_HD constexpr int source_element(int d, int half, int pw, int cin) { return 2 * d + half - left_pad(pw, cin); }

// Output channel of row i (0..15) of matrix-instruction tile t.  A lane owns rows 4 q .. 4 q + 3 of
// every tile; tiles 2 h and 2 h + 1 together give it 8 consecutive channels, 16 bytes of bf16
// output, and the four lanes q of a position cover 32 consecutive channels.
GE_ROWS_HD constexpr int channel_of(int t, int i) { return 32 * (t >> 1) + 8 * (i >> 2) + 4 * (t & 1) + (i & 3); }

// Mask of dword j (0..3) of lane group g's fragment: elements 8 g + 2 j and 8 g + 2 j + 1 of the K
// step are kept where they are below KW * Cin (what follows belongs to the next position).
GE_ROWS_HD constexpr unsigned k_mask(int g, int j, int kwcin)
{
    const int e = 8 * g + 2 * j;
    return (e < kwcin ? 0x0000ffffu : 0u) | (e + 1 < kwcin ? 0xffff0000u : 0u);
}

// Dwords of LDS in front of the filter bank's copy: the two sets of KH row images, or the table of the
// filters' fragments (16 bytes per lane, filter row and 16-channel tile) that is built there first.
GE_ROWS_HD constexpr int front_dwords(int KH, int pitch, int Cout)
{
    const int images = 2 * KH * pitch, table = KH * (Cout / 16) * 64 * 4;
    return images > table ? images : table;
}

// Dwords of LDS the kernel uses: the front, the filter bank and its padding.
GE_ROWS_HD constexpr int lds_dwords(int KH, int pitch, int Cout, int kwcin)
{
    return front_dwords(KH, pitch, Cout) + Cout * KH * kwcin / 2 + BANK_PAD;
}

}  // namespace ge_conv_rows
