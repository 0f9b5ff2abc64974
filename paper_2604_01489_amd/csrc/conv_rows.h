// Convolution kernel for layers with few input channels (a first layer: 3 channels, 7 x 7, stride 2),
// which have no 32 channels of one tap for the gathering kernel to make a K step of.  Here a K step is
// one filter ROW: in channels-last storage the KW * Cin elements an output position needs from one
// input row are contiguous (index functions and the reasoning in conv_rows_layout.h).
//
// A workgroup of four waves walks over output rows (image n, row oh), one at a time:
//   1. the KH input rows of the output row are staged in LDS, each as an image with the horizontal
//      padding written out as zeros (rows above or below the input: all zeros); two sets of images,
//      so that the rows of the next output row are fetched while this one is multiplied;
//   2. each wave takes tiles of 16 output columns: per filter row one matrix instruction per 16
//      output channels, the weights as the row operand (kept in registers for the whole walk: they
//      are the same for every output row), the lane's 16 bytes of the image as the column operand.
//      The window of a column starts at any even or odd element, so a lane reads five aligned dwords
//      and shifts; the elements of the K step beyond KW * Cin belong to the next position and are
//      masked to zero in registers (a zero weight would not silence an infinity there);
//   3. the consumer chain runs on the accumulators and a lane stores 8 consecutive channels of its
//      position in one piece (16 bytes of bf16).
// The weights are the same for every output row, which is why a workgroup keeps them and walks: the
// launch is sized to the workgroups the CUs hold at once.
#pragma once

#include <hip/hip_runtime.h>

#include "conv_rows_layout.h"
#include "ge_device.h"

namespace ge {

typedef __attribute__((ext_vector_type(4))) int rows_rsrc_t;

// A raw buffer over one input row: `bytes` of it from `base`, or nothing (every load returns 0).
__device__ inline rows_rsrc_t rows_make_rsrc(const void *base, unsigned bytes)
{
    const unsigned long long a = (unsigned long long)base;
    rows_rsrc_t r;
    r[0] = (int)(unsigned)a;
    r[1] = (int)((unsigned)(a >> 32) & 0xFFFFu);
    r[2] = (int)bytes;
    r[3] = (int)0x00020000u;             // raw buffer, 32-bit data format
    return r;
}

// 4 bytes per lane from a raw buffer straight into LDS at ldsAddr + 4 * lane; a lane whose offset is
// not inside the buffer lands a zero.  Inline assembly, as in the main kernels: the compiler does not
// track it, the caller awaits it with s_waitcnt vmcnt.
__device__ inline void rows_lds_dma4(rows_rsrc_t rs, unsigned ldsAddr, unsigned voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 :: "s"(ldsAddr), "v"(voff), "s"(rs) : "memory", "m0");
}

// NT: matrix-instruction tiles across the output channels (Cout = 16 NT: 32 or 64);
// PAIRS: an input row is 4-byte aligned and even in length, so the image is staged dword by dword;
// KHT: the number of filter rows when it is known at compile time (3 or 7), 0 for any other up to
// KH_MAX.  With a run-time count every filter row is a basic block of its own -- three LDS reads, a
// wait, the shifts, four matrix instructions -- and a tile pays the LDS latency once per filter row;
// with a constant the reads of all rows are issued ahead of the first multiply.
template <int NT, bool OUTBF16, bool PAIRS, int KHT>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))      // two workgroups to a CU: at most 256 registers
conv_rows_bf16_kernel(const GemmParams p, const int items)
{
    using namespace ge_conv_rows;
    static_assert(NT == 2 || NT == 4, "32 or 64 output channels");
    static_assert(KHT >= 0 && KHT <= KH_MAX, "filter rows kept in registers");
    constexpr int KHR = KHT ? KHT : KH_MAX;             // filter rows the registers are laid out for
    constexpr int ROWS_PER_WAVE = (KHR + 3) / 4;        // image rows a wave stages
    constexpr int DW_PER_LANE = 8;           // dwords of one image row per lane: pitch <= 512
    constexpr int BANK_PAD = ge_conv_rows::BANK_PAD;
    extern __shared__ __attribute__((aligned(16))) char rowsLds[];
    unsigned *img = (unsigned *)rowsLds;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int m = lane & 15, g = lane >> 4;
    const int H = p.convH, W = p.convW, Cin = p.convCin, KH = KHT ? KHT : p.convKH;
    const int kwcin = p.convKW * Cin, rowElems = W * Cin;
    const int OH = p.convOH, OW = p.convOW, Cout = p.N;
    const int pitch = pitch_dwords(W, Cin, OW, p.convSw, p.convPw);
    const int tilesW = (OW + PIX - 1) / PIX;
    const unsigned short *X = (const unsigned short *)p.A;
    const unsigned short *Wt = (const unsigned short *)p.B;

    unsigned kmask[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) kmask[j] = k_mask(g, j, kwcin);

    // The weights of every filter row, as row operands: lane (m, g) holds 8 k of channel_of(t, m).  A
    // lane's 8 elements lie at any even or odd element of the filter bank and neighbouring lanes are
    // whole filters apart, so fetched from memory they would be eight two-byte loads per fragment,
    // each touching sixteen cache lines (measured: 36 us of a 57 us launch).  The bank (a few KB) is
    // copied to LDS once, dword by dword; the workgroup then cuts every fragment from it once -- five
    // aligned dwords, a shift, the mask of the step's unused elements, as for the input windows -- into
    // a table in fragment order, 16 bytes per lane, from which each wave fills its registers without
    // bank conflicts (cut by every wave for itself, the scattered reads of the bank were 30 % of the
    // kernel's LDS instructions and half its LDS cycles).  The table lies where the row images will
    // (and may reach beyond them: front_dwords).
    const int bankDwords = Cout * KH * kwcin / 2;                 // Cout is even
    unsigned *bank = img + front_dwords(KH, pitch, Cout);         // behind the row images (and the table)
    for (int d = threadIdx.x; d < bankDwords + BANK_PAD; d += 256)
        bank[d] = d < bankDwords ? ((const unsigned *)Wt)[d] : 0u;
    __syncthreads();
    i32x4_t *table = (i32x4_t *)img;                              // [kh][t][lane]
    for (int f = threadIdx.x; f < KH * NT * 64; f += 256) {
        const int fl = f & 63, ft = (f >> 6) % NT, fkh = (f >> 6) / NT;
        const int fm = fl & 15, fg = fl >> 4;
        const int e0 = (channel_of(ft, fm) * KH + fkh) * kwcin + 8 * fg;
        const unsigned sh = (unsigned)(e0 & 1) * 2u;
        const unsigned *src = bank + (e0 >> 1);
        i32x4_t dv;
#pragma unroll
        for (int j = 0; j < 4; ++j) dv[j] = (int)(__builtin_amdgcn_alignbyte(src[j + 1], src[j], sh) & k_mask(fg, j, kwcin));
        table[f] = dv;
    }
    __syncthreads();
    bf16x8_t wf[KHR][NT];
#pragma unroll
    for (int kh = 0; kh < KHR; ++kh) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            i32x4_t dv = {0, 0, 0, 0};
            if (KHT || kh < KH) dv = table[(kh * NT + t) * 64 + lane];
            wf[kh][t] = __builtin_bit_cast(bf16x8_t, dv);
        }
    }
    // bias of the lane's channels: rows 4 g + r of tile t
    float bv[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) bv[t][r] = p.bias ? p.bias[channel_of(t, 4 * g + r)] : 0.0f;
    __syncthreads();                                   // the table has been read: the images may be written

    // The rows of one output row: wave w fetches filter rows w and w + 4.
    // PAIRS: straight into LDS, 4 bytes per lane and load, through a raw buffer over the row: a lane
    // left of the row (its byte offset is negative: a huge unsigned one) or right of it lands a
    // zero, which is the horizontal padding, and a row above or below the input is an empty buffer.
    // No register, no bounds arithmetic and no LDS store is spent on it.  Otherwise element by
    // element through registers, written to the image once they are needed.
    const int imageDwords = KH * pitch;            // two sets of images: one is read while the next is written
    const unsigned ldsBase = (unsigned)(size_t)(GE_LDS char *)rowsLds;
    // byte offset of the lane's dword i of a row, from the row's first element; left of it: out of range
    unsigned rowOff[PAIRS ? DW_PER_LANE : 1];
    if (PAIRS) {
#pragma unroll
        for (int i = 0; i < DW_PER_LANE; ++i) {
            const int o = 4 * (lane + 64 * i) - 2 * left_pad(p.convPw, Cin);
            rowOff[i] = o < 0 ? 0x80000000u : (unsigned)o;
        }
    }
    unsigned staged[PAIRS ? 1 : ROWS_PER_WAVE][PAIRS ? 1 : DW_PER_LANE];
    auto fetch_rows = [&](int item, int set) __attribute__((always_inline)) {
        const int n = item / OH, oh = item - n * OH;
        const int ih0 = oh * p.convSh - p.convPh;
#pragma unroll
        for (int rr = 0; rr < ROWS_PER_WAVE; ++rr) {
            const int kh = wave + 4 * rr;
            const int ih = ih0 + kh * p.convDh;
            const bool rowOk = kh < KH && ih >= 0 && ih < H;
            const unsigned short *src = X + ((long long)n * H + (rowOk ? ih : 0)) * rowElems;
            if (PAIRS) {
                if (kh < KH) {
                    const rows_rsrc_t rs = rows_make_rsrc(src, rowOk ? (unsigned)rowElems * 2u : 0u);
                    const unsigned row = ldsBase + (unsigned)((set * KH + kh) * pitch) * 4u;
#pragma unroll
                    for (int i = 0; i < DW_PER_LANE; ++i)
                        if (64 * i < pitch) rows_lds_dma4(rs, row + 256u * i, rowOff[i]);      // pitch is a multiple of 64
                }
            } else {
#pragma unroll
                for (int i = 0; i < DW_PER_LANE; ++i) {
                    const int d = lane + 64 * i;
                    const int j0 = source_element(d, 0, p.convPw, Cin);
                    unsigned v = 0u;
                    if (rowOk && d < pitch && j0 >= 0 && j0 < rowElems) v = (unsigned)src[j0];
                    if (rowOk && d < pitch && j0 + 1 >= 0 && j0 + 1 < rowElems) v |= ((unsigned)src[j0 + 1]) << 16;
                    staged[PAIRS ? 0 : rr][PAIRS ? 0 : i] = v;
                }
            }
        }
    };
    auto land_rows = [&](int set) __attribute__((always_inline)) {
        if (PAIRS) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else {
#pragma unroll
            for (int rr = 0; rr < ROWS_PER_WAVE; ++rr) {
                const int kh = wave + 4 * rr;
                if (kh < KH) {
#pragma unroll
                    for (int i = 0; i < DW_PER_LANE; ++i) {
                        const int d = lane + 64 * i;
                        if (d < pitch) img[(set * KH + kh) * pitch + d] = staged[PAIRS ? 0 : rr][PAIRS ? 0 : i];
                    }
                }
            }
        }
    };

    int cur = 0;
    if ((int)blockIdx.x < items) {
        fetch_rows(blockIdx.x, 0);
        land_rows(0);
    }
    __syncthreads();
    const bool hasR = p.R != nullptr;
    for (int item = blockIdx.x; item < items; item += gridDim.x) {
        const int n = item / OH, oh = item - n * OH;
        const unsigned *image = img + cur * imageDwords;
        // the next output row's input is on its way while this one is multiplied
        const int next = item + gridDim.x;
        if (next < items) fetch_rows(next, cur ^ 1);

        for (int tile = wave; tile < tilesW; tile += 4) {
            const int ow = tile * PIX + m;
            const int e0 = window_start(ow, p.convSw, Cin, p.convPw) + 8 * g;
            const unsigned sh = (unsigned)(e0 & 1) * 2u;
            const unsigned *first = image + (e0 >> 1);
            f32x4_t acc[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int kh = 0; kh < KHR; ++kh) {
                if (KHT || kh < KH) {
                    const unsigned *row = first + kh * pitch;
                    unsigned q[5];
#pragma unroll
                    for (int j = 0; j < 5; ++j) q[j] = row[j];
                    i32x4_t f;
#pragma unroll
                    for (int j = 0; j < 4; ++j) f[j] = (int)(__builtin_amdgcn_alignbyte(q[j + 1], q[j], sh) & kmask[j]);
                    const bf16x8_t xf = __builtin_bit_cast(bf16x8_t, f);
#pragma unroll
                    for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[kh][t], xf, acc[t], 0, 0, 0);
                }
            }
            if (ow < OW) {
                const long long at = (((long long)n * OH + oh) * OW + ow) * Cout;
#pragma unroll
                for (int h = 0; h < NT / 2; ++h) {
                    const int cb = 32 * h + 8 * g;               // channel_of(2 h, 4 g) .. + 7
                    f32x4_t v[2];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        v[0][r] = p.alpha * acc[2 * h][r] + bv[2 * h][r];
                        v[1][r] = p.alpha * acc[2 * h + 1][r] + bv[2 * h + 1][r];
                    }
                    if (hasR) {
                        if (p.rType == DT_BF16) {
                            const i32x4_t rv = *(const i32x4_t *)((const unsigned short *)p.R + at + cb);
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                v[j >> 1][2 * (j & 1)] += p.beta * __uint_as_float(((unsigned)rv[j]) << 16);
                                v[j >> 1][2 * (j & 1) + 1] += p.beta * __uint_as_float(((unsigned)rv[j]) & 0xffff0000u);
                            }
                        } else {
                            const f32x4_t r0 = *(const f32x4_t *)((const float *)p.R + at + cb);
                            const f32x4_t r1 = *(const f32x4_t *)((const float *)p.R + at + cb + 4);
#pragma unroll
                            for (int r = 0; r < 4; ++r) { v[0][r] += p.beta * r0[r]; v[1][r] += p.beta * r1[r]; }
                        }
                    }
                    act_clamp_row_block<2>(p, v);
                    if (OUTBF16) {
                        const i32x4_t o = {(int)pack_bf16_pair(v[0][0], v[0][1]), (int)pack_bf16_pair(v[0][2], v[0][3]),
                                           (int)pack_bf16_pair(v[1][0], v[1][1]), (int)pack_bf16_pair(v[1][2], v[1][3])};
                        *(i32x4_t *)((unsigned short *)p.C + at + cb) = o;
                    } else {
                        *(f32x4_t *)((float *)p.C + at + cb) = v[0];
                        *(f32x4_t *)((float *)p.C + at + cb + 4) = v[1];
                    }
                }
            }
        }
        if (next < items) land_rows(cur ^ 1);
        // the image just read may be overwritten, the one just written may be read
        __syncthreads();
        cur ^= 1;
    }
}

}  // namespace ge
