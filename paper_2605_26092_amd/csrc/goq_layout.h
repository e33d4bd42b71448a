// Packed device layout of a dual-PoT layer (the stored representation of Sec. 3.3 item 3:
// PoT code per weight, 2-bit pattern + 4 pair signs per 8-weight micro-block, two fp16
// coefficients per 128-weight macro-block), arranged for coalesced 16-byte-per-lane loads.
//
// Unit of the layout: a ROW BLOCK of 64 consecutive output channels times one macro-block
// (128 input channels).  It is stored as CH "chunks" of 1 KiB; chunk h holds, for every row
// r = 0..63 of the block, one 16-byte quad at byte offset r*16: 32 consecutive weights of the
// row (four micro-blocks), which is one k-slice group of a matrix-core operand.  A wavefront
// whose lanes read 16 consecutive quads of each of four chunks (or 64 of one) issues loads made
// of full 256-byte runs, and the unit's bytes are each read exactly once.
//
//   dword index of (row block R, macro-block g, chunk h, row r, dword q)
//        = ((((R * G_n + g) * CH + h) * 64 + r) * 4 + q            G_n = in / 128
//
// bw = 3 (CH = 4, 64 B per macro-block row = 4.0 bit/weight): dword q of chunk h is micro-block
//   m = 4h + q.  Byte j of the dword:  bits 0..2 code[8m+j], bits 3..5 code[8m+j+4],
//   bits 6..7 an auxiliary pair a_j:  a_0 = pattern (s-1), a_1 = signs bits 0..1,
//   a_2 = signs bits 2..3, a_3 = two bits of the coefficient word CW = c1 | c2 << 16, namely
//   bits (31-2m, 30-2m): folding cw = (cw << 2) | (dword >> 30) over m = 0..15 rebuilds CW.
//
// bw = 4 (CH = 5, 80 B per macro-block row = 5.0 bit/weight): chunks 0..3 as above but a dword
//   is eight 4-bit codes, byte j = code[8m+j] | code[8m+j+4] << 4.  Chunk 4 holds the metadata,
//   dword q for the four micro-blocks of chunk q: bits 6i..6i+5 = pattern | signs << 2 of
//   micro-block m = 4q + i (i = 0..3), bits 24..31 = byte q of CW.  The lane that decodes chunk q
//   of a row thus needs this one dword besides its quad.
//
// Rows are padded to a multiple of 64 with zero-valued codes and zero coefficients.
#pragma once
#include <stdint.h>

#define GOQ_N 128
#define GOQ_G 8
#define GOQ_ROWS 64

#if defined(__HIPCC__)
#define GOQ_HD __host__ __device__ __forceinline__
#else
#define GOQ_HD inline
#endif

GOQ_HD int goq_chunks(int bw) { return bw == 3 ? 4 : 5; }

GOQ_HD int64_t goq_row_blocks(int64_t out) { return (out + GOQ_ROWS - 1) / GOQ_ROWS; }

// dword index of the first dword of the quad of (R, g, h, r)
GOQ_HD int64_t goq_quad_index(int ch, int64_t gn, int64_t R, int64_t g, int h, int r)
{
    return ((((R * gn + g) * ch + h) * GOQ_ROWS + r) * 4);
}

GOQ_HD int64_t goq_packed_dwords(int bw, int64_t out, int64_t in)
{
    return goq_row_blocks(out) * (in / GOQ_N) * goq_chunks(bw) * GOQ_ROWS * 4;
}

// canonical code of the zero state
GOQ_HD int goq_zero_code(int bw) { return (1 << (bw - 1)) - 1; }
