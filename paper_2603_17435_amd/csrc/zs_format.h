// Geometry constants of the TCA-TBE blob (Section 4.2 of the ZipServ paper), shared by
// the host packer and the HIP kernels of this library.
#ifndef ZS_FORMAT_H
#define ZS_FORMAT_H

#define ZS_WINDOW 7            /* consecutive exponents with a 3-bit codeword             */
#define ZS_FT_DIM 8            /* FragTile 8 x 8                                          */
#define ZS_FT_ELEMS 64
#define ZS_FT_BITMAP_BYTES 24  /* three uint64 bit-planes                                 */
#define ZS_TT_ROWS 16          /* TensorCoreTile 16 (N) x 32 (K): one MFMA 16x16x32 A operand */
#define ZS_TT_COLS 32
#define ZS_TT_ELEMS 512
#define ZS_FT_PER_TT 8
#define ZS_TT_BITMAP_BYTES 192
#define ZS_BT_DIM 64           /* BlockTile 64 x 64                                       */
#define ZS_BT_ELEMS 4096
#define ZS_TT_PER_BT 8
#define ZS_BT_BITMAP_BYTES 1536
#define ZS_SECTION_ALIGN 256

#endif
