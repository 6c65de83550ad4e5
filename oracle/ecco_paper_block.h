/* CPU oracle for the paper's own self-contained 4x block -- TEST INFRASTRUCTURE ONLY.
 *
 * Section 3.2 "Model Compression" (two-level normalisation with an FP8 group scale, 15 centroids plus a
 * reserved index for the absolute maximum, H Huffman codebooks per pattern, clipping and outlier padding)
 * and Section 4.2 / 4.3 (decompressor and compressor of the 4x scheme), in the reading stated at the top
 * of ecco_paper_block.cpp.  Shares no code with the HIP library.  All pointers are host pointers; fp16
 * travels as uint16_t bit patterns.
 */
#ifndef ECCO_PAPER_BLOCK_ORACLE_H
#define ECCO_PAPER_BLOCK_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { PB_GROUP = 128, PB_CENTROIDS = 15, PB_SYMBOLS = 16, PB_BOOKS = 4, PB_BLOCK_BYTES = 64,
       PB_MIN_LEN = 2, PB_MAX_LEN = 8, PB_MAX_S = 64, PB_OUTLIER_BITS = 15 };

/* the 8-bit float of this format: 1 sign, 4 exponent (bias 7), 3 mantissa bits, subnormals, no infinities or NaN */
double pb_fp8_value(uint8_t b);
uint8_t pb_fp8_round(double v); /* nearest, ties to even mantissa, saturating at +-480 */

/* a model: S patterns of 15 sorted centroids, 4 codebooks of 16 code lengths per pattern, code lengths of the
 * pattern ids, and the exponent of the per-tensor power-of-two FP16-to-FP8 scale */
typedef struct {
    int S;
    int texp;                                              /* tensor scale = 2^texp, -15..7 */
    const uint16_t* cent;                                  /* [S][15] fp16 bits */
    const uint8_t* lens;                                   /* [S][4][16], 2..8 */
    const uint8_t* kp_lens;                                /* [S], 1..8 */
} pb_model;

/* 0 = every invariant holds, else the number of the failed check */
int pb_verify_model(const pb_model* m);

/* what the encoder decides for one group before packing (for tests): position of the absolute maximum, FP8
 * scale byte, pattern, codebook, the 128 indices */
void pb_quantize_group(const pb_model* m, const uint16_t* x, int* amax_pos, uint8_t* scale8, int* pattern, int* book,
                       uint8_t* idx);
void pb_encode(const pb_model* m, const uint16_t* src, size_t n_groups, uint8_t* blocks);
/* decode to fp16; n_coded / n_outliers (may be NULL) receive per block how many values were inside the block and
 * how many outlier entries followed */
void pb_decode(const pb_model* m, const uint8_t* blocks, size_t n_groups, uint16_t* dst, uint8_t* n_coded, uint8_t* n_outliers);

/* y[r] = sum_c w[r][c] * x[c] over the decoded weights (rows x cols, cols % 128 == 0, blocks row-major), in double */
void pb_gemv(const pb_model* m, const uint8_t* blocks, int rows, int cols, const uint16_t* x, double* y);

#ifdef __cplusplus
}
#endif
#endif
