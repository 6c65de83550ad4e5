/* libecco, second block format: the self-contained 4x block as the paper describes it.
 *
 * Section 3.2 "Model Compression" (two-level normalisation, 15 centroids plus a reserved index, H = 4
 * Huffman codebooks per shared pattern, clipping and outlier padding) and the 4x decompressor / compressor
 * of Sections 4.2 and 4.3.  Nothing lives outside the 64-byte block: no meta word, 4.00x against FP16.
 *
 * Format (one block = 128 FP16 values = 512 stream bits; stream bit j is bit 31 - (j & 31) of the
 * little-endian 32-bit word j >> 5, as in ecco.h; every field most significant bit first):
 *   bits 0..7    group scale, an 8-bit float: 1 sign, 4 exponent (bias 7), 3 mantissa bits, subnormals, every
 *                bit pattern a finite number (largest 480); it is the element of largest magnitude (first
 *                position on ties) divided by the per-tensor power-of-two scale 2^texp, rounded to nearest
 *                (ties to even, saturating), sign included
 *   bits 8..9    ID_HF, which of the pattern's four codebooks codes the data (the one with the shortest total
 *                length, lowest on ties)
 *   then         ID_KP, the pattern id in the model's canonical prefix code (1..8 bits)
 *   then         the codes (2..8 bits each) of the 128 indices in order: 0..14 = centroid of the pattern,
 *                15 = the element of largest magnitude itself
 *   clipping     the stream is cut at bit 512.  A value is present iff its whole code lies inside the block;
 *                values that are not present decode to +0
 *   padding      if all 128 values are present, floor(spare bits / 15) entries follow (at most 16): 7-bit
 *                position, 8-bit float of that element on the tensor scale; the elements are taken by
 *                decreasing magnitude (lower position first on ties), the largest excluded.  Remaining bits 0
 * Reconstruction: index k < 15 -> fp16(centroid[pattern][k] * |scale|) (exact FP32 product, one rounding),
 * index 15 -> the signed scale; a padded entry replaces the value at its position by its own 8-bit float
 * times 2^texp.  The encoder picks the pattern of least squared error over the 127 other elements against
 * those reconstructed centroids (nearest value, lowest index on ties; errors summed in FP32 in the balanced
 * pairwise tree; lowest pattern on ties).  The paper fixes the field widths, the reserved index, H = 4, the
 * 2..8-bit codes, clipping and the 15-bit padding entries; the 8-bit float layout, the field order, the bit
 * order and the tie rules are this library's reading (the paper's figure of the block is not available).
 *
 * Conventions as in ecco.h: status return values, device pointers owned by the caller, work enqueued on the
 * caller's stream, no CPU fallback.
 */
#ifndef ECCO_PAPER_BLOCK_H
#define ECCO_PAPER_BLOCK_H

#include <stddef.h>
#include <stdint.h>

#include "ecco.h"

#ifdef __cplusplus
extern "C" {
#endif

#define ECCO_PB_CENTROIDS 15
#define ECCO_PB_BOOKS 4
#define ECCO_PB_MIN_LEN 2
#define ECCO_PB_MAX_LEN 8

typedef struct ecco_pb_model ecco_pb_model; /* opaque; owned by the library; freed with ecco_pb_model_free */

/* CPU.  Fits a model to host FP16 data (n_values % 128 == 0, all finite), following Section 3.2: tensor scale
 * 2^texp from the largest magnitude; per group a 15-cluster 1-D k-means on the 127 normalised values besides
 * the largest; S shared patterns by k-means over those; per pattern 4 codebooks from a 4-cluster k-means over
 * the groups' index frequencies (optimal code lengths within 2..8 bits); a length-limited code for the pattern
 * ids from their use counts.  Deterministic in (data, S, seed).  At most 65 536 groups are used (seeded sample).
 * Errors: EINVAL (null, n_values, S outside 1..64), ENOMEM. */
int ecco_pb_fit(const uint16_t* data, size_t n_values, int S, uint64_t seed, ecco_pb_model** out);

/* CPU.  A model from its tables: centroids [S][15] FP16 bits (sorted, within [-1,1]), code_lens [S][4][16]
 * (2..8, Kraft sum exactly 1 per codebook), kp_lens [S] (1..8, Kraft sum 1, or at most 1 when S == 1),
 * texp in -15..7.  Errors: EINVAL, EFORMAT (a table fails validation), ENOMEM. */
int ecco_pb_model_create(const uint16_t* centroids, const uint8_t* code_lens, const uint8_t* kp_lens, int S, int texp,
                         ecco_pb_model** out);
/* CPU.  The model as a blob ({ 'ECP0', version 1, S, texp }, centroids, code lengths, pattern-id lengths; 2.1 KB + header for
 * S = 64).  save: *written receives the size needed; buf == NULL only queries it; EINVAL if cap is too small.  load validates
 * like ecco_pb_model_create (EFORMAT on a bad header, size or table). */
int ecco_pb_model_save(const ecco_pb_model* m, void* buf, size_t cap, size_t* written);
int ecco_pb_model_load(const void* buf, size_t len, ecco_pb_model** out);
int ecco_pb_model_S(const ecco_pb_model* m);
int ecco_pb_model_texp(const ecco_pb_model* m);
const uint16_t* ecco_pb_model_centroids(const ecco_pb_model* m); /* [S][15], valid while the model lives */
const uint8_t* ecco_pb_model_code_lens(const ecco_pb_model* m);  /* [S][4][16] */
const uint8_t* ecco_pb_model_kp_lens(const ecco_pb_model* m);    /* [S] */
/* uploads the decode / encode tables once (about 70 KB for S = 64); needed before encode / decode */
int ecco_pb_model_to_device(ecco_pb_model* m, int device);
void ecco_pb_model_free(ecco_pb_model* m);

/* GPU.  src: n_groups * 128 FP16 (finite), 4-byte aligned; blocks: n_groups * 64 bytes, 64-byte aligned.
 * Errors: EINVAL, EALIGN, EHIP.  n_groups == 0 returns OK. */
int ecco_pb_encode(const ecco_pb_model* m, const uint16_t* src_fp16, size_t n_groups, void* blocks, void* stream);
/* GPU.  dst: n_groups * 128 FP16, 16-byte aligned.  Any 64 bytes decode to the values the format statement
 * gives them.  Errors: EINVAL, ESHAPE (n_groups >= 2^31), EALIGN, EHIP. */
int ecco_pb_decode(const ecco_pb_model* m, const void* blocks, size_t n_groups, uint16_t* dst_fp16, void* stream);

/* GPU.  The decode fused into the consuming matrix-vector product (Section 2.1), batch 1: the FP16 weights never
 * reach HBM.  W = rows x cols as rows * (cols / 128) blocks, row-major; x device, cols FP16, 16-byte aligned; y device,
 * rows FP32: y[r] = sum_c W[r][c] * x[c], FP32 accumulation in a fixed order (results are reproducible; no device
 * memory beyond the arguments is used).  cols % 128 == 0, cols <= 65536.
 * Errors: EINVAL, ESHAPE, EALIGN, EHIP. */
int ecco_pb_decode_gemv(const ecco_pb_model* m, const void* blocks, int rows, int cols, const uint16_t* x, float* y,
                        void* stream);

#ifdef __cplusplus
}
#endif
#endif
