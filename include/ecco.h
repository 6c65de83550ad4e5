/* libecco -- Ecco block codec for MI355X (gfx950): C ABI.
 *
 * Ecco (arxiv 2505.06901) stores every group of 128 FP16 weight or KV values in a fixed 64-byte
 * block: the values are normalised by the group's absolute maximum, quantised to 16 levels against
 * one of S shared, pre-defined k-means centroid patterns (the pattern of minimum squared error),
 * and the 4-bit level indices are Huffman coded (Section 3.1 "Compression Target", Section 3.2
 * "Model Compression").  This library holds the data-parallel hot path: block decode to FP16
 * (Section 4.2 "Decompressor Design"), decode fused into a batch-1..16 GEMV and into single-query
 * attention (the consumers of Section 2.1), and the per-group encoder (Section 4.3 "Compressor
 * Design") for bulk tensors and for appended KV tokens.  The pattern / codebook fit runs on the CPU.
 *
 * BLOCK FORMAT (the simplified format this build measures; the paper's self-contained block, which
 * keeps the scale, the pattern id and padded outliers inside the 64 bytes, is in ecco_paper_block.h):
 *   - group  = 128 consecutive FP16 values.  Matrices: row-major, group g = (row, col/128).
 *   - block  = 64 bytes of payload per group at byte offset 64*g: 16 little-endian 32-bit words
 *              holding a bit stream; stream bit j (0..511) is bit 31 - (j & 31) of word j >> 5
 *              (most significant bit of each word first).
 *       Huffman mode: the canonical codes of values 0..127 in order, each written first code
 *              bit (most significant) first, starting at stream bit 0; remaining bits are 0.
 *       Raw mode (used when the codes need more than 512 bits): value i's 4-bit index sits in
 *              stream bits 4i..4i+3, most significant bit first.
 *   - meta   = one uint32 per group: bits 15:0 scale (FP16 bit pattern of max|x|, sign 0),
 *              bits 21:16 pattern id, bit 22 raw flag, bits 31:23 the stream bit at which the
 *              code of value 64 begins (256 in raw mode).  A decoder reads values 0..63 from
 *              bit 0 and values 64..127 from that position, so a block is two independent
 *              chains of 64 values; the encoder writes the position where value 63 ended.
 *   - model  = S patterns x 16 FP16 centroids in [-1,1], ascending, plus S x 16 code lengths in
 *              1..12 with Kraft sum exactly 1.  Codes are canonical: symbols ordered by
 *              (length, symbol); first code 0; next = (previous + 1) << (length growth).
 *   - value  = fp16_rn( f32(centroid[pattern][index]) * f32(scale) )   (one rounding).
 *   Decoders never read outside a block: stream bits >= 512 read as 0; a pattern id >= S is
 *   treated as S-1.  Any 64 bytes + any meta word therefore decode to something defined.
 *
 * CONVENTIONS
 *   - every function returns an ecco_status (0 = ok, negative = error); nothing throws.
 *   - "host" / "device" in a parameter comment says where the pointer must point.  The library
 *     never allocates, frees or keeps caller buffers; device work is enqueued on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and the call returns without
 *     synchronising.  Argument errors are detected on the host before anything is launched, in
 *     this order: null pointers (EINVAL), sizes (ESHAPE), alignment (EALIGN), and last whether the
 *     model is on a device (EINVAL) -- so the first three can be checked on a machine without a GPU.
 *   - device work is launched on the calling thread's current device, which must be the device the
 *     model was uploaded to; with another device current the call returns ECCO_EINVAL.
 *   - FP16 travels as uint16_t bit patterns.
 */
#ifndef ECCO_H
#define ECCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ECCO_GROUP 128
#define ECCO_BLOCK_BYTES 64
#define ECCO_K 16
#define ECCO_MAX_LEN 12
#define ECCO_MAX_S 64

typedef struct ecco_model ecco_model; /* opaque; owned by the library; host copy + one device copy */

typedef enum {
    ECCO_OK = 0,
    ECCO_EINVAL = -1,  /* null pointer, value out of range, model not on a device */
    ECCO_ESHAPE = -2,  /* size not a multiple of 128, batch outside 1..16, ... */
    ECCO_EALIGN = -3,  /* pointer not aligned as documented */
    ECCO_ENOMEM = -4,
    ECCO_EFORMAT = -5, /* serialized model fails validation */
    ECCO_EHIP = -6     /* a HIP runtime call failed */
} ecco_status;

const char* ecco_strerror(int status);

/* ---- model: fit, (de)serialise, upload ------------------------------------------------------ */

/* Section 3.2, offline steps: partition into groups of 128, normalise by the group maximum,
 * 16-cluster k-means per group, S-cluster k-means over the sorted per-group centroid vectors
 * (the shared patterns), quantise with pattern selection, and one length-limited canonical Huffman
 * codebook per pattern from the pooled index counts.  CPU only, deterministic in (data, S, seed).
 *   data        host, n_values FP16 bit patterns, all finite; n_values % 128 == 0, n_values > 0
 *   S           1..64 patterns;  max_code_len 4..12
 *   out         receives a new model (free with ecco_model_free)
 * Errors: EINVAL (null, S / max_code_len out of range, non-finite data), ESHAPE (n_values). */
int ecco_fit_patterns(const uint16_t* data, size_t n_values, int S, int max_code_len,
                      uint64_t seed, ecco_model** out);

/* Builds a model from explicit tables (host): centroids[S*16] FP16 bits, code_lens[S*16].
 * Validates as ecco_model_load does.  Errors: EINVAL, EFORMAT. */
int ecco_model_create(const uint16_t* centroids, const uint8_t* code_lens, int S, ecco_model** out);

/* Serialised model: little-endian { u32 magic 'ECC0', u32 version 1, u32 S, u32 K=16,
 * S*16 u16 centroids, S*16 u8 code lengths }.  save: buf may be NULL to query *written.
 * load validates: S range, centroids finite, in [-1,1], ascending; lengths 1..12; Kraft sum 1.
 * Errors: EINVAL (null / cap too small), EFORMAT (validation). */
int ecco_model_save(const ecco_model* m, void* buf /*host*/, size_t cap, size_t* written);
int ecco_model_load(const void* buf /*host*/, size_t len, ecco_model** out);

/* Read-only views of the host tables (valid until ecco_model_free). */
int ecco_model_S(const ecco_model* m);
const uint16_t* ecco_model_centroids(const ecco_model* m); /* S*16 */
const uint8_t* ecco_model_code_lens(const ecco_model* m);  /* S*16 */

/* Uploads the decode / encode tables to `device` (Section 4.2: tensor-level metadata is loaded
 * once, before any compressed load).  Must precede every GPU call below.  Calling it again for the
 * same device is a no-op; another device moves the tables.  Errors: EINVAL, EHIP, ENOMEM. */
int ecco_model_to_device(ecco_model* m, int device);
void ecco_model_free(ecco_model* m);

/* ---- GPU entry points ------------------------------------------------------------------------ */

/* Section 3.2 step 5 + Section 4.3: per group, scale = max|x|; every pattern's centroids times
 * scale rounded to FP16; each value to the nearest reconstructed value (lowest index on ties);
 * squared errors summed per pattern in FP32 by the balanced tree (i, i^1), (.., i^2), ...; pattern
 * of least sum (lowest id on ties); Huffman pack, or raw mode when the codes exceed 512 bits.
 *   src     device, n_groups*128 FP16, finite          blocks  device, n_groups*64 bytes, 64-byte aligned
 *   meta    device, n_groups uint32
 * Errors: EINVAL (null, model not on device), EALIGN, EHIP.  n_groups == 0 is a no-op (pointers may be null). */
int ecco_encode(const ecco_model* m, const uint16_t* src, size_t n_groups,
                void* blocks, uint32_t* meta, void* stream);

/* Section 4.2: pattern retrieval, Huffman decode, centroid x scale.  dst: device, n_groups*128 FP16,
 * 16-byte aligned.  Same errors as ecco_encode, plus ESHAPE for n_groups >= 2^31 - 32. */
int ecco_decode(const ecco_model* m, const void* blocks, const uint32_t* meta, size_t n_groups,
                uint16_t* dst, void* stream);

/* Like ecco_decode but writes the 4-bit indices, one per byte (idx: device, n_groups*128 bytes,
 * 16-byte aligned).  For index-level parity checks. */
int ecco_decode_indices(const ecco_model* m, const void* blocks, const uint32_t* meta, size_t n_groups,
                        uint8_t* idx, void* stream);

/* Decode fused into the consuming GEMV (Section 2.1: decode-phase projections are memory-bound
 * matrix-vector products); the FP16 weights never reach HBM.
 *   W = rows x cols, stored as rows*(cols/128) blocks, row-major;   x  device, batch x cols FP16, 16-byte aligned
 *   y  device, batch x rows FP32:  y[b][r] = sum_c W[r][c] * x[b][c]  (FP32 accumulation)
 *   batch 1..16;  cols % 128 == 0;  cols <= 65536.
 * A row is never split over workgroups and no device memory beyond the arguments and the model's
 * tables is touched, so calls may overlap freely and the sum order is fixed (results are reproducible).
 * Errors: EINVAL, ESHAPE (cols, batch, rows <= 0), EALIGN, EHIP. */
int ecco_decode_gemv(const ecco_model* m, const void* blocks, const uint32_t* meta,
                     int rows, int cols, const uint16_t* x, int batch, float* y, void* stream);

/* Section 3.2 "KV Cache Compression", online part: encodes one new token per sequence.
 *   k_new, v_new   device, [B][H][128] FP16
 *   k_blocks ...   device caches, [B][H][T_max] blocks / meta words (block (b,h,t) at index (b*H+h)*T_max+t)
 *   seq_len        device, [B] int32: write position of each sequence; a position outside
 *                  0..T_max-1 writes nothing.  The caller advances seq_len afterwards.
 * Pattern selection is the full minimum-squared-error search of ecco_encode (mk for K, mv for V).
 * Errors: EINVAL, ESHAPE (B, H, T_max <= 0), EALIGN, EHIP. */
int ecco_kv_append(const ecco_model* mk, const ecco_model* mv,
                   const uint16_t* k_new, const uint16_t* v_new,
                   void* k_blocks, uint32_t* k_meta, void* v_blocks, uint32_t* v_meta,
                   const int32_t* seq_len, int B, int H, int T_max, void* stream);

/* The online compressor's cheap pattern selector (Section 3.2 "KV Cache Compression"; pattern selector of
 * Section 4.3): instead of quantising the group with every pattern, the group's least and greatest value are
 * compared with each pattern's first and last centroid, both in the group's scale:
 *     fitness[p] = (min_i x_i - fp16(c[p][0]*s))^2 + (max_i x_i - fp16(c[p][15]*s))^2     (FP32, each operation rounded)
 * the least fitness wins (lowest p on a tie) and only that pattern's value mapping and packing are done.
 * The extremes run over all 128 values: this format quantises the absmax element with the pattern like any
 * other value.  Blocks and meta words have the format of ecco_encode, so every decoder reads them.
 * Arguments, layout, ownership and errors as ecco_encode / ecco_kv_append. */
int ecco_encode_minmax(const ecco_model* m, const uint16_t* src_fp16, size_t n_groups,
                       void* blocks, uint32_t* meta, void* stream);
int ecco_kv_append_minmax(const ecco_model* mk, const ecco_model* mv,
                          const uint16_t* k_new, const uint16_t* v_new,
                          void* k_blocks, uint32_t* k_meta, void* v_blocks, uint32_t* v_meta,
                          const int32_t* seq_len, int B, int H, int T_max, void* stream);

/* ---- 2x activation codec (Section 3.2 "Activation Compression"; low-ratio units of Sections 4.2, 4.3) ----------
 * Uniform integer quantisation with a zero point, 7 bits per value: 64 FP16 values (128 bytes) become one 64-byte
 * block, no side data, no model.
 *   byte i of a block:  bits 6:0  the two's-complement code q_i (-64..63) of value i;  bit 7  one metadata bit.
 *   The metadata bits of bytes 0..15 are the FP16 scale s (bit i of s in byte i), those of bytes 16..31 the FP16
 *   zero point z (bit i-16 of z in byte i), those of bytes 32..63 are written 0 and ignored by the decoder.
 *   Reconstruction:  x_i = fp16( q_i * s + z ), the exact value rounded once (a fused FP16 multiply-add).
 *   Encoder, per group of 64 consecutive values (all finite):
 *     s = fp16((max - min) / 127),  z = fp16(min + 64 s)           FP32 operations, each rounded on its own
 *     q_i = round-to-nearest-even((x_i - z) * (1 / s)) clamped to -64..63;  s = 0 (constant group): q_i = 0;
 *     a code whose reconstruction would be infinite (only next to +-65504) moves one step towards 0, at most twice.
 *   The paper fixes the widths (7 data bits, 16-bit scale and zero point in the eighth bits, 512-bit block) and the
 *   sign extension; bit order, the formulas for s, z and q and the reserved upper half are this library's reading.
 *   src / dst   device, n_groups * 64 FP16, 16-byte aligned;   blocks   device, n_groups * 64 bytes, 64-byte aligned.
 * A block whose scale or zero point is not finite (never written by the encoder) decodes to unspecified values.
 * Errors: EINVAL (null pointer), ESHAPE (n_groups > 2^40), EALIGN, EHIP.  n_groups == 0 returns OK and touches nothing. */
int ecco_act_encode(const uint16_t* src_fp16, size_t n_groups, void* blocks, void* stream);
int ecco_act_decode(const void* blocks, size_t n_groups, uint16_t* dst_fp16, void* stream);

/* Single-query attention over the compressed caches (Section 2.1): per (b,h), scores
 * q.K_t / sqrt(128) for t < seq_len[b], softmax, out = sum_t p_t V_t.  No mask beyond seq_len.
 *   q  device [B][H][128] FP16, 16-byte aligned;  out  device [B][H][128] FP32 (zeros where seq_len[b] <= 0).
 * seq_len values above T_max are clamped to T_max.  Errors as ecco_kv_append. */
int ecco_kv_attend(const ecco_model* mk, const ecco_model* mv, const uint16_t* q,
                   const void* k_blocks, const uint32_t* k_meta, const void* v_blocks, const uint32_t* v_meta,
                   const int32_t* seq_len, int B, int H, int T_max, float* out, void* stream);

/* Measurement aid, not part of the codec: reads `bytes` bytes (a multiple of 16; src device, 16-byte aligned) with one launch
 * of 256 workgroups and writes a checksum word per workgroup to out[0..255] (device).  Timed over the same compressed bytes as
 * a decoder, it gives the rate at which the machine can merely read them: the practical ceiling that the benchmark prints
 * beside the data-sheet bandwidth.  Errors: EINVAL, ESHAPE (bytes % 16), EALIGN, EHIP. */
int ecco_read_stream(const void* src, size_t bytes, uint32_t* out, void* stream);
/* Measurement aid: what the runtime reports for `device` -- compute units, memory clock (kHz) and memory bus width
 * (bits), printed by the benchmark beside the data-sheet bandwidth its roofline uses.  All three outputs are host pointers.  Errors: EINVAL (null, device < 0), EHIP. */
int ecco_device_info(int device, int* compute_units, int* memory_clock_khz, int* memory_bus_bits);

/* Grouped-query form of ecco_kv_attend, split over the tokens (Section 5.3: with grouped-query attention several
 * query heads share one key/value head and the matrix-vector products become small matrix products).
 *   q, out      device, [B][Hq][128] (FP16, 16-byte aligned / FP32);  caches  [B][Hkv][T_max] blocks and meta words
 *   Hq % Hkv == 0, Hq / Hkv <= 16; query head h reads the cache of head h / (Hq / Hkv).
 *   n_splits    1..256: each (sequence, key/value head) is cut into n_splits token ranges handled by separate
 *               workgroups (use it when B * Hkv is well below the number of compute units);  with n_splits > 1
 *               `workspace` (device, 16-byte aligned, ecco_kv_attend_gqa_workspace(B, Hq, n_splits) bytes, owned by the
 *               caller, contents irrelevant before and after) receives the partial results and a second small kernel
 *               merges them;  with n_splits == 1 workspace may be null.
 * Every K and V block is decoded once for all query heads of its group; products run on the matrix cores with the
 * probabilities rounded to FP16 (the denominator sums the rounded values).  Slots of the cache at or behind seq_len
 * may be uninitialised.  Calls that share a workspace must not overlap.
 * Errors: EINVAL, ESHAPE (sizes, Hq % Hkv, group > 16, n_splits), EALIGN, EHIP. */
size_t ecco_kv_attend_gqa_workspace(int B, int Hq, int n_splits);
/* A split count for ecco_kv_attend_gqa: enough token ranges to give every compute unit of `device` a workgroup
 * (B * Hkv * n_splits >= compute units where the sequences allow it), at least 256 tokens each, at most 256 splits.
 * `tokens` is the longest sequence to be read.  Returns >= 1, or ESHAPE for a size <= 0.  An unknown device counts
 * as 256 compute units. */
int ecco_kv_attend_gqa_splits(int device, int B, int Hkv, int tokens);
int ecco_kv_attend_gqa(const ecco_model* mk, const ecco_model* mv, const uint16_t* q,
                       const void* k_blocks, const uint32_t* k_meta, const void* v_blocks, const uint32_t* v_meta,
                       const int32_t* seq_len, int B, int Hq, int Hkv, int T_max, int n_splits, void* workspace,
                       float* out, void* stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): ecco_kv_attend_gqa with the token splits' partial results kept in a static
 * device array inside the library instead of a caller's workspace.  Same arguments (without `workspace`), same kernels,
 * same results bit for bit.  The call allocates and frees nothing.
 *   Limit: ecco_kv_attend_gqa_workspace(B, Hq, n_splits) = B * Hq * n_splits * 520 bytes must not exceed
 *   ECCO_GQA_SCRATCH_BYTES (8 MiB: B * Hq * n_splits <= 16131); larger sizes return ESHAPE and launch nothing.
 *   n_splits == 1 uses no scratch and has no limit.
 *   The array exists once per GPU and is shared by every call on that GPU: calls that overlap on one GPU (different
 *   streams, or host threads) race on it and must be serialised by the caller.  Nothing in it has to start at zero (every
 *   word that is read was written by the same call), and its contents after a call are unspecified.
 *   Its device address is looked up when a model is uploaded (ecco_model_to_device), so this call touches no runtime
 *   service beyond the two kernel launches.
 * Errors: as ecco_kv_attend_gqa; ESHAPE also for a size beyond the limit. */
#define ECCO_GQA_SCRATCH_BYTES (8u << 20)
int ecco_kv_attend_gqa_noalloc(const ecco_model* mk, const ecco_model* mv, const uint16_t* q,
                               const void* k_blocks, const uint32_t* k_meta, const void* v_blocks, const uint32_t* v_meta,
                               const int32_t* seq_len, int B, int Hq, int Hkv, int T_max, int n_splits,
                               float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif
