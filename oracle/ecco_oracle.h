/* CPU oracle for the Ecco block codec -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, step-by-step implementation of what the hot path computes, written from the
 * paper (Section 3.2 "Model Compression", Section 4.2 "Decompressor Design", Section 4.3
 * "Compressor Design") in the simplified block format this build measures (see include/ecco.h
 * for the format statement; the oracle restates it in its own code).  It shares no code with
 * the HIP library: only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Parity status of each function is stated in ecco_oracle.cpp's header.
 *
 * All pointers are host pointers.  fp16 travels as uint16_t bit patterns.
 */
#ifndef ECCO_ORACLE_H
#define ECCO_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORACLE_GROUP = 128, ORACLE_K = 16, ORACLE_BLOCK_BYTES = 64, ORACLE_MAX_LEN = 12, ORACLE_MAX_S = 64 };

/* number of threads the group-parallel loops use (1 = serial); returns the value in force */
int oracle_set_threads(int n);

/* fp16 <-> fp32, written out by hand (round to nearest even, subnormals kept) */
float    oracle_h2f(uint16_t h);
uint16_t oracle_f2h(float f);

/* dequantisation rule: fp16_rn( f32(c) * f32(s) ) */
uint16_t oracle_dequant(uint16_t c, uint16_t s);

/* ---- Huffman ---------------------------------------------------------------------------- */
/* optimal prefix-code lengths, no length limit (classic two-queue Huffman); n <= 64 */
int oracle_huffman_lengths(const uint64_t* counts, int n, uint8_t* lens);
/* optimal prefix-code lengths with every length <= max_len (package-merge); n <= 64 */
int oracle_limited_lengths(const uint64_t* counts, int n, int max_len, uint8_t* lens);
/* canonical code assignment: symbols ordered by (length, symbol); first code 0 */
void oracle_canonical_codes(const uint8_t* lens, int n, uint16_t* codes);

/* ---- model ------------------------------------------------------------------------------ */
/* checks every invariant of a model (S range, sortedness, finiteness, [-1,1], lengths in
 * [1,max], Kraft equality, prefix-freeness).  0 = ok, else the number of the failed check. */
int oracle_verify_model(const uint16_t* centroids, const uint8_t* lens, int S);

/* 1-D Lloyd k-means with K clusters on n values, quantile initialisation; returns iterations
 * done.  objective[it] (it = 0..iters) receives the sum of squared distances before each
 * update and after the last one.  cent_out is sorted ascending. */
int oracle_kmeans_1d(const float* v, int n, int K, int max_iter, double* cent_out, double* objective);

/* the whole fit of Section 3.2 steps 1-7 in this build's reading (each step is commented in the function body):
 * centroids[S*16] fp16 bits, lens[S*16], hist[S*16] (may be NULL), n_fit_groups (may be NULL) */
int oracle_fit(const uint16_t* data, size_t n_values, int S, int max_len, uint64_t seed,
               uint16_t* centroids, uint8_t* lens, uint64_t* hist, size_t* n_fit_groups);
/* the same fit, also handing out what its steps produced (each pointer may be NULL): pick[n_fit_groups] the indices
 * of the groups used (step 1; ascending), group_patterns[n_fit_groups*16] the sorted per-group centroids (step 3),
 * objective[0..*n_objective-1] the sum of squared distances to the nearest shared pattern at every assignment pass of
 * step 4 (at most 50 entries) */
int oracle_fit_trace(const uint16_t* data, size_t n_values, int S, int max_len, uint64_t seed,
                     uint16_t* centroids, uint8_t* lens, uint64_t* hist, size_t* n_fit_groups,
                     uint64_t* pick, double* group_patterns, double* objective, int* n_objective);

/* ---- encoder (Section 3.2 step 5 + Section 4.3) ---------------------------------------- */
/* one group: scale bits, chosen pattern, 128 indices, SSE of every pattern (sse may be NULL) */
void oracle_quantize_group(const uint16_t* centroids, int S, const uint16_t* x,
                           uint16_t* scale, int* pattern, uint8_t* idx, float* sse);
/* n_groups groups of 128 fp16 -> 64-byte blocks + one meta word per group */
void oracle_encode(const uint16_t* centroids, const uint8_t* lens, int S,
                   const uint16_t* src, size_t n_groups, uint8_t* blocks, uint32_t* meta);

/* min/max pattern selector of the online compressor (Section 3.2 "KV Cache Compression", Section 4.3):
 * fitness[p] = (group min - fp16(c[p][0]*s))^2 + (group max - fp16(c[p][15]*s))^2 in fp32; least wins,
 * lowest pattern on ties.  fitness may be NULL. */
void oracle_select_minmax(const uint16_t* centroids, int S, const uint16_t* x,
                          uint16_t* scale, int* pattern, float* fitness);
/* nearest reconstructed value of pattern p for each of the 128 values (lowest index on ties) */
void oracle_map_values(const uint16_t* centroids, int p, uint16_t scale, const uint16_t* x, uint8_t* idx);
/* as oracle_encode / oracle_kv_append, with the min/max selector in place of the least-squared-error search */
void oracle_encode_minmax(const uint16_t* centroids, const uint8_t* lens, int S,
                          const uint16_t* src, size_t n_groups, uint8_t* blocks, uint32_t* meta);

/* ---- decoder (Section 4.2) -------------------------------------------------------------- */
void oracle_decode_indices(const uint8_t* lens, int S, const uint8_t* blocks, const uint32_t* meta,
                           size_t n_groups, uint8_t* idx /* n_groups*128 */, uint16_t* used_bits /* may be NULL */);
void oracle_decode(const uint16_t* centroids, const uint8_t* lens, int S, const uint8_t* blocks,
                   const uint32_t* meta, size_t n_groups, uint16_t* dst /* n_groups*128 fp16 */);

/* ---- 2x activation codec (Section 3.2 "Activation Compression", Section 4.2 / 4.3 low-ratio units) ----
 * 64 FP16 values -> one 64-byte block: byte i = 7-bit two's-complement code q_i in bits 6:0, one
 * metadata bit in bit 7.  The metadata bits of bytes 0..15 are the FP16 scale s (bit i of s in byte i),
 * those of bytes 16..31 the FP16 zero point z, those of bytes 32..63 are 0.  Reconstruction:
 * x_i = fp16( q_i * s + z ), the exact value rounded once (what a fused FP16 multiply-add gives). */
enum { ORACLE_ACT_GROUP = 64 };
/* the reconstruction rule for one code (q in -64..63; s, z finite FP16 bit patterns) */
uint16_t oracle_act_dequant(int q, uint16_t s_bits, uint16_t z_bits);
/* scale and zero point of one group of 64 values */
void oracle_act_params(const uint16_t* x, uint16_t* s_bits, uint16_t* z_bits);
void oracle_act_encode(const uint16_t* src, size_t n_groups, uint8_t* blocks /* n_groups*64 */);
void oracle_act_decode(const uint8_t* blocks, size_t n_groups, uint16_t* dst /* n_groups*64 */);

/* ---- consumers -------------------------------------------------------------------------- */
/* y[b][r] = sum_c w[r][c] * x[b][c], accumulated in double over the decoded fp16 weights */
void oracle_gemv(const uint16_t* centroids, const uint8_t* lens, int S, const uint8_t* blocks,
                 const uint32_t* meta, int rows, int cols, const uint16_t* x, int batch, double* y);

/* append one token per sequence: k_new/v_new [B][H][128]; caches [B][H][T_max] blocks */
void oracle_kv_append(const uint16_t* ck, const uint8_t* lk, int Sk, const uint16_t* cv, const uint8_t* lv, int Sv,
                      const uint16_t* k_new, const uint16_t* v_new,
                      uint8_t* k_blocks, uint32_t* k_meta, uint8_t* v_blocks, uint32_t* v_meta,
                      const int32_t* seq_len, int B, int H, int T_max);

void oracle_kv_append_minmax(const uint16_t* ck, const uint8_t* lk, int Sk, const uint16_t* cv, const uint8_t* lv, int Sv,
                             const uint16_t* k_new, const uint16_t* v_new,
                             uint8_t* k_blocks, uint32_t* k_meta, uint8_t* v_blocks, uint32_t* v_meta,
                             const int32_t* seq_len, int B, int H, int T_max);

/* single-query attention over the compressed caches, double precision; out [B][H][128] */
void oracle_kv_attend(const uint16_t* ck, const uint8_t* lk, int Sk, const uint16_t* cv, const uint8_t* lv, int Sv,
                      const uint16_t* q, const uint8_t* k_blocks, const uint32_t* k_meta,
                      const uint8_t* v_blocks, const uint32_t* v_meta,
                      const int32_t* seq_len, int B, int H, int T_max, double* out);

/* grouped-query form: q and out [B][Hq][128], caches [B][Hkv][T_max]; query head h uses cache head h / (Hq / Hkv);
 * Hq must be a multiple of Hkv */
void oracle_kv_attend_gqa(const uint16_t* ck, const uint8_t* lk, int Sk, const uint16_t* cv, const uint8_t* lv, int Sv,
                          const uint16_t* q, const uint8_t* k_blocks, const uint32_t* k_meta,
                          const uint8_t* v_blocks, const uint32_t* v_meta,
                          const int32_t* seq_len, int B, int Hq, int Hkv, int T_max, double* out);

#ifdef __cplusplus
}
#endif
#endif
