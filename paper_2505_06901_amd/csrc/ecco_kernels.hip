// HIP kernels (gfx950) and GPU entry points of libecco.
//
// Mapping used throughout: one lane owns one 64-byte block and decodes its 128 indices in order;
// a wavefront therefore works on 64 blocks at once and all lanes sit at the same index position,
// whatever their bit positions.  Block payloads are brought into LDS with coalesced 16-byte loads
// and stored there with a 17-word stride, so that the per-lane word fetches of the bit window hit
// distinct banks.  The per-pattern decode tables are staged in LDS once per workgroup.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <algorithm>

#include "ecco_internal.h"

using namespace ecco;

namespace {

constexpr int kThreads = 256;
constexpr int kStride = kBlockWords + 1;  // LDS words per staged block

#define ECCO_HIP_CHECK(expr) do { if ((expr) != hipSuccess) return ECCO_EHIP; } while (0)

struct Tables {           // LDS copies of the model's decode tables
    const uint8_t* lut8;  // [kLutSlots][256]
    const uint32_t* longtab;  // [S][16]
    const __half* cent;   // [S][16]
};

// ---- staging ------------------------------------------------------------------------------------
// copies `bytes` (multiple of 4) from global to LDS, all threads of the workgroup
__device__ inline void stage_words(uint32_t* dst, const void* src, int bytes) {
    const uint32_t* s = static_cast<const uint32_t*>(src);
    for (int i = threadIdx.x; i < bytes / 4; i += blockDim.x) dst[i] = s[i];
}

// brings `count` consecutive blocks (starting at block index first) into LDS, stride kStride words
__device__ inline void stage_payload(uint32_t* lds, const uint4* blocks, size_t first, int count) {
    const uint4* src = blocks + first * 4;
    for (int i = threadIdx.x; i < count * 4; i += blockDim.x) {
        uint4 v = src[i];
        uint32_t* d = lds + (i >> 2) * kStride + (i & 3) * 4;
        d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
    }
}

struct MetaWord {
    uint32_t scale_bits, pattern, slot;
};
__device__ inline MetaWord unpack_meta(uint32_t m, int S) {
    MetaWord r;
    r.scale_bits = m & 0xFFFFu;
    uint32_t p = (m >> 16) & 0x3Fu;
    r.pattern = p < (uint32_t)S ? p : (uint32_t)(S - 1);
    r.slot = ((m >> 22) & 1u) ? (uint32_t)kRawSlot : r.pattern;
    return r;
}

// ---- the decoder --------------------------------------------------------------------------------
// Walks one staged block, calling sink(i, index) for i = 0..127.  `w` points at the block's 16 words
// in LDS; words past the block read as zero.  The window always holds more than 32 valid bits
// before a lookup, so a 12-bit code never runs out of bits.
template <class Sink>
__device__ inline void decode_block(const uint32_t* w, const uint8_t* lut, const uint32_t* longtab, Sink&& sink) {
    uint64_t win = (uint64_t)w[0] | ((uint64_t)w[1] << 32);
    int valid = 64, next = 2;
#pragma unroll 16
    for (int i = 0; i < kGroup; ++i) {
        uint32_t e = lut[(uint32_t)win & 0xFFu];
        uint32_t len = e >> 4, sym = e & 15u;
        if (len == 0) {
            // code longer than the peek: rank of the 12-bit prefix among the left-aligned canonical codes
            uint32_t v = __brev((uint32_t)win) >> (32 - kMaxLen);
            int rank = 0;
            for (int j = 1; j < kK; ++j) rank += ((longtab[j] & 0xFFFu) <= v) ? 1 : 0;
            uint32_t t = longtab[rank];
            sym = (t >> 12) & 15u;
            len = t >> 16;
        }
        sink(i, sym);
        win >>= len;
        valid -= (int)len;
        if (valid <= 32) {
            uint32_t nw = next < kBlockWords ? w[next] : 0u;
            ++next;
            win |= (uint64_t)nw << valid;
            valid += 32;
        }
    }
}

// dequantisation: one exact FP32 product, one rounding to FP16
__device__ inline __half dequant(__half c, float s) { return __float2half_rn(__half2float(c) * s); }

__device__ inline float scale_of(uint32_t bits) { return __half2float(__ushort_as_half((unsigned short)bits)); }

// LDS carve-up common to the decode-side kernels
struct DecodeLds {
    uint32_t* payload;
    Tables t;
};
__device__ inline DecodeLds setup_decode_lds(unsigned char* smem, const unsigned char* dev, int S, int threads, unsigned char** rest) {
    DecodeLds d;
    uint32_t* lut8 = reinterpret_cast<uint32_t*>(smem);
    uint32_t* longtab = lut8 + kLutSlots * 256 / 4;
    uint32_t* cent = longtab + kMaxS * kK;
    uint32_t* payload = cent + kMaxS * kK / 2;
    stage_words(lut8, dev + DevLayout::lut8, kLutSlots * 256);
    stage_words(longtab, dev + DevLayout::longtab, S * kK * 4);
    stage_words(cent, dev + DevLayout::cent, S * kK * 2);
    d.payload = payload;
    d.t.lut8 = reinterpret_cast<const uint8_t*>(lut8);
    d.t.longtab = longtab;
    d.t.cent = reinterpret_cast<const __half*>(cent);
    *rest = reinterpret_cast<unsigned char*>(payload + threads * kStride);
    return d;
}
constexpr size_t kDecodeLdsBytes = kLutSlots * 256 + kMaxS * kK * 4 + kMaxS * kK * 2 + (size_t)kThreads * kStride * 4;

// ---- ecco_decode / ecco_decode_indices -----------------------------------------------------------
template <bool kIndices>
__global__ __launch_bounds__(kThreads) void decode_kernel(const unsigned char* __restrict__ dev, int S,
                                                          const uint4* __restrict__ blocks, const uint32_t* __restrict__ meta,
                                                          size_t n_groups, void* __restrict__ dst) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* rest;
    DecodeLds L = setup_decode_lds(smem, dev, S, kThreads, &rest);
    for (size_t first = (size_t)blockIdx.x * kThreads; first < n_groups; first += (size_t)gridDim.x * kThreads) {
        const size_t left = n_groups - first;
        int count = left < (size_t)kThreads ? (int)left : kThreads;
        __syncthreads();
        stage_payload(L.payload, blocks, first, count);
        __syncthreads();
        if ((int)threadIdx.x < count) {
            size_t g = first + threadIdx.x;
            MetaWord mw = unpack_meta(meta[g], S);
            const uint32_t* w = L.payload + threadIdx.x * kStride;
            if (kIndices) {
                uint4* out = reinterpret_cast<uint4*>(static_cast<uint8_t*>(dst) + g * kGroup);
                uint32_t acc[4] = {0, 0, 0, 0};
                decode_block(w, L.t.lut8 + mw.slot * 256, L.t.longtab + mw.pattern * kK, [&](int i, uint32_t sym) {
                    acc[(i >> 2) & 3] |= sym << (8 * (i & 3));
                    if ((i & 15) == 15) {
                        out[i >> 4] = make_uint4(acc[0], acc[1], acc[2], acc[3]);
                        acc[0] = acc[1] = acc[2] = acc[3] = 0;
                    }
                });
            } else {
                uint4* out = reinterpret_cast<uint4*>(static_cast<uint16_t*>(dst) + g * kGroup);
                const __half* c = L.t.cent + mw.pattern * kK;
                const float s = scale_of(mw.scale_bits);
                uint32_t acc[4] = {0, 0, 0, 0};
                decode_block(w, L.t.lut8 + mw.slot * 256, L.t.longtab + mw.pattern * kK, [&](int i, uint32_t sym) {
                    uint32_t h = __half_as_ushort(dequant(c[sym], s));
                    acc[(i >> 1) & 3] |= h << (16 * (i & 1));
                    if ((i & 7) == 7) {
                        out[i >> 3] = make_uint4(acc[0], acc[1], acc[2], acc[3]);
                        acc[0] = acc[1] = acc[2] = acc[3] = 0;
                    }
                });
            }
        }
    }
}

// ---- ecco_decode_gemv, baseline kernel (any batch, one batch row per pass) -------------------------
// A workgroup owns `rows_per_wg` whole rows.  Column groups are taken in slabs of kSlabGroups; the
// slab's slice of x sits in LDS with 65 words per group, so lanes working on neighbouring column
// groups read different banks.  Each lane forms the dot product of its block with x in FP32
// (centroid x activation, scaled once per block), the per-block results go through LDS and one
// thread per row adds them in column order.
constexpr int kSlabGroups = 64;
constexpr int kXStride = kGroup / 2 + 1;  // words per column group of x in LDS

__global__ __launch_bounds__(kThreads) void gemv_rows_kernel(const unsigned char* __restrict__ dev, int S,
                                                             const uint4* __restrict__ blocks, const uint32_t* __restrict__ meta,
                                                             int rows, int gpr, int rows_per_wg,
                                                             const uint32_t* __restrict__ x, float* __restrict__ y) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* rest;
    DecodeLds L = setup_decode_lds(smem, dev, S, kThreads, &rest);
    uint32_t* xs = reinterpret_cast<uint32_t*>(rest);           // kSlabGroups * kXStride words
    float* part = reinterpret_cast<float*>(xs + kSlabGroups * kXStride);  // kThreads partial sums

    const int row0 = blockIdx.x * rows_per_wg;
    const int nrows = min(rows_per_wg, rows - row0);
    float row_acc = 0.0f;  // thread r < nrows accumulates row row0 + r
    for (int slab = 0; slab < gpr; slab += kSlabGroups) {
        const int sg = min(kSlabGroups, gpr - slab);  // column groups in this slab
        __syncthreads();
        for (int i = threadIdx.x; i < sg * (kGroup / 2); i += kThreads)
            xs[(i >> 6) * kXStride + (i & 63)] = x[(size_t)slab * (kGroup / 2) + i];
        const int total = nrows * sg;  // blocks of this slab, numbered row-major within the slab
        for (int base = 0; base < total; base += kThreads) {
            const int count = min(kThreads, total - base);
            __syncthreads();
            // stage: block j of the chunk is (row, cg) = divmod(base + j, sg)
            for (int i = threadIdx.x; i < count * 4; i += kThreads) {
                int j = base + (i >> 2);
                size_t g = (size_t)(row0 + j / sg) * gpr + slab + j % sg;
                uint4 v = blocks[g * 4 + (i & 3)];
                uint32_t* d = L.payload + (i >> 2) * kStride + (i & 3) * 4;
                d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
            }
            __syncthreads();
            if ((int)threadIdx.x < count) {
                int j = base + threadIdx.x;
                int cg = j % sg;
                size_t g = (size_t)(row0 + j / sg) * gpr + slab + cg;
                MetaWord mw = unpack_meta(meta[g], S);
                const __half* c = L.t.cent + mw.pattern * kK;
                const uint32_t* xg = xs + cg * kXStride;
                float acc = 0.0f;
                uint32_t xp = 0;
                decode_block(L.payload + threadIdx.x * kStride, L.t.lut8 + mw.slot * 256, L.t.longtab + mw.pattern * kK,
                             [&](int i, uint32_t sym) {
                                 if ((i & 1) == 0) xp = xg[i >> 1];
                                 float xv = __half2float(__ushort_as_half((unsigned short)((i & 1) ? (xp >> 16) : (xp & 0xFFFFu))));
                                 acc = fmaf(__half2float(c[sym]), xv, acc);
                             });
                part[threadIdx.x] = acc * scale_of(mw.scale_bits);
            }
            __syncthreads();
            if ((int)threadIdx.x < nrows) {
                // blocks of my row inside this chunk: j in [r*sg, (r+1)*sg) intersected with [base, base+count)
                int lo = max((int)threadIdx.x * sg, base), hi = min(((int)threadIdx.x + 1) * sg, base + count);
                for (int j = lo; j < hi; ++j) row_acc += part[j - base];
            }
        }
    }
    if ((int)threadIdx.x < nrows) y[row0 + threadIdx.x] = row_acc;
}

// ---- encoder ---------------------------------------------------------------------------------------
// One wavefront per group; lane l holds values 2l and 2l+1.
constexpr int kEncWaves = kThreads / 64;

__device__ inline float wave_xor_add(float v, int mask) { return __fadd_rn(v, __shfl_xor(v, mask)); }

struct EncLds {
    const __half* cent;     // [S][16]
    const uint32_t* enc;    // [S][16]
    float* recon;           // per wave [S][16]
    uint32_t* bits;         // per wave 16 words
};

// Encodes the group whose two values of this lane are (x0, x1); lanes 0..15 return one payload word
// each in *word, lane 0 the meta word in *meta.
__device__ inline void encode_group(const EncLds& E, int S, uint32_t hx0, uint32_t hx1, uint32_t* word, uint32_t* meta) {
    const int lane = threadIdx.x & 63;
    // scale: the largest magnitude, as an FP16 bit pattern
    uint32_t smax = max(hx0 & 0x7FFFu, hx1 & 0x7FFFu);
    for (int m = 1; m < 64; m <<= 1) smax = max(smax, (uint32_t)__shfl_xor((int)smax, m));
    const float s = scale_of(smax);
    // reconstructed values of every pattern: fp16(centroid * s) back in FP32
    for (int i = lane; i < S * kK; i += 64) E.recon[i] = __half2float(__float2half_rn(__half2float(E.cent[i]) * s));
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);  // LDS writes of this wave are done before the reads below
    const float x0 = __half2float(__ushort_as_half((unsigned short)hx0));
    const float x1 = __half2float(__ushort_as_half((unsigned short)hx1));
    float best = 0.0f;
    int best_p = 0;
    uint32_t best_idx = 0;
    for (int p = 0; p < S; ++p) {
        const float* r = E.recon + p * kK;
        float r0 = r[0];
        float d0 = fabsf(__fsub_rn(x0, r0)), d1 = fabsf(__fsub_rn(x1, r0));
        uint32_t k0 = 0, k1 = 0;
        float q0 = r0, q1 = r0;
#pragma unroll
        for (int k = 1; k < kK; ++k) {
            float rk = r[k];
            float a = fabsf(__fsub_rn(x0, rk)), b = fabsf(__fsub_rn(x1, rk));
            if (a < d0) { d0 = a; k0 = k; q0 = rk; }
            if (b < d1) { d1 = b; k1 = k; q1 = rk; }
        }
        float e0 = __fsub_rn(x0, q0), e1 = __fsub_rn(x1, q1);
        float v = __fadd_rn(__fmul_rn(e0, e0), __fmul_rn(e1, e1));  // tree level 0: values 2l and 2l+1
        for (int m = 1; m < 64; m <<= 1) v = wave_xor_add(v, m);    // levels 1..6
        if (p == 0 || v < best) { best = v; best_p = p; best_idx = k0 | (k1 << 4); }
    }
    // code lengths and codes of the chosen pattern
    const uint32_t c0 = E.enc[best_p * kK + (best_idx & 15u)], c1 = E.enc[best_p * kK + (best_idx >> 4)];
    const uint32_t l0 = c0 >> 16, l1 = c1 >> 16;
    uint32_t incl = l0 + l1;  // inclusive scan of bit counts over lanes
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = (uint32_t)__shfl_up((int)incl, d);
        if (lane >= d) incl += o;
    }
    const uint32_t total = (uint32_t)__shfl((int)incl, 63);
    const bool raw = total > 8u * ECCO_BLOCK_BYTES;
    if (lane < kBlockWords) E.bits[lane] = 0;
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);
    if (raw) {
        // value i in stream bits 4i..4i+3: lane l owns byte l of the payload
        atomicOr(&E.bits[lane >> 2], (best_idx & 0xFFu) << (8 * (lane & 3)));
    } else {
        uint32_t pos = incl - (l0 + l1);
        uint64_t v = (uint64_t)(c0 & 0xFFFFu) | ((uint64_t)(c1 & 0xFFFFu) << l0);  // up to 24 bits
        v <<= (pos & 31u);
        atomicOr(&E.bits[pos >> 5], (uint32_t)v);
        if ((v >> 32) != 0) atomicOr(&E.bits[(pos >> 5) + 1], (uint32_t)(v >> 32));
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);
    *word = lane < kBlockWords ? E.bits[lane] : 0u;
    *meta = smax | ((uint32_t)best_p << 16) | (raw ? (1u << 22) : 0u);
    __builtin_amdgcn_wave_barrier();
}

constexpr size_t kEncLdsBytes = kMaxS * kK * 2 + kMaxS * kK * 4 + (size_t)kEncWaves * (kMaxS * kK * 4 + kBlockWords * 4);

__device__ inline EncLds setup_enc_lds(unsigned char* smem, const unsigned char* dev, int S) {
    uint32_t* cent = reinterpret_cast<uint32_t*>(smem);
    uint32_t* enc = cent + kMaxS * kK / 2;
    float* recon = reinterpret_cast<float*>(enc + kMaxS * kK);
    uint32_t* bits = reinterpret_cast<uint32_t*>(recon + kEncWaves * kMaxS * kK);
    stage_words(cent, dev + DevLayout::cent, S * kK * 2);
    stage_words(enc, dev + DevLayout::enc, S * kK * 4);
    __syncthreads();
    const int wave = threadIdx.x >> 6;
    EncLds E;
    E.cent = reinterpret_cast<const __half*>(cent);
    E.enc = enc;
    E.recon = recon + wave * kMaxS * kK;
    E.bits = bits + wave * kBlockWords;
    return E;
}

__global__ __launch_bounds__(kThreads) void encode_kernel(const unsigned char* __restrict__ dev, int S,
                                                          const uint32_t* __restrict__ src, size_t n_groups,
                                                          uint32_t* __restrict__ blocks, uint32_t* __restrict__ meta) {
    extern __shared__ __align__(16) unsigned char smem[];
    EncLds E = setup_enc_lds(smem, dev, S);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (size_t g = (size_t)blockIdx.x * kEncWaves + wave; g < n_groups; g += (size_t)gridDim.x * kEncWaves) {
        uint32_t pair = src[g * (kGroup / 2) + lane];
        uint32_t word, mw;
        encode_group(E, S, pair & 0xFFFFu, pair >> 16, &word, &mw);
        if (lane < kBlockWords) blocks[g * kBlockWords + lane] = word;
        if (lane == 0) meta[g] = mw;
    }
}

// grid: B*H*2 wavefronts; even = K, odd = V
__global__ __launch_bounds__(kThreads) void kv_append_kernel(const unsigned char* __restrict__ dev_k, int Sk,
                                                             const unsigned char* __restrict__ dev_v, int Sv,
                                                             const uint32_t* __restrict__ k_new, const uint32_t* __restrict__ v_new,
                                                             uint32_t* __restrict__ k_blocks, uint32_t* __restrict__ k_meta,
                                                             uint32_t* __restrict__ v_blocks, uint32_t* __restrict__ v_meta,
                                                             const int32_t* __restrict__ seq_len, int B, int H, int T_max) {
    extern __shared__ __align__(16) unsigned char smem[];
    const bool is_v = blockIdx.y != 0;  // uniform per workgroup, so each workgroup stages one model
    const int S = is_v ? Sv : Sk;
    EncLds E = setup_enc_lds(smem, is_v ? dev_v : dev_k, S);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int bh = blockIdx.x * kEncWaves + wave;
    if (bh >= B * H) return;
    const int t = seq_len[bh / H];
    if (t < 0 || t >= T_max) return;
    const uint32_t* src = (is_v ? v_new : k_new) + (size_t)bh * (kGroup / 2);
    uint32_t pair = src[lane];
    uint32_t word, mw;
    encode_group(E, S, pair & 0xFFFFu, pair >> 16, &word, &mw);
    const size_t g = (size_t)bh * T_max + t;
    uint32_t* blocks = is_v ? v_blocks : k_blocks;
    uint32_t* meta = is_v ? v_meta : k_meta;
    if (lane < kBlockWords) blocks[g * kBlockWords + lane] = word;
    if (lane == 0) meta[g] = mw;
}

// ---- single-query attention over compressed K / V ----------------------------------------------------
// One workgroup per (sequence, head); tokens in chunks of 256, one token per lane.  Scores come from
// decoding K with q held in LDS (all lanes read the same q element at the same time).  Softmax is
// kept online: running maximum m, running denominator l, running output o rescaled per chunk.
// V blocks are decoded into an LDS tile [token][128] (129-word rows), then thread (d-pair, quarter)
// adds p_t * V_t over a quarter of the chunk's tokens.
constexpr int kVRow = kGroup / 2 + 1;

__device__ inline float wg_reduce(float v, float* scratch, bool is_max) {
    for (int m = 1; m < 64; m <<= 1) {
        float o = __shfl_xor(v, m);
        v = is_max ? fmaxf(v, o) : v + o;
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = scratch[0];
    for (int w = 1; w < kThreads / 64; ++w) r = is_max ? fmaxf(r, scratch[w]) : r + scratch[w];
    return r;
}

struct AttnLds {
    Tables tk, tv;
    uint32_t* payload;
    uint32_t* vtile;
    float* q;
    float* p;
    float* scratch;
};
constexpr size_t kAttnTableBytes = kLutSlots * 256 + kMaxS * kK * 4 + kMaxS * kK * 2;
constexpr size_t kAttnLdsBytes = 2 * kAttnTableBytes + (size_t)kThreads * kStride * 4 + (size_t)kThreads * kVRow * 4 +
                                 kGroup * 4 + kThreads * 4 + 64;

__device__ inline Tables stage_tables(uint32_t* base, const unsigned char* dev, int S) {
    uint32_t* lut8 = base;
    uint32_t* longtab = lut8 + kLutSlots * 256 / 4;
    uint32_t* cent = longtab + kMaxS * kK;
    stage_words(lut8, dev + DevLayout::lut8, kLutSlots * 256);
    stage_words(longtab, dev + DevLayout::longtab, S * kK * 4);
    stage_words(cent, dev + DevLayout::cent, S * kK * 2);
    Tables t;
    t.lut8 = reinterpret_cast<const uint8_t*>(lut8);
    t.longtab = longtab;
    t.cent = reinterpret_cast<const __half*>(cent);
    return t;
}

__global__ __launch_bounds__(kThreads) void kv_attend_kernel(const unsigned char* __restrict__ dev_k, int Sk,
                                                             const unsigned char* __restrict__ dev_v, int Sv,
                                                             const uint16_t* __restrict__ q,
                                                             const uint4* __restrict__ k_blocks, const uint32_t* __restrict__ k_meta,
                                                             const uint4* __restrict__ v_blocks, const uint32_t* __restrict__ v_meta,
                                                             const int32_t* __restrict__ seq_len, int H, int T_max,
                                                             float* __restrict__ out) {
    extern __shared__ __align__(16) unsigned char smem[];
    AttnLds A;
    uint32_t* base = reinterpret_cast<uint32_t*>(smem);
    A.tk = stage_tables(base, dev_k, Sk);
    A.tv = stage_tables(base + kAttnTableBytes / 4, dev_v, Sv);
    A.payload = base + 2 * kAttnTableBytes / 4;
    A.vtile = A.payload + kThreads * kStride;
    A.q = reinterpret_cast<float*>(A.vtile + kThreads * kVRow);
    A.p = A.q + kGroup;
    A.scratch = A.p + kThreads;

    const int bh = blockIdx.x;
    const int T = min(seq_len[bh / H], T_max);
    if (threadIdx.x < kGroup) A.q[threadIdx.x] = __half2float(__ushort_as_half(q[(size_t)bh * kGroup + threadIdx.x]));
    const int dp = threadIdx.x & 63, quarter = threadIdx.x >> 6;  // output pair (2dp, 2dp+1), token quarter
    float o0 = 0.0f, o1 = 0.0f, run_max = -INFINITY, run_den = 0.0f;
    const float inv_sqrt_d = 0.08838834764831845f;  // 1 / sqrt(128)
    for (int t0 = 0; t0 < T; t0 += kThreads) {
        const int count = min(kThreads, T - t0);
        const size_t first = (size_t)bh * T_max + t0;
        __syncthreads();
        stage_payload(A.payload, k_blocks, first, count);
        __syncthreads();
        float score = -INFINITY;
        if ((int)threadIdx.x < count) {
            MetaWord mw = unpack_meta(k_meta[first + threadIdx.x], Sk);
            const __half* c = A.tk.cent + mw.pattern * kK;
            // the softmax is sensitive to the scores (keys with large per-channel scales), so K takes the
            // exact dequantisation rule, FP16 rounding included
            const float s = scale_of(mw.scale_bits);
            float acc = 0.0f;
            decode_block(A.payload + threadIdx.x * kStride, A.tk.lut8 + mw.slot * 256, A.tk.longtab + mw.pattern * kK,
                         [&](int i, uint32_t sym) { acc = fmaf(__half2float(dequant(c[sym], s)), A.q[i], acc); });
            score = acc * inv_sqrt_d;
        }
        const float chunk_max = wg_reduce(score, A.scratch, true);
        const float new_max = fmaxf(run_max, chunk_max);
        const float p = ((int)threadIdx.x < count) ? __expf(score - new_max) : 0.0f;
        const float chunk_den = wg_reduce(p, A.scratch, false);
        const float rescale = (run_max == -INFINITY) ? 0.0f : __expf(run_max - new_max);
        run_den = run_den * rescale + chunk_den;
        run_max = new_max;
        o0 *= rescale;
        o1 *= rescale;
        A.p[threadIdx.x] = p;
        __syncthreads();
        stage_payload(A.payload, v_blocks, first, count);
        __syncthreads();
        if ((int)threadIdx.x < count) {
            MetaWord mw = unpack_meta(v_meta[first + threadIdx.x], Sv);
            const __half* c = A.tv.cent + mw.pattern * kK;
            const float s = scale_of(mw.scale_bits);
            uint32_t* row = A.vtile + threadIdx.x * kVRow;
            uint32_t lo = 0;
            decode_block(A.payload + threadIdx.x * kStride, A.tv.lut8 + mw.slot * 256, A.tv.longtab + mw.pattern * kK,
                         [&](int i, uint32_t sym) {
                             uint32_t h = __half_as_ushort(dequant(c[sym], s));
                             if (i & 1) row[i >> 1] = lo | (h << 16); else lo = h;
                         });
        }
        __syncthreads();
        for (int t = quarter; t < count; t += kThreads / 64) {
            uint32_t v = A.vtile[t * kVRow + dp];
            float pt = A.p[t];
            o0 = fmaf(pt, __half2float(__ushort_as_half((unsigned short)(v & 0xFFFFu))), o0);
            o1 = fmaf(pt, __half2float(__ushort_as_half((unsigned short)(v >> 16))), o1);
        }
    }
    // combine the four token quarters
    __syncthreads();
    float* red = reinterpret_cast<float*>(A.vtile);
    red[quarter * kGroup + 2 * dp] = o0;
    red[quarter * kGroup + 2 * dp + 1] = o1;
    __syncthreads();
    if (threadIdx.x < kGroup) {
        float v = red[threadIdx.x] + red[kGroup + threadIdx.x] + red[2 * kGroup + threadIdx.x] + red[3 * kGroup + threadIdx.x];
        out[(size_t)bh * kGroup + threadIdx.x] = T > 0 ? v / run_den : 0.0f;
    }
}

// ---- host side -----------------------------------------------------------------------------------------
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline int model_ready(const ecco_model* m) { return (m && m->dev && m->device >= 0) ? ECCO_OK : ECCO_EINVAL; }

template <class K>
int allow_lds(K kernel, size_t bytes) {
    static_assert(sizeof(K) == sizeof(void*), "kernel pointer");
    if (bytes > 64 * 1024)
        ECCO_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    return ECCO_OK;
}

int grid_for(size_t work_items, int per_wg, int cap) {
    size_t g = (work_items + per_wg - 1) / per_wg;
    return (int)std::min<size_t>(std::max<size_t>(g, 1), (size_t)cap);
}

}  // namespace

extern "C" {

int ecco_encode(const ecco_model* m, const uint16_t* src, size_t n_groups, void* blocks, uint32_t* meta, void* stream) {
    if (model_ready(m) != ECCO_OK) return ECCO_EINVAL;
    if (n_groups == 0) return ECCO_OK;  // nothing to do; pointers may be null
    if (!src || !blocks || !meta) return ECCO_EINVAL;
    if (!aligned(blocks, 64) || !aligned(src, 4) || !aligned(meta, 4)) return ECCO_EALIGN;
    int grid = grid_for(n_groups, kEncWaves, 1 << 16);
    hipLaunchKernelGGL(encode_kernel, dim3(grid), dim3(kThreads), kEncLdsBytes, static_cast<hipStream_t>(stream), m->dev, m->S,
                       reinterpret_cast<const uint32_t*>(src), n_groups, static_cast<uint32_t*>(blocks), meta);
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

static int decode_common(const ecco_model* m, const void* blocks, const uint32_t* meta, size_t n_groups, void* dst,
                         void* stream, bool indices) {
    if (model_ready(m) != ECCO_OK) return ECCO_EINVAL;
    if (n_groups == 0) return ECCO_OK;  // nothing to do; pointers may be null
    if (!blocks || !meta || !dst) return ECCO_EINVAL;
    if (!aligned(blocks, 64) || !aligned(dst, 16) || !aligned(meta, 4)) return ECCO_EALIGN;
    int grid = grid_for(n_groups, kThreads, 1 << 14);
    if (indices)
        hipLaunchKernelGGL(decode_kernel<true>, dim3(grid), dim3(kThreads), kDecodeLdsBytes, static_cast<hipStream_t>(stream),
                           m->dev, m->S, static_cast<const uint4*>(blocks), meta, n_groups, dst);
    else
        hipLaunchKernelGGL(decode_kernel<false>, dim3(grid), dim3(kThreads), kDecodeLdsBytes, static_cast<hipStream_t>(stream),
                           m->dev, m->S, static_cast<const uint4*>(blocks), meta, n_groups, dst);
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

int ecco_decode(const ecco_model* m, const void* blocks, const uint32_t* meta, size_t n_groups, uint16_t* dst, void* stream) {
    return decode_common(m, blocks, meta, n_groups, dst, stream, false);
}

int ecco_decode_indices(const ecco_model* m, const void* blocks, const uint32_t* meta, size_t n_groups, uint8_t* idx, void* stream) {
    return decode_common(m, blocks, meta, n_groups, idx, stream, true);
}

int ecco_decode_gemv(const ecco_model* m, const void* blocks, const uint32_t* meta, int rows, int cols,
                     const uint16_t* x, int batch, float* y, void* stream) {
    if (!blocks || !meta || !x || !y) return ECCO_EINVAL;
    if (model_ready(m) != ECCO_OK) return ECCO_EINVAL;
    if (rows <= 0 || cols <= 0 || cols % kGroup != 0 || cols > 65536 || batch < 1 || batch > 16) return ECCO_ESHAPE;
    if (!aligned(blocks, 64) || !aligned(x, 4) || !aligned(y, 4) || !aligned(meta, 4)) return ECCO_EALIGN;
    const int gpr = cols / kGroup;
    // rows per workgroup: about two chunks of 256 blocks, at least one row
    int rows_per_wg = std::max(1, std::min(kThreads, (2 * kThreads) / gpr));
    int grid = (rows + rows_per_wg - 1) / rows_per_wg;
    size_t lds = kDecodeLdsBytes + (size_t)kSlabGroups * kXStride * 4 + kThreads * 4;
    int rc = allow_lds(gemv_rows_kernel, lds);
    if (rc != ECCO_OK) return rc;
    for (int b = 0; b < batch; ++b) {
        hipLaunchKernelGGL(gemv_rows_kernel, dim3(grid), dim3(kThreads), lds, static_cast<hipStream_t>(stream), m->dev, m->S,
                           static_cast<const uint4*>(blocks), meta, rows, gpr, rows_per_wg,
                           reinterpret_cast<const uint32_t*>(x + (size_t)b * cols), y + (size_t)b * rows);
        ECCO_HIP_CHECK(hipGetLastError());
    }
    return ECCO_OK;
}

int ecco_kv_append(const ecco_model* mk, const ecco_model* mv, const uint16_t* k_new, const uint16_t* v_new,
                   void* k_blocks, uint32_t* k_meta, void* v_blocks, uint32_t* v_meta,
                   const int32_t* seq_len, int B, int H, int T_max, void* stream) {
    if (!k_new || !v_new || !k_blocks || !k_meta || !v_blocks || !v_meta || !seq_len) return ECCO_EINVAL;
    if (model_ready(mk) != ECCO_OK || model_ready(mv) != ECCO_OK || mk->device != mv->device) return ECCO_EINVAL;
    if (B <= 0 || H <= 0 || T_max <= 0) return ECCO_ESHAPE;
    if (!aligned(k_blocks, 64) || !aligned(v_blocks, 64) || !aligned(k_new, 4) || !aligned(v_new, 4)) return ECCO_EALIGN;
    dim3 grid((B * H + kEncWaves - 1) / kEncWaves, 2);
    hipLaunchKernelGGL(kv_append_kernel, grid, dim3(kThreads), kEncLdsBytes, static_cast<hipStream_t>(stream), mk->dev, mk->S,
                       mv->dev, mv->S, reinterpret_cast<const uint32_t*>(k_new), reinterpret_cast<const uint32_t*>(v_new),
                       static_cast<uint32_t*>(k_blocks), k_meta, static_cast<uint32_t*>(v_blocks), v_meta, seq_len, B, H, T_max);
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

int ecco_kv_attend(const ecco_model* mk, const ecco_model* mv, const uint16_t* q,
                   const void* k_blocks, const uint32_t* k_meta, const void* v_blocks, const uint32_t* v_meta,
                   const int32_t* seq_len, int B, int H, int T_max, float* out, void* stream) {
    if (!q || !k_blocks || !k_meta || !v_blocks || !v_meta || !seq_len || !out) return ECCO_EINVAL;
    if (model_ready(mk) != ECCO_OK || model_ready(mv) != ECCO_OK || mk->device != mv->device) return ECCO_EINVAL;
    if (B <= 0 || H <= 0 || T_max <= 0) return ECCO_ESHAPE;
    if (!aligned(k_blocks, 64) || !aligned(v_blocks, 64) || !aligned(q, 2) || !aligned(out, 4)) return ECCO_EALIGN;
    int rc = allow_lds(kv_attend_kernel, kAttnLdsBytes);
    if (rc != ECCO_OK) return rc;
    hipLaunchKernelGGL(kv_attend_kernel, dim3(B * H), dim3(kThreads), kAttnLdsBytes, static_cast<hipStream_t>(stream), mk->dev,
                       mk->S, mv->dev, mv->S, q, static_cast<const uint4*>(k_blocks), k_meta, static_cast<const uint4*>(v_blocks),
                       v_meta, seq_len, H, T_max, out);
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

}  // extern "C"
