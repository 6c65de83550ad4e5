// Decoder and encoder of the self-contained 4x block (include/ecco_paper_block.h) for gfx950.
//
// Decoder: the block has one code stream of 128 values behind a variable-length header, so a lane owns a whole
// block: 64 blocks (4 KB) per wavefront pass, loaded with 16-byte pieces on consecutive addresses into a private
// LDS buffer (17-word slots) one pass ahead, decoded in lockstep (value i of 64 blocks at a time) with an 8-bit
// peek into a byte table per (pattern, codebook) -- 4 x S tables of 256 bytes, 64 KB for S = 64 -- and a second
// small table for the centroid.  Values past the cut (code ends beyond bit 512) become zeros; the lane keeps
// counting bits, so the test stays true once it fails.  Decoded values leave through a private LDS image, 32 per
// lane at a time, as 64-byte pieces (four lanes per block).  The padded entries are only known when the stream
// has been walked to its end: the lane then overwrites those positions in global memory, after the wavefront's
// earlier stores have completed.
//
// Encoder: one wavefront per group, two values per lane, the same search and packing scheme as the other
// format's encoder (reconstructed centroids in LDS, nearest value by a strict-< scan, balanced FP32 error tree,
// bit positions by a wavefront scan, payload assembled with LDS atomic OR), plus: the element of largest
// magnitude takes index 15 and no error; the codebook is the one of least total length; the stream is cut at
// bit 512; if it ends before, the largest remaining magnitudes are found one by one (a wavefront maximum over a
// key of magnitude and position) and appended as 15-bit entries.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <algorithm>
#include <cstdint>
#include <type_traits>

#include "ecco_pb_internal.h"

namespace {

using namespace ecco_pb;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

#define ECCO_HIP_CHECK(expr) do { if ((expr) != hipSuccess) return ECCO_EHIP; } while (0)

constexpr int kSlot = kBlockWords + 1;    // LDS words per staged block; the last one is a zero pad
constexpr int kUnit = 64;                 // blocks per wavefront pass, one per lane
constexpr int kPayWords = kUnit * kSlot + 4;
constexpr int kPassValues = 32;           // values per lane between two write-outs
constexpr int kImgWords = 32 * 32;        // the write-out image: 32 lines of 128 bytes
// the header takes at most 18 bits and a code at most 8: value i ends at or before bit 18 + 8 (i + 1), inside the block for i <= 60
constexpr int kAlwaysPresent = (kBlockBits - 18) / kMaxLen;
constexpr int kDecThreads = 512;
constexpr int kDecWaves = kDecThreads / 64;

__device__ inline void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ inline void stage_words(uint32_t* dst, const uint32_t* __restrict__ src, int words) {  // words % 4 == 0, 16-byte aligned
    const uint4* s = reinterpret_cast<const uint4*>(src);
    uint4* d = reinterpret_cast<uint4*>(dst);
    for (int i = threadIdx.x; i < (words >> 2); i += blockDim.x) d[i] = s[i];
}

inline size_t dec_lds_bytes(int S) { return (DevLayout{S}.decode_words() + (size_t)kDecWaves * (kPayWords + kImgWords)) * 4; }

struct PieceLoad {
    uint4 v[4];
};
__device__ __forceinline__ PieceLoad load_pieces(const uint4* __restrict__ blocks, size_t g0, size_t n_groups, int lane) {
    PieceLoad L;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int q = lane + 64 * r;  // piece q of the pass: block q / 4, part q % 4
        const size_t g = min(g0 + (size_t)(q >> 2), n_groups - 1);
        L.v[r] = blocks[g * 4 + (q & 3)];
    }
    return L;
}
__device__ __forceinline__ void store_pieces(uint32_t* pay, const PieceLoad& L, int lane) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int q = lane + 64 * r;
        uint32_t* d = pay + (q >> 2) * kSlot + (q & 3) * 4;
        d[0] = L.v[r].x; d[1] = L.v[r].y; d[2] = L.v[r].z; d[3] = L.v[r].w;
    }
}

__global__ __launch_bounds__(kDecThreads) void pb_decode_kernel(const uint32_t* __restrict__ dev, int S,
                                                               const uint4* __restrict__ blocks, size_t n_groups,
                                                               uint16_t* __restrict__ dst) {
    extern __shared__ __align__(16) uint32_t smem[];
    const DevLayout D{S};
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint8_t* lut = reinterpret_cast<const uint8_t*>(smem + D.lut());
    const uint16_t* kplut = reinterpret_cast<const uint16_t*>(smem + D.kplut());
    const uint16_t* cent = reinterpret_cast<const uint16_t*>(smem + D.cent());
    const uint16_t* fp8 = reinterpret_cast<const uint16_t*>(smem + D.fp8());
    uint32_t* pay = smem + D.decode_words() + wave * (kPayWords + kImgWords);
    uint32_t* img = pay + kPayWords;

    const size_t n_units = (n_groups + kUnit - 1) / kUnit;
    const size_t first = (size_t)blockIdx.x * kDecWaves + wave, step = (size_t)gridDim.x * kDecWaves;
    PieceLoad pre;
    if (first < n_units) pre = load_pieces(blocks, first * kUnit, n_groups, lane);
    stage_words(smem, dev, (int)D.decode_words());
    pay[lane * kSlot + kBlockWords] = 0u;
    if (lane < 4) pay[kUnit * kSlot + lane] = 0u;
    __syncthreads();

    for (size_t u = first; u < n_units; u += step) {
        const size_t g0 = u * kUnit;
        wave_lds_fence();
        store_pieces(pay, pre, lane);
        wave_lds_fence();
        if (u + step < n_units) pre = load_pieces(blocks, (u + step) * kUnit, n_groups, lane);
        const uint32_t* w = pay + lane * kSlot;
        const uint32_t w0 = w[0];
        const uint32_t kpe = kplut[(w0 >> 14) & 0xFFu];
        const uint32_t p = kpe >> 8;
        const uint32_t sv = fp8[w0 >> 24];                 // the signed scale, FP16 bits
        const __half sabs = __ushort_as_half((unsigned short)(sv & 0x7FFFu));
        const uint8_t* tab = lut + (p * kBooks + ((w0 >> 22) & 3u)) * 256u;
        const uint16_t* cp = cent + p * 16u;
        uint32_t fetch = 10u + (kpe & 0xFFu);              // where the next run is fetched from; stops at 512
        uint32_t reach = fetch;                             // where the codes read so far end; keeps counting past 512
#pragma unroll 1
        for (int pp = 0; pp < kGroup / (2 * kPassValues); ++pp) {
            // 64 values per lane = one 128-byte line of output, kept in registers until the line is complete: a store
            // instruction that leaves half a line for later costs a second write of that line
            uint32_t packed[kPassValues];
#pragma unroll
            for (int i0 = 0; i0 < 2 * kPassValues; i0 += 4) {
                const uint32_t wi = fetch >> 5;
                uint64_t win = (((uint64_t)w[wi] << 32) | (uint64_t)w[wi + 1]) << (fetch & 31u);
                uint32_t used = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t e = tab[(uint32_t)(win >> 56)];
                    const uint32_t len = e & 15u;
                    reach += len;
                    used += len;
                    win <<= len;
                    const __half prod = __hmul(__ushort_as_half(cp[e >> 4]), sabs);   // one rounding: fp16(c * |s|)
                    uint32_t val = e >= 0xF0u ? sv : (uint32_t)__half_as_ushort(prod);
                    val = reach <= (uint32_t)kBlockBits ? val : 0u;                     // a code that ends beyond the block is absent
                    const int i = i0 + j;
                    if (i & 1) packed[i >> 1] |= val << 16; else packed[i >> 1] = val;
                }
                fetch = min(fetch + used, (uint32_t)kBlockBits);
            }
            // write-out: the lines of lanes 0..31, then of lanes 32..63, through the image (32 rows of eight 16-byte
            // pieces, piece k of row r at column k ^ (r & 7)); every store instruction carries whole lines, 8 lanes each
            uint4* image = reinterpret_cast<uint4*>(img);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                wave_lds_fence();
                if ((lane >> 5) == h) {
                    const int row = lane & 31;
#pragma unroll
                    for (int k = 0; k < 8; ++k)
                        image[row * 8 + (k ^ (row & 7))] = make_uint4(packed[4 * k], packed[4 * k + 1], packed[4 * k + 2], packed[4 * k + 3]);
                }
                wave_lds_fence();
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = (lane >> 3) + 8 * r, part = lane & 7;
                    const uint4 v = image[row * 8 + (part ^ (row & 7))];
                    const size_t b = g0 + 32 * h + row;
                    if (b < n_groups) reinterpret_cast<uint4*>(dst)[b * 16 + pp * 8 + part] = v;
                }
            }
        }
        // padded entries: only if all 128 values were present
        if (reach <= (uint32_t)kBlockBits && g0 + lane < n_groups) {
            const uint32_t n_out = ((uint32_t)kBlockBits - reach) / kOutlierBits;
            if (__builtin_amdgcn_ballot_w64(n_out > 0) != 0ull) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the stores above have landed
            for (uint32_t j = 0; j < n_out; ++j) {
                const uint32_t at = reach + j * kOutlierBits, wi = at >> 5;
                const uint64_t win = (((uint64_t)w[wi] << 32) | (uint64_t)w[wi + 1]) << (at & 31u);
                const uint32_t entry = (uint32_t)(win >> 49);   // 7-bit position, 8-bit float
                dst[(g0 + lane) * kGroup + (entry >> 8)] = fp8[entry & 0xFFu];
            }
        }
    }
}

template <int kCtrl>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, kCtrl, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t lane_u32(uint32_t v, int l) { return (uint32_t)__builtin_amdgcn_readlane((int)v, l); }
// an associative, commutative, exact operation over the 64 lanes (cross-lane moves inside rows of 16, then the four
// row results through scalar registers); every lane returns the result
template <class Op>
__device__ __forceinline__ uint32_t wave_all_u32(uint32_t t, Op op) {
    t = op(t, dpp_u32<0xB1>(t));   // quad_perm [1,0,3,2]
    t = op(t, dpp_u32<0x4E>(t));   // quad_perm [2,3,0,1]
    t = op(t, dpp_u32<0x141>(t));  // row_half_mirror
    t = op(t, dpp_u32<0x140>(t));  // row_mirror
    return op(op(lane_u32(t, 0), lane_u32(t, 16)), op(lane_u32(t, 32), lane_u32(t, 48)));
}
// FP32 sum in the balanced tree: aligned blocks of 2, 4, 8, 16 lanes, then (row 0 + row 1) + (row 2 + row 3)
__device__ __forceinline__ float wave_tree_sum(float t) {
    const auto f = [](float v) { return __builtin_bit_cast(uint32_t, v); };
    const auto g = [](uint32_t v) { return __builtin_bit_cast(float, v); };
    t = __fadd_rn(t, g(dpp_u32<0xB1>(f(t))));
    t = __fadd_rn(t, g(dpp_u32<0x4E>(f(t))));
    t = __fadd_rn(t, g(dpp_u32<0x141>(f(t))));
    t = __fadd_rn(t, g(dpp_u32<0x140>(f(t))));
    return __fadd_rn(__fadd_rn(g(lane_u32(f(t), 0)), g(lane_u32(f(t), 16))), __fadd_rn(g(lane_u32(f(t), 32)), g(lane_u32(f(t), 48))));
}

// Sixteen such sums at once: at each of the first four levels a lane keeps the half of its entries that matches its
// own lane bit and sends the other half to its partner (lanes l and l ^ 1, ^ 2, ^ 4, ^ 8), then the two remaining
// levels (^ 16, ^ 32) on the one entry left: lane l returns the total of entry l & 15, summed in the same tree.
__device__ __forceinline__ float wave_tree_sum16(const float (&q)[16], int lane) {
    const auto x1 = [](float v) { return __uint_as_float(dpp_u32<0xB1>(__float_as_uint(v))); };
    const auto x2 = [](float v) { return __uint_as_float(dpp_u32<0x4E>(__float_as_uint(v))); };
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4, b3 = lane & 8;
    float a[8], b[4], c[2];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = __fadd_rn(b0 ? q[2 * i + 1] : q[2 * i], x1(b0 ? q[2 * i] : q[2 * i + 1]));
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = __fadd_rn(b1 ? a[2 * i + 1] : a[2 * i], x2(b1 ? a[2 * i] : a[2 * i + 1]));
#pragma unroll
    for (int i = 0; i < 2; ++i) c[i] = __fadd_rn(b2 ? b[2 * i + 1] : b[2 * i], __shfl_xor(b2 ? b[2 * i] : b[2 * i + 1], 4));
    float t = __fadd_rn(b3 ? c[1] : c[0], __shfl_xor(b3 ? c[0] : c[1], 8));
    t = __fadd_rn(t, __shfl_xor(t, 16));
    return __fadd_rn(t, __shfl_xor(t, 32));
}

// ---- decode fused into the matrix-vector product --------------------------------------------------------------------
// y = W x without writing W: a workgroup owns a band of rows (its blocks are consecutive in memory); a wavefront
// takes 64 consecutive blocks of the band at a time, one per lane, exactly as the decoder does.  The lane keeps the
// 128 activations of its block's column group in 64 registers and adds centroid * x for every value that is present
// (index 15 counts as +-1); the sum is multiplied by |scale| at the end.  The 128 indices are kept as nibbles in 16
// registers: when padded entries follow, the lane takes back centroid * x at their positions and adds the entries'
// own values (times x) instead -- from the last entry to the first, each position once, which is what a sequential
// reader of the block ends up with.  Per-block sums go to LDS, and each row's blocks are added in a fixed tree.
constexpr int kGvThreads = 512;
constexpr int kGvWaves = kGvThreads / 64;
constexpr int kGvPartFloats = 2048;      // per-block sums of a band: band rows x column groups
constexpr int kGvXMaxCols = 8192;        // activations are staged in LDS up to this many columns, read through L2 beyond
constexpr int kNibStride = 17;           // words per lane of the index store (16 + 1)

inline size_t gv_lds_bytes(int S, int cols) {
    return (DevLayout{S}.decode_words() + (size_t)kGvWaves * (kPayWords + 64 * kNibStride) + kGvPartFloats +
            (cols <= kGvXMaxCols ? cols / 2 : 0)) * 4;
}

template <bool kXLds>
__global__ __launch_bounds__(kGvThreads) void pb_gemv_kernel(const uint32_t* __restrict__ dev, int S,
                                                             const uint4* __restrict__ blocks, int rows, int gpr, int band,
                                                             const uint4* __restrict__ x, float* __restrict__ y) {
    extern __shared__ __align__(16) uint32_t smem[];
    const DevLayout D{S};
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint8_t* lut = reinterpret_cast<const uint8_t*>(smem + D.lut());
    const uint16_t* kplut = reinterpret_cast<const uint16_t*>(smem + D.kplut());
    const uint16_t* cent = reinterpret_cast<const uint16_t*>(smem + D.cent());
    const uint16_t* fp8 = reinterpret_cast<const uint16_t*>(smem + D.fp8());
    uint32_t* pay = smem + D.decode_words() + wave * (kPayWords + 64 * kNibStride);
    uint32_t* nibs = pay + kPayWords + lane * kNibStride;
    float* part = reinterpret_cast<float*>(smem + D.decode_words() + kGvWaves * (kPayWords + 64 * kNibStride));
    uint32_t* xl = reinterpret_cast<uint32_t*>(part + kGvPartFloats);

    const int r0 = blockIdx.x * band, nrows = min(band, rows - r0);
    const size_t base = (size_t)r0 * gpr;                 // first block of the band
    const int n_blocks = nrows * gpr;                     // <= kGvPartFloats
    const int n_units = (n_blocks + kUnit - 1) / kUnit;
    PieceLoad pre;
    if (wave < n_units) pre = load_pieces(blocks + base * 4, (size_t)wave * kUnit, (size_t)n_blocks, lane);
    stage_words(smem, dev, (int)D.decode_words());
    if (kXLds)
        for (int i = threadIdx.x; i < gpr * 16; i += kGvThreads) reinterpret_cast<uint4*>(xl)[i] = x[i];
    pay[lane * kSlot + kBlockWords] = 0u;
    if (lane < 4) pay[kUnit * kSlot + lane] = 0u;
    __syncthreads();

    for (int u = wave; u < n_units; u += kGvWaves) {
        wave_lds_fence();
        store_pieces(pay, pre, lane);
        wave_lds_fence();
        if (u + kGvWaves < n_units) pre = load_pieces(blocks + base * 4, (size_t)(u + kGvWaves) * kUnit, (size_t)n_blocks, lane);
        const int bl = u * kUnit + lane;                  // block of the band; slots past the band hold a copy of its last block
        const int cg = min(bl, n_blocks - 1) % gpr;       // its column group
        const uint4* xsrc = kXLds ? reinterpret_cast<const uint4*>(xl) + cg * 16 : x + (size_t)cg * 16;
        uint32_t xs[kGroup / 4];  // the activations of half a column group at a time
        const uint32_t* w = pay + lane * kSlot;
        const uint32_t w0 = w[0];
        const uint32_t kpe = kplut[(w0 >> 14) & 0xFFu];
        const uint32_t p = kpe >> 8;
        const uint32_t sv = fp8[w0 >> 24];
        const uint8_t* tab = lut + (p * kBooks + ((w0 >> 22) & 3u)) * 256u;
        const uint16_t* cp = cent + p * 16u;
        uint32_t fetch = 10u + (kpe & 0xFFu), reach = fetch;
        float acc = 0.0f;
        uint32_t nib[kGroup / 8];
#pragma unroll
        for (int i0 = 0; i0 < kGroup; i0 += 4) {
            if ((i0 & 63) == 0) {
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const uint4 v = xsrc[(i0 >> 6) * 8 + k];
                    xs[4 * k] = v.x; xs[4 * k + 1] = v.y; xs[4 * k + 2] = v.z; xs[4 * k + 3] = v.w;
                }
            }
            const uint32_t wi = fetch >> 5;
            uint64_t win = (((uint64_t)w[wi] << 32) | (uint64_t)w[wi + 1]) << (fetch & 31u);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = i0 + j;
                const uint32_t e = tab[(uint32_t)(win >> 56)];
                const uint32_t len = e & 15u, idx = e >> 4;
                reach += len;
                win <<= len;
                // FP16 operands go straight into mixed-precision multiply-adds: the activations stay packed in their
                // registers (converted ahead of time they would need 128)
                const half2_t x2 = __builtin_bit_cast(half2_t, xs[(i & 63) >> 1]);
                const _Float16 xh = (i & 1) ? x2[1] : x2[0];
                uint32_t cb = cp[idx], keep = idx;
                if (i >= kAlwaysPresent) {  // only these values can lie beyond the cut: they then count as zero and as index 0
                    const bool present = reach <= (uint32_t)kBlockBits;
                    cb = present ? cb : 0u;
                    keep = present ? idx : 0u;
                }
                acc = fmaf((float)__builtin_bit_cast(_Float16, (unsigned short)cb), (float)xh, acc);
                nib[i >> 3] = (i & 7) ? ((nib[i >> 3] << 4) | keep) : keep;
                if ((i & 3) == 3) asm volatile("" : "+v"(acc), "+v"(nib[i >> 3]), "+v"(xs[(i & 63) >> 1]));  // keeps the arithmetic next to its table reads
            }
            fetch = min(reach, (uint32_t)kBlockBits);
        }
        const uint16_t* xh16 = kXLds ? reinterpret_cast<const uint16_t*>(xl) + cg * kGroup : reinterpret_cast<const uint16_t*>(x) + (size_t)cg * kGroup;
        if (sv & 0x8000u) {
            // index 15 was added as +1 times its activation; the scale is negative, so it is -1: find the positions with
            // index 15 (all four bits of the nibble set; an absent value was recorded as index 0, unless it really is
            // index 0 ... which is not 15 either) and take twice their activations back
#pragma unroll
            for (int k = 0; k < kGroup / 8; ++k) {
                uint32_t hit = nib[k] & (nib[k] >> 1) & (nib[k] >> 2) & (nib[k] >> 3) & 0x11111111u;
                while (hit) {
                    const uint32_t b = 31u - (uint32_t)__builtin_clz(hit);   // bit 4 * (7 - position in the register)
                    hit &= ~(1u << b);
                    const uint32_t pos = 8u * k + (7u - (b >> 2));
                    acc = fmaf(-2.0f, __half2float(__ushort_as_half(xh16[pos])), acc);
                }
            }
        }
        float extra = 0.0f;  // padded entries: absolute values, not multiples of the scale
        const uint32_t n_out = reach <= (uint32_t)kBlockBits ? ((uint32_t)kBlockBits - reach) / kOutlierBits : 0u;
        if (__builtin_amdgcn_ballot_w64(n_out > 0u) != 0ull) {
#pragma unroll
            for (int k = 0; k < kGroup / 8; ++k) nibs[k] = nib[k];
            const uint16_t* xh = xh16;
            uint64_t seen_lo = 0, seen_hi = 0;
            for (int j = (int)n_out - 1; j >= 0; --j) {
                const uint32_t at = reach + (uint32_t)j * kOutlierBits, wi = at >> 5;
                const uint64_t win = (((uint64_t)w[wi] << 32) | (uint64_t)w[wi + 1]) << (at & 31u);
                const uint32_t entry = (uint32_t)(win >> 49), pos = entry >> 8;
                const uint64_t bit = 1ull << (pos & 63u);
                const bool dup = ((pos < 64u ? seen_lo : seen_hi) & bit) != 0ull;
                if (pos < 64u) seen_lo |= bit; else seen_hi |= bit;
                if (dup) continue;  // a later entry for this position has been applied already
                const uint32_t idx = (nibs[pos >> 3] >> (4u * (7u - (pos & 7u)))) & 15u;
                const float xi = __half2float(__ushort_as_half(xh[pos]));
                float c = __half2float(__ushort_as_half(cp[idx]));
                if (idx == 15u && (sv & 0x8000u)) c = -c;
                acc = fmaf(-c, xi, acc);
                extra = fmaf(__half2float(__ushort_as_half(fp8[entry & 0xFFu])), xi, extra);
            }
        }
        if (bl < n_blocks) part[bl] = fmaf(acc, __half2float(__ushort_as_half((unsigned short)(sv & 0x7FFFu))), extra);
    }
    __syncthreads();
    // row sums: the blocks of a row in a fixed order (lane-strided partial sums, then the wavefront tree)
    for (int r = wave; r < nrows; r += kGvWaves) {
        float sum = 0.0f;
        for (int c = lane; c < gpr; c += 64) sum += part[r * gpr + c];
        sum = wave_tree_sum(sum);
        if (lane == 0) y[r0 + r] = sum;
    }
}

// ---- encoder ---------------------------------------------------------------------------------------------------
constexpr int kEncThreads = 256;
constexpr int kEncWaves = kEncThreads / 64;
constexpr int kBitWords = kBlockWords + 2;

__device__ __forceinline__ float half_bits_f(uint32_t bits) { return __half2float(__ushort_as_half((unsigned short)bits)); }

// v to the format's 8-bit float: nearest, ties to the even code, saturating at +-480
__device__ __forceinline__ uint32_t fp8_round_dev(float v) {
    const uint32_t sign = (__float_as_uint(v) >> 24) & 0x80u;
    const float a = fabsf(v);
    uint32_t code;
    if (a < 0.015625f) {
        code = (uint32_t)rintf(a * 512.0f);  // below 2^-6 the values are multiples of 2^-9; 8 is the smallest normal number
    } else {
        const uint32_t b = __float_as_uint(a);
        const uint32_t r = b + 0x7FFFFu + ((b >> 20) & 1u);  // to three mantissa bits, ties to even
        const int e = (int)(r >> 23) - 120;
        code = e > 15 ? 127u : (((uint32_t)e << 3) | ((r >> 20) & 7u));
    }
    return sign | code;
}

inline size_t enc_lds_bytes(int S) { return (DevLayout{S}.encode_words() + (size_t)kEncWaves * ((size_t)S * 16 + kBitWords)) * 4; }

// ORs the low `nbits` of `value` into the block image at stream bit `at`, most significant bit first; bits at or
// beyond 512 are dropped (the cut)
__device__ __forceinline__ void put_bits(uint32_t* bits, uint32_t at, uint32_t value, uint32_t nbits) {
    const uint64_t v = (uint64_t)value << (64u - nbits - (at & 31u));
    const uint32_t wi = at >> 5;
    if (wi < (uint32_t)kBlockWords && (uint32_t)(v >> 32) != 0u) atomicOr(&bits[wi], (uint32_t)(v >> 32));
    if (wi + 1 < (uint32_t)kBlockWords && (uint32_t)v != 0u) atomicOr(&bits[wi + 1], (uint32_t)v);
}

__global__ __launch_bounds__(kEncThreads) void pb_encode_kernel(const uint32_t* __restrict__ dev, int S, float inv_tscale,
                                                               const uint32_t* __restrict__ src, size_t n_groups,
                                                               uint32_t* __restrict__ blocks) {
    extern __shared__ __align__(16) uint32_t smem[];
    const DevLayout D{S};
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    stage_words(smem, dev + D.cent(), (int)D.encode_words());
    __syncthreads();
    const uint16_t* cent = reinterpret_cast<const uint16_t*>(smem);                                   // [S][16]
    const uint16_t* fp8 = reinterpret_cast<const uint16_t*>(smem + (D.fp8() - D.cent()));             // [256]
    const uint32_t* enc = smem + (D.enc() - D.cent());                                                // [S * 4][16]
    const uint32_t* kpenc = smem + (D.kpenc() - D.cent());                                            // [S]
    float* recon = reinterpret_cast<float*>(smem + D.encode_words()) + wave * (S * 16 + kBitWords);   // [S][16], this wavefront's
    uint32_t* bits = reinterpret_cast<uint32_t*>(recon + S * 16);                                     // [18]
    const auto umax = [](uint32_t a, uint32_t b) { return max(a, b); };
    const auto uadd = [](uint32_t a, uint32_t b) { return a + b; };

    for (size_t g = (size_t)blockIdx.x * kEncWaves + wave; g < n_groups; g += (size_t)gridDim.x * kEncWaves) {
        const uint32_t pair = src[g * (kGroup / 2) + lane];
        const uint32_t hx0 = pair & 0xFFFFu, hx1 = pair >> 16;                   // values 2l and 2l + 1
        // the element of largest magnitude, first position on ties: largest key of (magnitude, 127 - position)
        const uint32_t pos0 = 2u * lane, pos1 = pos0 + 1u;
        uint32_t key0 = ((hx0 & 0x7FFFu) << 7) | (127u - pos0), key1 = ((hx1 & 0x7FFFu) << 7) | (127u - pos1);
        const uint32_t top = wave_all_u32(max(key0, key1), umax);
        const uint32_t a = 127u - (top & 127u);
        const uint32_t xa = lane_u32((a & 1u) ? hx1 : hx0, (int)(a >> 1));
        const uint32_t s8 = fp8_round_dev(half_bits_f(xa) * inv_tscale);
        const uint32_t sv = fp8[s8];
        const float s = half_bits_f(sv & 0x7FFFu);
        const float x0 = half_bits_f(hx0), x1 = half_bits_f(hx1);
        const bool is0 = pos0 == a, is1 = pos1 == a;
        // reconstructed centroids of every pattern
        for (int i = lane; i < S * 16; i += 64) recon[i] = half_bits_f((uint32_t)__half_as_ushort(__float2half_rn(half_bits_f(cent[i]) * s)));
        if (lane < kBitWords) bits[lane] = 0u;
        wave_lds_fence();
        // pattern of least squared error over the other 127 elements
        // Rating a pattern needs every element's least distance, not the index that attains it (the squared error is
        // that distance squared): a subtraction per candidate and a three-way minimum per two candidates.  The index
        // scan runs once, for the winner.
        // Sixteen patterns at a time: q[e] is this lane's part of the squared error of pattern pb + e; the sixteen sums
        // over the wavefront are formed together (wave_tree_sum16: lane l ends up with the total of pattern
        // pb + (l & 15)), every lane keeps the least it has seen, and the lanes are compared at the end.
        float mine = __builtin_inff();
        int mine_p = 0;
        for (int pb = 0; pb < S; pb += 16) {
            float q[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                q[e] = __builtin_inff();
                if (pb + e < S) {  // uniform
                    const float* r = recon + (pb + e) * 16;
                    float d0 = fabsf(__fsub_rn(x0, r[0])), d1 = fabsf(__fsub_rn(x1, r[0]));
                    static_assert(kCent % 2 == 1, "candidates 1 .. kCent - 1 in pairs");
#pragma unroll
                    for (int k = 1; k < kCent; k += 2) {
                        const float ra = r[k], rb = r[k + 1];
                        d0 = fminf(fminf(d0, fabsf(__fsub_rn(x0, ra))), fabsf(__fsub_rn(x0, rb)));
                        d1 = fminf(fminf(d1, fabsf(__fsub_rn(x1, ra))), fabsf(__fsub_rn(x1, rb)));
                    }
                    const float q0 = is0 ? 0.0f : __fmul_rn(d0, d0), q1 = is1 ? 0.0f : __fmul_rn(d1, d1);
                    q[e] = __fadd_rn(q0, q1);
                }
            }
            const float t = wave_tree_sum16(q, lane);
            if (t < mine) {  // strict <: an earlier batch keeps a tie
                mine = t;
                mine_p = pb + (lane & 15);
            }
        }
        // least sum over the lanes, and the lowest pattern among the lanes that hold it
        const float least = __uint_as_float(wave_all_u32(__float_as_uint(mine), [](uint32_t a, uint32_t b) { return __float_as_uint(fminf(__uint_as_float(a), __uint_as_float(b))); }));
        const uint32_t cand = (mine == least && mine_p < S) ? (uint32_t)mine_p : 0x7FFFFFFFu;
        const uint32_t win = wave_all_u32(cand, [](uint32_t a, uint32_t b) { return min(a, b); });
        const int best_p = win < (uint32_t)S ? (int)win : 0;
        uint32_t best_idx;
        {
            // the reconstructed values ascend with k and FP32 rounding is monotone, so the distance falls (weakly) to its
            // least value and rises (weakly) after it: the first index of the least distance -- what a scan with a strict <
            // finds -- is the last k at which the distance strictly drops
            const float* r = recon + best_p * 16;
            float d0 = fabsf(__fsub_rn(x0, r[0])), d1 = fabsf(__fsub_rn(x1, r[0]));
            uint32_t k0 = 0, k1 = 0;
#pragma unroll
            for (int k = 1; k < kCent; ++k) {
                const float rk = r[k];
                const float u = fabsf(__fsub_rn(x0, rk)), v = fabsf(__fsub_rn(x1, rk));
                k0 = u < d0 ? (uint32_t)k : k0;
                k1 = v < d1 ? (uint32_t)k : k1;
                d0 = u;
                d1 = v;
            }
            best_idx = k0 | (k1 << 4);
        }
        const uint32_t i0 = is0 ? 15u : (best_idx & 15u), i1 = is1 ? 15u : (best_idx >> 4);
        // the codebook of least total length
        uint32_t c0 = 0, c1 = 0, best_total = 0;
        int best_h = 0;
        for (int h = 0; h < kBooks; ++h) {
            const uint32_t* t = enc + (best_p * kBooks + h) * kSym;
            const uint32_t a0 = t[i0], a1 = t[i1];
            const uint32_t total = wave_all_u32((a0 >> 16) + (a1 >> 16), uadd);
            if (h == 0 || total < best_total) {
                best_total = total;
                best_h = h;
                c0 = a0;
                c1 = a1;
            }
        }
        // header, then the codes at their positions (inclusive scan of the lengths over the lanes)
        const uint32_t kp = kpenc[best_p], base = 10u + (kp >> 16);
        if (lane == 0) bits[0] = (s8 << 24) | ((uint32_t)best_h << 22) | ((kp & 0xFFFFu) << (22u - (kp >> 16)));
        wave_lds_fence();
        const uint32_t l0 = c0 >> 16, l1 = c1 >> 16;
        uint32_t incl = l0 + l1;
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = (uint32_t)__shfl_up((int)incl, d);
            if (lane >= d) incl += o;
        }
        put_bits(bits, base + incl - (l0 + l1), ((c0 & 0xFFFFu) << l1) | (c1 & 0xFFFFu), l0 + l1);
        const uint32_t end = base + best_total;
        if (end <= (uint32_t)kBlockBits) {
            // room left: the largest remaining magnitudes, one per round, as (position, 8-bit float) entries
            const uint32_t slots = ((uint32_t)kBlockBits - end) / kOutlierBits;
            key0 = is0 ? 0u : key0 + 1u;
            key1 = is1 ? 0u : key1 + 1u;
            for (uint32_t j = 0; j < slots; ++j) {
                const uint32_t best = wave_all_u32(max(key0, key1), umax);
                if (best == 0u) break;
                if (key0 == best || key1 == best) {
                    const bool first = key0 == best;
                    const uint32_t v8 = fp8_round_dev((first ? x0 : x1) * inv_tscale);
                    put_bits(bits, end + j * kOutlierBits, ((first ? pos0 : pos1) << 8) | v8, kOutlierBits);
                    if (first) key0 = 0u; else key1 = 0u;
                }
            }
        }
        wave_lds_fence();
        if (lane < kBlockWords) blocks[g * kBlockWords + lane] = bits[lane];
        wave_lds_fence();
    }
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
// a model can be used once it is on a device, and only while that device is the calling thread's current one: the
// kernels are launched on the current device and read the model's tables through device pointers
inline int model_ready(const ecco_pb_model* m) {
    if (!m || !m->dev || m->device < 0) return ECCO_EINVAL;
    int cur = -1;
    return (hipGetDevice(&cur) == hipSuccess && cur == m->device) ? ECCO_OK : ECCO_EINVAL;
}

template <class K>
int allow_lds(K kernel, size_t bytes) {
    if (bytes > 64 * 1024)
        ECCO_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    return ECCO_OK;
}

}  // namespace

extern "C" {

int ecco_pb_encode(const ecco_pb_model* m, const uint16_t* src, size_t n_groups, void* blocks, void* stream) {
    if (!m) return ECCO_EINVAL;
    if (n_groups == 0) return model_ready(m);
    if (!src || !blocks) return ECCO_EINVAL;
    if (!aligned(src, 4) || !aligned(blocks, 64)) return ECCO_EALIGN;
    if (model_ready(m) != ECCO_OK) return ECCO_EINVAL;
    const size_t wgs = (n_groups + kEncWaves - 1) / kEncWaves;
    const int grid = (int)std::min<size_t>(wgs, 256 * 16);
    float inv_tscale = 1.0f;  // 2^-texp, exact
    for (int i = 0; i < (m->texp < 0 ? -m->texp : m->texp); ++i) inv_tscale *= m->texp < 0 ? 2.0f : 0.5f;
    hipLaunchKernelGGL(pb_encode_kernel, dim3(grid), dim3(kEncThreads), enc_lds_bytes(m->S), static_cast<hipStream_t>(stream), m->dev, m->S,
                       inv_tscale, reinterpret_cast<const uint32_t*>(src), n_groups, static_cast<uint32_t*>(blocks));
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

int ecco_pb_decode_gemv(const ecco_pb_model* m, const void* blocks, int rows, int cols, const uint16_t* x, float* y, void* stream) {
    if (!m || !blocks || !x || !y) return ECCO_EINVAL;
    if (rows <= 0 || cols <= 0 || cols % kGroup != 0 || cols > 65536) return ECCO_ESHAPE;
    if (!aligned(blocks, 64) || !aligned(x, 16) || !aligned(y, 4)) return ECCO_EALIGN;
    if (model_ready(m) != ECCO_OK) return ECCO_EINVAL;
    const int gpr = cols / kGroup;
    // a band of rows per workgroup: about one band per compute unit, at most kGvPartFloats blocks
    int band = std::max(1, (rows + 255) / 256);
    band = std::min(band, std::max(1, kGvPartFloats / gpr));
    const int grid = (rows + band - 1) / band;
    const size_t lds = gv_lds_bytes(m->S, cols);
    hipStream_t st = static_cast<hipStream_t>(stream);
    auto launch = [&](auto kernel) -> int {
        const int rc = allow_lds(kernel, lds);
        if (rc != ECCO_OK) return rc;
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(kGvThreads), lds, st, m->dev, m->S, static_cast<const uint4*>(blocks), rows, gpr, band,
                           reinterpret_cast<const uint4*>(x), y);
        ECCO_HIP_CHECK(hipGetLastError());
        return ECCO_OK;
    };
    return cols <= kGvXMaxCols ? launch(pb_gemv_kernel<true>) : launch(pb_gemv_kernel<false>);
}

int ecco_pb_decode(const ecco_pb_model* m, const void* blocks, size_t n_groups, uint16_t* dst, void* stream) {
    if (!m) return ECCO_EINVAL;
    if (n_groups == 0) return model_ready(m);
    if (!blocks || !dst) return ECCO_EINVAL;
    if (n_groups >= ((size_t)1 << 31)) return ECCO_ESHAPE;
    if (!aligned(blocks, 64) || !aligned(dst, 16)) return ECCO_EALIGN;
    if (model_ready(m) != ECCO_OK) return ECCO_EINVAL;
    const size_t lds = dec_lds_bytes(m->S);
    const int rc = allow_lds(pb_decode_kernel, lds);
    if (rc != ECCO_OK) return rc;
    const size_t units = (n_groups + kUnit - 1) / kUnit;
    const int grid = (int)std::min<size_t>((units + kDecWaves - 1) / kDecWaves, 1024);
    hipLaunchKernelGGL(pb_decode_kernel, dim3(grid), dim3(kDecThreads), lds, static_cast<hipStream_t>(stream), m->dev, m->S,
                       static_cast<const uint4*>(blocks), n_groups, dst);
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

}  // extern "C"
