// HIP kernels (gfx950) and GPU entry points of libecco.
//
// Decoder design.  A Huffman stream is serial, so the unit of parallelism is the half block: the
// meta word says where the code of value 64 begins, hence every block offers two independent
// chains of 64 values.  One lane owns one chain.  All lanes of a wavefront sit at the same value
// position (whatever their bit positions), which makes the position-dependent operand of the
// consumer -- the activation x[i] in the fused GEMV, the query q[i] in attention -- a register with
// a static index.  Per value a lane does: peek 8 bits of its 64-bit window, one LDS table read that
// returns code length, index and the centroid as FP16, the consumer's multiply-add, one 64-bit
// shift; every four values the window is rebuilt from LDS at the chain's bit position.  Raw-mode
// blocks run the same instructions against a 16-entry table with a 4-bit peek.  All kernels work
// in units of 32 blocks per wavefront: 2 KB of payload fetched with coalesced 16-byte loads one
// unit ahead, kept in a per-wavefront LDS buffer with a 17-word stride per block (word 16 is a
// zero pad), so the per-lane window reads hit distinct banks and wavefronts never wait for each
// other inside the decode.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <utility>
#include <vector>

#include "ecco_internal.h"

using namespace ecco;

namespace {

constexpr int kStride = kBlockWords + 1;  // LDS words per staged block (last one is a zero pad)
constexpr int kHalf = kGroup / 2;         // values per chain

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

#define ECCO_HIP_CHECK(expr) do { if ((expr) != hipSuccess) return ECCO_EHIP; } while (0)

__device__ __forceinline__ float half_bits_f(uint32_t bits) { return __half2float(__ushort_as_half((unsigned short)bits)); }
// dequantisation: one exact FP32 product, one rounding to FP16
__device__ __forceinline__ uint32_t dequant_bits(uint32_t cent_bits, float s) {
    return __half_as_ushort(__float2half_rn(half_bits_f(cent_bits) * s));
}

// orders the LDS accesses of one wavefront (private buffers need no workgroup barrier)
__device__ inline void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- LDS tables -------------------------------------------------------------------------------------
struct Tables {
    const uint32_t* lut;      // [S][256]
    const uint32_t* rawlut;   // [S][16]
    const uint32_t* longtab;  // [S][16]
    const __half* cent;       // [S][16]
};
__host__ __device__ constexpr size_t table_words(int S) { return (size_t)S * (kPeekEntries + kK + kK + kK / 2); }  // LDS words of a model's decode tables

// copies `words` (a multiple of 4; both sides 16-byte aligned) from global memory to LDS with all
// threads of the workgroup, four 16-byte loads in flight per thread
__device__ inline void stage_vec(uint32_t* dst, const uint32_t* __restrict__ src, int words) {
    const uint4* s = reinterpret_cast<const uint4*>(src);
    uint4* d = reinterpret_cast<uint4*>(dst);
    const int n = words >> 2, step = blockDim.x;
    for (int i = threadIdx.x; i < n; i += 4 * step) {
        uint4 v0, v1, v2, v3;
        const int i1 = i + step, i2 = i + 2 * step, i3 = i + 3 * step;
        v0 = s[i];
        if (i1 < n) v1 = s[i1];
        if (i2 < n) v2 = s[i2];
        if (i3 < n) v3 = s[i3];
        d[i] = v0;
        if (i1 < n) d[i1] = v1;
        if (i2 < n) d[i2] = v2;
        if (i3 < n) d[i3] = v3;
    }
}

// Building the decode tables of a model in LDS from the compact tables in global memory.  Item
// (p, k) is index k of pattern p: its code of length l <= 8 is the prefix of 2^(8-l) consecutive
// 8-bit peeks, which all get the entry (centroid, index, length); a longer code marks its single
// 8-bit prefix with 0.  The two global loads of an item are split from the LDS writes so that a
// kernel can issue them first, put its payload loads behind them, and build the tables while the
// payload is still on its way.
struct TableItem {
    uint32_t enc, cent;
};
__device__ __forceinline__ TableItem load_table_item(const uint32_t* __restrict__ dev, int S, int t) {
    const DevLayout D{S};
    TableItem it;
    it.enc = dev[D.enc() + t];
    it.cent = reinterpret_cast<const uint16_t*>(dev + D.cent())[t];
    return it;
}
__device__ __forceinline__ void build_table_item(uint32_t* base, int S, int t, TableItem it) {
    uint32_t* lut = base;
    uint32_t* rawlut = lut + S * kPeekEntries;
    const uint32_t code = it.enc & 0xFFFFu, len = it.enc >> 16, k = (uint32_t)t & (kK - 1);
    const uint32_t value = (it.cent << 16) | (k << 8);
    rawlut[t] = value | 4u;
    uint32_t* row = lut + (t / kK) * kPeekEntries;
    if (len > (uint32_t)kPeekBits) {
        row[code >> (len - kPeekBits)] = 0u;  // several long codes may share this prefix: same value
    } else {
        const uint32_t entry = value | len, n = 1u << (kPeekBits - len);
        uint32_t* dst = row + (code << (kPeekBits - len));
        if (n >= 4) {
            // neighbouring items start their runs at different offsets: all rows begin on the same LDS
            // bank and equal-length codes are a multiple of the run length apart, so without the
            // rotation the 64 items of a wavefront would write to a handful of banks at a time
            const uint4 v = make_uint4(entry, entry, entry, entry);
            const uint32_t rot = ((uint32_t)t + ((uint32_t)t >> 4) + (code >> 2)) * 4u;
            for (uint32_t j = 0; j < n; j += 4) *reinterpret_cast<uint4*>(dst + ((j + rot) & (n - 1))) = v;
        } else {
            for (uint32_t j = 0; j < n; ++j) dst[j] = entry;
        }
    }
}
__device__ __forceinline__ Tables table_pointers(uint32_t* base, int S) {
    Tables tb;
    tb.lut = base;
    tb.rawlut = base + S * kPeekEntries;
    tb.longtab = base + S * (kPeekEntries + kK);
    tb.cent = reinterpret_cast<const __half*>(base + S * (kPeekEntries + 2 * kK));
    return tb;
}
// The whole job for a workgroup of at least S * 16 / 2 threads, with a payload prefetch in its shadow: every
// thread first requests its (up to) two table items, then calls `prefetch` (the loads of its first unit), then
// builds the tables.  Loads return in issue order and a wait names how many may still be outstanding, so with
// the items requested first -- the same loads on one straight path in every thread, indices clamped, threads
// beyond the items repeating the last one -- the build does not wait for the payload.  The lists of the long
// codes and the centroids are copied only for a model that needs them (behind the payload, then).  The caller
// synchronises afterwards.
template <bool kLong, class Prefetch>
__device__ __forceinline__ Tables stage_tables_around(uint32_t* base, const uint32_t* __restrict__ dev, int S, Prefetch&& prefetch) {
    const int n = S * kK;
    const int t0 = min((int)threadIdx.x, n - 1), t1 = min((int)(threadIdx.x + blockDim.x), n - 1);
    const TableItem i0 = load_table_item(dev, S, t0), i1 = load_table_item(dev, S, t1);
    __builtin_amdgcn_sched_barrier(0);
    prefetch();
    __builtin_amdgcn_sched_barrier(0);
    build_table_item(base, S, t0, i0);
    build_table_item(base, S, t1, i1);
    if (kLong) {
        const DevLayout D{S};
        stage_vec(base + S * (kPeekEntries + kK), dev + D.longtab(), S * kK);
        stage_vec(base + S * (kPeekEntries + 2 * kK), dev + D.cent(), S * kK / 2);
    }
    return table_pointers(base, S);
}

// what one lane needs to decode one chain
struct Lane {
    const uint32_t* lut;      // this lane's table (Huffman: 256 entries, raw: 16)
    uint32_t shift;           // 32 - peek width
    const uint32_t* longtab;  // pattern's canonical list (codes longer than the peek)
    const __half* cent;       // pattern's centroids
    float scale;
    uint32_t second_start;    // stream bit where value 64 begins
};
__device__ __forceinline__ Lane lane_setup(const Tables& T, uint32_t meta, int S) {
    Lane L;
    uint32_t p = (meta >> 16) & 0x3Fu;
    p = p < (uint32_t)S ? p : (uint32_t)(S - 1);
    const bool raw = (meta >> 22) & 1u;
    L.lut = raw ? T.rawlut + p * kK : T.lut + p * kPeekEntries;
    L.shift = raw ? 28u : (uint32_t)(32 - kPeekBits);
    L.longtab = T.longtab + p * kK;
    L.cent = T.cent + p * kK;
    L.scale = half_bits_f(meta & 0xFFFFu);
    L.second_start = raw ? 4u * kHalf : (meta >> 23);
    return L;
}

typedef __attribute__((address_space(3))) uint32_t lds_u32;  // a 32-bit word in LDS, addressed as such
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) u32x4 global_u4;   // sixteen bytes in global memory

// ---- the chain decoder ----------------------------------------------------------------------------------
// Decodes kCount values starting at stream bit `start` of the staged block `w` (16 words, a zero
// word, then two more readable words), calling sink(i, entry) with the table entry of each (length,
// index, centroid).  Values are taken in runs of 4 (2 when the model has codes longer than 8 bits:
// kLong).  A run works on a left-aligned 64-bit window made of the two words around its bit
// position: at least 33 valid bits, enough for the longest run of codes plus the last peek, so
// there is no refill test and no branch inside a run.  A run consumes at most 32 bits, so the next
// run needs the same two words or the next two: the third word is requested one run ahead and the
// window is rebuilt with two selects, which keeps the LDS latency of the stream itself off the
// dependent chain (only the table reads remain on it).  The position is clamped to 512, where the
// window's upper half is the zero word: bits past the block read as zero and arbitrary bytes decode
// without touching other memory (the lower half of that last window is never looked at).
template <bool kLong, int kCount, class Sink>
__device__ __forceinline__ void decode_chain(const uint32_t* w, uint32_t start, const Lane& L, Sink&& sink) {
    constexpr int kRun = kLong ? 2 : 4;
    static_assert(kCount % kRun == 0, "chain length");
    static_assert(kRun * (kLong ? kMaxLen : kPeekBits) <= 32, "a run stays inside two words");
    uint32_t pos = start;  // <= 511
    uint32_t wi = pos >> 5;
    uint32_t w0 = w[wi], w1 = w[wi + 1], w2 = w[wi + 2];
#pragma unroll
    for (int i0 = 0; i0 < kCount; i0 += kRun) {
        uint64_t win = (((uint64_t)w0 << 32) | (uint64_t)w1) << (pos & 31u);
        uint32_t used = 0;  // sum of the run's entries; its low byte is the number of bits consumed (at most 4 x 8 or 2 x 12)
#pragma unroll
        for (int j = 0; j < kRun; ++j) {
            uint32_t e = L.lut[(uint32_t)(win >> 32) >> L.shift];
            if (kLong) {
                if ((e & 0xFFu) == 0u) {
                    // code longer than the peek: rank of the next 12 bits among the left-aligned canonical codes
                    const uint32_t v = (uint32_t)(win >> 32) >> (32 - kMaxLen);
                    // the list is read here, on the rare path, not held in 16 registers throughout: its LDS byte address
                    // passes through an empty asm statement (a pointer passed through one would come back without its
                    // address space, and the reads below would become flat loads instead of LDS reads)
                    uint32_t lt_at = (uint32_t)(size_t)(const lds_u32*)L.longtab;
                    asm volatile("" : "+v"(lt_at));
                    const lds_u32* lt = (const lds_u32*)(size_t)lt_at;
                    int rank = 0;
                    for (int q = 1; q < kK; ++q) rank += ((lt[q] & 0xFFFu) <= v) ? 1 : 0;
                    const uint32_t t = lt[rank];
                    const uint32_t idx = (t >> 12) & 15u;
                    e = ((uint32_t)__half_as_ushort(L.cent[idx]) << 16) | (idx << 8) | (t >> 16);
                }
            }
            sink(i0 + j, e);
            used += e;
            win <<= (e & 0xFFu);
        }
        if (i0 + kRun < kCount) {
            pos = min(pos + (used & 0xFFu), (uint32_t)(kBlockWords * 32));
            const uint32_t nwi = pos >> 5;  // wi or wi + 1
            const bool adv = nwi != wi;
            w0 = adv ? w1 : w0;
            w1 = adv ? w2 : w1;
            w2 = w[nwi + 2];  // used one run later at the earliest
            wi = nwi;
        }
    }
}

// ---- payload staging ------------------------------------------------------------------------------------

constexpr int kGemvThreads = 1024;

// ---- ecco_decode_gemv, batch 1 ----------------------------------------------------------------------------
// A workgroup (one per compute unit) owns a band of R consecutive rows; its work is cut into units
// of one row x 32 column groups: 32 blocks, a contiguous 2 KB of payload, 64 chains -- one
// wavefront.  Lane l of the wavefront decodes chain l / 32 of block l % 32.  After the decode tables
// and x are in LDS (one workgroup barrier), the 16 wavefronts run on their own: each fetches the
// payload of its next unit into registers, decodes the current one out of a private 2 KB LDS
// buffer, adds the 64 lane sums with a wavefront reduction and goes on, without any further
// workgroup barrier, so a wavefront starts decoding as soon as its own bytes have arrived and the
// loads of one unit overlap the decode of the one before.  Units of a wavefront stay in one column
// tile as long as possible (a contiguous run of units when the row has several column tiles), and the
// lane keeps the 64 activations of its chain in registers across those units, so a value costs one
// mixed-precision FMA.  Rows are never split over workgroups:
// partial sums of a row's column tiles meet in LDS and are added in a fixed order.
constexpr int kUnitBlocks = 32;
constexpr int kWaves = kGemvThreads / 64;
constexpr int kUnitWords = kUnitBlocks * kStride + 4;  // private payload buffer of a wavefront (+ the two words a chain may read past the last slot)
constexpr int kXGroupWords = kGroup / 2 + 4;           // words per column group of x in LDS (skewed against bank conflicts)
constexpr int kXLdsGroups = 128;                       // x is staged in LDS up to this many column groups, read from L2 beyond
constexpr int kMaxBandRows = 128;
constexpr int kMaxColTiles = 65536 / kGroup / kUnitBlocks;
inline size_t gemv_lds_bytes(int S, int gpr) {
    const size_t xwords = gpr <= kXLdsGroups ? (size_t)gpr * kXGroupWords : 0;
    return (table_words(S) + (size_t)kWaves * kUnitWords + (size_t)kMaxBandRows * kMaxColTiles + xwords) * 4;
}

template <int kCtrl>
__device__ __forceinline__ float dpp_mov(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), kCtrl, 0xF, 0xF, true));
}
__device__ __forceinline__ float read_lane(float v, int l) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
// sum over the 64 lanes of a wavefront in a fixed order, on the VALU (cross-lane moves inside rows of
// 16 lanes, then the four row sums through scalar registers); every lane returns the total
__device__ __forceinline__ float wave_sum(float t) {
    t += dpp_mov<0xB1>(t);   // quad_perm [1,0,3,2]
    t += dpp_mov<0x4E>(t);   // quad_perm [2,3,0,1]
    t += dpp_mov<0x141>(t);  // row_half_mirror
    t += dpp_mov<0x140>(t);  // row_mirror
    return (read_lane(t, 0) + read_lane(t, 16)) + (read_lane(t, 32) + read_lane(t, 48));
}

// the same walk for any associative, commutative, exact operation (minimum, maximum): the order does not matter
template <class T, class Op>
__device__ __forceinline__ T wave_all(T v, Op op) {
    float t = __builtin_bit_cast(float, v);
    const auto f = [&](float a, float b) { return __builtin_bit_cast(float, op(__builtin_bit_cast(T, a), __builtin_bit_cast(T, b))); };
    t = f(t, dpp_mov<0xB1>(t));
    t = f(t, dpp_mov<0x4E>(t));
    t = f(t, dpp_mov<0x141>(t));
    t = f(t, dpp_mov<0x140>(t));
    return __builtin_bit_cast(T, f(f(read_lane(t, 0), read_lane(t, 16)), f(read_lane(t, 32), read_lane(t, 48))));
}

struct UnitLoad {
    uint4 v0, v1;
    uint32_t meta;
};
// the payload pieces and the meta word of this lane for unit (row, ct).  Block indices are clamped into
// the row, so every lane issues the same loads and a slot past the row end holds a copy of the row's
// last block: it decodes to finite values, which the caller drops.  Nothing here uses the loaded
// data, so the loads stay in flight while the previous unit is decoded.
__device__ __forceinline__ UnitLoad load_unit(const uint4* __restrict__ blocks, const uint32_t* __restrict__ meta,
                                              int row, int gpr, int ct, int lane) {
    UnitLoad u;
    const size_t row_base = (size_t)row * gpr;
    const int g0 = ct * kUnitBlocks + (lane >> 2), g1 = g0 + 16;
    u.v0 = blocks[(row_base + min(g0, gpr - 1)) * 4 + (lane & 3)];
    u.v1 = blocks[(row_base + min(g1, gpr - 1)) * 4 + (lane & 3)];
    const int g = ct * kUnitBlocks + (lane & (kUnitBlocks - 1));
    u.meta = meta[row_base + min(g, gpr - 1)];
    return u;
}
// Lane l writes pieces of blocks l / 4 and l / 4 + 16; the chains are then read by other lanes (lane b and b + 32
// read block b).  The exchange goes through the wavefront's private buffer without a workgroup barrier, so it is
// fenced on both sides at wavefront scope: the reads of the previous unit come before these writes, and these
// writes before the reads that follow.
__device__ __forceinline__ void store_unit(uint32_t* wbuf, const UnitLoad& u, int lane) {
    wave_lds_fence();
    uint32_t* d = wbuf + (lane >> 2) * kStride + (lane & 3) * 4;
    d[0] = u.v0.x; d[1] = u.v0.y; d[2] = u.v0.z; d[3] = u.v0.w;
    d += 16 * kStride;
    d[0] = u.v1.x; d[1] = u.v1.y; d[2] = u.v1.z; d[3] = u.v1.w;
    wave_lds_fence();
}

template <bool kLong>
__global__ __launch_bounds__(kGemvThreads) void gemv_kernel(const uint32_t* __restrict__ dev, int S,
                                                            const uint4* __restrict__ blocks, const uint32_t* __restrict__ meta,
                                                            int rows, int gpr, int band,
                                                            const uint32_t* __restrict__ x, float* __restrict__ y) {
    extern __shared__ __align__(16) uint32_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row0 = blockIdx.x * band;
    const int band_rows = min(band, rows - row0);
    const int col_tiles = (gpr + kUnitBlocks - 1) / kUnitBlocks;
    const int units = band_rows * col_tiles;  // unit u = (column tile u / band_rows, row u % band_rows)
    const bool x_in_lds = gpr <= kXLdsGroups;
    uint32_t* wbuf = smem + table_words(S) + wave * kUnitWords;
    float* part = reinterpret_cast<float*>(smem + table_words(S) + kWaves * kUnitWords);
    uint32_t* xt = reinterpret_cast<uint32_t*>(part + kMaxBandRows * kMaxColTiles);
    const uint4* x4 = reinterpret_cast<const uint4*>(x);

    // Loads in the order they are needed: table item, x, then the first unit's payload (from HBM).  Loads
    // return in issue order and a wait names how many may still be outstanding, so every thread issues the
    // same loads on one straight path (indices clamped instead of branches around them): only then can the
    // wait for the table item leave the payload in flight while the tables are built.
    // (The scheduling barriers keep the compiler from issuing them in another order.)
    const int ti = min(tid, S * kK - 1);  // threads beyond the items repeat the last one: same values to the same words
    const TableItem item = load_table_item(dev, S, ti);
    __builtin_amdgcn_sched_barrier(0);
    static_assert(ECCO_MAX_S * kK <= kGemvThreads, "one table item per thread");
    static_assert(kXLdsGroups * 16 == 2 * kGemvThreads, "two x pieces per thread");
    const uint4 xp0 = x4[min(tid, gpr * 16 - 1)];
    const uint4 xp1 = x4[min(tid + kGemvThreads, gpr * 16 - 1)];
    __builtin_amdgcn_sched_barrier(0);
    // With several column tiles a wavefront takes a contiguous run of units (column tile by column tile, row by
    // row; runs differ by one unit at most), so it changes its column tile -- and fetches 64 activations per
    // lane -- as rarely as possible.  With one column tile there is nothing to keep, and the wavefronts stride
    // through the rows together, so that the workgroup reads one contiguous stretch of memory at a time.
    const bool runs = col_tiles > 1;
    const int u_step = runs ? 1 : kWaves;
    int u = runs ? wave * units / kWaves : wave;
    const int u_end = runs ? (wave + 1) * units / kWaves : units;
    const int u_first = min(u, units - 1);  // a wavefront without work loads the band's last unit and drops it
    UnitLoad pre = load_unit(blocks, meta, row0 + u_first % band_rows, gpr, u_first / band_rows, lane);
    __builtin_amdgcn_sched_barrier(0);
    build_table_item(smem, S, ti, item);
    if (kLong) {
        const DevLayout D{S};
        for (int i = tid; i < S * kK; i += kGemvThreads) smem[S * (kPeekEntries + kK) + i] = dev[D.longtab() + i];
        for (int i = tid; i < S * kK / 2; i += kGemvThreads) smem[S * (kPeekEntries + 2 * kK) + i] = dev[D.cent() + i];
    }
    if (x_in_lds) {
        const int i0 = tid, i1 = tid + kGemvThreads;
        if (i0 < gpr * 16) *reinterpret_cast<uint4*>(xt + (i0 >> 4) * kXGroupWords + (i0 & 15) * 4) = xp0;
        if (i1 < gpr * 16) *reinterpret_cast<uint4*>(xt + (i1 >> 4) * kXGroupWords + (i1 & 15) * 4) = xp1;
    }
    if (lane < kUnitBlocks) wbuf[lane * kStride + kBlockWords] = 0u;  // zero pads of the private buffer
    if (lane == 0) wbuf[kUnitBlocks * kStride] = 0u;
    const Tables T = table_pointers(smem, S);
    __syncthreads();

    const int blk = lane & (kUnitBlocks - 1), half = lane >> 5;
    uint32_t xs[kHalf / 2];
    int cur_ct = -1;
    for (; u < u_end; u += u_step) {
        const int ct = u / band_rows, r = u - ct * band_rows;
        store_unit(wbuf, pre, lane);
        const uint32_t mw = pre.meta;
        const int cg = ct * kUnitBlocks + blk;
        if (ct != cur_ct) {  // the activations of this lane's chain: 64 FP16 = 8 x 16 bytes
            cur_ct = ct;
            const int cgx = min(cg, gpr - 1);
            if (x_in_lds) {
                const uint4* src = reinterpret_cast<const uint4*>(xt + cgx * kXGroupWords + half * (kHalf / 2));
#pragma unroll
                for (int j = 0; j < kHalf / 8; ++j) {
                    const uint4 v = src[j];
                    xs[4 * j] = v.x; xs[4 * j + 1] = v.y; xs[4 * j + 2] = v.z; xs[4 * j + 3] = v.w;
                }
            } else {
                const uint4* src = x4 + (size_t)cgx * 16 + half * 8;
#pragma unroll
                for (int j = 0; j < kHalf / 8; ++j) {
                    const uint4 v = src[j];
                    xs[4 * j] = v.x; xs[4 * j + 1] = v.y; xs[4 * j + 2] = v.z; xs[4 * j + 3] = v.w;
                }
            }
        }
        // the next unit's payload is requested after the activations: loads return in issue order, and the
        // activations (from cache) must not queue behind a fetch from HBM
        const int un = u + u_step;
        if (un < u_end) pre = load_unit(blocks, meta, row0 + un % band_rows, gpr, un / band_rows, lane);
        const Lane L = lane_setup(T, mw, S);
        float acc = 0.0f;
        decode_chain<kLong, kHalf>(wbuf + blk * kStride, half ? L.second_start : 0u, L, [&](int i, uint32_t e) {
            const uint32_t xp = xs[i >> 1];
            const float xv = half_bits_f((i & 1) ? (xp >> 16) : (xp & 0xFFFFu));
            acc = fmaf(half_bits_f(e >> 16), xv, acc);
            // pins the running sum every four values: otherwise the multiply-adds are sunk below the whole
            // chain and all 64 table entries stay in registers
            if ((i & 3) == 3) asm volatile("" : "+v"(acc));
        });
        const float t = wave_sum(cg < gpr ? acc * L.scale : 0.0f);
        if (lane == 0) {
            if (col_tiles == 1) y[row0 + r] = t;
            else part[r * col_tiles + ct] = t;
        }
    }
    if (col_tiles > 1) {
        __syncthreads();
        if (tid < band_rows) {
            // four reads in flight at a time (indices clamped, the surplus not added): same order of additions
            float sum = 0.0f;
            for (int ct0 = 0; ct0 < col_tiles; ct0 += 4) {
                float v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = part[tid * col_tiles + min(ct0 + j, col_tiles - 1)];
#pragma unroll
                for (int j = 0; j < 4; ++j) sum += ct0 + j < col_tiles ? v[j] : 0.0f;
            }
            y[row0 + tid] = sum;
        }
    }
}

// ---- ecco_decode / ecco_decode_indices ---------------------------------------------------------------
// The streaming scheme of the batch-1 GEMV on a linear array of blocks: a unit is 32 consecutive
// groups, lane l decodes chain l / 32 of block l % 32, a workgroup takes a contiguous range of units
// and its wavefronts stride through it.  A lane ends up with 128 contiguous output bytes, 16 at a
// time; written directly, one store instruction would touch 64 different lines with 16 bytes each,
// and the L2 request rate, not bandwidth, would bound the kernel (measured: 13 of 21 us on the
// 4096 x 4096 matrix).  So the FP16 values pass through a per-wavefront LDS image, 32 values per
// chain at a time, and are read back so that adjacent lanes hold adjacent 16-byte pieces: four lanes
// write the 64 contiguous bytes a segment gets per pass.  The image is swizzled (piece c of segment
// s sits at 4 s + (c ^ (s / 4) % 4)) so that the transposed reads are conflict-free.  The 4 KB image
// lies over the wavefront's 2.2 KB payload buffer, which is dead once both chains are decoded (the
// values wait in registers meanwhile), so sixteen wavefronts fit 160 KB of LDS next to the S = 64
// tables; the zero words that bound each block's stream are rewritten with every unit.
constexpr int kDecWaves = 16;
struct DecCfg {
    static constexpr int kLinePieces = kHalf / 8;                  // 16-byte pieces of a chain's 128 output bytes
    static constexpr int kImageWords = 32 * kLinePieces * 4;       // 32 lines at a time
    static constexpr int kWaveWords = kImageWords > kUnitWords ? kImageWords : kUnitWords;  // private LDS of a wavefront: payload, then image
};
inline size_t decode_lds_bytes(int S) { return (table_words(S) + (size_t)kDecWaves * DecCfg::kWaveWords) * 4; }

template <bool kLong, bool kIndices>
__global__ __launch_bounds__(kDecWaves * 64) void decode_kernel(const uint32_t* __restrict__ dev, int S,
                                                              const uint4* __restrict__ blocks, const uint32_t* __restrict__ meta,
                                                              int n_groups, int units_per_wg, void* __restrict__ dst) {
    using Cfg = DecCfg;
    extern __shared__ __align__(16) uint32_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    uint32_t* wbuf = smem + table_words(S) + wave * Cfg::kWaveWords;
    uint4* image = reinterpret_cast<uint4*>(wbuf);
    const int total_units = (n_groups + kUnitBlocks - 1) / kUnitBlocks;
    const int u_end = min(total_units, (int)(blockIdx.x + 1) * units_per_wg);
    int u = blockIdx.x * units_per_wg + wave;
    // table item first, then the first unit's payload, the same loads in every thread, and the tables are built
    // while the payload is on its way (see gemv_kernel)
    static_assert(ECCO_MAX_S * kK <= kDecWaves * 64, "one table item per thread");
    const int ti = min(tid, S * kK - 1);
    const TableItem item = load_table_item(dev, S, ti);
    __builtin_amdgcn_sched_barrier(0);
    UnitLoad pre = load_unit(blocks, meta, 0, n_groups, min(u, u_end - 1), lane);
    __builtin_amdgcn_sched_barrier(0);
    build_table_item(smem, S, ti, item);
    if (kLong) {
        const DevLayout D{S};
        for (int i = tid; i < S * kK; i += kDecWaves * 64) smem[S * (kPeekEntries + kK) + i] = dev[D.longtab() + i];
        for (int i = tid; i < S * kK / 2; i += kDecWaves * 64) smem[S * (kPeekEntries + 2 * kK) + i] = dev[D.cent() + i];
    }
    const Tables T = table_pointers(smem, S);
    __syncthreads();

    const int blk = lane & (kUnitBlocks - 1), half = lane >> 5;  // block of the unit and chain of this lane
    for (; u < u_end; u += kDecWaves) {
        store_unit(wbuf, pre, lane);  // fenced: the previous unit's image has been read
        if (lane < kUnitBlocks) wbuf[lane * kStride + kBlockWords] = 0u;  // zero pads of the payload buffer (the image lay over them)
        if (lane == 0) wbuf[kUnitBlocks * kStride] = 0u;
        wave_lds_fence();
        const uint32_t mw = pre.meta;
        if (u + kDecWaves < u_end) pre = load_unit(blocks, meta, 0, n_groups, u + kDecWaves, lane);
        const Lane L = lane_setup(T, mw, S);
        const int g = u * kUnitBlocks + blk;
        const uint32_t* w = wbuf + blk * kStride;
        const uint32_t start = half ? L.second_start : 0u;
        if (kIndices) {
            uint4* out = reinterpret_cast<uint4*>(static_cast<uint8_t*>(dst) + (size_t)g * kGroup + half * kHalf);
            uint32_t acc[4] = {0, 0, 0, 0};
            decode_chain<kLong, kHalf>(w, start, L, [&](int i, uint32_t e) {
                acc[(i >> 2) & 3] |= ((e >> 8) & 15u) << (8 * (i & 3));
                if ((i & 15) == 15) {
                    if (g < n_groups) out[i >> 4] = make_uint4(acc[0], acc[1], acc[2], acc[3]);
                    acc[0] = acc[1] = acc[2] = acc[3] = 0;
                }
            });
        } else {
            uint8_t* obase = static_cast<uint8_t*>(dst) + (size_t)u * kUnitBlocks * kGroup * 2;  // the unit's 8 KB of output
            const _Float16 sh = __builtin_bit_cast(_Float16, (unsigned short)(mw & 0xFFFFu));
            const half2_t s2 = {sh, sh};
            uint32_t vals[kHalf / 2];  // the chain's 64 values = one 128-byte line of output
            uint32_t pk = 0;
            decode_chain<kLong, kHalf>(w, start, L, [&](int i, uint32_t e) {
                if ((i & 1) == 0) {
                    pk = e >> 16;
                    return;
                }
                // fp16(centroid * scale) for two values: the packed FP16 product rounds once, like the FP32 rule
                vals[i >> 1] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, pk | (e & 0xFFFF0000u)) * s2);
                if ((i & 7) == 7) asm volatile("" : "+v"(vals[i >> 1]));  // finished here, not gathered at the end of the chain
            });
            // Write-out in whole 128-byte lines: a store instruction that leaves half a line for later costs a second
            // write of that line.  First the 32 lanes with the first chains put their lines into the image (32 rows of
            // eight 16-byte pieces, piece k of row r at column k ^ (r & 7)) and all 64 lanes store them, eight lanes per
            // line; then the same for the second chains.
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                wave_lds_fence();
                if (half == h) {
#pragma unroll
                    for (int k = 0; k < Cfg::kLinePieces; ++k)
                        image[blk * Cfg::kLinePieces + (k ^ (blk & 7))] = make_uint4(vals[4 * k], vals[4 * k + 1], vals[4 * k + 2], vals[4 * k + 3]);
                }
                wave_lds_fence();
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = (lane >> 3) + 8 * r, part = lane & 7;
                    const uint4 v = image[row * Cfg::kLinePieces + (part ^ (row & 7))];
                    if (u * kUnitBlocks + row < n_groups)
                        *reinterpret_cast<uint4*>(obase + row * (kGroup * 2) + h * (kHalf * 2) + part * 16) = v;
                }
            }
        }
    }
}

// ---- ecco_decode_gemv, batch 2..16: MFMA ------------------------------------------------------------------
// The streaming scheme of the batch-1 kernel with the multiply-adds on the matrix cores.  A unit is
// 16 rows x 2 column groups (32 blocks, 16 runs of 128 contiguous bytes): lane l decodes, for row
// l % 16, chain (l / 16) % 2 of column group l / 32.  Eight decoded values of the lane are exactly
// its A operand of v_mfma_f32_16x16x32_f16 (row l % 16, k slice l / 16); the B operand of the lane
// is eight activations of batch row l % 16 at the columns of the chain of slice l / 16, which it
// holds in registers for the unit (zeros past the batch); the 16 x 16 FP32 accumulator (rows x
// batch) stays in registers over all units of a 16-row block.  The weights enter as
// fp16(centroid * scale) -- packed FP16 multiplies, which round exactly like the
// FP32-multiply-then-round rule -- so no per-row scaling of the accumulator is needed.  A workgroup
// owns whole 16-row blocks (all their column groups), so nothing is split over workgroups: per row
// block the 16 wavefronts add their accumulators through LDS in a fixed order.
constexpr int kMmaRows = 16;
constexpr int kMaxBatch = 16;
typedef float float4_t __attribute__((ext_vector_type(4)));
constexpr int kRbChunk = 3;  // row blocks whose per-wavefront sums wait in LDS for one common reduction
static_assert((table_words(ECCO_MAX_S) + (size_t)(kGemvThreads / 64) * (32 * kStride + 4) + (size_t)kRbChunk * (kGemvThreads / 64) * 16 * 16) * 4 <= 160 * 1024, "the batched kernel's LDS fits a compute unit");
inline size_t gemm_lds_bytes(int S) { return (table_words(S) + (size_t)kWaves * kUnitWords + (size_t)kRbChunk * kWaves * kMmaRows * kMaxBatch) * 4; }

// this lane's payload pieces and meta word of unit (rb, u): block (r, c) of the unit -- row 16 rb + r,
// column group 2 u + c -- goes to slot 2 r + c.  Indices are clamped into the matrix (see load_unit).
__device__ __forceinline__ UnitLoad load_unit16(const uint4* __restrict__ blocks, const uint32_t* __restrict__ meta,
                                                int rows, int gpr, int rb, int u, int lane) {
    UnitLoad t;
    const int slot = lane >> 2, c = slot & 1;
    const int cg = min(2 * u + c, gpr - 1);
    const int r0 = min(rb * kMmaRows + (slot >> 1), rows - 1), r1 = min(rb * kMmaRows + 8 + (slot >> 1), rows - 1);
    t.v0 = blocks[((size_t)r0 * gpr + cg) * 4 + (lane & 3)];
    t.v1 = blocks[((size_t)r1 * gpr + cg) * 4 + (lane & 3)];
    const int mr = min(rb * kMmaRows + (lane & 15), rows - 1), mc = min(2 * u + (lane >> 5), gpr - 1);
    t.meta = meta[(size_t)mr * gpr + mc];
    return t;
}

template <bool kLong>
__global__ __launch_bounds__(kGemvThreads) void gemm_kernel(const uint32_t* __restrict__ dev, int S,
                                                            const uint4* __restrict__ blocks, const uint32_t* __restrict__ meta,
                                                            int rows, int gpr, int rb_per_wg, int batch,
                                                            const uint16_t* __restrict__ x, float* __restrict__ y) {
    extern __shared__ __align__(16) uint32_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    uint32_t* wbuf = smem + table_words(S) + wave * kUnitWords;
    float* part = reinterpret_cast<float*>(smem + table_words(S) + kWaves * kUnitWords);  // [row block of the chunk][wavefront][batch 16][row 16]
    const int total_rb = (rows + kMmaRows - 1) / kMmaRows;
    const int rb0 = blockIdx.x * rb_per_wg, rb1 = min(total_rb, rb0 + rb_per_wg);
    const int upr = (gpr + 1) / 2;  // units per row block
    const size_t cols = (size_t)gpr * kGroup;

    TableItem item{0u, 0u};
    if (tid < S * kK) item = load_table_item(dev, S, tid);
    UnitLoad pre;
    if (wave < upr) pre = load_unit16(blocks, meta, rows, gpr, rb0, wave, lane);
    if (tid < S * kK) build_table_item(smem, S, tid, item);
    if (kLong) {
        const DevLayout D{S};
        for (int i = tid; i < S * kK; i += kGemvThreads) smem[S * (kPeekEntries + kK) + i] = dev[D.longtab() + i];
        for (int i = tid; i < S * kK / 2; i += kGemvThreads) smem[S * (kPeekEntries + 2 * kK) + i] = dev[D.cent() + i];
    }
    if (lane < kUnitBlocks) wbuf[lane * kStride + kBlockWords] = 0u;
    if (lane == 0) wbuf[kUnitBlocks * kStride] = 0u;
    const Tables T = table_pointers(smem, S);
    __syncthreads();

    const int r = lane & 15, c = lane >> 5, half = (lane >> 4) & 1;  // this lane's chain: row r, column group 2 u + c, chain `half`
    const int n = lane & 15;                                          // its batch row in B and its column in the accumulator
    uint4 bx[kHalf / 8];  // B: 64 activations of batch row n at this chain's columns
    for (int c0 = rb0; c0 < rb1; c0 += kRbChunk) {
        const int nrb = min(kRbChunk, rb1 - c0);
        for (int u = wave; u < upr; u += kWaves) {
            const int cg = 2 * u + c;
            for (int k = 0; k < nrb; ++k) {
                store_unit(wbuf, pre, lane);
                uint32_t mw = pre.meta;
                // the meta word is taken here, ahead of the activation loads: a wait for it placed behind them
                // would have to wait for them as well (they sit under a condition, so their number is not known)
                asm volatile("" : "+v"(mw));
                if (k == 0) {
#pragma unroll
                    for (int j = 0; j < kHalf / 8; ++j) bx[j] = make_uint4(0, 0, 0, 0);
                    if (n < batch && cg < gpr) {
                        const uint4* src = reinterpret_cast<const uint4*>(x + (size_t)n * cols + (size_t)cg * kGroup + half * kHalf);
#pragma unroll
                        for (int j = 0; j < kHalf / 8; ++j) bx[j] = src[j];
                    }
                }
                // the next unit's payload is requested after the activations (loads return in issue order):
                // the next row block of the chunk at the same columns, else the wavefront's next columns,
                // else the first unit of the next chunk
                int un = u, rbn = c0 + k + 1;
                if (k + 1 == nrb) {
                    un = u + kWaves;
                    rbn = c0;
                    if (un >= upr) {
                        un = wave;
                        rbn = c0 + kRbChunk;
                    }
                }
                if (rbn >= rb1) {  // nothing follows: the unit in hand is requested again (from cache) and dropped, so that
                    rbn = c0 + k;  // the same loads are in flight on every path and the waits for the activations
                    un = u;        // below can leave them outstanding
                }
                pre = load_unit16(blocks, meta, rows, gpr, rbn, un, lane);
                const Lane L = lane_setup(T, mw, S);
                const _Float16 sh = __builtin_bit_cast(_Float16, (unsigned short)(mw & 0xFFFFu));
                const half2_t s2 = {sh, sh};
                uint32_t pk[4] = {0, 0, 0, 0};
                float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
                decode_chain<kLong, kHalf>(wbuf + (2 * r + c) * kStride, half ? L.second_start : 0u, L, [&](int i, uint32_t e) {
                    if ((i & 1) == 0) {
                        pk[(i >> 1) & 3] = e >> 16;
                        return;
                    }
                    pk[(i >> 1) & 3] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, pk[(i >> 1) & 3] | (e & 0xFFFF0000u)) * s2);
                    if ((i & 7) != 7) return;
                    const uint4 av = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av), __builtin_bit_cast(half8_t, bx[i >> 3]), acc, 0, 0, 0);
                });
                // accumulator layout of the 16 x 16 tile: register j of lane l is row 4 * (l / 16) + j, column l % 16.
                // The wavefront's sums of a row block live in its own slice of LDS: the first unit stores, later ones add.
                float4_t* slot = reinterpret_cast<float4_t*>(part + (k * kWaves + wave) * (kMmaRows * kMaxBatch) + n * kMmaRows + 4 * (lane >> 4));
                if (u != wave) acc += *slot;
                *slot = acc;
            }
        }
        if (wave >= upr) {  // a wavefront without units contributes zeros
            const float4_t zero = {0.0f, 0.0f, 0.0f, 0.0f};
            for (int k = 0; k < nrb; ++k) reinterpret_cast<float4_t*>(part + (k * kWaves + wave) * (kMmaRows * kMaxBatch))[lane] = zero;
        }
        __syncthreads();
        if (tid < kMmaRows * kMaxBatch) {
            // the thread index is taken afresh: addresses derived from it are then formed here and not kept in
            // registers across the decode loop above, which has none to spare
            int t = tid;
            asm volatile("" : "+v"(t));
            const int b = t >> 4;
            for (int k = 0; k < nrb; ++k) {
                // a fixed number of reads, all in flight at once (a loop with a run-time bound waits for one after the other)
                float sum = 0.0f;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) sum += part[(k * kWaves + w) * (kMmaRows * kMaxBatch) + t];
                const int row = (c0 + k) * kMmaRows + (t & 15);
                if (b < batch && row < rows) y[(size_t)b * rows + row] = sum;
            }
        }
        __syncthreads();
    }
}

// ---- encoder ---------------------------------------------------------------------------------------
// One wavefront per group; lane l holds values 2l and 2l+1.
constexpr int kEncThreads = 256;
constexpr int kEncWaves = kEncThreads / 64;


struct EncLds {
    const __half* cent;     // [S][16]
    const uint32_t* enc;    // [S][16]
    float* recon;           // per wave [S][16]
    uint32_t* bits;         // per wave 16 words
};

// The group's scale: the largest magnitude among the 128 values (two per lane), as an FP16 bit pattern.
__device__ inline uint32_t group_scale_bits(uint32_t hx0, uint32_t hx1) {
    return wave_all(max(hx0 & 0x7FFFu, hx1 & 0x7FFFu), [](uint32_t a, uint32_t b) { return max(a, b); });
}

// Sixteen sums over the 64 lanes at once, each in the balanced tree (lanes l and l ^ 1, then ^ 2, ^ 4, ... ^ 32):
// at every one of the first four levels a lane keeps the half of its entries that matches its own lane bit and
// sends the other half to its partner, so the work halves per level instead of being done sixteen times over.
// Lane l returns the total of entry l & 15.  (Addition is commutative, so own + received is the tree's sum.)
__device__ __forceinline__ float wave_sum16(const float (&q)[16], int lane) {
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4, b3 = lane & 8;
    float a[8], b[4], c[2];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = (b0 ? q[2 * i + 1] : q[2 * i]) + dpp_mov<0xB1>(b0 ? q[2 * i] : q[2 * i + 1]);    // entry 2i + b0
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = (b1 ? a[2 * i + 1] : a[2 * i]) + dpp_mov<0x4E>(b1 ? a[2 * i] : a[2 * i + 1]);    // entry 4i + (l & 3)
#pragma unroll
    for (int i = 0; i < 2; ++i) c[i] = (b2 ? b[2 * i + 1] : b[2 * i]) + __shfl_xor(b2 ? b[2 * i] : b[2 * i + 1], 4);    // entry 8i + (l & 7)
    float t = (b3 ? c[1] : c[0]) + __shfl_xor(b3 ? c[0] : c[1], 8);                                                    // entry l & 15
    t += __shfl_xor(t, 16);
    t += __shfl_xor(t, 32);
    return t;
}

struct EncChoice {
    float sse;         // squared error of the best pattern so far (uniform over the wavefront)
    int pattern;
    uint32_t idx;      // this lane's two indices: value 2l in bits 3:0, value 2l+1 in bits 7:4
};

// Pattern search over patterns [p0, p1) for the group whose two values of this lane are (x0, x1):
// reconstructed values fp16(centroid * s) of those patterns into E.recon, nearest value per element
// (strict <: the lowest index wins a tie), squared errors summed by the balanced tree, least sum
// wins (strict <: the lowest pattern wins a tie).  p0 < p1.
// Choosing the pattern needs the least distance of every element, not the index that attains it: the squared
// error of an element is that distance squared, whichever of several equally near values is taken.  So the
// patterns are rated with a subtraction per candidate and a three-way minimum per two candidates, and the
// index scan (a subtraction, a compare and a select per candidate) runs once, for the winner.
__device__ inline EncChoice search_patterns(const EncLds& E, int p0, int p1, float s, float x0, float x1) {
    const int lane = threadIdx.x & 63;
    for (int i = p0 * kK + lane; i < p1 * kK; i += 64) E.recon[i] = half_bits_f(dequant_bits(__half_as_ushort(E.cent[i]), s));
    wave_lds_fence();
    EncChoice best{0.0f, p0, 0u};
    if (p1 - p0 > 1) {
        // Sixteen patterns at a time: q[e] is this lane's part (two elements) of the squared error of pattern pb + e.
        // The sixteen sums over the wavefront are formed together (wave_sum16): lane l ends up with the total of
        // pattern pb + (l & 15), keeps the least it has seen over the batches, and the lanes are compared at the end.
        float mine = __builtin_inff();
        int mine_p = p0;
        for (int pb = p0; pb < p1; pb += 16) {
            float q[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                q[e] = __builtin_inff();
                if (pb + e < p1) {  // uniform
                    const float* r = E.recon + (pb + e) * kK;
                    float d0 = fabsf(__fsub_rn(x0, r[0])), d1 = fabsf(__fsub_rn(x1, r[0]));
                    static_assert(kK % 2 == 0, "candidates 1 .. kK - 2 in pairs, the last one alone");
#pragma unroll
                    for (int k = 1; k + 1 < kK; k += 2) {
                        const float ra = r[k], rb = r[k + 1];
                        d0 = fminf(fminf(d0, fabsf(__fsub_rn(x0, ra))), fabsf(__fsub_rn(x0, rb)));
                        d1 = fminf(fminf(d1, fabsf(__fsub_rn(x1, ra))), fabsf(__fsub_rn(x1, rb)));
                    }
                    d0 = fminf(d0, fabsf(__fsub_rn(x0, r[kK - 1])));
                    d1 = fminf(d1, fabsf(__fsub_rn(x1, r[kK - 1])));
                    q[e] = __fadd_rn(__fmul_rn(d0, d0), __fmul_rn(d1, d1));  // tree level 0: values 2l and 2l+1
                }
            }
            const float t = wave_sum16(q, lane);
            const int tp = pb + (lane & 15);
            if (t < mine) {  // strict <: an earlier batch keeps a tie
                mine = t;
                mine_p = tp;
            }
        }
        // least sum over the lanes, and the lowest pattern among the lanes that hold it (a pattern past p1 holds +inf;
        // if every sum is +inf or the input held a NaN, against the contract, p0 stays)
        best.sse = wave_all(mine, [](float a, float b) { return fminf(a, b); });
        const int cand = (mine == best.sse && mine_p < p1) ? mine_p : 0x7FFFFFFF;
        const int win = wave_all(cand, [](int a, int b) { return min(a, b); });
        best.pattern = win < p1 ? win : p0;
    }
    // The indices of the chosen pattern.  The reconstructed values ascend with k, and FP32 rounding is monotone, so
    // |x - r[k]| falls (weakly) up to its least value and rises (weakly) after it: the first index of the least
    // distance -- what a scan with a strict < finds -- is the last k at which the distance strictly drops.
    const float* r = E.recon + best.pattern * kK;
    float d0 = fabsf(__fsub_rn(x0, r[0])), d1 = fabsf(__fsub_rn(x1, r[0]));
    uint32_t k0 = 0, k1 = 0;
#pragma unroll
    for (int k = 1; k < kK; ++k) {
        const float rk = r[k];
        const float a = fabsf(__fsub_rn(x0, rk)), b = fabsf(__fsub_rn(x1, rk));
        k0 = a < d0 ? (uint32_t)k : k0;
        k1 = b < d1 ? (uint32_t)k : k1;
        d0 = a;
        d1 = b;
    }
    best.idx = k0 | (k1 << 4);
    if (p1 - p0 == 1) {
        const float e0 = __fsub_rn(x0, r[k0]), e1 = __fsub_rn(x1, r[k1]);
        best.sse = wave_sum(__fadd_rn(__fmul_rn(e0, e0), __fmul_rn(e1, e1)));
    }
    return best;
}

// Packs the group with the chosen pattern and indices: lanes 0..15 return one payload word each in
// *word, every lane the meta word in *meta.
__device__ inline void pack_group(const EncLds& E, uint32_t smax, int best_p, uint32_t best_idx, uint32_t* word, uint32_t* meta) {
    const int lane = threadIdx.x & 63;
    if (lane < kBlockWords) E.bits[lane] = 0;
    wave_lds_fence();
    // codes of the chosen pattern, bit positions by an inclusive scan over lanes
    const uint32_t c0 = E.enc[best_p * kK + (best_idx & 15u)], c1 = E.enc[best_p * kK + (best_idx >> 4)];
    const uint32_t l0 = c0 >> 16, l1 = c1 >> 16;
    uint32_t incl = l0 + l1;
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)incl, d);
        if (lane >= d) incl += o;
    }
    const uint32_t total = (uint32_t)__shfl((int)incl, 63);
    const uint32_t mid = (uint32_t)__shfl((int)incl, 31);  // bits used by values 0..63
    const bool raw = total > 8u * ECCO_BLOCK_BYTES;
    if (raw) {
        // value i in stream bits 4i..4i+3, top bit first: lane l owns the byte at stream bits 8l..8l+7
        atomicOr(&E.bits[lane >> 2], (((best_idx & 15u) << 4) | (best_idx >> 4)) << (24 - 8 * (lane & 3)));
    } else {
        const uint32_t pos = incl - (l0 + l1);
        const uint32_t both = ((c0 & 0xFFFFu) << l1) | (c1 & 0xFFFFu);       // l0 + l1 <= 24 bits
        const uint64_t v = (uint64_t)both << (64 - (l0 + l1) - (pos & 31u));  // left-aligned at stream bit pos
        atomicOr(&E.bits[pos >> 5], (uint32_t)(v >> 32));
        if ((uint32_t)v != 0u) atomicOr(&E.bits[(pos >> 5) + 1], (uint32_t)v);
    }
    wave_lds_fence();
    *word = lane < kBlockWords ? E.bits[lane] : 0u;
    *meta = smax | ((uint32_t)best_p << 16) | (raw ? (1u << 22) : 0u) | ((raw ? 4u * kHalf : mid) << 23);
    wave_lds_fence();
}

// Pattern selector of the online compressor (Section 3.2 "KV Cache Compression", pattern selector of Section 4.3):
// only the group's least and greatest value are compared with each pattern's ends, taken in the group's scale as
// fp16(centroid * s):  fitness = (min - first)^2 + (max - last)^2, every operation rounded to FP32 on its own.
// Lane p rates pattern p (S <= 64); the least fitness wins, the lowest pattern on a tie.  Uniform result.
__device__ inline int select_minmax(const EncLds& E, int S, float s, float x0, float x1) {
    const int lane = threadIdx.x & 63;
    const float lo = wave_all(fminf(x0, x1), [](float a, float b) { return fminf(a, b); });
    const float hi = wave_all(fmaxf(x0, x1), [](float a, float b) { return fmaxf(a, b); });
    float f = __builtin_inff();
    if (lane < S) {
        const float first = half_bits_f(dequant_bits(__half_as_ushort(E.cent[lane * kK]), s));
        const float last = half_bits_f(dequant_bits(__half_as_ushort(E.cent[lane * kK + kK - 1]), s));
        const float dlo = __fsub_rn(lo, first), dhi = __fsub_rn(hi, last);
        f = __fadd_rn(__fmul_rn(dlo, dlo), __fmul_rn(dhi, dhi));
    }
    const float least = wave_all(f, [](float a, float b) { return fminf(a, b); });
    // lowest lane holding the least fitness (no lane does if the input held a NaN, against the contract: pattern 0 then)
    return max(__ffsll((long long)__ballot(f == least)) - 1, 0);
}

// One wavefront encodes one group (hx0, hx1: this lane's two values as FP16 bits).  kMinMax: the pattern comes
// from the min/max selector and only that pattern's value mapping is done; otherwise every pattern is tried
// and the least squared error wins.
template <bool kMinMax>
__device__ inline void encode_group(const EncLds& E, int S, uint32_t hx0, uint32_t hx1, uint32_t* word, uint32_t* meta) {
    const uint32_t smax = group_scale_bits(hx0, hx1);
    const float s = half_bits_f(smax), x0 = half_bits_f(hx0), x1 = half_bits_f(hx1);
    int p0 = 0, p1 = S;
    if (kMinMax) {
        p0 = select_minmax(E, S, s, x0, x1);
        p1 = p0 + 1;
    }
    const EncChoice c = search_patterns(E, p0, p1, s, x0, x1);
    pack_group(E, smax, c.pattern, c.idx, word, meta);
}

constexpr size_t enc_lds_bytes(int S) { return (size_t)S * kK * 2 + (size_t)S * kK * 4 + (size_t)kEncWaves * ((size_t)S * kK * 4 + kBlockWords * 4); }

__device__ inline EncLds setup_enc_lds(unsigned char* smem, const uint32_t* dev, int S) {
    const DevLayout D{S};
    uint32_t* cent = reinterpret_cast<uint32_t*>(smem);
    uint32_t* enc = cent + S * kK / 2;
    float* recon = reinterpret_cast<float*>(enc + S * kK);
    uint32_t* bits = reinterpret_cast<uint32_t*>(recon + kEncWaves * S * kK);
    stage_vec(cent, dev + D.cent(), S * kK / 2);
    stage_vec(enc, dev + D.enc(), S * kK);
    __syncthreads();
    const int wave = threadIdx.x >> 6;
    EncLds E;
    E.cent = reinterpret_cast<const __half*>(cent);
    E.enc = enc;
    E.recon = recon + wave * S * kK;
    E.bits = bits + wave * kBlockWords;
    return E;
}

template <bool kMinMax>
__global__ __launch_bounds__(kEncThreads) void encode_kernel(const uint32_t* __restrict__ dev, int S,
                                                             const uint32_t* __restrict__ src, size_t n_groups,
                                                             uint32_t* __restrict__ blocks, uint32_t* __restrict__ meta) {
    extern __shared__ __align__(16) unsigned char smem_enc[];
    EncLds E = setup_enc_lds(smem_enc, dev, S);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (size_t g = (size_t)blockIdx.x * kEncWaves + wave; g < n_groups; g += (size_t)gridDim.x * kEncWaves) {
        const uint32_t pair = src[g * (kGroup / 2) + lane];
        uint32_t word, mw;
        encode_group<kMinMax>(E, S, pair & 0xFFFFu, pair >> 16, &word, &mw);
        if (lane < kBlockWords) blocks[g * kBlockWords + lane] = word;
        if (lane == 0) meta[g] = mw;
    }
}

// grid: (B*H, 2); y = 0 encodes K, y = 1 encodes V.  One workgroup per new group: the append is a
// latency problem (B*H*2 groups, far fewer than the chip has wavefront slots), so the four wavefronts
// of the workgroup split the pattern search, a quarter of the patterns each, and wavefront 0 packs
// the winner (ascending pattern ranges, strict <: the lowest pattern still wins a tie).
__global__ __launch_bounds__(kEncThreads) void kv_append_kernel(const uint32_t* __restrict__ dev_k, int Sk,
                                                                const uint32_t* __restrict__ dev_v, int Sv,
                                                                const uint32_t* __restrict__ k_new, const uint32_t* __restrict__ v_new,
                                                                uint32_t* __restrict__ k_blocks, uint32_t* __restrict__ k_meta,
                                                                uint32_t* __restrict__ v_blocks, uint32_t* __restrict__ v_meta,
                                                                const int32_t* __restrict__ seq_len, int B, int H, int T_max) {
    extern __shared__ __align__(16) unsigned char smem_enc[];
    __shared__ float cand_sse[kEncWaves];
    __shared__ int cand_pattern[kEncWaves];
    __shared__ uint32_t cand_idx[kEncWaves][64];
    const bool is_v = blockIdx.y != 0;  // uniform per workgroup, so each workgroup stages one model
    const int S = is_v ? Sv : Sk;
    EncLds E = setup_enc_lds(smem_enc, is_v ? dev_v : dev_k, S);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int bh = blockIdx.x;
    const int t = seq_len[bh / H];
    if (t < 0 || t >= T_max) return;  // uniform over the workgroup
    const uint32_t* src = (is_v ? v_new : k_new) + (size_t)bh * (kGroup / 2);
    const uint32_t pair = src[lane];
    const uint32_t smax = group_scale_bits(pair & 0xFFFFu, pair >> 16);
    const int per = (S + kEncWaves - 1) / kEncWaves;
    const int p0 = wave * per, p1 = min(S, p0 + per);
    if (p0 < p1) {
        const EncChoice c = search_patterns(E, p0, p1, half_bits_f(smax), half_bits_f(pair & 0xFFFFu), half_bits_f(pair >> 16));
        cand_idx[wave][lane] = c.idx;
        if (lane == 0) {
            cand_sse[wave] = c.sse;
            cand_pattern[wave] = c.pattern;
        }
    }
    __syncthreads();
    if (wave != 0) return;
    int win = 0;
    for (int w = 1; w < kEncWaves; ++w)
        if (w * per < S && cand_sse[w] < cand_sse[win]) win = w;
    uint32_t word, mw;
    pack_group(E, smax, cand_pattern[win], cand_idx[win][lane], &word, &mw);
    const size_t g = (size_t)bh * T_max + t;
    uint32_t* blocks = is_v ? v_blocks : k_blocks;
    uint32_t* meta = is_v ? v_meta : k_meta;
    if (lane < kBlockWords) blocks[g * kBlockWords + lane] = word;
    if (lane == 0) meta[g] = mw;
}

// The append with the min/max selector: grid (ceil(B*H / 4), 2); one wavefront per new group, since the
// selector leaves a single pattern to map and nothing to split.
__global__ __launch_bounds__(kEncThreads) void kv_append_minmax_kernel(const uint32_t* __restrict__ dev_k, int Sk,
                                                                       const uint32_t* __restrict__ dev_v, int Sv,
                                                                       const uint32_t* __restrict__ k_new, const uint32_t* __restrict__ v_new,
                                                                       uint32_t* __restrict__ k_blocks, uint32_t* __restrict__ k_meta,
                                                                       uint32_t* __restrict__ v_blocks, uint32_t* __restrict__ v_meta,
                                                                       const int32_t* __restrict__ seq_len, int B, int H, int T_max) {
    extern __shared__ __align__(16) unsigned char smem_enc[];
    const bool is_v = blockIdx.y != 0;
    const int S = is_v ? Sv : Sk;
    EncLds E = setup_enc_lds(smem_enc, is_v ? dev_v : dev_k, S);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int bh = blockIdx.x * kEncWaves + wave;
    if (bh >= B * H) return;  // no workgroup barrier below
    const int t = seq_len[bh / H];
    if (t < 0 || t >= T_max) return;
    const uint32_t pair = ((is_v ? v_new : k_new) + (size_t)bh * (kGroup / 2))[lane];
    uint32_t word, mw;
    encode_group<true>(E, S, pair & 0xFFFFu, pair >> 16, &word, &mw);
    const size_t g = (size_t)bh * T_max + t;
    uint32_t* blocks = is_v ? v_blocks : k_blocks;
    uint32_t* meta = is_v ? v_meta : k_meta;
    if (lane < kBlockWords) blocks[g * kBlockWords + lane] = word;
    if (lane == 0) meta[g] = mw;
}

// ---- single-query attention over compressed K / V ----------------------------------------------------
// One workgroup of 12 wavefronts per (sequence, head): three per SIMD, which leaves each lane the
// registers for 64 private accumulators next to the decoder state (8 wavefronts when the V model has
// codes longer than the table peek: that decoder needs more registers still).  The cache of a head is a band of T blocks,
// so the kernel reuses the streaming scheme of the batch-1 GEMV: a unit is 32 consecutive tokens
// (2 KB of payload), lane l of a wavefront decodes chain l / 32 of token l % 32, units are
// prefetched into registers and decoded out of the wavefront's private LDS buffer.  The sequence is
// walked in spans of kSpan tokens.  Per span: with the K tables in LDS the scores q.K_t / sqrt(128)
// are formed (the lane keeps the 64 query elements of its chain in registers) and kept in LDS; the
// span's maximum updates the running softmax (maximum, denominator, rescale of what has been
// accumulated); then the V tables replace the K tables and every lane adds p_t * V_t of its chain
// into 64 private FP32 accumulators (a static register per value position, nothing shared).  At the
// end the accumulators are added over the lanes of a wavefront on the VALU and over the wavefronts
// through LDS.  K and V enter as fp16(centroid * scale), formed two at a time by a packed FP16
// multiply, which rounds exactly like the FP32-multiply-then-round rule.  Only one model's tables
// are resident at a time, which keeps S = 64 for both K and V within 160 KB of LDS.
constexpr int kAttnThreads = 768;      // workgroup size; 512 for a V model with long codes
constexpr int kAttnWaves = kAttnThreads / 64;
constexpr int kSpan = 8192;
static_assert(2 * 512 >= ECCO_MAX_S * kK, "stage_tables_around: two table items per thread cover every model (the smallest attention workgroup has 512 threads)");
inline size_t attn_lds_bytes(int Sk, int Sv) {
    return (table_words(std::max(Sk, Sv)) + (size_t)kAttnWaves * kUnitWords + kSpan + kAttnWaves * 2 * kGroup + 64) * 4;
}

__device__ inline float wg_reduce(float v, float* scratch, bool is_max, int waves) {
    for (int m = 1; m < 64; m <<= 1) {
        float o = __shfl_xor(v, m);
        v = is_max ? fmaxf(v, o) : v + o;
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = scratch[0];
    for (int w = 1; w < waves; ++w) r = is_max ? fmaxf(r, scratch[w]) : r + scratch[w];
    return r;
}

template <bool kLongK, bool kLongV>
__global__ __launch_bounds__(kLongV ? 512 : kAttnThreads) void kv_attend_kernel(const uint32_t* __restrict__ dev_k, int Sk,
                                                                 const uint32_t* __restrict__ dev_v, int Sv,
                                                                 const uint16_t* __restrict__ q,
                                                                 const uint4* __restrict__ k_blocks, const uint32_t* __restrict__ k_meta,
                                                                 const uint4* __restrict__ v_blocks, const uint32_t* __restrict__ v_meta,
                                                                 const int32_t* __restrict__ seq_len, int H, int T_max,
                                                                 float* __restrict__ out) {
    extern __shared__ __align__(16) uint32_t smem[];
    const int Smax = max(Sk, Sv);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int waves = kLongV ? 8 : kAttnWaves, threads = waves * 64;
    uint32_t* wbuf = smem + table_words(Smax) + wave * kUnitWords;
    float* scores = reinterpret_cast<float*>(smem + table_words(Smax) + kAttnWaves * kUnitWords);
    float* wred = scores + kSpan;               // [wavefront][row of 16 lanes][64] at the end
    float* scratch = wred + kAttnWaves * 2 * kGroup;
    if (lane < kUnitBlocks) wbuf[lane * kStride + kBlockWords] = 0u;
    if (lane == 0) wbuf[kUnitBlocks * kStride] = 0u;

    const int bh = blockIdx.x;
    const int T = min(seq_len[bh / H], T_max);
    const int blk = lane & (kUnitBlocks - 1), half = lane >> 5;
    float my_out = 0.0f;  // threads 0..127: output element `tid`, not yet divided by the denominator
    float run_max = -INFINITY, run_den = 0.0f;
    const float inv_sqrt_d = 0.08838834764831845f;  // 1 / sqrt(128)
    for (int s0 = 0; s0 < T; s0 += kSpan) {
        const int span = min(kSpan, T - s0);
        const int units = (span + kUnitBlocks - 1) / kUnitBlocks, unit0 = s0 / kUnitBlocks;
        // ---- scores of the span
        __syncthreads();
        int u = wave;
        UnitLoad pre;
        const Tables TK = stage_tables_around<kLongK>(smem, dev_k, Sk, [&] { pre = load_unit(k_blocks, k_meta, bh, T_max, unit0 + min(u, units - 1), lane); });
        __syncthreads();
        float my_max = -INFINITY;
        {
            uint32_t qx[kHalf / 2];  // the query elements of this lane's chain, FP16 pairs
            // reloaded per span (from cache) rather than kept alive across the V phase; the pointer that comes back from
            // the empty asm statement is given its address space again, or its loads would be flat loads
            const uint4* qgen = reinterpret_cast<const uint4*>(q + (size_t)bh * kGroup + half * kHalf);
            asm volatile("" : "+v"(qgen));
            const global_u4* qsrc = (const global_u4*)qgen;
#pragma unroll
            for (int j = 0; j < kHalf / 8; ++j) {
                const u32x4 v = qsrc[j];
                qx[4 * j] = v.x; qx[4 * j + 1] = v.y; qx[4 * j + 2] = v.z; qx[4 * j + 3] = v.w;
            }
            for (; u < units; u += waves) {
                store_unit(wbuf, pre, lane);
                const uint32_t mw = pre.meta;
                if (u + waves < units) pre = load_unit(k_blocks, k_meta, bh, T_max, unit0 + u + waves, lane);
                // the query stays packed: without this the conversions to FP32 are hoisted out of the loop and
                // occupy 64 registers instead of 32
#pragma unroll
                for (int j = 0; j < kHalf / 2; ++j) asm volatile("" : "+v"(qx[j]));
                const Lane L = lane_setup(TK, mw, Sk);
                const _Float16 sh = __builtin_bit_cast(_Float16, (unsigned short)(mw & 0xFFFFu));
                const half2_t s2 = {sh, sh};
                uint32_t pk = 0;
                float acc = 0.0f;
                decode_chain<kLongK, kHalf>(wbuf + blk * kStride, half ? L.second_start : 0u, L, [&](int i, uint32_t e) {
                    if ((i & 1) == 0) {
                        pk = e >> 16;
                    } else {
                        const half2_t w2 = __builtin_bit_cast(half2_t, pk | (e & 0xFFFF0000u)) * s2;
                        const half2_t q2 = __builtin_bit_cast(half2_t, qx[i >> 1]);
                        acc = fmaf((float)w2[0], (float)q2[0], acc);
                        acc = fmaf((float)w2[1], (float)q2[1], acc);
                        if ((i & 3) == 3) asm volatile("" : "+v"(acc));  // keeps the multiply-adds next to their table reads
                    }
                });
                acc += __shfl_xor(acc, 32);
                const int t = u * kUnitBlocks + blk;
                const float sc = t < span ? acc * inv_sqrt_d : -INFINITY;
                if (half == 0) scores[t] = sc;
                my_max = fmaxf(my_max, sc);
            }
        }
        // ---- running softmax
        const float new_max = fmaxf(run_max, wg_reduce(my_max, scratch, true, waves));
        float my_den = 0.0f;
        for (int t = tid; t < units * kUnitBlocks; t += threads) {
            const float p = __expf(scores[t] - new_max);  // 0 for the tokens past the span
            scores[t] = p;
            my_den += p;
        }
        const float rescale = (run_max == -INFINITY) ? 0.0f : __expf(run_max - new_max);
        run_den = run_den * rescale + wg_reduce(my_den, scratch, false, waves);
        run_max = new_max;
        // ---- weighted sum of V over the span
        __syncthreads();
        u = wave;
        const Tables TV = stage_tables_around<kLongV>(smem, dev_v, Sv, [&] { pre = load_unit(v_blocks, v_meta, bh, T_max, unit0 + min(u, units - 1), lane); });
        __syncthreads();
        {
            float o[kHalf];
#pragma unroll
            for (int i = 0; i < kHalf; ++i) o[i] = 0.0f;
            for (; u < units; u += waves) {
                store_unit(wbuf, pre, lane);
                // a slot past the sequence end may hold anything (the cache behind seq_len need not be initialised):
                // its scale is taken as 0, so that its values are zeros and not, say, NaN times a zero weight
                const uint32_t mw = (u * kUnitBlocks + blk < span) ? pre.meta : (pre.meta & 0xFFFF0000u);
                if (u + waves < units) pre = load_unit(v_blocks, v_meta, bh, T_max, unit0 + u + waves, lane);
                const Lane L = lane_setup(TV, mw, Sv);
                const _Float16 sh = __builtin_bit_cast(_Float16, (unsigned short)(mw & 0xFFFFu));
                const half2_t s2 = {sh, sh};
                const float p = scores[u * kUnitBlocks + blk];
                uint32_t pk = 0;
                decode_chain<kLongV, kHalf>(wbuf + blk * kStride, half ? L.second_start : 0u, L, [&](int i, uint32_t e) {
                    if ((i & 1) == 0) {
                        pk = e >> 16;
                    } else {
                        const half2_t w2 = __builtin_bit_cast(half2_t, pk | (e & 0xFFFF0000u)) * s2;
                        o[i - 1] = fmaf(p, (float)w2[0], o[i - 1]);
                        o[i] = fmaf(p, (float)w2[1], o[i]);
                    }
                });
            }
            // the span's sums: over the lanes of a wavefront on the VALU (lanes 0..31 hold values 0..63, lanes
            // 32..63 values 64..127), then over the wavefronts through LDS into the running output
            int ln = lane;  // taken afresh: what is derived from it is then formed here, not kept across the loop above
            asm volatile("" : "+v"(ln));
            const bool row_first = (ln & 15) == 0;
            float* wrow = wred + (wave * 4 + (ln >> 4)) * kHalf;
#pragma unroll
            for (int i = 0; i < kHalf; ++i) {
                float t = o[i];
                t += dpp_mov<0xB1>(t);   // quad_perm [1,0,3,2]
                t += dpp_mov<0x4E>(t);   // quad_perm [2,3,0,1]
                t += dpp_mov<0x141>(t);  // row_half_mirror
                t += dpp_mov<0x140>(t);  // row_mirror: every lane of a row of 16 now holds the row's sum
                // the first lane of each row stores it: rows 0 and 1 belong to values 0..63, rows 2 and 3 to 64..127
                if (row_first) wrow[i] = t;
            }
        }
        __syncthreads();
        if (tid < kGroup) {
            float v = 0.0f;
            const int hrow = (tid >> 6) * 2, i = tid & (kHalf - 1);
#pragma unroll 4
            for (int w = 0; w < waves; ++w) v += wred[(w * 4 + hrow) * kHalf + i] + wred[(w * 4 + hrow + 1) * kHalf + i];
            my_out = my_out * rescale + v;
        }
    }
    if (tid < kGroup) out[(size_t)bh * kGroup + tid] = T > 0 ? my_out / run_den : 0.0f;
}

// ---- grouped-query attention over compressed K / V, split over the tokens ---------------------------------
// Several query heads share one key/value head (Section 5.3: with grouped-query attention the batched
// matrix-vector products become small matrix products).  One workgroup of 8 wavefronts per (sequence,
// key/value head, token split) decodes every K and V block of its token range once and serves all
// grp = Hq / Hkv query heads of the group with it, on the matrix cores:
//   scores  S[token][head] = sum_dim K[token][dim] q[head][dim]:  v_mfma_f32_32x32x16_f16 with the 32 tokens
//           of a unit as rows; lane l decodes chain l / 32 of token l % 32, which is exactly the A layout (row
//           l % 32, eight consecutive k per lane, k group l / 32) once the 16 k of a step are taken to be
//           dimensions 8j..8j+7 of chain 0 and of chain 1; B holds the queries (head l % 32, zero past grp).
//   output  O[dim][head] = sum_token V[token][dim] P[head][token]: here the reduction runs over the tokens, so the
//           decoded values have to be turned: every 16 values the wavefront writes a 32 dims x 32 tokens FP16 tile
//           to its private LDS buffer (neighbouring lanes first swap halves so that each writes two tokens of one
//           dimension), reads it back as A operands (row = dimension, eight tokens per lane) and multiplies with
//           the FP16 probabilities; the four 32 x 32 accumulator tiles (64 registers) live across the spans.
// The sequence is walked in spans; per span the scores go to LDS, each head's running maximum and
// denominator are updated (one wavefront per head), the accumulators of a lane -- all of one head -- are
// rescaled, and the probabilities are stored as FP16 (the denominator sums the rounded values).  With one
// split the result is normalised and written; otherwise (maximum, denominator, unnormalised output) of the
// split go to the caller's workspace and kv_attend_combine_kernel merges the splits.
constexpr int kGqaThreads = 512;
constexpr int kGqaWaves = kGqaThreads / 64;
constexpr int kGqaMaxGroup = 16;
constexpr int kTileStride = 20;                 // words per row of the transposition tile: 32 tokens (16 words) + 4 of padding
constexpr int kTileWords = 32 * kTileStride;
constexpr int kGqaSpanBudget = 7680;            // query heads x tokens of a span kept in LDS (FP32 scores + FP16 probabilities)
typedef float float16_t __attribute__((ext_vector_type(16)));

__host__ __device__ constexpr int gqa_span(int grp) { return (kGqaSpanBudget / grp) & ~(kUnitBlocks - 1); }
__host__ __device__ constexpr int gqa_score_stride(int span) { return span + 1; }   // words; odd, so that heads fall on different banks
__host__ __device__ constexpr int gqa_prob_stride(int span) { return span + 8; }    // halves; rows stay 16-byte aligned
// LDS words of the span's scores (FP32, rounded up to a 16-byte boundary) and probabilities (FP16); the same region
// holds the cross-wavefront sum of one accumulator tile at the end
__host__ __device__ constexpr int gqa_score_words(int grp, int span) { return (grp * gqa_score_stride(span) + 3) & ~3; }
__host__ __device__ constexpr int gqa_shared_words(int grp, int span) {
    const int a = gqa_score_words(grp, span) + (grp * gqa_prob_stride(span) + 1) / 2, b = kGqaWaves * 16 * 64;
    return a > b ? a : b;
}
constexpr int kGqaStateWords = 64;  // running maximum, denominator and rescale factor per query head
inline size_t gqa_lds_bytes(int Sk, int Sv, int grp) {
    return (table_words(std::max(Sk, Sv)) + (size_t)kGqaWaves * (kUnitWords + kTileWords) + kGqaStateWords +
            gqa_shared_words(grp, gqa_span(grp))) * 4;
}

template <bool kLongK, bool kLongV>
__global__ __launch_bounds__(kGqaThreads) void kv_attend_gqa_kernel(const uint32_t* __restrict__ dev_k, int Sk,
                                                                    const uint32_t* __restrict__ dev_v, int Sv,
                                                                    const uint16_t* __restrict__ q,
                                                                    const uint4* __restrict__ k_blocks, const uint32_t* __restrict__ k_meta,
                                                                    const uint4* __restrict__ v_blocks, const uint32_t* __restrict__ v_meta,
                                                                    const int32_t* __restrict__ seq_len, int Hq, int Hkv, int T_max,
                                                                    float* __restrict__ out, float* __restrict__ ws) {
    extern __shared__ __align__(16) uint32_t smem[];
    const int Smax = max(Sk, Sv);
    const int grp = Hq / Hkv, span_max = gqa_span(grp);
    const int sstride = gqa_score_stride(span_max), pstride = gqa_prob_stride(span_max);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    uint32_t* wbuf = smem + table_words(Smax) + wave * kUnitWords;
    uint32_t* tile = smem + table_words(Smax) + kGqaWaves * kUnitWords + wave * kTileWords;
    float* st_max = reinterpret_cast<float*>(smem + table_words(Smax) + kGqaWaves * (kUnitWords + kTileWords));
    float* st_den = st_max + kGqaMaxGroup;
    float* st_alpha = st_den + kGqaMaxGroup;
    uint32_t* shared0 = smem + table_words(Smax) + kGqaWaves * (kUnitWords + kTileWords) + kGqaStateWords;
    float* scores = reinterpret_cast<float*>(shared0);                                             // [grp][sstride]
    _Float16* probs = reinterpret_cast<_Float16*>(shared0 + gqa_score_words(grp, span_max));       // [grp][pstride]
    float* red = reinterpret_cast<float*>(shared0);                                                // [wavefront][16][64], after the last span
    if (lane < kUnitBlocks) wbuf[lane * kStride + kBlockWords] = 0u;
    if (lane == 0) wbuf[kUnitBlocks * kStride] = 0u;
    if (tid < kGqaMaxGroup) {
        st_max[tid] = -INFINITY;
        st_den[tid] = 0.0f;
        st_alpha[tid] = 1.0f;
    }

    const int bkv = blockIdx.x, b = bkv / Hkv, hkv = bkv - b * Hkv;
    const int n_splits = gridDim.y, split = blockIdx.y;
    const int T = max(0, min(seq_len[b], T_max));
    const int units_total = (T + kUnitBlocks - 1) / kUnitBlocks;
    const int units_per_split = (units_total + n_splits - 1) / n_splits;
    const int t_begin = min(T, split * units_per_split * kUnitBlocks), t_end = min(T, (split + 1) * units_per_split * kUnitBlocks);
    const int blk = lane & (kUnitBlocks - 1), half = lane >> 5;   // token of the unit and chain of this lane; also MFMA row / column and k group
    const bool head_ok = blk < grp;
    const size_t q_row = ((size_t)b * Hq + (size_t)hkv * grp + (head_ok ? blk : 0)) * kGroup;
    const float inv_sqrt_d = 0.08838834764831845f;  // 1 / sqrt(128)
    const uint32_t swap_sel = (lane & 1) ? 0x03020706u : 0x05040100u;  // odd lanes keep the high halves, even lanes the low halves
    float16_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[j][i] = 0.0f;

    for (int s0 = t_begin; s0 < t_end; s0 += span_max) {
        const int span = min(span_max, t_end - s0);
        const int units = (span + kUnitBlocks - 1) / kUnitBlocks, unit0 = s0 / kUnitBlocks;  // s0 is a multiple of 32
        // ---- scores of the span, all query heads of the group
        __syncthreads();
        int u = wave;
        UnitLoad pre;
        const Tables TK = stage_tables_around<kLongK>(smem, dev_k, Sk, [&] { pre = load_unit(k_blocks, k_meta, bkv, T_max, unit0 + min(u, units - 1), lane); });
        __syncthreads();
        {
            uint4 bq[kHalf / 8];  // B operands: the query of head blk, dimensions 64 * half + 8j .. + 7
            // reloaded per span rather than kept alive across the V phase (address space restored as above)
            const uint4* qgen = reinterpret_cast<const uint4*>(q + q_row + half * kHalf);
            asm volatile("" : "+v"(qgen));
            const global_u4* qsrc = (const global_u4*)qgen;
#pragma unroll
            for (int j = 0; j < kHalf / 8; ++j) {
                const u32x4 v = qsrc[j];
                bq[j] = head_ok ? make_uint4(v.x, v.y, v.z, v.w) : make_uint4(0u, 0u, 0u, 0u);
            }
            for (; u < units; u += kGqaWaves) {
                store_unit(wbuf, pre, lane);
                const uint32_t mw = pre.meta;
                if (u + kGqaWaves < units) pre = load_unit(k_blocks, k_meta, bkv, T_max, unit0 + u + kGqaWaves, lane);
                const Lane L = lane_setup(TK, mw, Sk);
                const _Float16 sh = __builtin_bit_cast(_Float16, (unsigned short)(mw & 0xFFFFu));
                const half2_t s2 = {sh, sh};
                uint32_t pk[4];
                float16_t acc;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
                decode_chain<kLongK, kHalf>(wbuf + blk * kStride, half ? L.second_start : 0u, L, [&](int i, uint32_t e) {
                    if ((i & 1) == 0) {
                        pk[(i >> 1) & 3] = e >> 16;
                        return;
                    }
                    pk[(i >> 1) & 3] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, pk[(i >> 1) & 3] | (e & 0xFFFF0000u)) * s2);
                    if ((i & 7) != 7) return;
                    const uint4 av = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, av), __builtin_bit_cast(half8_t, bq[i >> 3]), acc, 0, 0, 0);
                });
                // accumulator layout of the 32 x 32 tile: register i of lane l is row 8 * (i / 4) + 4 * (l / 32) + i % 4, column l % 32
                if (head_ok) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int t = u * kUnitBlocks + 8 * (i >> 2) + 4 * half + (i & 3);
                        scores[blk * sstride + t] = t < span ? acc[i] * inv_sqrt_d : -INFINITY;
                    }
                }
            }
        }
        __syncthreads();
        // ---- running softmax, one wavefront per query head
        for (int g = wave; g < grp; g += kGqaWaves) {
            const int n = units * kUnitBlocks;
            // both passes take four scores per lane at a time, so that their LDS reads are in flight together (a loop
            // over single reads waits for each); indices past the end are clamped for the read (a repeated score does
            // not change a maximum) and left out of the second pass; the additions keep their order
            float mx = -INFINITY;
            for (int t0 = lane; t0 < n; t0 += 4 * 64) {
                float a[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) a[j] = scores[g * sstride + min(t0 + 64 * j, n - 1)];
#pragma unroll
                for (int j = 0; j < 4; ++j) mx = fmaxf(mx, a[j]);
            }
            mx = wave_all(mx, [](float a, float c) { return fmaxf(a, c); });
            const float old_max = st_max[g], new_max = fmaxf(old_max, mx);
            float den = 0.0f;
            for (int t0 = lane; t0 < n; t0 += 4 * 64) {
                float a[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) a[j] = scores[g * sstride + min(t0 + 64 * j, n - 1)];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (t0 + 64 * j < n) {
                        const _Float16 ph = (_Float16)__expf(a[j] - new_max);  // 0 for the tokens past the span
                        probs[g * pstride + t0 + 64 * j] = ph;
                        den += (float)ph;
                    }
                }
            }
            den = wave_sum(den);
            if (lane == 0) {
                const float alpha = (old_max == -INFINITY) ? 0.0f : __expf(old_max - new_max);
                st_alpha[g] = alpha;
                st_den[g] = st_den[g] * alpha + den;
                st_max[g] = new_max;
            }
        }
        // ---- weighted sum of V over the span
        __syncthreads();
        u = wave;
        const Tables TV = stage_tables_around<kLongV>(smem, dev_v, Sv, [&] { pre = load_unit(v_blocks, v_meta, bkv, T_max, unit0 + min(u, units - 1), lane); });
        __syncthreads();
        {
            const float alpha = head_ok ? st_alpha[blk] : 1.0f;  // every accumulator of a lane belongs to head l % 32
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[j][i] *= alpha;
            for (; u < units; u += kGqaWaves) {
                store_unit(wbuf, pre, lane);
                // a slot past the range may hold anything: scale 0, so that its values are zeros (NaN * 0 would poison the sum)
                const uint32_t mw = (u * kUnitBlocks + blk < span) ? pre.meta : (pre.meta & 0xFFFF0000u);
                if (u + kGqaWaves < units) pre = load_unit(v_blocks, v_meta, bkv, T_max, unit0 + u + kGqaWaves, lane);
                const Lane L = lane_setup(TV, mw, Sv);
                const _Float16 sh = __builtin_bit_cast(_Float16, (unsigned short)(mw & 0xFFFFu));
                const half2_t s2 = {sh, sh};
                // B operands: probabilities of head blk for tokens 16 ks + 8 * half .. + 7 of the unit
                uint4 pb[2];
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
                    pb[ks] = head_ok ? *reinterpret_cast<const uint4*>(probs + blk * pstride + u * kUnitBlocks + 16 * ks + 8 * half)
                                     : make_uint4(0u, 0u, 0u, 0u);
                uint32_t pk[8];
                decode_chain<kLongV, kHalf>(wbuf + blk * kStride, half ? L.second_start : 0u, L, [&](int i, uint32_t e) {
                    if ((i & 1) == 0) {
                        pk[(i >> 1) & 7] = e >> 16;
                        return;
                    }
                    pk[(i >> 1) & 7] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, pk[(i >> 1) & 7] | (e & 0xFFFF0000u)) * s2);
                    if ((i & 15) != 15) return;
                    // 16 values of this lane's token -> rows 16 * half + r of the tile (dimension 64 * half + 16 * (i / 16) + r);
                    // an even lane takes dimension 2 r2 of its own and its neighbour's token, the odd neighbour dimension 2 r2 + 1
                    wave_lds_fence();
#pragma unroll
                    for (int r2 = 0; r2 < 8; ++r2) {
                        const uint32_t other = (uint32_t)__builtin_amdgcn_mov_dpp((int)pk[r2], 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
                        tile[(16 * half + 2 * r2 + (lane & 1)) * kTileStride + (blk >> 1)] = __builtin_amdgcn_perm(other, pk[r2], swap_sel);
                    }
                    wave_lds_fence();
                    const uint4 a0 = *reinterpret_cast<const uint4*>(tile + blk * kTileStride + 4 * half);
                    const uint4 a1 = *reinterpret_cast<const uint4*>(tile + blk * kTileStride + 8 + 4 * half);
                    o[i >> 4] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a0), __builtin_bit_cast(half8_t, pb[0]), o[i >> 4], 0, 0, 0);
                    o[i >> 4] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a1), __builtin_bit_cast(half8_t, pb[1]), o[i >> 4], 0, 0, 0);
                });
            }
        }
    }
    // ---- sum over the wavefronts, one accumulator tile at a time; tile j row m is dimension 64 * (m / 16) + 16 j + m % 16
    const size_t part = ((size_t)b * Hq + (size_t)hkv * grp) * n_splits;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 16; ++i) red[(wave * 16 + i) * 64 + lane] = o[j][i];
        __syncthreads();
        for (int e = tid; e < 16 * 64; e += kGqaThreads) {
            float sum = 0.0f;
            for (int w = 0; w < kGqaWaves; ++w) sum += red[w * 16 * 64 + e];
            const int i = e >> 6, ln = e & 63, head = ln & 31;
            if (head >= grp) continue;
            const int m = 8 * (i >> 2) + 4 * (ln >> 5) + (i & 3);
            const int dim = 64 * (m >> 4) + 16 * j + (m & 15);
            if (n_splits == 1) {
                const float den = st_den[head];
                out[((size_t)b * Hq + (size_t)hkv * grp + head) * kGroup + dim] = den > 0.0f ? sum / den : 0.0f;
            } else {
                ws[((part + (size_t)head * n_splits) + split) * kGroup + dim] = sum;
            }
        }
    }
    if (n_splits > 1 && tid < grp) {
        // behind the partial outputs: [B * Hq][n_splits][2] = (maximum, denominator)
        float* ml = ws + (size_t)gridDim.x / Hkv * Hq * n_splits * kGroup;
        const size_t at = (part + (size_t)tid * n_splits + split) * 2;
        ml[at] = st_max[tid];
        ml[at + 1] = st_den[tid];
    }
}

// merges the token splits of one (sequence, query head): grid B * Hq, 128 threads
__global__ __launch_bounds__(kGroup) void kv_attend_combine_kernel(const float* __restrict__ ws, int n_heads, int n_splits, float* __restrict__ out) {
    const size_t bh = blockIdx.x;
    const float* ml = ws + (size_t)n_heads * n_splits * kGroup + bh * n_splits * 2;
    const float* part = ws + bh * n_splits * kGroup + threadIdx.x;
    // the largest of the splits' maxima: a few splits per lane and a wavefront maximum (exact whatever the order),
    // instead of a chain of n_splits dependent loads
    float mx = -INFINITY;
    for (int s = threadIdx.x & 63; s < n_splits; s += 64) mx = fmaxf(mx, ml[2 * s]);
    mx = wave_all(mx, [](float a, float b) { return fmaxf(a, b); });
    // Sixteen splits at a time with all their loads in flight together (indices clamped, the surplus given weight 0
    // by a select, no branch); the additions run in split order.  An empty split (maximum -inf, zeros) gets weight
    // 0, also when every split is empty (mx = -inf).
    float num = 0.0f, den = 0.0f;
    if (n_splits <= 8) {  // few splits: four at a time cost fewer surplus loads
#pragma unroll 4
        for (int s = 0; s < n_splits; ++s) {
            const float m = ml[2 * s], d = ml[2 * s + 1], v = part[(size_t)s * kGroup];
            const float w = m == -INFINITY ? 0.0f : __expf(m - mx);
            num += w * v;
            den += w * d;
        }
    } else
    for (int s0 = 0; s0 < n_splits; s0 += 16) {
        float m[16], d[16], v[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int sj = min(s0 + j, n_splits - 1);
            m[j] = ml[2 * sj];
            d[j] = ml[2 * sj + 1];
            v[j] = part[(size_t)sj * kGroup];
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if (s0 + j < n_splits) {  // uniform
                const float w = m[j] == -INFINITY ? 0.0f : __expf(m[j] - mx);
                num += w * v[j];
                den += w * d[j];
            }
        }
    }
    out[bh * kGroup + threadIdx.x] = den > 0.0f ? num / den : 0.0f;
}

// ---- device scratch of the entry point that allocates nothing -----------------------------------------------
// ecco_kv_attend_gqa_noalloc keeps the token splits' partial results here instead of in a caller's workspace.
// Each GPU the library runs on holds its own copy of the array, at its own address, until the process ends.  In host
// code the array's name is only a handle: the address kernels can use comes from hipGetSymbolAddress, asked once
// per device with that device current, and is what every launch and every host call is given.
static __device__ __align__(256) float scratch[ECCO_GQA_SCRATCH_BYTES / sizeof(float)];

constexpr int kMaxDevices = 16;
std::mutex scratch_lock;
float* scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, once asked

// The address of `scratch` on `device`, which must be the current device.  nullptr if the runtime refuses.
float* scratch_on_current_device(int device) {
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> hold(scratch_lock);
    if (!scratch_ptr[device]) {
        float* p = nullptr;
        if (hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        scratch_ptr[device] = p;
    }
    return scratch_ptr[device];
}

// ---- host side -----------------------------------------------------------------------------------------
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// a model can be used once it is on a device, and only while that device is the calling thread's current one: the
// kernels are launched on the current device and read the model's tables through device pointers
inline int model_ready(const ecco_model* m) {
    if (!m || !m->dev || m->device < 0) return ECCO_EINVAL;
    int cur = -1;
    return (hipGetDevice(&cur) == hipSuccess && cur == m->device) ? ECCO_OK : ECCO_EINVAL;
}

// A kernel that needs more than 64 KB of LDS has to be told so; the attribute belongs to the kernel (on the
// current device), not to a launch, so it is set the first time a kernel is launched on a device -- to the most
// any launch can ask for -- and remembered (a short list under a mutex: host threads may enter together).
int allow_lds_once(const void* kernel, int device, size_t bytes) {
    if (bytes <= 64 * 1024) return ECCO_OK;
    static std::mutex lock;
    static std::vector<std::pair<const void*, int>> done;
    std::lock_guard<std::mutex> hold(lock);
    for (const auto& d : done)
        if (d.first == kernel && d.second == device) return ECCO_OK;
    ECCO_HIP_CHECK(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    done.emplace_back(kernel, device);
    return ECCO_OK;
}
template <class K>
int allow_lds(K kernel, int device, size_t bytes) { return allow_lds_once(reinterpret_cast<const void*>(kernel), device, bytes); }

// compute units of a device, asked once per device (atomics: host threads may race to fill the cache, with the same value)
int cu_count(int device) {
    static std::atomic<int> cached[16];
    if (device < 0 || device >= 16) return 256;
    int n = cached[device].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n <= 0) n = 256;
        cached[device].store(n, std::memory_order_relaxed);
    }
    return n;
}

}  // namespace

namespace ecco {
// Called by ecco_model_to_device with `device` current: asks for the scratch array's address on that device, so that
// the entry point that allocates nothing finds it ready (also under stream capture).
int init_device_scratch(int device) { return scratch_on_current_device(device) ? ECCO_OK : ECCO_EHIP; }
}  // namespace ecco

extern "C" {

static int encode_common(bool minmax, const ecco_model* m, const uint16_t* src, size_t n_groups, void* blocks, uint32_t* meta, void* stream) {
    if (!m) return ECCO_EINVAL;
    if (n_groups == 0) return model_ready(m);  // nothing to do; pointers may be null
    if (!src || !blocks || !meta) return ECCO_EINVAL;
    if (!aligned(blocks, 64) || !aligned(src, 4) || !aligned(meta, 4)) return ECCO_EALIGN;
    if (model_ready(m) != ECCO_OK) return ECCO_EINVAL;
    const size_t wgs = (n_groups + kEncWaves - 1) / kEncWaves;
    const int grid = (int)std::min<size_t>(wgs, (size_t)cu_count(m->device) * 16);
    hipLaunchKernelGGL(minmax ? encode_kernel<true> : encode_kernel<false>, dim3(grid), dim3(kEncThreads), enc_lds_bytes(m->S), static_cast<hipStream_t>(stream), m->dev,
                       m->S, reinterpret_cast<const uint32_t*>(src), n_groups, static_cast<uint32_t*>(blocks), meta);
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

int ecco_encode(const ecco_model* m, const uint16_t* src, size_t n_groups, void* blocks, uint32_t* meta, void* stream) {
    return encode_common(false, m, src, n_groups, blocks, meta, stream);
}

int ecco_encode_minmax(const ecco_model* m, const uint16_t* src, size_t n_groups, void* blocks, uint32_t* meta, void* stream) {
    return encode_common(true, m, src, n_groups, blocks, meta, stream);
}

static int decode_common(const ecco_model* m, const void* blocks, const uint32_t* meta, size_t n_groups, void* dst,
                         void* stream, bool indices) {
    if (!m) return ECCO_EINVAL;
    if (n_groups == 0) return model_ready(m);  // nothing to do; pointers may be null
    if (!blocks || !meta || !dst) return ECCO_EINVAL;
    if (n_groups > (size_t)0x7FFFFFFF - kUnitBlocks) return ECCO_ESHAPE;
    if (!aligned(blocks, 64) || !aligned(dst, 16) || !aligned(meta, 4)) return ECCO_EALIGN;
    if (model_ready(m) != ECCO_OK) return ECCO_EINVAL;
    const int units = (int)((n_groups + kUnitBlocks - 1) / kUnitBlocks);
    const int cus = cu_count(m->device);
    const int units_per_wg = std::max(1, (units + cus - 1) / cus);  // small inputs: few units on many compute units (a wavefront's chain is the floor)
    const int grid = (units + units_per_wg - 1) / units_per_wg;
    const size_t lds = decode_lds_bytes(m->S);
    const bool lng = m->max_len > kPeekBits;
    const int dev_id = m->device;
    auto launch = [&](auto kernel) -> int {
        int rc = allow_lds(kernel, dev_id, lds);
        if (rc != ECCO_OK) return rc;
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(kDecWaves * 64), lds, static_cast<hipStream_t>(stream), m->dev, m->S,
                           static_cast<const uint4*>(blocks), meta, (int)n_groups, units_per_wg, dst);
        ECCO_HIP_CHECK(hipGetLastError());
        return ECCO_OK;
    };
    if (indices) return lng ? launch(decode_kernel<true, true>) : launch(decode_kernel<false, true>);
    return lng ? launch(decode_kernel<true, false>) : launch(decode_kernel<false, false>);
}

int ecco_decode(const ecco_model* m, const void* blocks, const uint32_t* meta, size_t n_groups, uint16_t* dst, void* stream) {
    return decode_common(m, blocks, meta, n_groups, dst, stream, false);
}

int ecco_decode_indices(const ecco_model* m, const void* blocks, const uint32_t* meta, size_t n_groups, uint8_t* idx, void* stream) {
    return decode_common(m, blocks, meta, n_groups, idx, stream, true);
}

int ecco_decode_gemv(const ecco_model* m, const void* blocks, const uint32_t* meta, int rows, int cols,
                     const uint16_t* x, int batch, float* y, void* stream) {
    if (!m || !blocks || !meta || !x || !y) return ECCO_EINVAL;
    if (rows <= 0 || cols <= 0 || cols % kGroup != 0 || cols > 65536 || batch < 1 || batch > 16) return ECCO_ESHAPE;
    if (!aligned(blocks, 64) || !aligned(x, 16) || !aligned(y, 4) || !aligned(meta, 4)) return ECCO_EALIGN;
    if (model_ready(m) != ECCO_OK) return ECCO_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int gpr = cols / kGroup;
    const int cus = cu_count(m->device);
    const bool lng = m->max_len > kPeekBits;
    if (batch == 1) {
        // one band of rows per workgroup, one workgroup per compute unit where the matrix allows it
        const int band = std::min(kMaxBandRows, std::max(1, (rows + cus - 1) / cus));
        const size_t lds = gemv_lds_bytes(m->S, gpr);
        int rc = lng ? allow_lds(gemv_kernel<true>, m->device, lds) : allow_lds(gemv_kernel<false>, m->device, lds);
        if (rc != ECCO_OK) return rc;
        const uint32_t* xb = reinterpret_cast<const uint32_t*>(x);
        const int grid = (rows + band - 1) / band;
        if (lng)
            hipLaunchKernelGGL(gemv_kernel<true>, dim3(grid), dim3(kGemvThreads), lds, st, m->dev, m->S,
                               static_cast<const uint4*>(blocks), meta, rows, gpr, band, xb, y);
        else
            hipLaunchKernelGGL(gemv_kernel<false>, dim3(grid), dim3(kGemvThreads), lds, st, m->dev, m->S,
                               static_cast<const uint4*>(blocks), meta, rows, gpr, band, xb, y);
    } else {
        // whole 16-row blocks per workgroup, one workgroup per compute unit where the matrix allows it
        const int total_rb = (rows + kMmaRows - 1) / kMmaRows;
        const int rb_per_wg = std::max(1, (total_rb + cus - 1) / cus);
        const int grid = (total_rb + rb_per_wg - 1) / rb_per_wg;
        const size_t glds = gemm_lds_bytes(m->S);
        int rc = lng ? allow_lds(gemm_kernel<true>, m->device, glds) : allow_lds(gemm_kernel<false>, m->device, glds);
        if (rc != ECCO_OK) return rc;
        if (lng)
            hipLaunchKernelGGL(gemm_kernel<true>, dim3(grid), dim3(kGemvThreads), glds, st, m->dev, m->S,
                               static_cast<const uint4*>(blocks), meta, rows, gpr, rb_per_wg, batch, x, y);
        else
            hipLaunchKernelGGL(gemm_kernel<false>, dim3(grid), dim3(kGemvThreads), glds, st, m->dev, m->S,
                               static_cast<const uint4*>(blocks), meta, rows, gpr, rb_per_wg, batch, x, y);
    }
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

static int kv_append_common(bool minmax, const ecco_model* mk, const ecco_model* mv, const uint16_t* k_new, const uint16_t* v_new,
                            void* k_blocks, uint32_t* k_meta, void* v_blocks, uint32_t* v_meta,
                            const int32_t* seq_len, int B, int H, int T_max, void* stream) {
    if (!mk || !mv || !k_new || !v_new || !k_blocks || !k_meta || !v_blocks || !v_meta || !seq_len) return ECCO_EINVAL;
    if (B <= 0 || H <= 0 || T_max <= 0 || (long long)B * H > 0x7FFFFFFF) return ECCO_ESHAPE;
    if (!aligned(k_blocks, 64) || !aligned(v_blocks, 64) || !aligned(k_new, 4) || !aligned(v_new, 4)) return ECCO_EALIGN;
    if (model_ready(mk) != ECCO_OK || model_ready(mv) != ECCO_OK || mk->device != mv->device) return ECCO_EINVAL;
    const dim3 grid(minmax ? (B * H + kEncWaves - 1) / kEncWaves : B * H, 2);
    hipLaunchKernelGGL(minmax ? kv_append_minmax_kernel : kv_append_kernel, grid, dim3(kEncThreads),
                       enc_lds_bytes(std::max(mk->S, mv->S)),
                       static_cast<hipStream_t>(stream), mk->dev, mk->S, mv->dev, mv->S,
                       reinterpret_cast<const uint32_t*>(k_new), reinterpret_cast<const uint32_t*>(v_new),
                       static_cast<uint32_t*>(k_blocks), k_meta, static_cast<uint32_t*>(v_blocks), v_meta, seq_len, B, H, T_max);
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

int ecco_kv_append(const ecco_model* mk, const ecco_model* mv, const uint16_t* k_new, const uint16_t* v_new,
                   void* k_blocks, uint32_t* k_meta, void* v_blocks, uint32_t* v_meta,
                   const int32_t* seq_len, int B, int H, int T_max, void* stream) {
    return kv_append_common(false, mk, mv, k_new, v_new, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, H, T_max, stream);
}

int ecco_kv_append_minmax(const ecco_model* mk, const ecco_model* mv, const uint16_t* k_new, const uint16_t* v_new,
                          void* k_blocks, uint32_t* k_meta, void* v_blocks, uint32_t* v_meta,
                          const int32_t* seq_len, int B, int H, int T_max, void* stream) {
    return kv_append_common(true, mk, mv, k_new, v_new, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, H, T_max, stream);
}

int ecco_kv_attend_gqa_splits(int device, int B, int Hkv, int tokens) {
    if (B <= 0 || Hkv <= 0 || tokens <= 0) return ECCO_ESHAPE;
    const long long heads = (long long)B * Hkv;
    const long long by_units = std::max<long long>(1, cu_count(device) / heads);  // a workgroup for every compute unit
    const long long by_tokens = ((long long)tokens + 255) / 256;                  // but at least 256 tokens per split
    return (int)std::min<long long>(std::min(by_units, by_tokens), 256);
}

size_t ecco_kv_attend_gqa_workspace(int B, int Hq, int n_splits) {
    if (B <= 0 || Hq <= 0 || n_splits <= 1) return 0;
    return (size_t)B * Hq * n_splits * (kGroup + 2) * sizeof(float);
}

// argument checks shared by the two grouped-query entry points (everything but the workspace)
static int gqa_check(const ecco_model* mk, const ecco_model* mv, const uint16_t* q,
                     const void* k_blocks, const uint32_t* k_meta, const void* v_blocks, const uint32_t* v_meta,
                     const int32_t* seq_len, int B, int Hq, int Hkv, int T_max, int n_splits, const float* out) {
    if (!mk || !mv || !q || !k_blocks || !k_meta || !v_blocks || !v_meta || !seq_len || !out) return ECCO_EINVAL;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || T_max <= 0 || Hq % Hkv != 0 || Hq / Hkv > kGqaMaxGroup) return ECCO_ESHAPE;
    if (n_splits < 1 || n_splits > 256 || (long long)B * Hkv > 0x7FFFFFFF || (long long)B * Hq > 0x7FFFFFFF) return ECCO_ESHAPE;
    return ECCO_OK;
}

// the two launches: the attention kernel over (sequence, key/value head, split), then the merge of the splits
static int gqa_launch(const ecco_model* mk, const ecco_model* mv, const uint16_t* q,
                      const void* k_blocks, const uint32_t* k_meta, const void* v_blocks, const uint32_t* v_meta,
                      const int32_t* seq_len, int B, int Hq, int Hkv, int T_max, int n_splits, float* workspace,
                      float* out, void* stream) {
    const size_t lds = gqa_lds_bytes(mk->S, mv->S, Hq / Hkv);
    const bool lk = mk->max_len > kPeekBits, lv = mv->max_len > kPeekBits;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int dev_id = mk->device;
    auto launch = [&](auto kernel) -> int {
        int rc = allow_lds(kernel, dev_id, lds);
        if (rc != ECCO_OK) return rc;
        hipLaunchKernelGGL(kernel, dim3(B * Hkv, n_splits), dim3(kGqaThreads), lds, st, mk->dev, mk->S, mv->dev, mv->S, q,
                           static_cast<const uint4*>(k_blocks), k_meta, static_cast<const uint4*>(v_blocks), v_meta, seq_len,
                           Hq, Hkv, T_max, out, workspace);
        ECCO_HIP_CHECK(hipGetLastError());
        return ECCO_OK;
    };
    const int rc = lk ? (lv ? launch(kv_attend_gqa_kernel<true, true>) : launch(kv_attend_gqa_kernel<true, false>))
                      : (lv ? launch(kv_attend_gqa_kernel<false, true>) : launch(kv_attend_gqa_kernel<false, false>));
    if (rc != ECCO_OK || n_splits == 1) return rc;
    hipLaunchKernelGGL(kv_attend_combine_kernel, dim3(B * Hq), dim3(kGroup), 0, st, workspace, B * Hq, n_splits, out);
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

int ecco_kv_attend_gqa(const ecco_model* mk, const ecco_model* mv, const uint16_t* q,
                       const void* k_blocks, const uint32_t* k_meta, const void* v_blocks, const uint32_t* v_meta,
                       const int32_t* seq_len, int B, int Hq, int Hkv, int T_max, int n_splits, void* workspace,
                       float* out, void* stream) {
    const int rc = gqa_check(mk, mv, q, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, Hq, Hkv, T_max, n_splits, out);
    if (rc != ECCO_OK) return rc;
    if (n_splits > 1 && !workspace) return ECCO_EINVAL;
    if (!aligned(k_blocks, 64) || !aligned(v_blocks, 64) || !aligned(q, 16) || !aligned(out, 4) || !aligned(workspace, 16)) return ECCO_EALIGN;
    if (model_ready(mk) != ECCO_OK || model_ready(mv) != ECCO_OK || mk->device != mv->device) return ECCO_EINVAL;
    return gqa_launch(mk, mv, q, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, Hq, Hkv, T_max, n_splits,
                      static_cast<float*>(workspace), out, stream);
}

int ecco_kv_attend_gqa_noalloc(const ecco_model* mk, const ecco_model* mv, const uint16_t* q,
                               const void* k_blocks, const uint32_t* k_meta, const void* v_blocks, const uint32_t* v_meta,
                               const int32_t* seq_len, int B, int Hq, int Hkv, int T_max, int n_splits,
                               float* out, void* stream) {
    const int rc = gqa_check(mk, mv, q, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, Hq, Hkv, T_max, n_splits, out);
    if (rc != ECCO_OK) return rc;
    // the partial results of the splits must fit the static array
    if (n_splits > 1 && ecco_kv_attend_gqa_workspace(B, Hq, n_splits) > (size_t)ECCO_GQA_SCRATCH_BYTES) return ECCO_ESHAPE;
    if (!aligned(k_blocks, 64) || !aligned(v_blocks, 64) || !aligned(q, 16) || !aligned(out, 4)) return ECCO_EALIGN;
    if (model_ready(mk) != ECCO_OK || model_ready(mv) != ECCO_OK || mk->device != mv->device) return ECCO_EINVAL;
    float* ws = nullptr;
    if (n_splits > 1) {
        // this device's copy of the array: asked for when the model was uploaded; looked up here otherwise, which
        // needs the model's device to be the current one
        {
            std::lock_guard<std::mutex> hold(scratch_lock);
            ws = mk->device < kMaxDevices ? scratch_ptr[mk->device] : nullptr;
        }
        if (!ws) {
            int cur = -1;
            if (hipGetDevice(&cur) != hipSuccess || cur != mk->device) return ECCO_EINVAL;
            ws = scratch_on_current_device(cur);
            if (!ws) return ECCO_EHIP;
        }
    }
    return gqa_launch(mk, mv, q, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, Hq, Hkv, T_max, n_splits, ws, out, stream);
}

int ecco_kv_attend(const ecco_model* mk, const ecco_model* mv, const uint16_t* q,
                   const void* k_blocks, const uint32_t* k_meta, const void* v_blocks, const uint32_t* v_meta,
                   const int32_t* seq_len, int B, int H, int T_max, float* out, void* stream) {
    if (!mk || !mv || !q || !k_blocks || !k_meta || !v_blocks || !v_meta || !seq_len || !out) return ECCO_EINVAL;
    if (B <= 0 || H <= 0 || T_max <= 0 || (long long)B * H > 0x7FFFFFFF) return ECCO_ESHAPE;
    if (!aligned(k_blocks, 64) || !aligned(v_blocks, 64) || !aligned(q, 16) || !aligned(out, 4)) return ECCO_EALIGN;
    if (model_ready(mk) != ECCO_OK || model_ready(mv) != ECCO_OK || mk->device != mv->device) return ECCO_EINVAL;
    const size_t lds = attn_lds_bytes(mk->S, mv->S);
    const bool lk = mk->max_len > kPeekBits, lv = mv->max_len > kPeekBits;
    const int dev_id = mk->device;
    auto launch = [&](auto kernel) -> int {
        int rc = allow_lds(kernel, dev_id, lds);
        if (rc != ECCO_OK) return rc;
        hipLaunchKernelGGL(kernel, dim3(B * H), dim3(lv ? 512 : kAttnThreads), lds, static_cast<hipStream_t>(stream), mk->dev, mk->S, mv->dev,
                           mv->S, q, static_cast<const uint4*>(k_blocks), k_meta, static_cast<const uint4*>(v_blocks), v_meta,
                           seq_len, H, T_max, out);
        ECCO_HIP_CHECK(hipGetLastError());
        return ECCO_OK;
    };
    if (lk) return lv ? launch(kv_attend_kernel<true, true>) : launch(kv_attend_kernel<true, false>);
    return lv ? launch(kv_attend_kernel<false, true>) : launch(kv_attend_kernel<false, false>);
}

}  // extern "C"
