// The 2x activation codec for gfx950: uniform 7-bit quantisation with a zero point, 64 FP16 values per
// 64-byte block (Section 3.2 "Activation Compression"; the low-ratio decompressor and compressor of
// Sections 4.2 and 4.3).  Format and rules are stated in include/ecco.h.
//
// Both kernels are plain streaming kernels: a lane owns one 8-byte piece of a block (8 values), eight
// lanes own one block, and the only cross-lane traffic is among those eight (DPP): the minimum / maximum
// of the group on the way in, the scale and the zero point -- gathered from the spare bits of pieces
// 0..3 -- on the way out.  Every load and store instruction covers consecutive addresses with
// consecutive lanes (8 bytes per lane on the compressed side, 16 on the FP16 side); 16-byte pieces with
// two half-dense FP16 stores per lane ran at 4.7 instead of 5.6 TB/s.
// The decoder follows the paper's two-operation scheme: the 7-bit code is placed in the mantissa of an
// FP16 number with a fixed exponent (a value of 1088 + q, exact), and one packed subtraction plus one
// packed fused multiply-add give fp16(q * s + z) with a single rounding.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "ecco.h"

namespace {

#define ECCO_HIP_CHECK(expr) do { if ((expr) != hipSuccess) return ECCO_EHIP; } while (0)

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int kActThreads = 256;
constexpr int kPiecesPerBlock = ECCO_BLOCK_BYTES / 8;  // 8 lanes per group

template <int kCtrl>
__device__ __forceinline__ uint32_t quad_dpp(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, kCtrl, 0xF, 0xF, true);
}
template <int kCtrl>
__device__ __forceinline__ float quad_dpp(float v) {
    return __builtin_bit_cast(float, quad_dpp<kCtrl>(__builtin_bit_cast(uint32_t, v)));
}

// bit 7 of each of the four bytes of d, gathered into bits 3:0 (byte k -> bit k)
__device__ __forceinline__ uint32_t spare_bits(uint32_t d) {
    return (((d >> 7) & 0x01010101u) * 0x01020408u) >> 24;
}
// bits 3:0 of n spread to bit 7 of bytes 0..3
__device__ __forceinline__ uint32_t spread_bits(uint32_t n) {
    return ((n * 0x00204081u) & 0x01010101u) << 7;
}

// two codes (bytes k0 and k0 + 1 of d, already xor-ed with 0x40) -> two FP16 values fp16(q * s + z)
template <uint32_t kSel>
__device__ __forceinline__ uint32_t dequant_pair(uint32_t d, half2_t s2, half2_t z2) {
    const uint32_t p = __builtin_amdgcn_perm(0u, d, kSel);                 // the two bytes in the low byte of each half
    const uint32_t h = (p & 0x007F007Fu) | 0x64006400u;                    // FP16 1024 + (q + 64) each
    const half2_t q2 = __builtin_bit_cast(half2_t, h) - (half2_t){(_Float16)1088.0f, (_Float16)1088.0f};  // exact
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(q2, s2, z2));
}

__global__ __launch_bounds__(kActThreads) void act_decode_kernel(const uint2* __restrict__ blocks, size_t n_pieces,
                                                                  uint4* __restrict__ dst) {
    const size_t stride = (size_t)gridDim.x * kActThreads;
    for (size_t i = (size_t)blockIdx.x * kActThreads + threadIdx.x; i < n_pieces; i += stride) {  // whole groups of 8 lanes pass or fail
        const uint2 w = blocks[i];
        const uint32_t j = (uint32_t)i & 7u;
        // pieces 0..3 hold the 32 metadata bits, a byte each: OR them over the first quad, then hand them to the second
        uint32_t side = j < 4u ? (spare_bits(w.x) | (spare_bits(w.y) << 4)) << (8u * j) : 0u;
        side |= quad_dpp<0xB1>(side);
        side |= quad_dpp<0x4E>(side);
        side |= quad_dpp<0x141>(side);  // mirror within 8 lanes
        const uint32_t sb = side & 0xFFFFu, zb = side >> 16;
        const half2_t s2 = __builtin_bit_cast(half2_t, sb | (sb << 16)), z2 = __builtin_bit_cast(half2_t, zb | (zb << 16));
        uint4 o;
        uint32_t d = w.x ^ 0x40404040u;
        o.x = dequant_pair<0x0C010C00u>(d, s2, z2);
        o.y = dequant_pair<0x0C030C02u>(d, s2, z2);
        d = w.y ^ 0x40404040u;
        o.z = dequant_pair<0x0C010C00u>(d, s2, z2);
        o.w = dequant_pair<0x0C030C02u>(d, s2, z2);
        dst[i] = o;
    }
}

__device__ __forceinline__ float half_lo(uint32_t v) { return (float)__builtin_bit_cast(half2_t, v).x; }
__device__ __forceinline__ float half_hi(uint32_t v) { return (float)__builtin_bit_cast(half2_t, v).y; }
__device__ __forceinline__ uint32_t to_half_bits(float f) {
    const _Float16 h = (_Float16)f;  // round to nearest even
    return (uint32_t)__builtin_bit_cast(unsigned short, h);
}

__global__ __launch_bounds__(kActThreads) void act_encode_kernel(const uint4* __restrict__ src, size_t n_pieces,
                                                                 uint2* __restrict__ blocks) {
    const size_t stride = (size_t)gridDim.x * kActThreads;
    for (size_t i = (size_t)blockIdx.x * kActThreads + threadIdx.x; i < n_pieces; i += stride) {  // whole groups of 8 lanes pass or fail
        const uint4 a = src[i];
        const uint32_t raw[4] = {a.x, a.y, a.z, a.w};
        float x[8];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            x[2 * k] = half_lo(raw[k]);
            x[2 * k + 1] = half_hi(raw[k]);
        }
        float lo = x[0], hi = x[0];
#pragma unroll
        for (int k = 1; k < 8; ++k) {
            lo = fminf(lo, x[k]);
            hi = fmaxf(hi, x[k]);
        }
        lo = fminf(lo, quad_dpp<0xB1>(lo));   // quad_perm [1,0,3,2]
        hi = fmaxf(hi, quad_dpp<0xB1>(hi));
        lo = fminf(lo, quad_dpp<0x4E>(lo));   // quad_perm [2,3,0,1]
        hi = fmaxf(hi, quad_dpp<0x4E>(hi));
        lo = fminf(lo, quad_dpp<0x141>(lo));  // mirror within 8 lanes
        hi = fmaxf(hi, quad_dpp<0x141>(hi));
        // s = fp16((max - min) / 127), z = fp16(min + 64 s): every step rounded to FP32 on its own
        const uint32_t sb = to_half_bits(__fdiv_rn(__fsub_rn(hi, lo), 127.0f));
        const float s = half_lo(sb);
        const uint32_t zb = to_half_bits(__fadd_rn(lo, __fmul_rn(64.0f, s)));
        const float z = half_lo(zb);
        const float inv = s == 0.0f ? 0.0f : __fdiv_rn(1.0f, s);
        float r[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            // nearest code, ties to even, clamped to -64..63; s = 0: (x - z) * 0 = 0
            r[k] = fminf(fmaxf(rintf(__fmul_rn(__fsub_rn(x[k], z), inv)), -64.0f), 63.0f);
        }
        if (fabsf(z) + 64.0f * s > 65000.0f) {
            // only next to the largest FP16 magnitudes can a code reconstruct to infinity: step towards 0
            const _Float16 sh = __builtin_bit_cast(_Float16, (unsigned short)sb), zh = __builtin_bit_cast(_Float16, (unsigned short)zb);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                for (int it = 0; it < 2; ++it) {
                    const _Float16 v = __builtin_fmaf16((_Float16)r[k], sh, zh);
                    const bool inf = ((uint32_t)__builtin_bit_cast(unsigned short, v) & 0x7FFFu) == 0x7C00u;
                    if (inf) r[k] += r[k] > 0.0f ? -1.0f : 1.0f;
                }
            }
        }
        // pieces 0..3 of the block carry a byte each of (scale | zero point << 16) in their spare bits
        const uint32_t j = (uint32_t)i & 7u;
        const uint32_t side = j < 4u ? ((sb | (zb << 16)) >> (8u * j)) & 0xFFu : 0u;
        uint32_t out[2];
#pragma unroll
        for (int dw = 0; dw < 2; ++dw) {
            uint32_t v = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) v = __builtin_amdgcn_cvt_pk_u8_f32(r[4 * dw + k] + 64.0f, k, v);  // code + 64 in 0..127
            out[dw] = (v ^ 0x40404040u) | spread_bits((side >> (4 * dw)) & 0xFu);  // back to two's complement, 7 bits
        }
        blocks[i] = make_uint2(out[0], out[1]);
    }
}

// A read-only streaming kernel: every lane reads 16-byte pieces on consecutive addresses and folds them into one word
// per workgroup.  It does nothing useful; timed over the same bytes as a decoder it gives the rate at which this
// machine can merely read them with one launch (the practical ceiling beside the 8 TB/s of the data sheet).
__global__ __launch_bounds__(1024) void read_stream_kernel(const uint4* __restrict__ src, size_t n16, uint32_t* __restrict__ out) {
    uint32_t acc = 0;
    const size_t step = (size_t)gridDim.x * 1024;
    size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
    for (; i + 3 * step < n16; i += 4 * step) {  // four loads in flight per lane
        const uint4 a = src[i], b = src[i + step], c = src[i + 2 * step], d = src[i + 3 * step];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    uint4 t[3] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};
#pragma unroll
    for (int k = 0; k < 3; ++k)
        if (i + k * step < n16) t[k] = src[i + k * step];
#pragma unroll
    for (int k = 0; k < 3; ++k) acc ^= t[k].x ^ t[k].y ^ t[k].z ^ t[k].w;
    for (int m = 1; m < 64; m <<= 1) acc ^= (uint32_t)__shfl_xor((int)acc, m);
    __shared__ uint32_t part[16];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t all = 0;
        for (int w = 0; w < 16; ++w) all ^= part[w];
        out[blockIdx.x] = all;  // one plain store per workgroup
    }
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline int act_grid(size_t n_pieces) {
    const size_t wgs = (n_pieces + kActThreads - 1) / kActThreads;
    return (int)std::min<size_t>(wgs, 256 * 32);  // grid-stride beyond 32 workgroups per CU
}

}  // namespace

extern "C" {

int ecco_act_encode(const uint16_t* src, size_t n_groups, void* blocks, void* stream) {
    if (n_groups == 0) return ECCO_OK;
    if (!src || !blocks) return ECCO_EINVAL;
    if (n_groups > ((size_t)1 << 40)) return ECCO_ESHAPE;
    if (!aligned(src, 16) || !aligned(blocks, 64)) return ECCO_EALIGN;
    const size_t n_pieces = n_groups * kPiecesPerBlock;
    hipLaunchKernelGGL(act_encode_kernel, dim3(act_grid(n_pieces)), dim3(kActThreads), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const uint4*>(src), n_pieces, static_cast<uint2*>(blocks));
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

int ecco_device_info(int device, int* compute_units, int* memory_clock_khz, int* memory_bus_bits) {
    if (!compute_units || !memory_clock_khz || !memory_bus_bits || device < 0) return ECCO_EINVAL;
    ECCO_HIP_CHECK(hipDeviceGetAttribute(compute_units, hipDeviceAttributeMultiprocessorCount, device));
    ECCO_HIP_CHECK(hipDeviceGetAttribute(memory_clock_khz, hipDeviceAttributeMemoryClockRate, device));
    ECCO_HIP_CHECK(hipDeviceGetAttribute(memory_bus_bits, hipDeviceAttributeMemoryBusWidth, device));
    return ECCO_OK;
}

int ecco_read_stream(const void* src, size_t bytes, uint32_t* out, void* stream) {
    if (!src || !out) return ECCO_EINVAL;
    if (bytes % 16 != 0) return ECCO_ESHAPE;
    if (!aligned(src, 16) || !aligned(out, 4)) return ECCO_EALIGN;
    if (bytes == 0) return ECCO_OK;
    hipLaunchKernelGGL(read_stream_kernel, dim3(256), dim3(1024), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), bytes / 16, out);
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

int ecco_act_decode(const void* blocks, size_t n_groups, uint16_t* dst, void* stream) {
    if (n_groups == 0) return ECCO_OK;
    if (!blocks || !dst) return ECCO_EINVAL;
    if (n_groups > ((size_t)1 << 40)) return ECCO_ESHAPE;
    if (!aligned(blocks, 64) || !aligned(dst, 16)) return ECCO_EALIGN;
    const size_t n_pieces = n_groups * kPiecesPerBlock;
    hipLaunchKernelGGL(act_decode_kernel, dim3(act_grid(n_pieces)), dim3(kActThreads), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint2*>(blocks), n_pieces, reinterpret_cast<uint4*>(dst));
    ECCO_HIP_CHECK(hipGetLastError());
    return ECCO_OK;
}

}  // extern "C"
