// Measurement program (not part of libecco): what the LDS of a gfx950 compute unit charges for the access patterns a
// table-driven Huffman decoder can use, and how fast the decode loop's instruction mix can run.  Three parts:
//
//   1. LDS access patterns: cycles per wavefront instruction and compute unit for reads whose addresses the host
//      chooses (linear, random, one bank, few entries, few active lanes; 32-, 64- and 128-bit; ds_bpermute).
//   2. The decode chain as a closed loop: per value a few dependent VALU instructions, one dependent random LDS
//      read, and a varying number of independent VALU instructions; 8, 12 and 16 wavefronts, 1, 2 or 4 chains per lane.
//   3. One 32-bit table read per value (the shipped loop's mix, with the window refill) against one 64-bit read per
//      two values plus a second, dependent read on a fraction of the lanes (what a two-values-per-entry table needs
//      for pairs that do not fit the peek, and for raw-mode blocks).
//
// Cycles are at the nominal 2.4 GHz from HIP event time; one workgroup per compute unit, 256 workgroups.  Every
// address is inside the dynamic LDS allocation of its kernel (checked on the host before the launch).
// Build: python -m paper_2505_06901_amd.build   Run: ./paper_2505_06901_amd/probe_lds [1|2|3]
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <functional>
#include <random>
#include <string>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); std::exit(1); } } while (0)

namespace {

constexpr double kClockHz = 2.4e9;
constexpr int kGrid = 256;

__device__ inline uint32_t hash32(uint32_t h) { h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h *= 3266489917u; h ^= h >> 16; return h; }

double time_ms(const std::function<void()>& launch) {
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    launch();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    launch();
    CK(hipEventRecord(e1));
    CK(hipDeviceSynchronize());
    float ms = 0.0f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return ms;
}

// ---- part 1: access patterns ---------------------------------------------------------------------------------------
constexpr int kPatIter = 4096, kPatAddrs = 8, kPatLdsBytes = 131072;

// OP 0: ds_read_b32, 1: ds_read_b64, 2: ds_read_b128, 3: ds_bpermute_b32, 4: ds_read_u16
template <int OP>
__global__ __launch_bounds__(1024) void pattern_kernel(uint32_t* out, const uint32_t* addrs, const uint32_t* active) {
    extern __shared__ __align__(16) uint32_t lds[];
    for (int i = threadIdx.x; i < kPatLdsBytes / 4; i += blockDim.x) lds[i] = i * 2654435761u;
    __syncthreads();
    uint32_t a[kPatAddrs];
    for (int j = 0; j < kPatAddrs; ++j) a[j] = addrs[threadIdx.x * kPatAddrs + j];
    uint32_t acc = 0, src = threadIdx.x * 77u;
    if (active[threadIdx.x] != 0) {
        for (int i = 0; i < kPatIter; ++i) {
            uint32_t v[kPatAddrs];
            uint2 v2[kPatAddrs];
            uint4 v4[kPatAddrs];
#pragma unroll
            for (int j = 0; j < kPatAddrs; ++j) {
                if (OP == 0) asm volatile("ds_read_b32 %0, %1" : "=v"(v[j]) : "v"(a[j]));
                else if (OP == 1) asm volatile("ds_read_b64 %0, %1" : "=v"(v2[j]) : "v"(a[j]));
                else if (OP == 2) asm volatile("ds_read_b128 %0, %1" : "=v"(v4[j]) : "v"(a[j]));
                else if (OP == 3) asm volatile("ds_bpermute_b32 %0, %1, %2" : "=v"(v[j]) : "v"(a[j]), "v"(src));
                else asm volatile("ds_read_u16 %0, %1" : "=v"(v[j]) : "v"(a[j]));
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int j = 0; j < kPatAddrs; ++j) acc += OP == 1 ? (v2[j].x ^ v2[j].y) : OP == 2 ? (v4[j].x ^ v4[j].w) : v[j];
        }
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

double run_pattern(int op, const std::vector<uint32_t>& addrs, const std::vector<uint32_t>& active) {
    const int threads = 1024, width = op == 1 ? 8 : op == 2 ? 16 : op == 4 ? 2 : 4;
    for (uint32_t a : addrs)
        if (op != 3 && (a % width != 0 || a + width > (uint32_t)kPatLdsBytes)) { std::printf("address %u out of range\n", a); std::exit(1); }
    uint32_t *out, *da, *dact;
    CK(hipMalloc(&out, (size_t)kGrid * threads * 4));
    CK(hipMalloc(&da, addrs.size() * 4));
    CK(hipMalloc(&dact, active.size() * 4));
    CK(hipMemcpy(da, addrs.data(), addrs.size() * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(dact, active.data(), active.size() * 4, hipMemcpyHostToDevice));
    const void* kernels[5] = {(const void*)pattern_kernel<0>, (const void*)pattern_kernel<1>, (const void*)pattern_kernel<2>,
                              (const void*)pattern_kernel<3>, (const void*)pattern_kernel<4>};
    CK(hipFuncSetAttribute(kernels[op], hipFuncAttributeMaxDynamicSharedMemorySize, kPatLdsBytes));
    const double ms = time_ms([&] {
        switch (op) {
            case 0: hipLaunchKernelGGL(pattern_kernel<0>, dim3(kGrid), dim3(threads), kPatLdsBytes, 0, out, da, dact); break;
            case 1: hipLaunchKernelGGL(pattern_kernel<1>, dim3(kGrid), dim3(threads), kPatLdsBytes, 0, out, da, dact); break;
            case 2: hipLaunchKernelGGL(pattern_kernel<2>, dim3(kGrid), dim3(threads), kPatLdsBytes, 0, out, da, dact); break;
            case 3: hipLaunchKernelGGL(pattern_kernel<3>, dim3(kGrid), dim3(threads), kPatLdsBytes, 0, out, da, dact); break;
            default: hipLaunchKernelGGL(pattern_kernel<4>, dim3(kGrid), dim3(threads), kPatLdsBytes, 0, out, da, dact); break;
        }
    });
    CK(hipFree(out));
    CK(hipFree(da));
    CK(hipFree(dact));
    return ms * 1e-3 * kClockHz / ((double)kPatIter * kPatAddrs * (threads / 64.0));
}

void part1() {
    std::printf("\n== 1. LDS access patterns: cycles per wavefront instruction per compute unit (16 wavefronts, 8 reads in flight each)\n");
    std::mt19937 rng(12345);
    auto U = [&](uint32_t n) { return (uint32_t)(rng() % n); };
    struct Case { std::string name; int op; std::function<uint32_t(int, int)> addr; std::function<bool(int)> act; };
    auto all = [](int) { return true; };
    const std::vector<Case> cases = {
        {"32-bit, lane i reads word i (no conflict)", 0, [&](int t, int j) { return (uint32_t)((t & 63) * 4 + j * 256 + (t >> 6) * 2048); }, all},
        {"32-bit, random over 64 KB (a decode table of 64 patterns)", 0, [&](int, int) { return U(16384) * 4; }, all},
        {"32-bit, bank = lane % 32, random row (lanes i and i + 32 share a bank)", 0, [&](int t, int) { return (U(512) * 32 + (t & 31)) * 4; }, all},
        {"32-bit, 16 even banks only, random row (2 lanes of a half per bank)", 0, [&](int t, int) { return (U(512) * 32 + (t & 15) * 2) * 4; }, all},
        {"32-bit, stride of 32 words (every lane on one bank)", 0, [&](int t, int) { return (uint32_t)((t & 63) * 32) * 4; }, all},
        {"32-bit, stride of 16 words (two banks)", 0, [&](int t, int) { return (uint32_t)((t & 63) * 16) * 4; }, all},
        {"32-bit, random among 16 words (a 4-bit table of one pattern)", 0, [&](int, int) { return U(16) * 4; }, all},
        {"32-bit, random among 32 words", 0, [&](int, int) { return U(32) * 4; }, all},
        {"32-bit, random among 64 words", 0, [&](int, int) { return U(64) * 4; }, all},
        {"32-bit, random among 256 words (an 8-bit table of one pattern)", 0, [&](int, int) { return U(256) * 4; }, all},
        {"32-bit, random over 64 KB, 32 of 64 lanes active", 0, [&](int, int) { return U(16384) * 4; }, [](int t) { return (t & 1) == 0; }},
        {"32-bit, random over 64 KB, 16 of 64 lanes active", 0, [&](int, int) { return U(16384) * 4; }, [](int t) { return (t & 3) == 0; }},
        {"32-bit, random over 64 KB, 8 of 64 lanes active", 0, [&](int, int) { return U(16384) * 4; }, [](int t) { return (t & 7) == 0; }},
        {"32-bit, random over 64 KB, 1 of 64 lanes active", 0, [&](int, int) { return U(16384) * 4; }, [](int t) { return (t & 63) == 0; }},
        {"64-bit, lane i reads entry i (no conflict)", 1, [&](int t, int j) { return (uint32_t)((t & 63) * 8 + j * 512 + ((t >> 6) & 7) * 4096); }, all},
        {"64-bit, random over 128 KB", 1, [&](int, int) { return U(16384) * 8; }, all},
        {"64-bit, slot = lane % 32, random row", 1, [&](int t, int) { return (U(512) * 32 + (t & 31)) * 8; }, all},
        {"64-bit, random over 128 KB, 16 of 64 lanes active", 1, [&](int, int) { return U(16384) * 8; }, [](int t) { return (t & 3) == 0; }},
        {"128-bit, lane i reads entry i (no conflict)", 2, [&](int t, int j) { return (uint32_t)((t & 63) * 16 + j * 1024 + ((t >> 6) & 3) * 8192); }, all},
        {"128-bit, random over 128 KB", 2, [&](int, int) { return U(8192) * 16; }, all},
        {"16-bit, random over 64 KB", 4, [&](int, int) { return U(32768) * 2; }, all},
        {"ds_bpermute_b32, random source lane (a 64-entry table held in one register)", 3, [&](int, int) { return U(64) * 4; }, all},
        {"ds_bpermute_b32, own lane", 3, [&](int t, int) { return (uint32_t)(t & 63) * 4; }, all},
    };
    for (const Case& c : cases) {
        std::vector<uint32_t> addrs(1024 * kPatAddrs), active(1024);
        for (int t = 0; t < 1024; ++t) {
            for (int j = 0; j < kPatAddrs; ++j) addrs[t * kPatAddrs + j] = c.addr(t, j);
            active[t] = c.act(t) ? 1u : 0u;
        }
        std::printf("  %-78s %6.2f\n", c.name.c_str(), run_pattern(c.op, addrs, active));
        std::fflush(stdout);
    }
}

// ---- parts 2 and 3: the decode loop as a closed loop ---------------------------------------------------------------
constexpr int kValues = 4096;  // values per chain
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// F: independent VALU work per value on top of the dependent chain (0: none; 3: a multiply-add on the entry; 5, 7: more)
template <int F, int ILP>
__global__ __launch_bounds__(1024) void chain_kernel(uint32_t* out, int zero) {
    extern __shared__ __align__(16) uint32_t lds[];
    for (int i = threadIdx.x; i < 16384; i += blockDim.x) lds[i] = hash32(i + 1);
    __syncthreads();
    uint64_t win[ILP];
    float acc[ILP];
    uint32_t used[ILP];
    for (int c = 0; c < ILP; ++c) {
        win[c] = ((uint64_t)hash32(threadIdx.x * 747796405u + c * 2891336453u + 12345u) << 32) | hash32(threadIdx.x * 277803737u + c);
        acc[c] = 0.f;
        used[c] = 0;
    }
    for (int i = 0; i < kValues; ++i) {
        uint32_t e[ILP];
#pragma unroll
        for (int c = 0; c < ILP; ++c) e[c] = lds[((uint32_t)(win[c] >> 32) >> 18) + zero];
#pragma unroll
        for (int c = 0; c < ILP; ++c) {
            win[c] = (win[c] << (e[c] & 15u)) ^ (uint64_t)e[c];  // the xor keeps the window random: this loop has no payload to refill from
            if (F >= 1) acc[c] = __builtin_fmaf(__builtin_bit_cast(float, (e[c] & 0x007FFFFFu) | 0x3F800000u), 0.5f, acc[c]);
            if (F >= 4) used[c] += e[c];
            if (F >= 5) used[c] = (used[c] >> 3) ^ e[c];
            if (F >= 7) acc[c] = acc[c] * 1.0001f + 0.25f;
        }
    }
    uint32_t r = 0;
    for (int c = 0; c < ILP; ++c) r += (uint32_t)win[c] + (uint32_t)(win[c] >> 32) + __builtin_bit_cast(uint32_t, acc[c]) + used[c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

template <int F, int ILP>
void run_chain(int threads, int valu_per_value) {
    uint32_t* out;
    CK(hipMalloc(&out, (size_t)kGrid * 1024 * 4));
    const double ms = time_ms([&] { hipLaunchKernelGGL((chain_kernel<F, ILP>), dim3(kGrid), dim3(threads), 65536, 0, out, 0); });
    CK(hipFree(out));
    const double waves = threads / 64.0;
    std::printf("  %2.0f wavefronts, %d chain(s) per lane, %2d VALU per value: %6.2f cycles per wavefront and value\n", waves, ILP, valu_per_value,
                ms * 1e-3 * kClockHz / kValues / (waves * ILP));
    std::fflush(stdout);
}

void part2() {
    std::printf("\n== 2. The decode chain as a closed loop: one dependent random 32-bit read (64 KB table) per value\n"
                "   (the read alone costs 7.3 cycles per wavefront, part 1; VALU issue is 4 cycles per instruction and SIMD, i.e. one\n"
                "   cycle per instruction and value with 16 wavefronts: the loop runs at the larger of the two)\n");
    for (int threads : {512, 768, 1024}) {
        run_chain<0, 1>(threads, 6);
        run_chain<3, 1>(threads, 8);
        run_chain<5, 1>(threads, 10);
        run_chain<7, 1>(threads, 11);
        run_chain<3, 2>(threads, 8);
        run_chain<3, 4>(threads, 8);
    }
}

// MODE 0: one 32-bit read per value, window refilled every 4 values (one linear read).  MODE 1: one 64-bit read per two
// values, a second dependent 64-bit read for the lanes whose entry says so (byte 3 of its upper word below the
// threshold), window refilled every 8 values (three linear reads).
template <int MODE, int ILP>
__global__ __launch_bounds__(1024) void loop_kernel(uint32_t* out, int need2_thresh, int zero) {
    extern __shared__ __align__(16) uint32_t lds[];
    const int table_words = MODE ? 32768 : 16384;  // 128 KB of 8-byte entries / 64 KB of 4-byte entries
    for (int i = threadIdx.x; i < table_words; i += blockDim.x) {
        uint32_t h = hash32(i + 1);
        // the word that carries lengths (every word of the 4-byte table, the upper word of an 8-byte entry): bits 5:0 a
        // length 1..8, bits 15:8 a length 1..4; byte 3 stays random (it decides the second read)
        if (!MODE || (i & 1)) h = (h & 0xFF000000u) | ((1u + ((h >> 8) & 3u)) << 8) | (1u + (h & 7u)) | (MODE ? 0u : (h & 0xFFFF0000u));
        lds[i] = h;
    }
    uint32_t* wbuf = lds + table_words;  // stands for the staged payload: 17 words per lane
    for (int i = threadIdx.x; i < 64 * 17 + 8; i += blockDim.x) wbuf[i] = hash32(i * 7 + 3);
    __syncthreads();
    const int lane = threadIdx.x & 63;
    uint64_t win[ILP];
    float acc[ILP];
    uint32_t used[ILP], pos[ILP], xr[ILP][4];
    for (int c = 0; c < ILP; ++c) {
        win[c] = ((uint64_t)hash32(threadIdx.x * 747796405u + c * 2891336453u + 12345u) << 32) | hash32(threadIdx.x * 277803737u + c);
        acc[c] = 0.f;
        used[c] = 0;
        pos[c] = hash32(threadIdx.x + c) & 31u;
        for (int j = 0; j < 4; ++j) xr[c][j] = 0x3C003C00u + ((threadIdx.x + j) & 0xFF);
    }
    // table base and peek shift sit in vector registers the compiler cannot see through, as in the real kernels (they
    // depend on the block's pattern and mode); both hold their plain values at run time
    const uint32_t tbase = out[blockIdx.x * blockDim.x + threadIdx.x + zero];
    const char* ldsb = reinterpret_cast<const char*>(lds);
    const uint32_t sh = 18u + tbase;
    const uint32_t* wl = wbuf + lane * 17;
    if (MODE == 0) {
        for (int i = 0; i < kValues; i += 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t e[ILP];
#pragma unroll
                for (int c = 0; c < ILP; ++c) e[c] = *reinterpret_cast<const uint32_t*>(ldsb + ((((uint32_t)(win[c] >> 32) >> sh) << 2) + tbase));
#pragma unroll
                for (int c = 0; c < ILP; ++c) {
                    win[c] <<= (e[c] & 63u);
                    const half2_t ev = __builtin_bit_cast(half2_t, e[c]);
                    const half2_t xv = __builtin_bit_cast(half2_t, xr[c][j >> 1]);
                    acc[c] = __builtin_fmaf((float)ev[1], (float)((j & 1) ? xv[1] : xv[0]), acc[c]);
                    used[c] += e[c];
                }
            }
#pragma unroll
            for (int c = 0; c < ILP; ++c) {
                pos[c] = min(pos[c] + (used[c] & 7u) + 9u, 512u);
                const uint32_t w2 = wl[((pos[c] >> 5) & 15u) + c];
                const bool adv = (pos[c] & 32u) != 0;
                uint32_t hi = (uint32_t)(win[c] >> 32), lo = (uint32_t)win[c];
                hi = adv ? lo : (hi ^ w2);
                lo = adv ? w2 : (lo + w2);
                win[c] = (((uint64_t)hi << 32) | lo) << (pos[c] & 31u);
                pos[c] &= 255u;
                used[c] = 0;
            }
        }
    } else {
        for (int i = 0; i < kValues; i += 8) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint2 e[ILP];
#pragma unroll
                for (int c = 0; c < ILP; ++c) {
                    const uint64_t v = *reinterpret_cast<const uint64_t*>(ldsb + ((((uint32_t)(win[c] >> 32) >> sh) << 3) + tbase));
                    e[c] = make_uint2((uint32_t)v, (uint32_t)(v >> 32));
                }
#pragma unroll
                for (int c = 0; c < ILP; ++c) {
                    if ((int)(e[c].y >> 24) < need2_thresh) {
                        const uint64_t w2 = win[c] << (e[c].y & 63u);
                        const uint64_t v = *reinterpret_cast<const uint64_t*>(ldsb + ((((uint32_t)(w2 >> 32) >> sh) << 3) + tbase));
                        e[c].x = __builtin_amdgcn_perm((uint32_t)v, e[c].x, 0x05040100u);
                        e[c].y += ((uint32_t)(v >> 32) >> 8) & 0xFFu;
                    }
                    win[c] <<= (e[c].y & 63u);
                    acc[c] = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, e[c].x), __builtin_bit_cast(half2_t, xr[c][j]), acc[c], false);
                    used[c] += e[c].y;
                }
            }
#pragma unroll
            for (int c = 0; c < ILP; ++c) {
                pos[c] = min(pos[c] + (used[c] & 15u) + 17u, 512u);
                const uint32_t wi = (pos[c] >> 5) & 7u;
                const uint32_t w0 = wl[wi + c], w1 = wl[wi + c + 1], w2 = wl[wi + c + 2];
                const uint64_t a = (((uint64_t)w0 << 32) | w1) << (pos[c] & 31u);
                const uint64_t b = (((uint64_t)w1 << 32) | w2) << (pos[c] & 31u);
                win[c] = ((a & 0xFFFFFFFF00000000ull) | (b >> 32)) + (win[c] >> 40);
                pos[c] &= 255u;
                used[c] = 0;
            }
        }
    }
    uint32_t r = 0;
    for (int c = 0; c < ILP; ++c) r += (uint32_t)win[c] + (uint32_t)(win[c] >> 32) + __builtin_bit_cast(uint32_t, acc[c]) + used[c];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}

template <int MODE, int ILP>
void run_loop(int threads, int need2_pct) {
    uint32_t* out;
    const size_t out_bytes = (size_t)kGrid * 1024 * 4 + 64;
    CK(hipMalloc(&out, out_bytes));
    CK(hipMemset(out, 0, out_bytes));
    const int lds_bytes = (MODE ? 131072 : 65536) + (64 * 17 + 8) * 4;
    CK(hipFuncSetAttribute((const void*)loop_kernel<MODE, ILP>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
    const int thresh = need2_pct * 256 / 100;
    const double ms = time_ms([&] {
        CK(hipMemsetAsync(out, 0, out_bytes, 0));  // the kernel reads its table base (0) from here and overwrites it
        hipLaunchKernelGGL((loop_kernel<MODE, ILP>), dim3(kGrid), dim3(threads), lds_bytes, 0, out, thresh, 0);
    });
    CK(hipFree(out));
    const double waves = threads / 64.0;
    const double cyc = ms * 1e-3 * kClockHz / kValues / (waves * ILP);
    if (MODE == 0)
        std::printf("  %2.0f wavefronts, %d chain(s) per lane, one 32-bit read per value:                        %6.2f cycles per wavefront and value (%5.1f us for the 8192 x 28672 matrix)\n",
                    waves, ILP, cyc, cyc * 14336 / 2.4e3);
    else
        std::printf("  %2.0f wavefronts, %d chain(s) per lane, one 64-bit read per pair, second read on %3d %% of lanes: %6.2f cycles per wavefront and value (%5.1f us)\n",
                    waves, ILP, need2_pct, cyc, cyc * 14336 / 2.4e3);
    std::fflush(stdout);
}

void part3() {
    std::printf("\n== 3. One table read per value against one per two values (time includes a small memset per launch)\n");
    for (int threads : {1024, 768, 640}) {
        run_loop<0, 1>(threads, 0);
        run_loop<0, 2>(threads, 0);
        for (int pct : {0, 10, 28, 100}) run_loop<1, 1>(threads, pct);
        run_loop<1, 2>(threads, 28);
    }
}

}  // namespace

int main(int argc, char** argv) {
    const int only = argc > 1 ? std::atoi(argv[1]) : 0;
    int cus = 0;
    CK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
    std::printf("probe_lds: %d compute units; cycles at 2.4 GHz from event time, 256 workgroups (one per compute unit)\n", cus);
    if (only == 0 || only == 1) part1();
    if (only == 0 || only == 2) part2();
    if (only == 0 || only == 3) part3();
    return 0;
}
