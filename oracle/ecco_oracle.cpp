// CPU oracle for the Ecco block codec -- TEST INFRASTRUCTURE ONLY (see ecco_oracle.h).
//
// Written from the paper, in the paper's order of steps:
//   fit      Section 3.2 "Model Compression", steps 1-4 (partition, normalise, per-group k-means,
//            shared-pattern k-means) and steps 6-7 (index statistics -> Huffman codebooks, H = 1)
//   encode   Section 3.2 step 5 (round to nearest centroid of every shared pattern, keep the
//            pattern of minimum squared error) and Section 4.3 (value mappers, Huffman encode,
//            concatenate, length check) with a raw 4-bit fallback instead of clipping; also with the
//            online compressor's min/max pattern selector (Section 3.2 "KV Cache Compression")
//   decode   Section 4.2 (pattern retrieval, Huffman decode, centroid x scale)
//   gemv / attention: the consumers of the decompressed values (Section 2.1), in double.
//   act      the 2x activation codec (Section 3.2 "Activation Compression", low-ratio units of Sections 4.2, 4.3)
//
// Parity status:
//   fp16 helpers, dequant rule ........ pinned (exhaustive, against integer arithmetic and numpy)
//   Huffman lengths / canonical codes .. pinned (Kraft, prefix-freeness, dyadic closed form, brute force)
//   encode / decode ................... pinned (brute force on tiny inputs, round trip, uniform 4-bit special case)
//   min/max pattern selector .......... pinned (hand-worked example, exact rational brute force, mirror symmetry,
//                                       single-pattern case equals the least-squared-error encoder)
//   2x activation codec ............... pinned (reconstruction rule against exact rationals for every code, hand-packed
//                                       block, power-of-two scale = plain round-to-nearest integers, constant and
//                                       extreme groups, error bound of a uniform quantiser)
//   k-means ........................... pinned (monotone objective, Lloyd-Max quantiser of a Gaussian)
//   gemv / attention .................. pinned (unit vectors, ones, seq_len 1, q = 0)
//   fitted pattern VALUES and code LENGTHS for a given tensor: parity unpinned -- the paper prints
//   no pattern values (its pattern figure is not available); only their invariants are checked.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fopenmp -shared -fPIC (see oracle/build.py).
// No intrinsics, no code shared with the HIP library.

#include "ecco_oracle.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

int g_threads = 1;

constexpr int G = ORACLE_GROUP;
constexpr int K = ORACLE_K;

// ------------------------------------------------------------------------------------------
// random numbers the fit draws: splitmix64 sequence (Steele, Lea, Flood 2014), restated here.
struct SplitMix {
    uint64_t s;
    explicit SplitMix(uint64_t seed) : s(seed) {}
    uint64_t next() {
        s += 0x9E3779B97F4A7C15ull;
        uint64_t z = s;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    double uniform() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }
};

// ------------------------------------------------------------------------------------------
// bit stream of one 64-byte block: 16 little-endian 32-bit words; stream bit j is bit 31 - (j & 31)
// of word j >> 5 (most significant bit of each word first).  Bits at positions >= 512 read as 0
// and are never written.
inline int get_bit(const uint8_t* blk, int j) {
    if (j >= 8 * ORACLE_BLOCK_BYTES) return 0;
    int in_word = 31 - (j & 31);                       // bit number inside the 32-bit word
    return (blk[(j >> 5) * 4 + (in_word >> 3)] >> (in_word & 7)) & 1;  // little-endian byte order
}
inline void put_bit(uint8_t* blk, int j, int b) {
    int in_word = 31 - (j & 31);
    if (b) blk[(j >> 5) * 4 + (in_word >> 3)] = (uint8_t)(blk[(j >> 5) * 4 + (in_word >> 3)] | (1u << (in_word & 7)));
}

struct Meta {
    uint16_t scale;
    int pattern;
    int raw;
    int mid;  // stream bit at which the code of value 64 begins
};
inline Meta unpack_meta(uint32_t m, int S) {
    Meta r;
    r.scale = (uint16_t)(m & 0xFFFFu);
    r.pattern = (int)((m >> 16) & 0x3Fu);
    if (r.pattern >= S) r.pattern = S - 1;  // corrupt meta: clamp, never index outside the model
    r.raw = (int)((m >> 22) & 1u);
    r.mid = (int)(m >> 23);
    return r;
}
inline uint32_t pack_meta(uint16_t scale, int pattern, int raw, int mid) {
    return (uint32_t)scale | ((uint32_t)pattern << 16) | ((uint32_t)raw << 22) | ((uint32_t)mid << 23);
}

}  // namespace

extern "C" {

int oracle_set_threads(int n) {
    if (n < 1) n = 1;
#ifdef _OPENMP
    int mx = omp_get_num_procs();
    if (n > mx) n = mx;
    g_threads = n;
#else
    g_threads = 1;
#endif
    return g_threads;
}

// ------------------------------------------------------------------------------------------
// fp16 <-> fp32 by bit manipulation (IEEE 754 binary16: 1 sign, 5 exponent, 10 fraction bits).
float oracle_h2f(uint16_t h) {
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1Fu;
    uint32_t m = h & 0x3FFu;
    uint32_t bits;
    if (e == 0) {
        if (m == 0) {
            bits = sign;
        } else {  // subnormal: m * 2^-24, renormalise
            int sh = 0;
            while (!(m & 0x400u)) { m <<= 1; ++sh; }
            m &= 0x3FFu;
            bits = sign | ((uint32_t)(113 - sh) << 23) | (m << 13);
        }
    } else if (e == 31) {
        bits = sign | 0x7F800000u | (m << 13);
    } else {
        bits = sign | ((e + 112u) << 23) | (m << 13);
    }
    float f;
    std::memcpy(&f, &bits, 4);
    return f;
}

uint16_t oracle_f2h(float f) {
    uint32_t bits;
    std::memcpy(&bits, &f, 4);
    uint16_t sign = (uint16_t)((bits >> 16) & 0x8000u);
    uint32_t x = bits & 0x7FFFFFFFu;
    if (x > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);   // NaN
    if (x >= 0x47800000u) return (uint16_t)(sign | 0x7C00u);  // >= 65536: infinity
    uint32_t e = x >> 23;
    uint32_t m = x & 0x7FFFFFu;
    uint32_t h;
    if (e < 113) {             // below the smallest normal half (2^-14): result in units of 2^-24
        if (e < 102) return sign;  // below 2^-25: rounds to zero
        m |= 0x800000u;
        uint32_t shift = 126 - e;  // 14..24
        h = m >> shift;
        uint32_t rem = m & ((1u << shift) - 1u);
        uint32_t half = 1u << (shift - 1);
        if (rem > half || (rem == half && (h & 1u))) ++h;
    } else {
        h = ((e - 112u) << 10) | (m >> 13);
        uint32_t rem = m & 0x1FFFu;
        if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;  // may carry into the exponent, up to infinity
    }
    return (uint16_t)(sign | h);
}

// Section 4.2: "the chosen k-means pattern is multiplied by the scale factor".  The product of two
// fp16 numbers is exact in fp32 (11-bit x 11-bit significands), so there is one rounding, to fp16.
uint16_t oracle_dequant(uint16_t c, uint16_t s) {
    float p = oracle_h2f(c) * oracle_h2f(s);
    return oracle_f2h(p);
}

// ------------------------------------------------------------------------------------------
// Huffman (1952): merge the two lightest subtrees until one is left; a leaf's code length is the
// number of merges its subtree took part in.
int oracle_huffman_lengths(const uint64_t* counts, int n, uint8_t* lens) {
    if (n < 1 || n > 64) return -1;
    if (n == 1) { lens[0] = 1; return 0; }
    struct Node { uint64_t w; std::vector<int> leaves; };
    std::vector<Node> nodes;
    for (int i = 0; i < n; ++i) nodes.push_back(Node{counts[i], {i}});
    std::vector<int> depth(n, 0);
    while (nodes.size() > 1) {
        // lightest two (first found on ties)
        size_t a = 0;
        for (size_t i = 1; i < nodes.size(); ++i) if (nodes[i].w < nodes[a].w) a = i;
        Node na = nodes[a];
        nodes.erase(nodes.begin() + (long)a);
        size_t b = 0;
        for (size_t i = 1; i < nodes.size(); ++i) if (nodes[i].w < nodes[b].w) b = i;
        Node nb = nodes[b];
        nodes.erase(nodes.begin() + (long)b);
        Node m{na.w + nb.w, na.leaves};
        m.leaves.insert(m.leaves.end(), nb.leaves.begin(), nb.leaves.end());
        for (int leaf : m.leaves) ++depth[leaf];
        nodes.push_back(m);
    }
    for (int i = 0; i < n; ++i) lens[i] = (uint8_t)depth[i];
    return 0;
}

// Length-limited optimal prefix code by package-merge (Larmore & Hirschberg 1990): max_len lists
// of "coins"; list for the deepest level holds the n leaves; each shallower list is the leaves
// merged with the pairs ("packages") of the list below; the 2n-2 cheapest entries of the top
// list are bought, and a symbol's length is the number of bought entries that contain it.
int oracle_limited_lengths(const uint64_t* counts, int n, int max_len, uint8_t* lens) {
    if (n < 1 || n > 64 || max_len < 1 || max_len > 32) return -1;
    if (n == 1) { lens[0] = 1; return 0; }
    if ((max_len < 6) && ((1 << max_len) < n)) return -2;  // no prefix code with such short lengths
    struct Coin { uint64_t w; std::vector<uint8_t> mult; };
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return counts[a] < counts[b]; });
    std::vector<Coin> leaves;
    for (int i : order) {
        Coin c{counts[i], std::vector<uint8_t>(n, 0)};
        c.mult[i] = 1;
        leaves.push_back(c);
    }
    std::vector<Coin> cur = leaves;
    for (int level = max_len - 1; level >= 1; --level) {
        std::vector<Coin> packages;
        for (size_t i = 0; i + 1 < cur.size(); i += 2) {
            Coin p{cur[i].w + cur[i + 1].w, cur[i].mult};
            for (int s = 0; s < n; ++s) p.mult[s] = (uint8_t)(p.mult[s] + cur[i + 1].mult[s]);
            packages.push_back(p);
        }
        std::vector<Coin> merged;
        size_t a = 0, b = 0;
        while (a < leaves.size() || b < packages.size()) {
            if (b >= packages.size() || (a < leaves.size() && leaves[a].w <= packages[b].w)) merged.push_back(leaves[a++]);
            else merged.push_back(packages[b++]);
        }
        cur.swap(merged);
    }
    std::vector<int> len(n, 0);
    for (int i = 0; i < 2 * n - 2; ++i)
        for (int s = 0; s < n; ++s) len[s] += cur[(size_t)i].mult[s];
    for (int s = 0; s < n; ++s) lens[s] = (uint8_t)len[s];
    return 0;
}

// Canonical assignment: symbols in order of (length, symbol); the first gets code 0 and each
// following one gets (previous + 1) shifted left by the growth in length.
void oracle_canonical_codes(const uint8_t* lens, int n, uint16_t* codes) {
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return lens[a] < lens[b]; });
    uint32_t code = 0;
    for (int j = 0; j < n; ++j) {
        if (j > 0) code = (code + 1u) << (lens[order[j]] - lens[order[j - 1]]);
        codes[order[j]] = (uint16_t)code;
    }
}

int oracle_verify_model(const uint16_t* centroids, const uint8_t* lens, int S) {
    if (S < 1 || S > ORACLE_MAX_S) return 1;
    for (int p = 0; p < S; ++p) {
        const uint16_t* c = centroids + p * K;
        const uint8_t* l = lens + p * K;
        for (int k = 0; k < K; ++k) {
            if (((c[k] >> 10) & 0x1F) == 31) return 2;                 // Inf / NaN
            if (std::fabs(oracle_h2f(c[k])) > 1.0f) return 3;          // outside [-1,1]
            if (k > 0 && oracle_h2f(c[k]) < oracle_h2f(c[k - 1])) return 4;  // not sorted
            if (l[k] < 1 || l[k] > ORACLE_MAX_LEN) return 5;
        }
        uint32_t kraft = 0;
        for (int k = 0; k < K; ++k) kraft += 1u << (ORACLE_MAX_LEN - l[k]);
        if (kraft != (1u << ORACLE_MAX_LEN)) return 6;
        uint16_t code[K];
        oracle_canonical_codes(l, K, code);
        for (int a = 0; a < K; ++a)
            for (int b = 0; b < K; ++b) {
                if (a == b || l[a] > l[b]) continue;
                if ((code[b] >> (l[b] - l[a])) == code[a]) return 7;  // a is a prefix of b
            }
    }
    return 0;
}

// ------------------------------------------------------------------------------------------
// Lloyd's algorithm in one dimension (Section 3.2 step 3).  Reading of what the paper leaves open:
// start at the (k + 0.5)/K quantiles of the sorted values, at most max_iter rounds, stop when no
// assignment changes, an empty cluster keeps its centroid, ties go to the lower centroid index.
int oracle_kmeans_1d(const float* v, int n, int Kc, int max_iter, double* cent, double* objective) {
    std::vector<double> x(v, v + n);
    std::sort(x.begin(), x.end());
    for (int k = 0; k < Kc; ++k) cent[k] = x[(size_t)(((2 * k + 1) * n) / (2 * Kc))];
    std::vector<int> assign(n, -1);
    int it = 0;
    for (;;) {
        bool changed = false;
        double obj = 0.0;
        for (int i = 0; i < n; ++i) {
            int best = 0;
            double bd = std::fabs(x[i] - cent[0]);
            for (int k = 1; k < Kc; ++k) {
                double d = std::fabs(x[i] - cent[k]);
                if (d < bd) { bd = d; best = k; }
            }
            if (best != assign[i]) { assign[i] = best; changed = true; }
            obj += bd * bd;
        }
        if (objective) objective[it] = obj;
        if (!changed || it >= max_iter) break;
        for (int k = 0; k < Kc; ++k) {
            double sum = 0.0;
            int cnt = 0;
            for (int i = 0; i < n; ++i) if (assign[i] == k) { sum += x[i]; ++cnt; }
            if (cnt > 0) cent[k] = sum / cnt;
        }
        ++it;
    }
    std::sort(cent, cent + Kc);
    return it;
}

// ------------------------------------------------------------------------------------------
// Encoder, one group.  Steps (Section 3.2 step 5, Section 4.3):
//  1. scale s = largest |x_i| (an fp16 value, found exactly)
//  2. every pattern's centroids times s, rounded to fp16 -- the values the decoder will produce
//  3. each x_i goes to the reconstructed value at minimum |difference| (lowest index on ties)
//  4. squared errors are summed per pattern in a fixed balanced tree (pairs i, i^1; then i^2; ...)
//     in fp32, so that any implementation following the same tree gets the same bits
//  5. the pattern with the smallest sum wins (lowest index on ties)
void oracle_quantize_group(const uint16_t* centroids, int S, const uint16_t* x,
                           uint16_t* scale, int* pattern, uint8_t* idx, float* sse_out) {
    uint16_t s_bits = 0;
    for (int i = 0; i < G; ++i) {
        uint16_t a = (uint16_t)(x[i] & 0x7FFFu);
        if (a > s_bits) s_bits = a;  // finite fp16 magnitudes order like their bit patterns
    }
    int best_p = 0;
    float best_sse = 0.0f;
    uint8_t best_idx[G];
    for (int p = 0; p < S; ++p) {
        float r[K];
        for (int k = 0; k < K; ++k) r[k] = oracle_h2f(oracle_dequant(centroids[p * K + k], s_bits));
        float e[G];
        uint8_t id[G];
        for (int i = 0; i < G; ++i) {
            float xi = oracle_h2f(x[i]);
            int bk = 0;
            float bd = std::fabs(xi - r[0]);
            for (int k = 1; k < K; ++k) {
                float d = std::fabs(xi - r[k]);
                if (d < bd) { bd = d; bk = k; }
            }
            float d = xi - r[bk];
            e[i] = d * d;
            id[i] = (uint8_t)bk;
        }
        for (int stride = 1; stride < G; stride <<= 1)       // level j adds partners differing in bit j
            for (int i = 0; i < G; i += 2 * stride) e[i] = e[i] + e[i + stride];
        float sse = e[0];
        if (sse_out) sse_out[p] = sse;
        if (p == 0 || sse < best_sse) {
            best_sse = sse;
            best_p = p;
            std::memcpy(best_idx, id, G);
        }
    }
    *scale = s_bits;
    *pattern = best_p;
    std::memcpy(idx, best_idx, G);
}

// ------------------------------------------------------------------------------------------
// Pattern selector of the online (KV cache) compressor: Section 3.2 "KV Cache Compression" and the
// pattern selector of Section 4.3.  Instead of quantising the group with every pattern, only the
// group's smallest and largest value are compared with each pattern's smallest and largest centroid:
//     fitness_p = (group min - pattern min)^2 + (group max - pattern max)^2,   least fitness wins.
// This build's reading: the pattern's ends are taken in the group's own scale, i.e. as the
// reconstructed values fp16(c[p][0] * s) and fp16(c[p][15] * s), so no division is needed; the
// group's extremes run over all 128 values (the paper leaves the absmax element out because its
// format stores that element apart from the pattern; here it is quantised by the pattern like any
// other value, so the pattern's ends cover it); differences, squares and the sum are fp32, each
// rounded on its own; the lowest pattern wins a tie.
void oracle_select_minmax(const uint16_t* centroids, int S, const uint16_t* x,
                          uint16_t* scale, int* pattern, float* fitness_out) {
    uint16_t s_bits = 0;
    float lo = oracle_h2f(x[0]), hi = lo;
    for (int i = 0; i < G; ++i) {
        uint16_t a = (uint16_t)(x[i] & 0x7FFFu);
        if (a > s_bits) s_bits = a;
        float v = oracle_h2f(x[i]);
        if (v < lo) lo = v;
        if (v > hi) hi = v;
    }
    int best_p = 0;
    float best_f = 0.0f;
    for (int p = 0; p < S; ++p) {
        float pmin = oracle_h2f(oracle_dequant(centroids[p * K], s_bits));
        float pmax = oracle_h2f(oracle_dequant(centroids[p * K + K - 1], s_bits));
        float dlo = lo - pmin, dhi = hi - pmax;
        float qlo = dlo * dlo, qhi = dhi * dhi;
        float f = qlo + qhi;
        if (fitness_out) fitness_out[p] = f;
        if (p == 0 || f < best_f) { best_f = f; best_p = p; }
    }
    *scale = s_bits;
    *pattern = best_p;
}

// Value mapping with one given pattern (Section 4.3, the parallel value mappers): every value goes
// to the nearest reconstructed value of that pattern, lowest index on ties.
void oracle_map_values(const uint16_t* centroids, int p, uint16_t s_bits, const uint16_t* x, uint8_t* idx) {
    float r[K];
    for (int k = 0; k < K; ++k) r[k] = oracle_h2f(oracle_dequant(centroids[p * K + k], s_bits));
    for (int i = 0; i < G; ++i) {
        float xi = oracle_h2f(x[i]);
        int bk = 0;
        float bd = std::fabs(xi - r[0]);
        for (int k = 1; k < K; ++k) {
            float d = std::fabs(xi - r[k]);
            if (d < bd) { bd = d; bk = k; }
        }
        idx[i] = (uint8_t)bk;
    }
}

// selector: 0 = least squared error over all patterns, 1 = min/max fitness
static void encode_one(const uint16_t* centroids, const uint8_t* lens, const uint16_t* codes, int S,
                       const uint16_t* x, uint8_t* blk, uint32_t* meta, int selector = 0) {
    uint16_t s;
    int p;
    uint8_t idx[G];
    if (selector == 0) {
        oracle_quantize_group(centroids, S, x, &s, &p, idx, nullptr);
    } else {
        oracle_select_minmax(centroids, S, x, &s, &p, nullptr);
        oracle_map_values(centroids, p, s, x, idx);
    }
    int total = 0;
    for (int i = 0; i < G; ++i) total += lens[p * K + idx[i]];
    std::memset(blk, 0, ORACLE_BLOCK_BYTES);
    if (total <= 8 * ORACLE_BLOCK_BYTES) {
        int pos = 0, mid = 0;
        for (int i = 0; i < G; ++i) {
            if (i == G / 2) mid = pos;  // where the second half of the values starts
            int l = lens[p * K + idx[i]];
            uint16_t c = codes[p * K + idx[i]];
            for (int b = l - 1; b >= 0; --b) put_bit(blk, pos++, (c >> b) & 1);  // first bit = top bit of the code
        }
        *meta = pack_meta(s, p, 0, mid);
    } else {  // does not fit: plain 4-bit indices, value i in stream bits 4i..4i+3, top bit first
        for (int i = 0; i < G; ++i)
            for (int b = 0; b < 4; ++b) put_bit(blk, 4 * i + b, (idx[i] >> (3 - b)) & 1);
        *meta = pack_meta(s, p, 1, 4 * (G / 2));
    }
}

void oracle_encode(const uint16_t* centroids, const uint8_t* lens, int S,
                   const uint16_t* src, size_t n_groups, uint8_t* blocks, uint32_t* meta) {
    std::vector<uint16_t> codes((size_t)S * K);
    for (int p = 0; p < S; ++p) oracle_canonical_codes(lens + p * K, K, codes.data() + p * K);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (long g = 0; g < (long)n_groups; ++g)
        encode_one(centroids, lens, codes.data(), S, src + (size_t)g * G,
                   blocks + (size_t)g * ORACLE_BLOCK_BYTES, meta + g);
}

void oracle_encode_minmax(const uint16_t* centroids, const uint8_t* lens, int S,
                          const uint16_t* src, size_t n_groups, uint8_t* blocks, uint32_t* meta) {
    std::vector<uint16_t> codes((size_t)S * K);
    for (int p = 0; p < S; ++p) oracle_canonical_codes(lens + p * K, K, codes.data() + p * K);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (long g = 0; g < (long)n_groups; ++g)
        encode_one(centroids, lens, codes.data(), S, src + (size_t)g * G,
                   blocks + (size_t)g * ORACLE_BLOCK_BYTES, meta + g, 1);
}

// ------------------------------------------------------------------------------------------
// Decoder, one block: walk the stream one bit at a time; a symbol is recognised as soon as the
// bits read so far equal one of the 16 codes of the group's pattern.  Values 0..63 are read from
// stream bit 0 on; values 64..127 from the position the meta word gives (for a block written by
// the encoder that is exactly where value 63 ended).
static int decode_one(const uint8_t* lens, const uint16_t* codes, int S, const uint8_t* blk, uint32_t m,
                      uint8_t* idx) {
    Meta mt = unpack_meta(m, S);
    if (mt.raw) {
        for (int i = 0; i < G; ++i) {
            int v = 0;
            for (int b = 0; b < 4; ++b) v |= get_bit(blk, 4 * i + b) << (3 - b);
            idx[i] = (uint8_t)v;
        }
        return 4 * G;
    }
    const uint8_t* l = lens + mt.pattern * K;
    const uint16_t* c = codes + mt.pattern * K;
    int pos = 0;
    for (int i = 0; i < G; ++i) {
        if (i == G / 2) pos = mt.mid;
        uint32_t code = 0;
        int len = 0, sym = -1;
        while (sym < 0 && len < ORACLE_MAX_LEN) {
            code = (code << 1) | (uint32_t)get_bit(blk, pos++);
            ++len;
            for (int k = 0; k < K; ++k)
                if (l[k] == len && c[k] == code) sym = k;
        }
        idx[i] = (uint8_t)(sym < 0 ? 0 : sym);  // unreachable for a complete (Kraft = 1) code
    }
    return pos;
}

void oracle_decode_indices(const uint8_t* lens, int S, const uint8_t* blocks, const uint32_t* meta,
                           size_t n_groups, uint8_t* idx, uint16_t* used_bits) {
    std::vector<uint16_t> codes((size_t)S * K);
    for (int p = 0; p < S; ++p) oracle_canonical_codes(lens + p * K, K, codes.data() + p * K);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (long g = 0; g < (long)n_groups; ++g) {
        int used = decode_one(lens, codes.data(), S, blocks + (size_t)g * ORACLE_BLOCK_BYTES, meta[g], idx + (size_t)g * G);
        if (used_bits) used_bits[g] = (uint16_t)used;
    }
}

void oracle_decode(const uint16_t* centroids, const uint8_t* lens, int S, const uint8_t* blocks,
                   const uint32_t* meta, size_t n_groups, uint16_t* dst) {
    std::vector<uint16_t> codes((size_t)S * K);
    for (int p = 0; p < S; ++p) oracle_canonical_codes(lens + p * K, K, codes.data() + p * K);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (long g = 0; g < (long)n_groups; ++g) {
        uint8_t idx[G];
        decode_one(lens, codes.data(), S, blocks + (size_t)g * ORACLE_BLOCK_BYTES, meta[g], idx);
        Meta mt = unpack_meta(meta[g], S);
        for (int i = 0; i < G; ++i)
            dst[(size_t)g * G + i] = oracle_dequant(centroids[mt.pattern * K + idx[i]], mt.scale);
    }
}

// ------------------------------------------------------------------------------------------
// 2x activation codec: uniform integer quantisation with a zero point, 7 bits per value, the scale
// and the zero point spread over the spare bit of every byte (Section 3.2 "Activation Compression";
// decompressor and compressor of Sections 4.2 and 4.3).  The paper fixes the widths (7-bit data,
// 16-bit scale, 16-bit zero point, 512-bit block) and that the codes are sign-extended; this
// build's reading of the rest:
//   s = fp16( (max - min) / 127 )            difference and quotient in fp32
//   z = fp16( min + 64 * s )                 the value of code 0; fp32 sum
//   q = round-to-nearest-even( (x - z) * (1 / s) ), clamped to -64..63       fp32, each step rounded;
//       s = 0 (constant group): q = 0;  a code whose reconstruction would not be finite moves
//       towards 0 (at most twice) -- only possible next to the largest FP16 magnitudes
//   x' = fp16( q * s + z )                   exact value, one rounding
// Every finite FP16 value is an integer multiple of 2^-24, so the last rule is done in integers.
static int64_t half_scaled(uint16_t h) {  // value * 2^24 of a finite fp16
    int e = (h >> 10) & 0x1F, m = h & 0x3FF;
    int64_t a = e == 0 ? m : ((int64_t)(m | 0x400) << (e - 1));
    return (h & 0x8000) ? -a : a;
}

static uint16_t half_from_scaled(int64_t n) {  // fp16 nearest (ties to even) to n * 2^-24, n != 0
    uint16_t sign = n < 0 ? 0x8000 : 0;
    uint64_t a = (uint64_t)(n < 0 ? -n : n);
    if (a < 2048) return (uint16_t)(sign | a);  // subnormals and the first binade: bit pattern = a
    int t = 63;
    while (!((a >> t) & 1)) --t;
    int shift = t - 10;
    uint64_t mant = a >> shift, rem = a & ((1ull << shift) - 1), half = 1ull << (shift - 1);
    if (rem > half || (rem == half && (mant & 1))) ++mant;
    if (mant == 2048) { mant = 1024; ++shift; }
    int e = shift + 1;
    if (e >= 31) return (uint16_t)(sign | 0x7C00);
    return (uint16_t)(sign | (e << 10) | (mant - 1024));
}

uint16_t oracle_act_dequant(int q, uint16_t s_bits, uint16_t z_bits) {
    int64_t n = (int64_t)q * half_scaled(s_bits) + half_scaled(z_bits);
    if (n != 0) return half_from_scaled(n);
    // an exact zero: -0 only if both addends are -0 (IEEE 754 sum rule); the product of code 0 is +0 * s
    bool prod_is_zero = q == 0 || (s_bits & 0x7FFF) == 0;
    bool prod_neg = (q < 0) != ((s_bits & 0x8000) != 0);
    bool z_neg_zero = z_bits == 0x8000;
    return (prod_is_zero && prod_neg && z_neg_zero) ? 0x8000 : 0x0000;
}

void oracle_act_params(const uint16_t* x, uint16_t* s_bits, uint16_t* z_bits) {
    float lo = oracle_h2f(x[0]), hi = lo;
    for (int i = 1; i < ORACLE_ACT_GROUP; ++i) {
        float v = oracle_h2f(x[i]);
        if (v < lo) lo = v;
        if (v > hi) hi = v;
    }
    float range = hi - lo;
    float step = range / 127.0f;
    *s_bits = oracle_f2h(step);
    float s = oracle_h2f(*s_bits);
    float scaled = 64.0f * s;
    float zero = lo + scaled;
    *z_bits = oracle_f2h(zero);
}

static bool half_is_finite(uint16_t h) { return (h & 0x7C00) != 0x7C00; }

void oracle_act_encode(const uint16_t* src, size_t n_groups, uint8_t* blocks) {
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (long g = 0; g < (long)n_groups; ++g) {
        const uint16_t* x = src + (size_t)g * ORACLE_ACT_GROUP;
        uint8_t* blk = blocks + (size_t)g * ORACLE_BLOCK_BYTES;
        uint16_t s_bits, z_bits;
        oracle_act_params(x, &s_bits, &z_bits);
        float s = oracle_h2f(s_bits), z = oracle_h2f(z_bits);
        float inv = s == 0.0f ? 0.0f : 1.0f / s;
        uint32_t side = (uint32_t)s_bits | ((uint32_t)z_bits << 16);
        for (int i = 0; i < ORACLE_ACT_GROUP; ++i) {
            int q = 0;
            if (s != 0.0f) {
                float d = oracle_h2f(x[i]) - z;
                float u = d * inv;
                float r = std::nearbyint(u);  // default rounding mode: to nearest, ties to even
                if (r < -64.0f) r = -64.0f;
                if (r > 63.0f) r = 63.0f;
                q = (int)r;
                for (int it = 0; it < 2; ++it)
                    if (!half_is_finite(oracle_act_dequant(q, s_bits, z_bits))) q += q > 0 ? -1 : 1;
            }
            int side_bit = i < 32 ? (int)((side >> i) & 1u) : 0;
            blk[i] = (uint8_t)((q & 0x7F) | (side_bit << 7));
        }
    }
}

void oracle_act_decode(const uint8_t* blocks, size_t n_groups, uint16_t* dst) {
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (long g = 0; g < (long)n_groups; ++g) {
        const uint8_t* blk = blocks + (size_t)g * ORACLE_BLOCK_BYTES;
        uint32_t side = 0;
        for (int i = 0; i < 32; ++i) side |= (uint32_t)(blk[i] >> 7) << i;
        uint16_t s_bits = (uint16_t)(side & 0xFFFFu), z_bits = (uint16_t)(side >> 16);
        for (int i = 0; i < ORACLE_ACT_GROUP; ++i) {
            int q = blk[i] & 0x7F;
            if (q & 0x40) q -= 128;  // sign extension of the 7-bit code
            // a block the encoder never writes (scale or zero point not finite) has no defined values: NaN here
            dst[(size_t)g * ORACLE_ACT_GROUP + i] =
                (half_is_finite(s_bits) && half_is_finite(z_bits)) ? oracle_act_dequant(q, s_bits, z_bits) : (uint16_t)0x7E00;
        }
    }
}

// ------------------------------------------------------------------------------------------
void oracle_gemv(const uint16_t* centroids, const uint8_t* lens, int S, const uint8_t* blocks,
                 const uint32_t* meta, int rows, int cols, const uint16_t* x, int batch, double* y) {
    const int gpr = cols / G;  // groups per row
    std::vector<double> xd((size_t)batch * cols);
    for (size_t i = 0; i < xd.size(); ++i) xd[i] = (double)oracle_h2f(x[i]);
    std::vector<uint16_t> codes((size_t)S * K);
    for (int p = 0; p < S; ++p) oracle_canonical_codes(lens + p * K, K, codes.data() + p * K);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int r = 0; r < rows; ++r) {
        std::vector<double> w((size_t)cols);
        for (int gc = 0; gc < gpr; ++gc) {
            size_t g = (size_t)r * gpr + gc;
            uint8_t idx[G];
            decode_one(lens, codes.data(), S, blocks + g * ORACLE_BLOCK_BYTES, meta[g], idx);
            Meta mt = unpack_meta(meta[g], S);
            for (int i = 0; i < G; ++i)
                w[(size_t)gc * G + i] = (double)oracle_h2f(oracle_dequant(centroids[mt.pattern * K + idx[i]], mt.scale));
        }
        for (int b = 0; b < batch; ++b) {
            double acc = 0.0;
            for (int c = 0; c < cols; ++c) acc += w[c] * xd[(size_t)b * cols + c];
            y[(size_t)b * rows + r] = acc;
        }
    }
}

// ------------------------------------------------------------------------------------------
static void kv_append_with(int selector, const uint16_t* ck, const uint8_t* lk, int Sk, const uint16_t* cv, const uint8_t* lv, int Sv,
                           const uint16_t* k_new, const uint16_t* v_new,
                           uint8_t* k_blocks, uint32_t* k_meta, uint8_t* v_blocks, uint32_t* v_meta,
                           const int32_t* seq_len, int B, int H, int T_max) {
    std::vector<uint16_t> codes_k((size_t)Sk * K), codes_v((size_t)Sv * K);
    for (int p = 0; p < Sk; ++p) oracle_canonical_codes(lk + p * K, K, codes_k.data() + p * K);
    for (int p = 0; p < Sv; ++p) oracle_canonical_codes(lv + p * K, K, codes_v.data() + p * K);
    for (int b = 0; b < B; ++b) {
        int t = seq_len[b];
        if (t < 0 || t >= T_max) continue;  // full or invalid sequence: nothing is written
        for (int h = 0; h < H; ++h) {
            size_t src = ((size_t)b * H + h) * G;
            size_t dst = ((size_t)b * H + h) * T_max + t;
            encode_one(ck, lk, codes_k.data(), Sk, k_new + src, k_blocks + dst * ORACLE_BLOCK_BYTES, k_meta + dst, selector);
            encode_one(cv, lv, codes_v.data(), Sv, v_new + src, v_blocks + dst * ORACLE_BLOCK_BYTES, v_meta + dst, selector);
        }
    }
}

void oracle_kv_append(const uint16_t* ck, const uint8_t* lk, int Sk, const uint16_t* cv, const uint8_t* lv, int Sv,
                      const uint16_t* k_new, const uint16_t* v_new,
                      uint8_t* k_blocks, uint32_t* k_meta, uint8_t* v_blocks, uint32_t* v_meta,
                      const int32_t* seq_len, int B, int H, int T_max) {
    kv_append_with(0, ck, lk, Sk, cv, lv, Sv, k_new, v_new, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, H, T_max);
}

void oracle_kv_append_minmax(const uint16_t* ck, const uint8_t* lk, int Sk, const uint16_t* cv, const uint8_t* lv, int Sv,
                             const uint16_t* k_new, const uint16_t* v_new,
                             uint8_t* k_blocks, uint32_t* k_meta, uint8_t* v_blocks, uint32_t* v_meta,
                             const int32_t* seq_len, int B, int H, int T_max) {
    kv_append_with(1, ck, lk, Sk, cv, lv, Sv, k_new, v_new, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, H, T_max);
}

// Scaled dot-product attention for one query token per sequence (Section 2.1): scores
// q.K_t / sqrt(d) over the first seq_len tokens, softmax, weighted sum of V_t.  Double throughout.
//
// With grouped queries (Section 5.3 "Performance Evaluation": models with grouped-query attention) Hq query heads share Hkv
// key/value heads: query head h reads the cache of head h / (Hq / Hkv).  Hq = Hkv is the plain case.
static void attend_heads(const uint16_t* ck, const uint8_t* lk, int Sk, const uint16_t* cv, const uint8_t* lv, int Sv,
                         const uint16_t* q, const uint8_t* k_blocks, const uint32_t* k_meta,
                         const uint8_t* v_blocks, const uint32_t* v_meta,
                         const int32_t* seq_len, int B, int H, int Hkv, int T_max, double* out) {
    const int per_kv = H / Hkv;  // query heads per key/value head
    std::vector<uint16_t> codes_k((size_t)Sk * K), codes_v((size_t)Sv * K);
    for (int p = 0; p < Sk; ++p) oracle_canonical_codes(lk + p * K, K, codes_k.data() + p * K);
    for (int p = 0; p < Sv; ++p) oracle_canonical_codes(lv + p * K, K, codes_v.data() + p * K);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int bh = 0; bh < B * H; ++bh) {
        int b = bh / H;
        int T = seq_len[b];
        if (T > T_max) T = T_max;
        double* o = out + (size_t)bh * G;
        for (int d = 0; d < G; ++d) o[d] = 0.0;
        if (T <= 0) continue;
        std::vector<double> score((size_t)T);
        double qd[G];
        for (int d = 0; d < G; ++d) qd[d] = (double)oracle_h2f(q[(size_t)bh * G + d]);
        for (int t = 0; t < T; ++t) {
            size_t g = ((size_t)b * Hkv + (bh % H) / per_kv) * T_max + t;
            uint8_t idx[G];
            decode_one(lk, codes_k.data(), Sk, k_blocks + g * ORACLE_BLOCK_BYTES, k_meta[g], idx);
            Meta mt = unpack_meta(k_meta[g], Sk);
            double acc = 0.0;
            for (int d = 0; d < G; ++d)
                acc += qd[d] * (double)oracle_h2f(oracle_dequant(ck[mt.pattern * K + idx[d]], mt.scale));
            score[(size_t)t] = acc / std::sqrt((double)G);
        }
        double mx = score[0];
        for (int t = 1; t < T; ++t) mx = std::max(mx, score[(size_t)t]);
        double denom = 0.0;
        for (int t = 0; t < T; ++t) { score[(size_t)t] = std::exp(score[(size_t)t] - mx); denom += score[(size_t)t]; }
        for (int t = 0; t < T; ++t) {
            size_t g = ((size_t)b * Hkv + (bh % H) / per_kv) * T_max + t;
            uint8_t idx[G];
            decode_one(lv, codes_v.data(), Sv, v_blocks + g * ORACLE_BLOCK_BYTES, v_meta[g], idx);
            Meta mt = unpack_meta(v_meta[g], Sv);
            double pt = score[(size_t)t] / denom;
            for (int d = 0; d < G; ++d)
                o[d] += pt * (double)oracle_h2f(oracle_dequant(cv[mt.pattern * K + idx[d]], mt.scale));
        }
    }
}

void oracle_kv_attend(const uint16_t* ck, const uint8_t* lk, int Sk, const uint16_t* cv, const uint8_t* lv, int Sv,
                      const uint16_t* q, const uint8_t* k_blocks, const uint32_t* k_meta,
                      const uint8_t* v_blocks, const uint32_t* v_meta,
                      const int32_t* seq_len, int B, int H, int T_max, double* out) {
    attend_heads(ck, lk, Sk, cv, lv, Sv, q, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, H, H, T_max, out);
}

void oracle_kv_attend_gqa(const uint16_t* ck, const uint8_t* lk, int Sk, const uint16_t* cv, const uint8_t* lv, int Sv,
                          const uint16_t* q, const uint8_t* k_blocks, const uint32_t* k_meta,
                          const uint8_t* v_blocks, const uint32_t* v_meta,
                          const int32_t* seq_len, int B, int Hq, int Hkv, int T_max, double* out) {
    attend_heads(ck, lk, Sk, cv, lv, Sv, q, k_blocks, k_meta, v_blocks, v_meta, seq_len, B, Hq, Hkv, T_max, out);
}

// ------------------------------------------------------------------------------------------
// The fit (Section 3.2).  Where the paper leaves a step open, the comment at that step says which reading is taken.
// oracle_fit_trace is the fit itself; beside the model it hands out what the steps produced on the way, so that
// tests can check each step on its own: the groups picked in step 1, the per-group patterns of step 3, and the
// objective of step 4 (sum over the groups of the squared distance to the nearest shared pattern) at every
// assignment pass.  Any of the trace pointers may be NULL.
int oracle_fit_trace(const uint16_t* data, size_t n_values, int S, int max_len, uint64_t seed,
                     uint16_t* centroids, uint8_t* lens, uint64_t* hist_out, size_t* n_fit_groups,
                     uint64_t* pick_out, double* group_patterns_out, double* objective_out, int* n_objective) {
    if (n_objective) *n_objective = 0;
    if (!data || n_values == 0 || n_values % G != 0 || S < 1 || S > ORACLE_MAX_S || max_len < 4 || max_len > ORACLE_MAX_LEN)
        return -1;
    const size_t n_all = n_values / G;
    SplitMix rng(seed);

    // step 1: groups of 128 consecutive values; a seeded subset of 65 536 groups if there are more
    std::vector<size_t> pick;
    const size_t cap = 65536;
    if (n_all > cap) {
        std::vector<uint32_t> perm(n_all);
        for (size_t i = 0; i < n_all; ++i) perm[i] = (uint32_t)i;
        for (size_t i = 0; i < cap; ++i) {
            size_t j = i + (size_t)(rng.next() % (uint64_t)(n_all - i));
            std::swap(perm[i], perm[j]);
        }
        pick.assign(perm.begin(), perm.begin() + (long)cap);
        std::sort(pick.begin(), pick.end());
    } else {
        pick.resize(n_all);
        for (size_t i = 0; i < n_all; ++i) pick[i] = i;
    }
    const size_t n = pick.size();
    if (n_fit_groups) *n_fit_groups = n;
    if (pick_out) for (size_t i = 0; i < n; ++i) pick_out[i] = (uint64_t)pick[i];

    // steps 2-3: normalise by the group's absolute maximum, then 16-cluster k-means per group
    std::vector<double> pat(n * K);
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (long gi = 0; gi < (long)n; ++gi) {
        const uint16_t* x = data + pick[(size_t)gi] * G;
        uint16_t s_bits = 0;
        for (int i = 0; i < G; ++i) s_bits = std::max<uint16_t>(s_bits, (uint16_t)(x[i] & 0x7FFF));
        float s = oracle_h2f(s_bits);
        float v[G];
        for (int i = 0; i < G; ++i) v[i] = (s_bits == 0) ? 0.0f : oracle_h2f(x[i]) / s;
        oracle_kmeans_1d(v, G, K, 25, &pat[(size_t)gi * K], nullptr);
    }

    if (group_patterns_out) std::memcpy(group_patterns_out, pat.data(), sizeof(double) * n * K);

    // step 4: k-means with S clusters over the 16-vectors.  k-means++ seeding (Arthur & Vassilvitskii 2007)
    std::vector<double> cen((size_t)S * K);
    auto dist2 = [&](size_t g, const double* c) {
        double d = 0.0;
        for (int k = 0; k < K; ++k) { double t = pat[g * K + k] - c[k]; d += t * t; }
        return d;
    };
    {
        size_t first = (size_t)(rng.next() % (uint64_t)n);
        for (int k = 0; k < K; ++k) cen[k] = pat[first * K + k];
        std::vector<double> d2(n);
        for (size_t g = 0; g < n; ++g) d2[g] = dist2(g, &cen[0]);
        for (int s = 1; s < S; ++s) {
            double total = 0.0;
            for (size_t g = 0; g < n; ++g) total += d2[g];
            size_t chosen;
            uint64_t r64 = rng.next();
            if (total > 0.0) {
                double target = (double)(r64 >> 11) * (1.0 / 9007199254740992.0) * total;
                double cum = 0.0;
                chosen = n - 1;
                for (size_t g = 0; g < n; ++g) { cum += d2[g]; if (cum > target) { chosen = g; break; } }
            } else {
                chosen = (size_t)(r64 % (uint64_t)n);
            }
            for (int k = 0; k < K; ++k) cen[(size_t)s * K + k] = pat[chosen * K + k];
            for (size_t g = 0; g < n; ++g) d2[g] = std::min(d2[g], dist2(g, &cen[(size_t)s * K]));
        }
    }
    std::vector<int> assign(n, -1);
    std::vector<double> own(n);
    for (int it = 0; it < 50; ++it) {
        long changed = 0;
#pragma omp parallel for num_threads(g_threads) schedule(static) reduction(+ : changed)
        for (long gi = 0; gi < (long)n; ++gi) {
            int best = 0;
            double bd = dist2((size_t)gi, &cen[0]);
            for (int s = 1; s < S; ++s) {
                double d = dist2((size_t)gi, &cen[(size_t)s * K]);
                if (d < bd) { bd = d; best = s; }
            }
            if (best != assign[(size_t)gi]) { assign[(size_t)gi] = best; ++changed; }
            own[(size_t)gi] = bd;
        }
        if (objective_out) {  // reporting only: the fit does not use this sum
            double total = 0.0;
            for (size_t g = 0; g < n; ++g) total += own[g];
            objective_out[it] = total;
        }
        if (n_objective) *n_objective = it + 1;
        if (changed == 0) break;
        std::vector<double> sum((size_t)S * K, 0.0);
        std::vector<size_t> cnt((size_t)S, 0);
        for (size_t g = 0; g < n; ++g) {  // in group order: one fixed summation order
            for (int k = 0; k < K; ++k) sum[(size_t)assign[g] * K + k] += pat[g * K + k];
            ++cnt[(size_t)assign[g]];
        }
        std::vector<char> used(n, 0);
        for (int s = 0; s < S; ++s) {
            if (cnt[(size_t)s] > 0) {
                for (int k = 0; k < K; ++k) cen[(size_t)s * K + k] = sum[(size_t)s * K + k] / (double)cnt[(size_t)s];
            } else {  // empty cluster: move it onto the point farthest from its own centroid
                size_t far = 0;
                double fd = -1.0;
                for (size_t g = 0; g < n; ++g) if (!used[g] && own[g] > fd) { fd = own[g]; far = g; }
                used[far] = 1;
                for (int k = 0; k < K; ++k) cen[(size_t)s * K + k] = pat[far * K + k];
            }
        }
    }
    // shared patterns as fp16, inside [-1,1], sorted
    for (int s = 0; s < S; ++s) {
        float f[K];
        for (int k = 0; k < K; ++k) {
            double c = std::max(-1.0, std::min(1.0, cen[(size_t)s * K + k]));
            f[k] = oracle_h2f(oracle_f2h((float)c));
        }
        std::stable_sort(f, f + K);
        for (int k = 0; k < K; ++k) centroids[s * K + k] = oracle_f2h(f[k]);
    }

    // steps 5-6: quantise the fit groups, count index use per pattern
    std::vector<uint64_t> hist((size_t)S * K, 0);
    std::vector<uint64_t> groups_of((size_t)S, 0);
    {
        std::vector<int> pp(n);
        std::vector<uint8_t> ii(n * G);
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (long gi = 0; gi < (long)n; ++gi) {
            uint16_t s;
            oracle_quantize_group(centroids, S, data + pick[(size_t)gi] * G, &s, &pp[(size_t)gi], &ii[(size_t)gi * G], nullptr);
        }
        for (size_t g = 0; g < n; ++g) {
            ++groups_of[(size_t)pp[g]];
            for (int i = 0; i < G; ++i) ++hist[(size_t)pp[g] * K + ii[g * G + i]];
        }
    }
    if (hist_out) std::memcpy(hist_out, hist.data(), sizeof(uint64_t) * (size_t)S * K);

    // step 7: one codebook per pattern from the pooled counts (+1 each, so every index has a code)
    for (int s = 0; s < S; ++s) {
        if (groups_of[(size_t)s] == 0) {
            for (int k = 0; k < K; ++k) lens[s * K + k] = 4;
            continue;
        }
        uint64_t c[K];
        for (int k = 0; k < K; ++k) c[k] = hist[(size_t)s * K + k] + 1;
        int rc = oracle_limited_lengths(c, K, max_len, lens + s * K);
        if (rc != 0) return rc;
    }
    return 0;
}

int oracle_fit(const uint16_t* data, size_t n_values, int S, int max_len, uint64_t seed,
               uint16_t* centroids, uint8_t* lens, uint64_t* hist_out, size_t* n_fit_groups) {
    return oracle_fit_trace(data, n_values, S, max_len, seed, centroids, lens, hist_out, n_fit_groups,
                            nullptr, nullptr, nullptr, nullptr);
}

}  // extern "C"
