// ecco_fit_patterns: the offline part of Ecco's compression (Section 3.2, steps 1-4 and 6-7), on
// the CPU.  Groups of 128 values are normalised by their absolute maximum; a 16-level 1-D k-means
// per group yields the group's sorted centroid vector; an S-cluster k-means over those vectors
// yields the shared patterns; the fit groups are quantised with minimum-error pattern selection
// (step 5) and each pattern's pooled index counts give one length-limited canonical Huffman code.
//
// Work that is independent per group runs on a thread pool; every reduction is done by one thread
// in group order, so the result depends only on (data, S, max_code_len, seed).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <thread>
#include <vector>

#include "ecco_internal.h"

namespace ecco {
namespace {

struct Rng {  // splitmix64 sequence
    uint64_t s;
    uint64_t operator()() {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
};

template <class F>
void parallel_for(size_t n, F&& body) {
    unsigned hw = std::thread::hardware_concurrency();
    size_t nt = std::max<size_t>(1, std::min<size_t>(hw ? hw : 1, 32));
    if (n < 256) nt = 1;
    if (nt == 1) {
        for (size_t i = 0; i < n; ++i) body(i);
        return;
    }
    std::vector<std::thread> pool;
    size_t chunk = (n + nt - 1) / nt;
    for (size_t t = 0; t < nt; ++t) {
        size_t lo = t * chunk, hi = std::min(n, lo + chunk);
        if (lo >= hi) break;
        pool.emplace_back([lo, hi, &body] { for (size_t i = lo; i < hi; ++i) body(i); });
    }
    for (auto& th : pool) th.join();
}

// Lloyd iterations in one dimension.  Start at the (k+0.5)/16 quantiles of the sorted values; at
// most 25 rounds; stop when no value changes cluster; an empty cluster keeps its centroid; a value
// equally near two centroids goes to the lower one.
void group_pattern(const uint16_t* x, double* out) {
    uint16_t smax = 0;
    for (int i = 0; i < kGroup; ++i) smax = std::max<uint16_t>(smax, x[i] & 0x7FFF);
    float v32[kGroup];
    const float s = half_bits_to_float(smax);
    for (int i = 0; i < kGroup; ++i) v32[i] = smax ? half_bits_to_float(x[i]) / s : 0.0f;
    std::sort(v32, v32 + kGroup);
    double c[kK];
    for (int k = 0; k < kK; ++k) c[k] = v32[((2 * k + 1) * kGroup) / (2 * kK)];
    int8_t owner[kGroup];
    std::memset(owner, -1, sizeof owner);
    for (int round = 0;; ++round) {
        bool moved = false;
        for (int i = 0; i < kGroup; ++i) {
            int8_t b = 0;
            double bd = std::fabs((double)v32[i] - c[0]);
            for (int k = 1; k < kK; ++k) {
                double d = std::fabs((double)v32[i] - c[k]);
                if (d < bd) { bd = d; b = (int8_t)k; }
            }
            moved |= (b != owner[i]);
            owner[i] = b;
        }
        if (!moved || round >= 25) break;
        double sum[kK] = {0};
        int cnt[kK] = {0};
        for (int i = 0; i < kGroup; ++i) { sum[owner[i]] += (double)v32[i]; ++cnt[owner[i]]; }
        for (int k = 0; k < kK; ++k) if (cnt[k]) c[k] = sum[k] / cnt[k];
    }
    std::sort(c, c + kK);
    std::copy(c, c + kK, out);
}

inline double sqdist(const double* a, const double* b) {
    double d = 0.0;
    for (int k = 0; k < kK; ++k) { double t = a[k] - b[k]; d += t * t; }
    return d;
}

// Encoder rule of Section 3.2 step 5 on the host (used for the index statistics only): scale,
// reconstructed values per pattern, nearest value with ties to the lower index, squared errors
// summed by the balanced pairwise tree, pattern of least error.
void quantize_host(const uint16_t* cent, int S, const uint16_t* x, int* pattern, uint8_t* idx) {
    uint16_t smax = 0;
    for (int i = 0; i < kGroup; ++i) smax = std::max<uint16_t>(smax, x[i] & 0x7FFF);
    const float s = half_bits_to_float(smax);
    float xv[kGroup];
    for (int i = 0; i < kGroup; ++i) xv[i] = half_bits_to_float(x[i]);
    float best = 0.0f;
    uint8_t cand[kGroup];
    for (int p = 0; p < S; ++p) {
        float r[kK];
        for (int k = 0; k < kK; ++k)
            r[k] = half_bits_to_float(float_to_half_bits(half_bits_to_float(cent[p * kK + k]) * s));
        float e[kGroup];
        for (int i = 0; i < kGroup; ++i) {
            // r is ascending: find the first element >= x, then compare with its left neighbours
            int hi = (int)(std::lower_bound(r, r + kK, xv[i]) - r);
            int k;
            if (hi == 0) k = 0;
            else if (hi == kK) { k = kK - 1; while (k > 0 && r[k - 1] == r[k]) --k; }
            else {
                float dl = std::fabs(xv[i] - r[hi - 1]), dh = std::fabs(xv[i] - r[hi]);
                k = (dl <= dh) ? hi - 1 : hi;
                while (k > 0 && r[k - 1] == r[k]) --k;
            }
            cand[i] = (uint8_t)k;
            float d = xv[i] - r[k];
            e[i] = d * d;
        }
        for (int stride = 1; stride < kGroup; stride <<= 1)
            for (int i = 0; i < kGroup; i += 2 * stride) e[i] = e[i] + e[i + stride];
        if (p == 0 || e[0] < best) {
            best = e[0];
            *pattern = p;
            std::memcpy(idx, cand, kGroup);
        }
    }
}

// Optimal code lengths <= limit for n <= 16 weights: package-merge (Larmore & Hirschberg),
// with each coin carrying how often every symbol occurs in it.
void limited_lengths(const uint64_t* w, int n, int limit, uint8_t* len) {
    struct Coin { uint64_t w; uint8_t occ[kK]; };
    std::vector<Coin> base(n);
    std::vector<int> ord(n);
    std::iota(ord.begin(), ord.end(), 0);
    std::stable_sort(ord.begin(), ord.end(), [&](int a, int b) { return w[a] < w[b]; });
    for (int j = 0; j < n; ++j) {
        base[j].w = w[ord[j]];
        std::memset(base[j].occ, 0, sizeof base[j].occ);
        base[j].occ[ord[j]] = 1;
    }
    std::vector<Coin> level = base, next;
    for (int depth = 1; depth < limit; ++depth) {
        next.clear();
        size_t bi = 0;
        for (size_t j = 0; j + 1 < level.size(); j += 2) {
            Coin pk;
            pk.w = level[j].w + level[j + 1].w;
            for (int k = 0; k < kK; ++k) pk.occ[k] = (uint8_t)(level[j].occ[k] + level[j + 1].occ[k]);
            while (bi < base.size() && base[bi].w <= pk.w) next.push_back(base[bi++]);
            next.push_back(pk);
        }
        while (bi < base.size()) next.push_back(base[bi++]);
        level.swap(next);
    }
    int acc[kK] = {0};
    for (int j = 0; j < 2 * n - 2; ++j)
        for (int k = 0; k < n; ++k) acc[k] += level[j].occ[k];
    for (int k = 0; k < n; ++k) len[k] = (uint8_t)acc[k];
}

}  // namespace
}  // namespace ecco

using namespace ecco;

extern "C" int ecco_fit_patterns(const uint16_t* data, size_t n_values, int S, int max_code_len,
                                 uint64_t seed, ecco_model** out) {
    if (!data || !out) return ECCO_EINVAL;
    if (S < 1 || S > kMaxS || max_code_len < 4 || max_code_len > kMaxLen) return ECCO_EINVAL;
    if (n_values == 0 || n_values % kGroup != 0) return ECCO_ESHAPE;
    for (size_t i = 0; i < n_values; ++i)
        if ((data[i] & 0x7C00) == 0x7C00) return ECCO_EINVAL;  // Inf / NaN

    const size_t n_all = n_values / kGroup;
    Rng rng{seed};
    // step 1: at most 65 536 groups take part (a seeded sample without replacement, kept in order)
    const size_t cap = 65536;
    std::vector<uint32_t> pick;
    if (n_all > cap) {
        std::vector<uint32_t> perm(n_all);
        std::iota(perm.begin(), perm.end(), 0u);
        for (size_t i = 0; i < cap; ++i) std::swap(perm[i], perm[i + rng() % (n_all - i)]);
        pick.assign(perm.begin(), perm.begin() + cap);
        std::sort(pick.begin(), pick.end());
    } else {
        pick.resize(n_all);
        std::iota(pick.begin(), pick.end(), 0u);
    }
    const size_t n = pick.size();

    // steps 2-3
    std::vector<double> pat(n * kK);
    parallel_for(n, [&](size_t g) { group_pattern(data + (size_t)pick[g] * kGroup, &pat[g * kK]); });

    // step 4: k-means++ seeding, then Lloyd (<= 50 rounds)
    std::vector<double> cen((size_t)S * kK);
    {
        std::vector<double> d2(n);
        size_t first = rng() % n;
        std::copy(&pat[first * kK], &pat[first * kK] + kK, &cen[0]);
        parallel_for(n, [&](size_t g) { d2[g] = sqdist(&pat[g * kK], &cen[0]); });
        for (int s = 1; s < S; ++s) {
            double total = 0.0;
            for (size_t g = 0; g < n; ++g) total += d2[g];
            uint64_t r = rng();
            size_t chosen = n - 1;
            if (total > 0.0) {
                double target = (double)(r >> 11) * (1.0 / 9007199254740992.0) * total, cum = 0.0;
                for (size_t g = 0; g < n; ++g) { cum += d2[g]; if (cum > target) { chosen = g; break; } }
            } else {
                chosen = r % n;
            }
            double* c = &cen[(size_t)s * kK];
            std::copy(&pat[chosen * kK], &pat[chosen * kK] + kK, c);
            parallel_for(n, [&](size_t g) { d2[g] = std::min(d2[g], sqdist(&pat[g * kK], c)); });
        }
    }
    std::vector<int> assign(n, -1), fresh(n);
    std::vector<double> own(n);
    for (int it = 0; it < 50; ++it) {
        parallel_for(n, [&](size_t g) {
            int b = 0;
            double bd = sqdist(&pat[g * kK], &cen[0]);
            for (int s = 1; s < S; ++s) {
                double d = sqdist(&pat[g * kK], &cen[(size_t)s * kK]);
                if (d < bd) { bd = d; b = s; }
            }
            fresh[g] = b;
            own[g] = bd;
        });
        if (fresh == assign) break;
        assign = fresh;
        std::vector<double> sum((size_t)S * kK, 0.0);
        std::vector<size_t> cnt(S, 0);
        for (size_t g = 0; g < n; ++g) {
            double* dst = &sum[(size_t)assign[g] * kK];
            for (int k = 0; k < kK; ++k) dst[k] += pat[g * kK + k];
            ++cnt[assign[g]];
        }
        std::vector<char> taken(n, 0);
        for (int s = 0; s < S; ++s) {
            double* c = &cen[(size_t)s * kK];
            if (cnt[s]) {
                for (int k = 0; k < kK; ++k) c[k] = sum[(size_t)s * kK + k] / (double)cnt[s];
            } else {  // empty cluster: restart it on the worst-served point
                size_t far = 0;
                double fd = -1.0;
                for (size_t g = 0; g < n; ++g) if (!taken[g] && own[g] > fd) { fd = own[g]; far = g; }
                taken[far] = 1;
                std::copy(&pat[far * kK], &pat[far * kK] + kK, c);
            }
        }
    }

    ecco_model* m = new (std::nothrow) ecco_model;
    if (!m) return ECCO_ENOMEM;
    m->S = S;
    for (int s = 0; s < S; ++s) {
        float f[kK];
        for (int k = 0; k < kK; ++k) {
            double c = std::min(1.0, std::max(-1.0, cen[(size_t)s * kK + k]));
            f[k] = half_bits_to_float(float_to_half_bits((float)c));
        }
        std::stable_sort(f, f + kK);
        for (int k = 0; k < kK; ++k) m->cent[s * kK + k] = float_to_half_bits(f[k]);
    }

    // steps 5-7: index statistics of the fit groups -> one codebook per pattern
    std::vector<int> gp(n);
    std::vector<uint8_t> gi(n * kGroup);
    parallel_for(n, [&](size_t g) { quantize_host(m->cent, S, data + (size_t)pick[g] * kGroup, &gp[g], &gi[g * kGroup]); });
    std::vector<uint64_t> hist((size_t)S * kK, 0), used(S, 0);
    for (size_t g = 0; g < n; ++g) {
        ++used[gp[g]];
        for (int i = 0; i < kGroup; ++i) ++hist[(size_t)gp[g] * kK + gi[g * kGroup + i]];
    }
    for (int s = 0; s < S; ++s) {
        if (!used[s]) {
            std::memset(&m->lens[s * kK], 4, kK);
            continue;
        }
        uint64_t w[kK];
        for (int k = 0; k < kK; ++k) w[k] = hist[(size_t)s * kK + k] + 1;  // every index keeps a code
        limited_lengths(w, kK, max_code_len, &m->lens[s * kK]);
    }
    if (validate_tables(m->cent, m->lens, S) != ECCO_OK) {
        delete m;
        return ECCO_EFORMAT;
    }
    derive_codes(m);
    *out = m;
    return ECCO_OK;
}
