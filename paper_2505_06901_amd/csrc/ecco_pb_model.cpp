// Model object of the self-contained block format: validation, canonical codes, device tables, and the CPU fit
// (Section 3.2 "Model Compression": two-level normalisation, per-group 15-cluster k-means on the 127 values besides
// the largest, S shared patterns, H = 4 codebooks per pattern from a k-means over the groups' index frequencies).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <thread>
#include <vector>

#include "ecco_internal.h"
#include "ecco_pb_internal.h"

using namespace ecco_pb;
using ecco::float_to_half_bits;
using ecco::half_bits_to_float;

namespace {

// canonical codes of n symbols with the given lengths: ordered by (length, symbol), first code 0
void canonical_codes(const uint8_t* lens, int n, uint16_t* codes) {
    uint32_t code = 0;
    int prev = 0;
    bool first = true;
    for (int l = 1; l <= 16; ++l)
        for (int k = 0; k < n; ++k)
            if (lens[k] == l) {
                if (!first) code = (code + 1) << (l - prev);
                first = false;
                prev = l;
                codes[k] = (uint16_t)code;
            }
}

int validate(const uint16_t* cent, const uint8_t* lens, const uint8_t* kp_lens, int S, int texp) {
    if (S < 1 || S > kMaxS) return ECCO_EFORMAT;
    if (texp < -15 || texp > 7) return ECCO_EFORMAT;
    for (int p = 0; p < S; ++p) {
        for (int k = 0; k < kCent; ++k) {
            const uint16_t c = cent[p * kCent + k];
            if ((c & 0x7C00) == 0x7C00 || (c & 0x7FFF) > 0x3C00) return ECCO_EFORMAT;
            if (k && half_bits_to_float(c) < half_bits_to_float(cent[p * kCent + k - 1])) return ECCO_EFORMAT;
        }
        for (int h = 0; h < kBooks; ++h) {
            uint32_t kraft = 0;
            for (int k = 0; k < kSym; ++k) {
                const uint8_t l = lens[(p * kBooks + h) * kSym + k];
                if (l < kMinLen || l > kMaxLen) return ECCO_EFORMAT;
                kraft += 1u << (kMaxLen - l);
            }
            if (kraft != (1u << kMaxLen)) return ECCO_EFORMAT;
        }
    }
    uint32_t kraft = 0;
    for (int p = 0; p < S; ++p) {
        if (kp_lens[p] < 1 || kp_lens[p] > 8) return ECCO_EFORMAT;
        kraft += 1u << (8 - kp_lens[p]);
    }
    if (kraft > 256u || (S >= 2 && kraft != 256u)) return ECCO_EFORMAT;
    return ECCO_OK;
}

void build_image(const ecco_pb_model* m, uint32_t* img) {
    const DevLayout D{m->S};
    std::memset(img, 0, D.total_words() * 4);
    uint8_t* lut = reinterpret_cast<uint8_t*>(img + D.lut());
    uint16_t* kplut = reinterpret_cast<uint16_t*>(img + D.kplut());
    uint16_t* cent = reinterpret_cast<uint16_t*>(img + D.cent());
    uint16_t* fp8 = reinterpret_cast<uint16_t*>(img + D.fp8());
    uint32_t* enc = img + D.enc();
    uint32_t* kpenc = img + D.kpenc();
    for (int t = 0; t < m->S * kBooks; ++t)
        for (int k = 0; k < kSym; ++k) {
            const int l = m->lens[t * kSym + k];
            const uint32_t code = m->codes[t * kSym + k];
            enc[t * kSym + k] = code | ((uint32_t)l << 16);
            for (uint32_t j = 0; j < (1u << (kMaxLen - l)); ++j) lut[t * 256 + (code << (kMaxLen - l)) + j] = (uint8_t)((k << 4) | l);
        }
    for (int i = 0; i < 256; ++i) kplut[i] = (uint16_t)(((m->S - 1) << 8) | 8);
    for (int p = 0; p < m->S; ++p) {
        const int l = m->kp_lens[p];
        kpenc[p] = (uint32_t)m->kp_codes[p] | ((uint32_t)l << 16);
        for (uint32_t j = 0; j < (1u << (8 - l)); ++j) kplut[((uint32_t)m->kp_codes[p] << (8 - l)) + j] = (uint16_t)((p << 8) | l);
    }
    for (int p = 0; p < m->S; ++p)
    {
        for (int k = 0; k < kCent; ++k) cent[p * 16 + k] = m->cent[p * kCent + k];
        cent[p * 16 + 15] = 0x3C00;  // index 15 stands for the scale itself: 1.0 times the scale
    }
    for (int b = 0; b < 256; ++b) fp8[b] = float_to_half_bits((float)std::ldexp(fp8_value((uint8_t)b), m->texp));  // exact
}

// ---- fit helpers ------------------------------------------------------------------------------------------
struct Rng {  // splitmix64 sequence
    uint64_t s;
    uint64_t operator()() {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    double uniform() { return (double)((*this)() >> 11) * (1.0 / 9007199254740992.0); }
};

template <class F>
void parallel_for(size_t n, F&& body) {
    const unsigned hw = std::thread::hardware_concurrency();
    size_t nt = std::max<size_t>(1, std::min<size_t>(hw ? hw : 1, 32));
    if (n < 256) nt = 1;
    if (nt == 1) {
        for (size_t i = 0; i < n; ++i) body(i);
        return;
    }
    std::vector<std::thread> pool;
    const size_t chunk = (n + nt - 1) / nt;
    for (size_t t = 0; t < nt; ++t) {
        const size_t lo = t * chunk, hi = std::min(n, lo + chunk);
        if (lo >= hi) break;
        pool.emplace_back([lo, hi, &body] { for (size_t i = lo; i < hi; ++i) body(i); });
    }
    for (auto& th : pool) th.join();
}

uint8_t fp8_round(double v) {  // nearest, ties to even code, saturating
    const uint8_t sign = std::signbit(v) ? 0x80 : 0;
    const double a = std::fabs(v);
    if (a >= 480.0) return (uint8_t)(sign | 127);
    int lo = 0, hi = 127;
    while (hi - lo > 1) {
        const int mid = (lo + hi) / 2;
        if (fp8_value((uint8_t)mid) <= a) lo = mid; else hi = mid;
    }
    const double dl = a - fp8_value((uint8_t)lo), dh = fp8_value((uint8_t)hi) - a;
    return (uint8_t)(sign | (dl < dh ? lo : dh < dl ? hi : ((lo & 1) ? hi : lo)));
}

// position of the element of largest magnitude (first on ties) and the magnitude of the group scale as FP16 bits
void group_scale(const uint16_t* x, int texp, int* amax, uint16_t* sabs_bits) {
    int a = 0;
    for (int i = 1; i < kGroup; ++i)
        if ((x[i] & 0x7FFF) > (x[a] & 0x7FFF)) a = i;
    const uint8_t s8 = fp8_round(std::ldexp((double)half_bits_to_float(x[a]), -texp));
    *amax = a;
    *sabs_bits = (uint16_t)(float_to_half_bits((float)std::ldexp(fp8_value(s8), texp)) & 0x7FFF);
}

// 1-D Lloyd k-means on n sorted values: start at the (k + 0.5) / K quantiles, at most 25 rounds, stop when no value
// changes cluster, an empty cluster keeps its centroid, a value equally near two centroids goes to the lower one
void kmeans_1d(const float* v, int n, int K, double* c) {
    for (int k = 0; k < K; ++k) c[k] = v[std::min(n - 1, (int)(((double)k + 0.5) * n / K))];
    std::vector<int> assign(n, -1);
    for (int it = 0; it < 25; ++it) {
        bool moved = false;
        for (int i = 0; i < n; ++i) {
            int best = 0;
            double bd = std::fabs((double)v[i] - c[0]);
            for (int k = 1; k < K; ++k) {
                const double d = std::fabs((double)v[i] - c[k]);
                if (d < bd) { bd = d; best = k; }
            }
            if (best != assign[i]) { assign[i] = best; moved = true; }
        }
        if (!moved) break;
        for (int k = 0; k < K; ++k) {
            double sum = 0.0;
            int cnt = 0;
            for (int i = 0; i < n; ++i)
                if (assign[i] == k) { sum += v[i]; ++cnt; }
            if (cnt) c[k] = sum / cnt;
        }
    }
    std::sort(c, c + K);
}

// k-means over n points of dimension D: k-means++ seeding, at most `rounds` Lloyd rounds, an empty cluster restarts on
// the point farthest from its centroid; sums in double in point order, so the result depends on (points, K, seed) only
void kmeans_vectors(const double* pts, size_t n, int D, int K, uint64_t seed, int rounds, std::vector<double>& cent, std::vector<int>& assign) {
    cent.assign((size_t)K * D, 0.0);
    assign.assign(n, 0);
    if (n == 0) return;
    Rng rng{seed};
    auto dist = [&](size_t i, const double* c) {
        double s = 0.0;
        for (int d = 0; d < D; ++d) { const double t = pts[i * D + d] - c[d]; s += t * t; }
        return s;
    };
    std::vector<double> near(n);
    size_t first = (size_t)(rng.uniform() * (double)n);
    if (first >= n) first = n - 1;
    std::memcpy(&cent[0], pts + first * D, sizeof(double) * D);
    for (size_t i = 0; i < n; ++i) near[i] = dist(i, &cent[0]);
    for (int k = 1; k < K; ++k) {
        double total = 0.0;
        for (size_t i = 0; i < n; ++i) total += near[i];
        size_t pick = n - 1;
        if (total > 0.0) {
            double r = rng.uniform() * total;
            for (size_t i = 0; i < n; ++i) {
                r -= near[i];
                if (r < 0.0) { pick = i; break; }
            }
        } else {
            pick = (size_t)(rng.uniform() * (double)n) % n;
        }
        std::memcpy(&cent[(size_t)k * D], pts + pick * D, sizeof(double) * D);
        for (size_t i = 0; i < n; ++i) near[i] = std::min(near[i], dist(i, &cent[(size_t)k * D]));
    }
    std::vector<double> sums((size_t)K * D);
    std::vector<size_t> counts(K);
    for (int it = 0; it < rounds; ++it) {
        std::vector<int> next(n);
        parallel_for(n, [&](size_t i) {
            int best = 0;
            double bd = dist(i, &cent[0]);
            for (int k = 1; k < K; ++k) {
                const double d = dist(i, &cent[(size_t)k * D]);
                if (d < bd) { bd = d; best = k; }
            }
            next[i] = best;
            near[i] = bd;
        });
        const bool same = it > 0 && next == assign;
        assign.swap(next);
        if (same) break;
        std::fill(sums.begin(), sums.end(), 0.0);
        std::fill(counts.begin(), counts.end(), 0);
        for (size_t i = 0; i < n; ++i) {
            ++counts[assign[i]];
            for (int d = 0; d < D; ++d) sums[(size_t)assign[i] * D + d] += pts[i * D + d];
        }
        for (int k = 0; k < K; ++k) {
            if (counts[k]) {
                for (int d = 0; d < D; ++d) cent[(size_t)k * D + d] = sums[(size_t)k * D + d] / (double)counts[k];
            } else {
                size_t far = 0;
                for (size_t i = 1; i < n; ++i)
                    if (near[i] > near[far]) far = i;
                std::memcpy(&cent[(size_t)k * D], pts + far * D, sizeof(double) * D);
                near[far] = 0.0;
            }
        }
    }
}

// optimal prefix-code lengths within lmin..lmax and Kraft sum exactly 1, for n symbols: dynamic programme over the
// symbols by decreasing count (an optimal code gives them non-decreasing lengths), the previous length and the
// remaining Kraft budget in units of 2^-lmax
void optimal_lengths(const uint64_t* counts, int n, int lmin, int lmax, uint8_t* lens) {
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return counts[a] > counts[b]; });
    const int budget = 1 << lmax, span = lmax - lmin + 1;
    const uint64_t kInf = ~0ull;
    // cost[i][l - lmin][b]: least cost of symbols i.. with lengths >= l using exactly budget b
    std::vector<uint64_t> cost((size_t)(n + 1) * span * (budget + 1), kInf);
    std::vector<uint8_t> pick((size_t)(n + 1) * span * (budget + 1), 0);
    auto at = [&](int i, int l, int b) { return ((size_t)i * span + (l - lmin)) * (budget + 1) + b; };
    for (int l = lmin; l <= lmax; ++l) cost[at(n, l, 0)] = 0;
    for (int i = n - 1; i >= 0; --i)
        for (int l = lmax; l >= lmin; --l)
            for (int b = 0; b <= budget; ++b) {
                uint64_t best = kInf;
                uint8_t bl = 0;
                for (int t = l; t <= lmax; ++t) {
                    const int w = 1 << (lmax - t);
                    if (w > b) continue;
                    const uint64_t rest = cost[at(i + 1, t, b - w)];
                    if (rest == kInf) continue;
                    const uint64_t c = rest + counts[order[i]] * (uint64_t)t;
                    if (c < best) { best = c; bl = (uint8_t)t; }
                }
                cost[at(i, l, b)] = best;
                pick[at(i, l, b)] = bl;
            }
    int l = lmin, b = budget;
    for (int i = 0; i < n; ++i) {
        const uint8_t t = pick[at(i, l, b)];
        lens[order[i]] = t;
        b -= 1 << (lmax - t);
        l = t;
    }
}

// the encoder's decisions for one group on the host (same rules, FP32): pattern of least squared error, indices
void quantize_host(const uint16_t* cent, int S, int texp, const uint16_t* x, int* pattern, uint8_t* idx) {
    int a;
    uint16_t sabs_bits;
    group_scale(x, texp, &a, &sabs_bits);
    const float sabs = half_bits_to_float(sabs_bits);
    float best_sse = 0.0f;
    uint8_t id[kGroup], best_id[kGroup];
    int best_p = 0;
    for (int p = 0; p < S; ++p) {
        float r[kCent], e[kGroup];
        for (int k = 0; k < kCent; ++k) r[k] = half_bits_to_float(float_to_half_bits(half_bits_to_float(cent[p * kCent + k]) * sabs));
        for (int i = 0; i < kGroup; ++i) {
            if (i == a) { e[i] = 0.0f; id[i] = 15; continue; }
            const float xi = half_bits_to_float(x[i]);
            int bk = 0;
            float bd = std::fabs(xi - r[0]);
            for (int k = 1; k < kCent; ++k) {
                const float d = std::fabs(xi - r[k]);
                if (d < bd) { bd = d; bk = k; }
            }
            const float d = xi - r[bk];
            e[i] = d * d;
            id[i] = (uint8_t)bk;
        }
        for (int stride = 1; stride < kGroup; stride <<= 1)
            for (int i = 0; i < kGroup; i += 2 * stride) e[i] = e[i] + e[i + stride];
        if (p == 0 || e[0] < best_sse) { best_sse = e[0]; best_p = p; std::memcpy(best_id, id, kGroup); }
    }
    *pattern = best_p;
    std::memcpy(idx, best_id, kGroup);
}

}  // namespace

extern "C" {

int ecco_pb_model_create(const uint16_t* centroids, const uint8_t* code_lens, const uint8_t* kp_lens, int S, int texp,
                         ecco_pb_model** out) {
    if (!centroids || !code_lens || !kp_lens || !out) return ECCO_EINVAL;
    if (S < 1 || S > kMaxS) return ECCO_EINVAL;
    const int rc = validate(centroids, code_lens, kp_lens, S, texp);
    if (rc != ECCO_OK) return rc;
    ecco_pb_model* m = new (std::nothrow) ecco_pb_model;
    if (!m) return ECCO_ENOMEM;
    m->S = S;
    m->texp = texp;
    std::memcpy(m->cent, centroids, sizeof(uint16_t) * S * kCent);
    std::memcpy(m->lens, code_lens, (size_t)S * kBooks * kSym);
    std::memcpy(m->kp_lens, kp_lens, (size_t)S);
    for (int t = 0; t < S * kBooks; ++t) canonical_codes(m->lens + t * kSym, kSym, m->codes + t * kSym);
    canonical_codes(m->kp_lens, S, m->kp_codes);
    *out = m;
    return ECCO_OK;
}

// serialised form: { 'ECP0', version 1, S, texp } then centroids [S][15] FP16, code lengths [S][4][16], pattern-id lengths [S]
namespace {
constexpr uint32_t kPbMagic = 0x30504345u;  // "ECP0"
struct PbHeader { uint32_t magic, version; int32_t S, texp; };
size_t pb_blob_bytes(int S) { return sizeof(PbHeader) + (size_t)S * (kCent * 2 + kBooks * kSym + 1); }
}  // namespace

int ecco_pb_model_save(const ecco_pb_model* m, void* buf, size_t cap, size_t* written) {
    if (!m || !written) return ECCO_EINVAL;
    const size_t need = pb_blob_bytes(m->S);
    *written = need;
    if (!buf) return ECCO_OK;
    if (cap < need) return ECCO_EINVAL;
    const PbHeader h{kPbMagic, 1u, m->S, m->texp};
    unsigned char* p = static_cast<unsigned char*>(buf);
    std::memcpy(p, &h, sizeof h);
    p += sizeof h;
    std::memcpy(p, m->cent, (size_t)m->S * kCent * 2);
    p += (size_t)m->S * kCent * 2;
    std::memcpy(p, m->lens, (size_t)m->S * kBooks * kSym);
    p += (size_t)m->S * kBooks * kSym;
    std::memcpy(p, m->kp_lens, (size_t)m->S);
    return ECCO_OK;
}

int ecco_pb_model_load(const void* buf, size_t len, ecco_pb_model** out) {
    if (!buf || !out) return ECCO_EINVAL;
    if (len < sizeof(PbHeader)) return ECCO_EFORMAT;
    PbHeader h;
    std::memcpy(&h, buf, sizeof h);
    if (h.magic != kPbMagic || h.version != 1u || h.S < 1 || h.S > kMaxS) return ECCO_EFORMAT;
    if (len != pb_blob_bytes(h.S)) return ECCO_EFORMAT;
    const unsigned char* p = static_cast<const unsigned char*>(buf) + sizeof h;
    std::vector<uint16_t> cent((size_t)h.S * kCent);
    std::memcpy(cent.data(), p, cent.size() * 2);
    const uint8_t* lens = p + cent.size() * 2;
    return ecco_pb_model_create(cent.data(), lens, lens + (size_t)h.S * kBooks * kSym, h.S, h.texp, out);
}

int ecco_pb_model_S(const ecco_pb_model* m) { return m ? m->S : 0; }
int ecco_pb_model_texp(const ecco_pb_model* m) { return m ? m->texp : 0; }
const uint16_t* ecco_pb_model_centroids(const ecco_pb_model* m) { return m ? m->cent : nullptr; }
const uint8_t* ecco_pb_model_code_lens(const ecco_pb_model* m) { return m ? m->lens : nullptr; }
const uint8_t* ecco_pb_model_kp_lens(const ecco_pb_model* m) { return m ? m->kp_lens : nullptr; }

int ecco_pb_model_to_device(ecco_pb_model* m, int device) {
    if (!m || device < 0) return ECCO_EINVAL;
    if (m->dev && m->device == device) return ECCO_OK;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device >= count) return ECCO_EHIP;
    int prev = 0;
    if (hipGetDevice(&prev) != hipSuccess) return ECCO_EHIP;
    if (m->dev) {
        (void)hipSetDevice(m->device);
        (void)hipFree(m->dev);
        m->dev = nullptr;
        m->device = -1;
    }
    if (hipSetDevice(device) != hipSuccess) return ECCO_EHIP;
    const DevLayout D{m->S};
    std::vector<uint32_t> img(D.total_words());
    build_image(m, img.data());
    void* d = nullptr;
    hipError_t e = hipMalloc(&d, D.total_words() * 4);
    if (e != hipSuccess) {
        (void)hipSetDevice(prev);
        return e == hipErrorOutOfMemory ? ECCO_ENOMEM : ECCO_EHIP;
    }
    e = hipMemcpy(d, img.data(), D.total_words() * 4, hipMemcpyHostToDevice);
    (void)hipSetDevice(prev);
    if (e != hipSuccess) {
        (void)hipFree(d);
        return ECCO_EHIP;
    }
    m->dev = static_cast<uint32_t*>(d);
    m->device = device;
    return ECCO_OK;
}

void ecco_pb_model_free(ecco_pb_model* m) {
    if (!m) return;
    if (m->dev) {
        int prev = 0;
        if (hipGetDevice(&prev) == hipSuccess) {
            (void)hipSetDevice(m->device);
            (void)hipFree(m->dev);
            (void)hipSetDevice(prev);
        }
    }
    delete m;
}

int ecco_pb_fit(const uint16_t* data, size_t n_values, int S, uint64_t seed, ecco_pb_model** out) {
    if (!data || !out || n_values == 0 || n_values % kGroup != 0 || S < 1 || S > kMaxS) return ECCO_EINVAL;
    const size_t n_all = n_values / kGroup;
    // tensor scale: the smallest power of two that brings the largest magnitude within the 8-bit float's range
    uint16_t top = 0;
    for (size_t i = 0; i < n_values; ++i) top = std::max<uint16_t>(top, data[i] & 0x7FFF);
    int texp = -15;
    while (texp < 7 && std::ldexp((double)half_bits_to_float(top), -texp) > 480.0) ++texp;
    // fit groups: all of them, or a seeded sample of 65 536
    std::vector<size_t> pickg;
    constexpr size_t kMaxFit = 65536;
    if (n_all <= kMaxFit) {
        pickg.resize(n_all);
        for (size_t g = 0; g < n_all; ++g) pickg[g] = g;
    } else {
        Rng rng{seed ^ 0x5851F42D4C957F2Dull};
        std::vector<size_t> perm(n_all);
        for (size_t g = 0; g < n_all; ++g) perm[g] = g;
        for (size_t g = 0; g < kMaxFit; ++g) std::swap(perm[g], perm[g + (size_t)(rng() % (n_all - g))]);
        pickg.assign(perm.begin(), perm.begin() + kMaxFit);
        std::sort(pickg.begin(), pickg.end());
    }
    const size_t n = pickg.size();
    // per-group patterns: 15 clusters over the 127 values besides the largest, normalised by the group scale
    std::vector<double> pats(n * kCent);
    parallel_for(n, [&](size_t j) {
        const uint16_t* x = data + pickg[j] * kGroup;
        int a;
        uint16_t sb;
        group_scale(x, texp, &a, &sb);
        const float s = half_bits_to_float(sb);
        float v[kGroup - 1];
        int t = 0;
        for (int i = 0; i < kGroup; ++i)
            if (i != a) v[t++] = s > 0.0f ? std::min(1.0f, std::max(-1.0f, half_bits_to_float(x[i]) / s)) : 0.0f;
        std::sort(v, v + (kGroup - 1));
        kmeans_1d(v, kGroup - 1, kCent, &pats[j * kCent]);
    });
    // shared patterns
    std::vector<double> shared;
    std::vector<int> assign;
    const int Sfit = (int)std::min<size_t>((size_t)S, n);
    kmeans_vectors(pats.data(), n, kCent, Sfit, seed, 50, shared, assign);
    ecco_pb_model* m = new (std::nothrow) ecco_pb_model;
    if (!m) return ECCO_ENOMEM;
    m->S = S;
    m->texp = texp;
    for (int p = 0; p < S; ++p) {
        float c[kCent];
        for (int k = 0; k < kCent; ++k) {
            const double v = p < Sfit ? shared[(size_t)p * kCent + k] : -1.0 + 2.0 * (k + 0.5) / kCent;  // spare patterns: evenly spaced
            c[k] = half_bits_to_float(float_to_half_bits((float)std::min(1.0, std::max(-1.0, v))));
        }
        std::sort(c, c + kCent);
        for (int k = 0; k < kCent; ++k) m->cent[p * kCent + k] = float_to_half_bits(c[k]);
    }
    // quantise the fit groups; index counts per group
    std::vector<int> gp(n);
    std::vector<uint8_t> hist(n * kSym);
    parallel_for(n, [&](size_t j) {
        uint8_t idx[kGroup];
        quantize_host(m->cent, S, texp, data + pickg[j] * kGroup, &gp[j], idx);
        uint8_t* h = &hist[j * kSym];
        std::memset(h, 0, kSym);
        for (int i = 0; i < kGroup; ++i) ++h[idx[i]];
    });
    // codebooks: per pattern, 4 clusters over the groups' index frequencies; each cluster's pooled counts (+1 each) give
    // optimal lengths within 2..8; a cluster without groups takes the pattern's pooled counts
    std::vector<uint64_t> use(S, 0);
    for (int p = 0; p < S; ++p) {
        std::vector<size_t> members;
        for (size_t j = 0; j < n; ++j)
            if (gp[j] == p) members.push_back(j);
        use[p] = members.size();
        std::vector<double> freq(members.size() * kSym);
        for (size_t t = 0; t < members.size(); ++t)
            for (int k = 0; k < kSym; ++k) freq[t * kSym + k] = (double)hist[members[t] * kSym + k] / kGroup;
        std::vector<double> fc;
        std::vector<int> fa;
        const int H = (int)std::min<size_t>(kBooks, members.size());
        if (H > 0) kmeans_vectors(freq.data(), members.size(), kSym, H, seed + 1000003ull * (uint64_t)(p + 1), 25, fc, fa);
        uint64_t pooled[kSym];
        for (int k = 0; k < kSym; ++k) pooled[k] = 1;
        for (size_t t = 0; t < members.size(); ++t)
            for (int k = 0; k < kSym; ++k) pooled[k] += hist[members[t] * kSym + k];
        for (int h = 0; h < kBooks; ++h) {
            uint64_t cnt[kSym];
            size_t got = 0;
            for (int k = 0; k < kSym; ++k) cnt[k] = 1;
            for (size_t t = 0; t < members.size(); ++t)
                if (h < H && fa[t] == h) {
                    ++got;
                    for (int k = 0; k < kSym; ++k) cnt[k] += hist[members[t] * kSym + k];
                }
            optimal_lengths(got ? cnt : pooled, kSym, kMinLen, kMaxLen, m->lens + (p * kBooks + h) * kSym);
        }
    }
    // pattern ids: optimal lengths within 1..8 for the use counts (+1 each)
    if (S == 1) {
        m->kp_lens[0] = 1;
    } else {
        for (int p = 0; p < S; ++p) ++use[p];
        optimal_lengths(use.data(), S, 1, 8, m->kp_lens);
    }
    for (int t = 0; t < S * kBooks; ++t) canonical_codes(m->lens + t * kSym, kSym, m->codes + t * kSym);
    canonical_codes(m->kp_lens, S, m->kp_codes);
    if (validate(m->cent, m->lens, m->kp_lens, S, texp) != ECCO_OK) {
        delete m;
        return ECCO_EFORMAT;
    }
    *out = m;
    return ECCO_OK;
}

}  // extern "C"
