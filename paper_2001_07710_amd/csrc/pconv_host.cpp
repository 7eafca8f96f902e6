// Host side of libpconv: argument checks, pattern assignment, connectivity selection, packing, export.
// Pure C++ (no HIP calls here); the device upload lives in pconv_device.hip.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <numeric>

#include "pconv_internal.h"

namespace {

inline int popcount9(unsigned m) { return __builtin_popcount(m & 0x1FFu); }

// Library check shared by every entry point: K in [1,126], every mask a 9-bit value with exactly four bits
// (section 5.1 of the paper: four non-zero entries per kernel, at most C(9,4) = 126 masks).
int check_library(const uint16_t* lib, int K) {
    if (!lib) return PCONV_EINVAL;
    if (K < 1 || K > 126) return PCONV_EPATTERN;
    for (int j = 0; j < K; ++j)
        if (lib[j] >= 512u || popcount9(lib[j]) != 4) return PCONV_EPATTERN;
    return PCONV_OK;
}

int check_fc(int F, int C) {
    if (F <= 0 || C <= 0 || C >= 65536) return PCONV_ESHAPE;
    if ((long long)F * (long long)C > (1ll << 31) / 9) return PCONV_ESHAPE;
    return PCONV_OK;
}

// IEEE binary16 -> binary32, exact (subnormals, infinities and NaN payloads included).
inline float half_bits_to_float(uint16_t h) {
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1Fu, man = h & 0x3FFu, out;
    if (exp == 0) {
        if (man == 0) {
            out = sign;
        } else {
            int e = -1;
            do {
                man <<= 1;
                ++e;
            } while (!(man & 0x400u));
            out = sign | ((uint32_t)(127 - 15 - e) << 23) | ((man & 0x3FFu) << 13);
        }
    } else if (exp == 31) {
        out = sign | 0x7F800000u | (man << 13);
    } else {
        out = sign | ((exp + 112u) << 23) | (man << 13);
    }
    float f;
    std::memcpy(&f, &out, 4);
    return f;
}

// Rank of a four-bit mask among the 126 such masks in ascending order (the pattern code of the device layout).
inline uint32_t mask_rank(unsigned m) {
    uint32_t rank = 0;
    for (unsigned v = 0; v < m; ++v)
        if (popcount9(v) == 4) ++rank;
    return rank;
}

// Retained squared norm of one kernel under one mask: squares in double, added in ascending tap order.
inline double retained(const float* k9, unsigned m) {
    double acc = 0.0;
    bool first = true;
    for (int t = 0; t < 9; ++t) {
        if (!((m >> t) & 1u)) continue;
        const double v = (double)k9[t];
        const double sq = v * v;
        acc = first ? sq : acc + sq;
        first = false;
    }
    return acc;
}

}  // namespace

extern "C" int pconv_assign_patterns(const float* w, int F, int C, const uint16_t* lib, int K, uint8_t* pid_out) {
    if (!w || !pid_out) return PCONV_EINVAL;
    if (int rc = check_library(lib, K)) return rc;
    if (int rc = check_fc(F, C)) return rc;
    const long long n = (long long)F * C;
    for (long long i = 0; i < n; ++i) {
        const float* k9 = w + i * 9;
        int best = 0;
        double best_e = retained(k9, lib[0]);
        for (int j = 1; j < K; ++j) {
            const double e = retained(k9, lib[j]);
            if (e > best_e) {
                best_e = e;
                best = j;
            }
        }
        pid_out[i] = (uint8_t)best;
    }
    return PCONV_OK;
}

extern "C" int pconv_select_connectivity(const float* w, int F, int C, const uint16_t* lib, int K, const uint8_t* pid,
                                         double keep, uint8_t* mask_out) {
    if (!w || !pid || !mask_out) return PCONV_EINVAL;
    if (int rc = check_library(lib, K)) return rc;
    if (int rc = check_fc(F, C)) return rc;
    if (!(keep >= 0.0 && keep <= 1.0)) return PCONV_EINVAL;
    const long long n = (long long)F * C;
    for (long long i = 0; i < n; ++i)
        if (pid[i] >= K) return PCONV_EPATTERN;
    std::vector<double> score;
    std::vector<uint32_t> idx;
    try {
        score.resize((size_t)n);
        idx.resize((size_t)n);
    } catch (const std::bad_alloc&) {
        return PCONV_ENOMEM;
    }
    for (long long i = 0; i < n; ++i) score[(size_t)i] = retained(w + i * 9, lib[pid[i]]);
    std::iota(idx.begin(), idx.end(), 0u);
    long long k = (long long)std::floor(keep * (double)n + 0.5);
    k = std::max(0ll, std::min(k, n));
    auto before = [&](uint32_t a, uint32_t b) {
        if (score[a] != score[b]) return score[a] > score[b];
        return a < b;
    };
    if (k > 0 && k < n) std::nth_element(idx.begin(), idx.begin() + (k - 1), idx.end(), before);
    std::memset(mask_out, 0, (size_t)n);
    for (long long i = 0; i < k; ++i) mask_out[idx[(size_t)i]] = 1;
    return PCONV_OK;
}

extern "C" int pconv_pack(const void* w_oihw, int dtype, int F, int C, const uint16_t* lib, int K, const uint8_t* pid,
                          const uint8_t* mask, unsigned flags, pconv_packed** out) {
    if (!out) return PCONV_EINVAL;
    *out = nullptr;
    if (!w_oihw || !pid || !mask) return PCONV_EINVAL;
    if (dtype != PCONV_F32 && dtype != PCONV_F16) return PCONV_EINVAL;
    if (flags & ~(unsigned)PCONV_PACK_HOST_ONLY) return PCONV_EINVAL;
    if (int rc = check_library(lib, K)) return rc;
    if (int rc = check_fc(F, C)) return rc;
    const size_t esize = dtype == PCONV_F16 ? 2 : 4;
    const unsigned char* wb = static_cast<const unsigned char*>(w_oihw);

    for (long long i = 0; i < (long long)F * C; ++i)
        if (mask[i] && pid[i] >= K) return PCONV_EPATTERN;

    pconv_packed* p = new (std::nothrow) pconv_packed;
    if (!p) return PCONV_ENOMEM;
    try {
        p->F = F;
        p->C = C;
        p->K = K;
        p->dtype = dtype;
        p->lib.assign(lib, lib + K);

        // taps of every mask, ascending
        std::vector<int> taps((size_t)K * 4);
        for (int j = 0; j < K; ++j) {
            int q = 0;
            for (int t = 0; t < 9; ++t)
                if ((lib[j] >> t) & 1u) taps[(size_t)j * 4 + q++] = t;
        }

        // filter order: kept-kernel count descending, filter index ascending
        std::vector<uint32_t> count((size_t)F, 0);
        size_t n_kept = 0;
        for (int f = 0; f < F; ++f) {
            uint32_t n = 0;
            for (int c = 0; c < C; ++c) n += mask[(size_t)f * C + c] ? 1u : 0u;
            count[(size_t)f] = n;
            n_kept += n;
        }
        p->n_kept = n_kept;
        p->filter_order.resize((size_t)F);
        std::iota(p->filter_order.begin(), p->filter_order.end(), 0u);
        std::stable_sort(p->filter_order.begin(), p->filter_order.end(),
                         [&](uint32_t a, uint32_t b) { return count[a] > count[b]; });

        // canonical arrays: per (position i, pattern j) the kept kernels in ascending channel
        p->grp_ptr.assign((size_t)F * K + 1, 0);
        p->cin.resize(n_kept);
        p->w4.resize(n_kept * 4 * esize);
        size_t e = 0;
        for (int i = 0; i < F; ++i) {
            const uint32_t f = p->filter_order[(size_t)i];
            for (int j = 0; j < K; ++j) {
                p->grp_ptr[(size_t)i * K + j] = (uint32_t)e;
                for (int c = 0; c < C; ++c) {
                    const size_t fc = (size_t)f * C + c;
                    if (!mask[fc] || pid[fc] != j) continue;
                    p->cin[e] = (uint16_t)c;
                    for (int q = 0; q < 4; ++q)
                        std::memcpy(&p->w4[(e * 4 + q) * esize], wb + (fc * 9 + taps[(size_t)j * 4 + q]) * esize, esize);
                    ++e;
                }
            }
        }
        p->grp_ptr[(size_t)F * K] = (uint32_t)e;

        // device layout, derived from the canonical one: per (position i, channel bucket) the entries by pattern,
        // then channel; weights widened to fp32
        const int chunk = pconv::kBucket;
        p->n_buckets = (C + chunk - 1) / chunk;
        p->ent.resize(n_kept);
        p->eptr.assign((size_t)F * p->n_buckets + 1, 0);
        std::vector<uint32_t> cursor((size_t)K);
        size_t d = 0;
        for (int i = 0; i < F; ++i) {
            for (int j = 0; j < K; ++j) cursor[(size_t)j] = p->grp_ptr[(size_t)i * K + j];
            for (int k = 0; k < p->n_buckets; ++k) {
                p->eptr[(size_t)i * p->n_buckets + k] = (uint32_t)d;
                const int c_end = std::min(C, (k + 1) * chunk);
                for (int j = 0; j < K; ++j) {
                    const uint32_t g_end = p->grp_ptr[(size_t)i * K + j + 1];
                    uint32_t& cur = cursor[(size_t)j];
                    while (cur < g_end && (int)p->cin[cur] < c_end) {
                        pconv::DevEntry& de = p->ent[d++];
                        for (int q = 0; q < 4; ++q) {
                            if (dtype == PCONV_F16) {
                                uint16_t hb;
                                std::memcpy(&hb, &p->w4[((size_t)cur * 4 + q) * 2], 2);
                                de.w[q] = half_bits_to_float(hb);
                            } else {
                                std::memcpy(&de.w[q], &p->w4[((size_t)cur * 4 + q) * 4], 4);
                            }
                        }
                        de.c = p->cin[cur];
                        de.mask9 = lib[j];
                        de.code = mask_rank(lib[j]);
                        de.joff = de.code * (uint32_t)pconv::kLeafStride;
                        ++cur;
                    }
                }
            }
        }
        p->eptr[(size_t)F * p->n_buckets] = (uint32_t)d;
    } catch (const std::bad_alloc&) {
        delete p;
        return PCONV_ENOMEM;
    }

    if (!(flags & PCONV_PACK_HOST_ONLY)) {
        const int rc = pconv::upload_packed(p);
        if (rc != PCONV_OK) {
            pconv::release_device(p);
            delete p;
            return rc;
        }
    }
    *out = p;
    return PCONV_OK;
}

extern "C" int pconv_packed_export(const pconv_packed* p, uint32_t* filter_order, uint32_t* grp_ptr, uint16_t* cin,
                                   void* w4, size_t* n_kept) {
    if (!p) return PCONV_EINVAL;
    if (filter_order) std::memcpy(filter_order, p->filter_order.data(), p->filter_order.size() * sizeof(uint32_t));
    if (grp_ptr) std::memcpy(grp_ptr, p->grp_ptr.data(), p->grp_ptr.size() * sizeof(uint32_t));
    if (cin && !p->cin.empty()) std::memcpy(cin, p->cin.data(), p->cin.size() * sizeof(uint16_t));
    if (w4 && !p->w4.empty()) std::memcpy(w4, p->w4.data(), p->w4.size());
    if (n_kept) *n_kept = p->n_kept;
    return PCONV_OK;
}

extern "C" int pconv_packed_stats(const pconv_packed* p, int* F, int* C, int* K, int* dtype, size_t* n_kept) {
    if (!p) return PCONV_EINVAL;
    if (F) *F = p->F;
    if (C) *C = p->C;
    if (K) *K = p->K;
    if (dtype) *dtype = p->dtype;
    if (n_kept) *n_kept = p->n_kept;
    return PCONV_OK;
}

extern "C" void pconv_free(pconv_packed* p) {
    if (!p) return;
    pconv::release_device(p);
    delete p;
}

extern "C" const char* pconv_strerror(int code) {
    switch (code) {
        case PCONV_OK: return "ok";
        case PCONV_EINVAL: return "invalid argument (null pointer, bad enum or flag)";
        case PCONV_EPATTERN: return "bad pattern library or pattern id (masks need exactly four of nine bits, 1 <= K <= 126, id < K)";
        case PCONV_ESHAPE: return "bad shape (non-positive extent, C >= 65536, empty output or size overflow)";
        case PCONV_EUNSUPPORTED: return "unsupported stride (1 or 2) or pad (0 or 1)";
        case PCONV_ENOMEM: return "out of memory";
        case PCONV_EHIP: return "HIP runtime error (see pconv_last_hip_error)";
        case PCONV_ESTATE: return "packed handle has no device copy (packed host-only) or belongs to another device";
        default: return "unknown pconv error code";
    }
}
