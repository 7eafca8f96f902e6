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

// The library of a layer re-packed over parity planes: any masks with one to four bits.
int check_partial_library(const uint16_t* lib, int K) {
    if (!lib) return PCONV_EINVAL;
    if (K < 1 || K > 255) return PCONV_EPATTERN;
    for (int j = 0; j < K; ++j)
        if (lib[j] >= 512u || popcount9(lib[j]) < 1 || popcount9(lib[j]) > 4) return PCONV_EPATTERN;
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

// Rank of a mask among the 255 masks with one to four bits in ascending order (the pattern code of the device
// layout: the tiled kernel has one code section per such mask).
inline uint32_t mask_rank(unsigned m) {
    uint32_t rank = 0;
    for (unsigned v = 1; v < m; ++v)
        if (popcount9(v) >= 1 && popcount9(v) <= 4) ++rank;
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

namespace {

// Builds the balanced layout of `p` for one tiling (see pconv::BalancedLayout).
void build_balanced(const pconv_packed* p, int fw, int nf, int cc, pconv::BalancedLayout* out) {
    const int F = p->F, C = p->C, K = p->K;
    const int fg = fw * nf;
    out->fw = fw;
    out->nf = nf;
    out->cc = cc;
    out->n_groups = (F + fg - 1) / fg;
    out->n_chunks = (C + cc - 1) / cc;
    const int nch = out->n_chunks, npos = nch * cc;
    out->perm.assign((size_t)out->n_groups * npos, pconv::kNoChannel);
    out->ent.resize(p->n_kept);
    out->eptr.assign((size_t)F * nch + 1, 0);

    // kept kernels of every filter position as (channel, canonical entry index), from the canonical arrays
    std::vector<std::vector<std::pair<uint16_t, uint32_t>>> kept((size_t)F);
    for (int i = 0; i < F; ++i)
        for (uint32_t e = p->grp_ptr[(size_t)i * K]; e < p->grp_ptr[(size_t)(i + 1) * K]; ++e)
            kept[(size_t)i].push_back({p->cin[e], e});
    std::vector<uint8_t> pattern_of(p->n_kept);
    for (int i = 0; i < F; ++i)
        for (int j = 0; j < K; ++j)
            for (uint32_t e = p->grp_ptr[(size_t)i * K + j]; e < p->grp_ptr[(size_t)i * K + j + 1]; ++e)
                pattern_of[e] = (uint8_t)j;

    std::vector<uint32_t> pos_of((size_t)C);          // position of a channel in the group's staging order
    std::vector<std::vector<uint8_t>> uses;           // [wave][channel] kept kernels of the wave's filters
    size_t d = 0;
    std::vector<std::vector<std::pair<uint32_t, uint32_t>>> per_chunk;   // scratch: (sort key, entry) per chunk
    // entries must be emitted in filter-position order; groups are consecutive positions, so go group by group
    for (int g = 0; g < out->n_groups; ++g) {
        const int i0 = g * fg, i1 = std::min(F, i0 + fg);
        uses.assign((size_t)fw, std::vector<uint8_t>((size_t)C, 0));
        std::vector<uint32_t> weight((size_t)C, 0);
        for (int i = i0; i < i1; ++i) {
            const int w = (i - i0) % fw;                 // wave w holds positions i0 + w + a*fw
            for (auto& ce : kept[(size_t)i]) {
                ++uses[(size_t)w][ce.first];
                ++weight[ce.first];
            }
        }
        // channels by decreasing number of users (unused ones are dropped), then index
        std::vector<uint32_t> order;
        for (int c = 0; c < C; ++c)
            if (weight[(size_t)c]) order.push_back((uint32_t)c);
        std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return weight[a] > weight[b]; });
        // greedy vector bin packing: put each channel into the chunk where the busiest wave stays least busy
        std::vector<std::vector<uint32_t>> load((size_t)nch, std::vector<uint32_t>((size_t)fw, 0));
        std::vector<uint32_t> fill((size_t)nch, 0), total((size_t)nch, 0);
        std::vector<std::vector<uint32_t>> members((size_t)nch);
        for (uint32_t c : order) {
            int best = -1;
            uint32_t best_max = 0, best_total = 0;
            for (int k = 0; k < nch; ++k) {
                if ((int)fill[(size_t)k] >= cc) continue;
                uint32_t mx = 0;
                for (int w = 0; w < fw; ++w) mx = std::max(mx, load[(size_t)k][(size_t)w] + uses[(size_t)w][c]);
                if (best < 0 || mx < best_max || (mx == best_max && total[(size_t)k] < best_total)) {
                    best = k;
                    best_max = mx;
                    best_total = total[(size_t)k];
                }
            }
            for (int w = 0; w < fw; ++w) load[(size_t)best][(size_t)w] += uses[(size_t)w][c];
            total[(size_t)best] += weight[c];
            ++fill[(size_t)best];
            members[(size_t)best].push_back(c);
        }
        for (int k = 0; k < nch; ++k) {
            std::sort(members[(size_t)k].begin(), members[(size_t)k].end());
            for (size_t m = 0; m < members[(size_t)k].size(); ++m) {
                const uint32_t c = members[(size_t)k][m];
                pos_of[c] = (uint32_t)(k * cc + (int)m);
                out->perm[(size_t)g * npos + pos_of[c]] = c;
            }
        }
        // entries of the group's filters: by chunk, then pattern, then position
        for (int i = i0; i < i1; ++i) {
            per_chunk.assign((size_t)nch, {});
            for (auto& ce : kept[(size_t)i]) {
                const uint32_t pos = pos_of[ce.first];
                per_chunk[pos / (uint32_t)cc].push_back({((uint32_t)pattern_of[ce.second] << 20) | pos, ce.second});
            }
            for (int k = 0; k < nch; ++k) {
                out->eptr[(size_t)i * nch + k] = (uint32_t)d;
                auto& v = per_chunk[(size_t)k];
                std::sort(v.begin(), v.end());
                for (auto& ke : v) {
                    pconv::DevEntry de = p->ent[p->ent_of_canonical[ke.second]];
                    de.c = ke.first & 0xFFFFFu;
                    de.hdr = (de.c & 0xFFu) | (de.code << 8);
                    out->ent[d++] = de;
                }
            }
        }
    }
    out->eptr[(size_t)F * nch] = (uint32_t)d;
}

// The layer's weights in matrix-core order for workgroup tiles of mt filters (see pconv::MfmaWeights), from the
// canonical arrays.  fp16 storage only: the 16-bit patterns are copied as they are.
void build_mfma_weights(const pconv_packed* p, int mt, int groups, pconv::MfmaWeights* out) {
    const int F = p->F, C = p->C, K = p->K;
    out->mt = mt;
    out->groups = groups;
    out->n_mtiles = (F + mt - 1) / mt;
    out->n_cblocks = (C / groups + 15) / 16;
    // taps that occur: the union of the masks of the patterns that have kept kernels
    unsigned present = 0;
    for (int i = 0; i < F; ++i)
        for (int j = 0; j < K; ++j)
            if (p->grp_ptr[(size_t)i * K + j + 1] > p->grp_ptr[(size_t)i * K + j]) present |= p->lib[(size_t)j];
    int slot_of[9];
    out->n_taps = 0;
    for (int t = 0; t < 9; ++t) {
        slot_of[t] = -1;
        if ((present >> t) & 1u) {
            slot_of[t] = out->n_taps;
            out->taps[out->n_taps++] = (uint8_t)t;
        }
    }
    // (channel ranges in the place of taps: as many tap slots as ranges, all of them the layer's one tap)
    if (groups > 1) {
        for (int g = 1; g < groups; ++g) out->taps[g] = out->taps[0];
        out->n_taps = groups;
    }
    const int nt = out->n_taps;
    const size_t group_channels = (size_t)(C / groups);
    // Channels that the filters of every tile keep.  Lists are made where they save at least a tenth of the blocks;
    // otherwise every tile takes all channels in their own order.
    std::vector<std::vector<uint8_t>> used((size_t)out->n_mtiles, std::vector<uint8_t>((size_t)C, 0));
    for (int i = 0; i < F; ++i) {
        const uint32_t f = p->filter_order[(size_t)i];
        for (uint32_t e = p->grp_ptr[(size_t)i * K]; e < p->grp_ptr[(size_t)(i + 1) * K]; ++e)
            used[f / (uint32_t)mt][p->cin[e]] = 1;
    }
    std::vector<std::vector<uint32_t>> pos_of((size_t)out->n_mtiles);     // with lists: position of a channel in its tile
    std::vector<size_t> first_block((size_t)out->n_mtiles, 0);
    size_t listed = 0;
    for (int t = 0; t < out->n_mtiles; ++t) {
        size_t n = 0;
        for (int c = 0; c < C; ++c) n += used[(size_t)t][(size_t)c];
        listed += std::max<size_t>(1, (n + 15) / 16);
    }
    const bool lists = groups == 1 && listed * 10 <= (size_t)out->n_mtiles * out->n_cblocks * 9;
    out->clist.clear();
    out->tinfo.clear();
    out->min_blocks = out->n_cblocks;
    out->total_blocks = out->n_mtiles * out->n_cblocks;
    if (lists) {
        out->min_blocks = 1 << 30;
        size_t at_block = 0;
        for (int t = 0; t < out->n_mtiles; ++t) {
            pos_of[(size_t)t].assign((size_t)C, 0);
            size_t n = 0;
            for (int c = 0; c < C; ++c)
                if (used[(size_t)t][(size_t)c]) {
                    pos_of[(size_t)t][(size_t)c] = (uint32_t)n++;
                    out->clist.push_back((uint32_t)c);
                }
            const size_t nb = std::max<size_t>(1, (n + 15) / 16);
            out->clist.resize((at_block + nb) * 16, pconv::kNoChannel);
            out->tinfo.push_back((uint32_t)nb);
            out->tinfo.push_back((uint32_t)at_block);
            first_block[(size_t)t] = at_block;
            out->min_blocks = std::min(out->min_blocks, (int)nb);
            at_block += nb;
        }
        out->total_blocks = (int)at_block;
    } else {
        for (int t = 0; t < out->n_mtiles; ++t) first_block[(size_t)t] = (size_t)t * out->n_cblocks;
    }
    out->w.assign((size_t)out->total_blocks * nt * 2 * mt * 8, 0);
    for (int i = 0; i < F; ++i) {
        const uint32_t f = p->filter_order[(size_t)i];
        const size_t tile = f / (uint32_t)mt, fl = f % (uint32_t)mt;
        for (int j = 0; j < K; ++j) {
            int taps[4], q = 0;
            for (int t = 0; t < 9; ++t)
                if ((p->lib[(size_t)j] >> t) & 1u) taps[q++] = t;
            for (uint32_t e = p->grp_ptr[(size_t)i * K + j]; e < p->grp_ptr[(size_t)i * K + j + 1]; ++e) {
                size_t c = lists ? pos_of[tile][p->cin[e]] : p->cin[e];      // position among the tile's channels
                const size_t range = groups > 1 ? c / group_channels : 0;
                if (groups > 1) c -= range * group_channels;
                const size_t cb = c / 16, kb = (c % 16) / 8, c8 = c % 8;
                for (int k = 0; k < q; ++k) {
                    const size_t ts = groups > 1 ? range : (size_t)slot_of[taps[k]];
                    const size_t at = ((((first_block[tile] + cb) * nt + ts) * 2 + kb) * mt + fl) * 8 + c8;
                    std::memcpy(&out->w[at], &p->w4[((size_t)e * 4 + k) * 2], 2);
                }
            }
        }
    }
}

}  // namespace

// pconv_pack, and the packing of a layer re-packed over parity planes (`partial`: masks of one to four taps, up to
// 255 of them; missing taps of a kernel are stored as zero weights).
static int pack_impl(const void* w_oihw, int dtype, int F, int C, const uint16_t* lib, int K, const uint8_t* pid,
                     const uint8_t* mask, unsigned flags, bool partial, bool want_mfma, pconv_packed** out,
                     bool one_by_one = false) {
    if (!out) return PCONV_EINVAL;
    *out = nullptr;
    if (!w_oihw || !pid || !mask) return PCONV_EINVAL;
    if (dtype != PCONV_F32 && dtype != PCONV_F16) return PCONV_EINVAL;
    if (flags & ~(unsigned)PCONV_PACK_HOST_ONLY) return PCONV_EINVAL;
    if (int rc = partial ? check_partial_library(lib, K) : check_library(lib, K)) return rc;
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

        // taps of every mask, ascending (-1: the mask has fewer than four)
        std::vector<int> taps((size_t)K * 4, -1);
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
                    for (int q = 0; q < 4; ++q) {
                        const int t = taps[(size_t)j * 4 + q];
                        if (t >= 0) std::memcpy(&p->w4[(e * 4 + q) * esize], wb + (fc * 9 + t) * esize, esize);
                        else std::memset(&p->w4[(e * 4 + q) * esize], 0, esize);
                    }
                    ++e;
                }
            }
        }
        p->grp_ptr[(size_t)F * K] = (uint32_t)e;
        p->canon.resize(n_kept * 2);
        for (int i = 0; i < F; ++i)
            for (int j = 0; j < K; ++j)
                for (uint32_t q = p->grp_ptr[(size_t)i * K + j]; q < p->grp_ptr[(size_t)i * K + j + 1]; ++q) {
                    p->canon[(size_t)q * 2] = p->filter_order[(size_t)i];
                    p->canon[(size_t)q * 2 + 1] = (uint32_t)p->cin[q] | ((uint32_t)lib[j] << 16);
                }

        // device layout, derived from the canonical one: per (position i, channel bucket) the entries by pattern,
        // then channel; weights widened to fp32
        const int chunk = pconv::kBucket;
        p->n_buckets = (C + chunk - 1) / chunk;
        p->ent.resize(n_kept);
        p->ent_of_canonical.resize(n_kept);
        p->eptr.assign((size_t)F * p->n_buckets + 1, 0);
        std::vector<uint32_t> cursor((size_t)K), code_of((size_t)K);
        for (int j = 0; j < K; ++j) code_of[(size_t)j] = mask_rank(lib[j]);
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
                        p->ent_of_canonical[cur] = (uint32_t)d;
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
                        de.code = code_of[(size_t)j];
                        de.hdr = (de.c & 0xFFu) | (de.code << 8);
                        ++cur;
                    }
                }
            }
        }
        p->eptr[(size_t)F * p->n_buckets] = (uint32_t)d;

        // balanced layouts for the tilings of the automatic choice (waves, filters per wave, channels per chunk);
        // the 16-channel ones are the quad kernel's
        static const int tilings[5][3] = {{16, 2, 32}, {16, 1, 32}, {8, 1, 32}, {16, 2, 16}, {16, 1, 16}};
        p->balanced.resize(5);
        for (int t = 0; t < 5; ++t)
            build_balanced(p, tilings[t][0], tilings[t][1], tilings[t][2], &p->balanced[(size_t)t]);
        if (dtype == PCONV_F16 && want_mfma) {
            const int nh = (int)(sizeof(pconv::kMfmaTileHeights) / sizeof(int));
            p->mfma.resize((size_t)nh);
            for (int h = 0; h < nh; ++h) build_mfma_weights(p, pconv::kMfmaTileHeights[h], 1, &p->mfma[(size_t)h]);
            // (a 1x1 layer is bound by the round trips of its many short channel blocks: kept a second time with
            // several channel ranges per block)
            if (one_by_one && K == 1 && C % (16 * pconv::kOneByOneGroups) == 0) {
                p->mfma.resize((size_t)(2 * nh));
                for (int h = 0; h < nh; ++h)
                    build_mfma_weights(p, pconv::kMfmaTileHeights[h], pconv::kOneByOneGroups, &p->mfma[(size_t)(nh + h)]);
            }
        }
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

extern "C" int pconv_pack(const void* w_oihw, int dtype, int F, int C, const uint16_t* lib, int K, const uint8_t* pid,
                          const uint8_t* mask, unsigned flags, pconv_packed** out) {
    return pack_impl(w_oihw, dtype, F, C, lib, K, pid, mask, flags, false, true, out);
}

// Bit t = 3*ky + kx of a mask moved to 3*(2-ky) + (2-kx) = 8 - t: the kernel rotated by 180 degrees.
static inline uint16_t rotate_mask(uint16_t m) {
    unsigned r = 0;
    for (int t = 0; t < 9; ++t)
        if ((m >> t) & 1u) r |= 1u << (8 - t);
    return (uint16_t)r;
}

extern "C" int pconv_packed_transpose(const pconv_packed* p, unsigned flags, pconv_packed** out) {
    if (!out) return PCONV_EINVAL;
    *out = nullptr;
    if (!p) return PCONV_EINVAL;
    if (flags & ~(unsigned)PCONV_PACK_HOST_ONLY) return PCONV_EINVAL;
    if (check_library(p->lib.data(), p->K) != PCONV_OK || p->is_1x1) return PCONV_EUNSUPPORTED;   // (a derived form)
    const int F = p->F, C = p->C, K = p->K;
    if (F >= 65536) return PCONV_ESHAPE;                 // (the filters become the input channels: 16-bit indices)
    const size_t esize = p->dtype == PCONV_F16 ? 2 : 4;
    try {
        std::vector<uint16_t> lib((size_t)K);
        for (int j = 0; j < K; ++j) lib[(size_t)j] = rotate_mask(p->lib[(size_t)j]);
        std::vector<unsigned char> w((size_t)C * F * 9 * esize, 0);
        std::vector<uint8_t> pid((size_t)C * F, 0), mask((size_t)C * F, 0);
        for (int i = 0; i < F; ++i) {
            const uint32_t f = p->filter_order[(size_t)i];
            for (int j = 0; j < K; ++j) {
                int taps[4], q = 0;
                for (int t = 0; t < 9; ++t)
                    if ((p->lib[(size_t)j] >> t) & 1u) taps[q++] = t;
                for (uint32_t e = p->grp_ptr[(size_t)i * K + j]; e < p->grp_ptr[(size_t)i * K + j + 1]; ++e) {
                    const size_t cf = (size_t)p->cin[e] * F + f;
                    pid[cf] = (uint8_t)j;
                    mask[cf] = 1;
                    for (int k = 0; k < 4; ++k)
                        std::memcpy(&w[(cf * 9 + (size_t)(8 - taps[k])) * esize], &p->w4[((size_t)e * 4 + k) * esize], esize);
                }
            }
        }
        return pack_impl(w.data(), p->dtype, C, F, lib.data(), K, pid.data(), mask.data(), flags, false, true, out);
    } catch (const std::bad_alloc&) {
        return PCONV_ENOMEM;
    }
}

extern "C" int pconv_pack_1x1(const void* w_fc, int dtype, int F, int C, const uint16_t* lib, int K, const uint8_t* pid,
                              const uint8_t* mask, unsigned flags, pconv_packed** out) {
    if (!out) return PCONV_EINVAL;
    *out = nullptr;
    if (!w_fc || !pid || !mask) return PCONV_EINVAL;
    if (dtype != PCONV_F32 && dtype != PCONV_F16) return PCONV_EINVAL;
    if (int rc = check_library(lib, K)) return rc;
    if (int rc = check_fc(F, C)) return rc;
    const int G = (C + 8) / 9;
    for (long long i = 0; i < (long long)F * G; ++i)
        if (mask[i] && pid[i] >= K) return PCONV_EPATTERN;
    const size_t esize = dtype == PCONV_F16 ? 2 : 4;
    const unsigned char* wb = static_cast<const unsigned char*>(w_fc);
    try {
        // the same layer as a 3x3 layer whose kernels keep their centre tap only: kernel (f,c) exists where channel c
        // is a kept position of its group's pattern
        std::vector<unsigned char> w9((size_t)F * C * 9 * esize, 0);
        std::vector<uint8_t> pid9((size_t)F * C, 0), mask9((size_t)F * C, 0);
        for (int f = 0; f < F; ++f)
            for (int c = 0; c < C; ++c) {
                const size_t fg = (size_t)f * G + (size_t)(c / 9);
                if (!mask[fg] || !((lib[pid[fg]] >> (c % 9)) & 1u)) continue;
                const size_t fc = (size_t)f * C + c;
                mask9[fc] = 1;
                std::memcpy(&w9[(fc * 9 + 4) * esize], wb + fc * esize, esize);
            }
        const uint16_t centre = 0x010;
        const int rc = pack_impl(w9.data(), dtype, F, C, &centre, 1, pid9.data(), mask9.data(), flags, true, true, out, true);
        if (rc == PCONV_OK) (*out)->is_1x1 = true;
        return rc;
    } catch (const std::bad_alloc&) {
        return PCONV_ENOMEM;
    }
}

int pconv::derive_for_stride2(const pconv_packed* p, int pad, bool upload, pconv_packed** out) {
    if (!p || !out || (pad != 0 && pad != 1)) return PCONV_EINVAL;
    *out = nullptr;
    const int F = p->F, C = p->C, K = p->K, C4 = 4 * C;
    if (C4 >= 65536) return PCONV_EUNSUPPORTED;
    const size_t esize = p->dtype == PCONV_F16 ? 2 : 4;
    try {
        // where tap t of a kernel goes: plane (0..3) and tap inside the plane's kernel
        int plane_of[9], tap_of[9];
        for (int t = 0; t < 9; ++t) {
            const int dy = t / 3 - pad, dx = t % 3 - pad;            // -1..2
            const int a = dy & 1, b = dx & 1;                          // parity (two's complement: -1 & 1 == 1)
            const int ky = (dy - a) / 2 + pad, kx = (dx - b) / 2 + pad;   // floor(d/2) + pad, in {0,1}
            plane_of[t] = 2 * a + b;
            tap_of[t] = 3 * ky + kx;
        }
        std::vector<unsigned char> w((size_t)F * C4 * 9 * esize, 0);
        std::vector<uint16_t> m9((size_t)F * C4, 0);
        for (int i = 0; i < F; ++i) {
            const uint32_t f = p->filter_order[(size_t)i];
            for (int j = 0; j < K; ++j) {
                int taps[4], q = 0;
                for (int t = 0; t < 9; ++t)
                    if ((p->lib[(size_t)j] >> t) & 1u) taps[q++] = t;
                for (uint32_t e = p->grp_ptr[(size_t)i * K + j]; e < p->grp_ptr[(size_t)i * K + j + 1]; ++e) {
                    const size_t c = p->cin[e];
                    for (int k = 0; k < q; ++k) {          // (q < 4: a layer whose kernels keep fewer taps, the 1x1 form)
                        const size_t fc = (size_t)f * C4 + 4 * c + (size_t)plane_of[taps[k]];
                        std::memcpy(&w[(fc * 9 + (size_t)tap_of[taps[k]]) * esize], &p->w4[((size_t)e * 4 + k) * esize], esize);
                        m9[fc] |= (uint16_t)(1u << tap_of[taps[k]]);
                    }
                }
            }
        }
        // library of the re-packed layer: the masks that occur, ascending
        std::vector<int> index_of(512, -1);
        std::vector<uint16_t> lib;
        std::vector<char> used(512, 0);
        for (size_t i = 0; i < m9.size(); ++i) used[m9[i]] = 1;
        for (unsigned v = 1; v < 512; ++v)
            if (used[v]) {
                index_of[v] = (int)lib.size();
                lib.push_back((uint16_t)v);
            }
        if (lib.empty()) lib.push_back(1);   // a layer with nothing kept
        std::vector<uint8_t> pid(m9.size(), 0), mask(m9.size(), 0);
        for (size_t i = 0; i < m9.size(); ++i)
            if (m9[i]) {
                pid[i] = (uint8_t)index_of[m9[i]];
                mask[i] = 1;
            }
        return pack_impl(w.data(), p->dtype, F, C4, lib.data(), (int)lib.size(), pid.data(), mask.data(),
                         upload ? 0u : (unsigned)PCONV_PACK_HOST_ONLY, true, false, out);
    } catch (const std::bad_alloc&) {
        return PCONV_ENOMEM;
    }
}

extern "C" int pconv_filter_similarity_order(const uint8_t* mask, int F, int C, int group, uint32_t* order_out) {
    if (!mask || !order_out) return PCONV_EINVAL;
    if (int rc = check_fc(F, C)) return rc;
    if (group < 1) return PCONV_EINVAL;
    try {
        // the channels every filter keeps, as bit sets
        const size_t words = ((size_t)C + 63) / 64;
        std::vector<uint64_t> support((size_t)F * words, 0);
        std::vector<uint32_t> count((size_t)F, 0);
        for (int f = 0; f < F; ++f)
            for (int c = 0; c < C; ++c)
                if (mask[(size_t)f * C + c]) {
                    support[(size_t)f * words + (size_t)c / 64] |= 1ull << (c % 64);
                    ++count[(size_t)f];
                }
        std::vector<char> taken((size_t)F, 0);
        std::vector<uint64_t> uni(words);
        int placed = 0;
        while (placed < F) {
            // a group starts with the filter that keeps the most kernels (lowest index among equals) ...
            int seed = -1;
            for (int f = 0; f < F; ++f)
                if (!taken[(size_t)f] && (seed < 0 || count[(size_t)f] > count[(size_t)seed])) seed = f;
            taken[(size_t)seed] = 1;
            order_out[placed++] = (uint32_t)seed;
            std::copy(support.begin() + (size_t)seed * words, support.begin() + (size_t)(seed + 1) * words, uni.begin());
            // ... and takes, one at a time, the filter that adds the fewest channels to the group's union; among
            // equals the one that shares the most with it, then the lowest index
            for (int k = 1; k < group && placed < F; ++k) {
                int best = -1;
                uint32_t best_add = 0, best_share = 0;
                for (int f = 0; f < F; ++f) {
                    if (taken[(size_t)f]) continue;
                    uint32_t add = 0, share = 0;
                    const uint64_t* sf = &support[(size_t)f * words];
                    for (size_t w = 0; w < words; ++w) {
                        add += (uint32_t)__builtin_popcountll(sf[w] & ~uni[w]);
                        share += (uint32_t)__builtin_popcountll(sf[w] & uni[w]);
                    }
                    if (best < 0 || add < best_add || (add == best_add && share > best_share)) {
                        best = f;
                        best_add = add;
                        best_share = share;
                    }
                }
                taken[(size_t)best] = 1;
                order_out[placed++] = (uint32_t)best;
                const uint64_t* sb = &support[(size_t)best * words];
                for (size_t w = 0; w < words; ++w) uni[w] |= sb[w];
            }
        }
    } catch (const std::bad_alloc&) {
        return PCONV_ENOMEM;
    }
    return PCONV_OK;
}

extern "C" int pconv_packed_mfma_blocks(const pconv_packed* p, int tile_filters, int* listed_blocks, int* all_blocks) {
    if (!p) return PCONV_EINVAL;
    for (const pconv::MfmaWeights& m : p->mfma)
        if (m.mt == tile_filters) {
            if (listed_blocks) *listed_blocks = m.total_blocks;
            if (all_blocks) *all_blocks = m.n_mtiles * m.n_cblocks;
            return PCONV_OK;
        }
    return PCONV_EUNSUPPORTED;
}

extern "C" int pconv_packed_parity_form(const pconv_packed* p, int pad, pconv_packed** out) {
    return pconv::derive_for_stride2(p, pad, false, out);
}

extern "C" int pconv_packed_library(const pconv_packed* p, uint16_t* lib_out) {
    if (!p || !lib_out) return PCONV_EINVAL;
    std::memcpy(lib_out, p->lib.data(), p->lib.size() * sizeof(uint16_t));
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

// The inverse of pconv_packed_export: the canonical arrays are checked, spread back into a dense masked tensor with its
// pattern ids and connectivity mask, and packed again, so that an imported layer is in every respect the layer that
// pconv_pack would have made from the original weights.
extern "C" int pconv_packed_import(const uint32_t* filter_order, const uint32_t* grp_ptr, const uint16_t* cin,
                                   const void* w4, int dtype, int F, int C, const uint16_t* lib, int K,
                                   unsigned flags, pconv_packed** out) {
    if (!out) return PCONV_EINVAL;
    *out = nullptr;
    if (!filter_order || !grp_ptr) return PCONV_EINVAL;
    if (dtype != PCONV_F32 && dtype != PCONV_F16) return PCONV_EINVAL;
    if (int rc = check_library(lib, K)) return rc;
    if (int rc = check_fc(F, C)) return rc;
    const size_t esize = dtype == PCONV_F16 ? 2 : 4;
    const size_t n_groups = (size_t)F * K;
    const size_t n_kept = grp_ptr[n_groups];
    if (grp_ptr[0] != 0 || n_kept > (size_t)F * C) return PCONV_EINVAL;
    for (size_t g = 0; g < n_groups; ++g)
        if (grp_ptr[g] > grp_ptr[g + 1]) return PCONV_EINVAL;
    if (n_kept && (!cin || !w4)) return PCONV_EINVAL;
    try {
        std::vector<unsigned char> seen((size_t)F, 0);
        for (int i = 0; i < F; ++i) {
            if (filter_order[i] >= (uint32_t)F || seen[filter_order[i]]) return PCONV_EINVAL;
            seen[filter_order[i]] = 1;
        }
        std::vector<int> taps((size_t)K * 4);
        for (int j = 0; j < K; ++j) {
            int n = 0;
            for (int t = 0; t < 9; ++t)
                if (lib[j] >> t & 1) taps[(size_t)j * 4 + n++] = t;
        }
        std::vector<unsigned char> w((size_t)F * C * 9 * esize, 0);
        std::vector<uint8_t> pid((size_t)F * C, 0), mask((size_t)F * C, 0);
        const unsigned char* src = static_cast<const unsigned char*>(w4);
        for (int i = 0; i < F; ++i) {
            const size_t f = filter_order[i];
            for (int j = 0; j < K; ++j) {
                const size_t a = grp_ptr[(size_t)i * K + j], b = grp_ptr[(size_t)i * K + j + 1];
                for (size_t e = a; e < b; ++e) {
                    const size_t c = cin[e];
                    // inside a group channels ascend; over the groups of a filter no channel comes twice
                    if (c >= (size_t)C || (e > a && cin[e - 1] >= c) || mask[f * C + c]) return PCONV_EINVAL;
                    mask[f * C + c] = 1;
                    pid[f * C + c] = (uint8_t)j;
                    for (int k = 0; k < 4; ++k)
                        std::memcpy(&w[((f * C + c) * 9 + taps[(size_t)j * 4 + k]) * esize], src + (e * 4 + k) * esize,
                                    esize);
                }
            }
        }
        return pack_impl(w.data(), dtype, F, C, lib, K, pid.data(), mask.data(), flags, false, true, out);
    } catch (const std::bad_alloc&) {
        return PCONV_ENOMEM;
    }
}

extern "C" int pconv_packed_balance(const pconv_packed* p, int waves, int filters_per_wave, int balanced,
                                    double* mean_per_wave, double* mean_of_max) {
    if (!p || !mean_per_wave || !mean_of_max) return PCONV_EINVAL;
    if (waves < 1 || filters_per_wave < 1) return PCONV_EINVAL;
    const int F = p->F, fg = waves * filters_per_wave, cc = 32;
    const pconv::BalancedLayout* bl = nullptr;
    for (const pconv::BalancedLayout& b : p->balanced)
        if (b.fw == waves && b.nf == filters_per_wave && b.cc == cc) bl = &b;
    if (balanced && !bl) return PCONV_EUNSUPPORTED;
    const int nch = balanced ? bl->n_chunks : (p->C + cc - 1) / cc;
    const int per = cc / pconv::kBucket;
    auto count = [&](int pos, int k) -> uint32_t {
        if (balanced) return bl->eptr[(size_t)pos * nch + k + 1] - bl->eptr[(size_t)pos * nch + k];
        const int b0 = k * per, b1 = std::min(p->n_buckets, b0 + per);
        return p->eptr[(size_t)pos * p->n_buckets + b1] - p->eptr[(size_t)pos * p->n_buckets + b0];
    };
    double sum = 0.0, sum_max = 0.0;
    long long n_wave_chunks = 0, n_chunks = 0;
    for (int g = 0; g * fg < F; ++g)
        for (int k = 0; k < nch; ++k) {
            uint32_t mx = 0;
            for (int w = 0; w < waves; ++w) {
                uint32_t load = 0;
                for (int a = 0; a < filters_per_wave; ++a) {
                    const int pos = g * fg + w + a * waves;
                    if (pos < F) load += count(pos, k);
                }
                mx = std::max(mx, load);
                sum += load;
                ++n_wave_chunks;
            }
            sum_max += mx;
            ++n_chunks;
        }
    *mean_per_wave = n_wave_chunks ? sum / (double)n_wave_chunks : 0.0;
    *mean_of_max = n_chunks ? sum_max / (double)n_chunks : 0.0;
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
    for (pconv_packed*& child : p->by_parity) {
        pconv_free(child);
        child = nullptr;
    }
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
        case PCONV_ESTATE: return "packed handle has no device copy (packed host-only), belongs to another device, or lacks a form of the layer that only an allocating call can build";
        case PCONV_ESCRATCH: return "the launch needs more scratch memory than the fixed arena of pconv_conv3x3_noalloc holds";
        default: return "unknown pconv error code";
    }
}
