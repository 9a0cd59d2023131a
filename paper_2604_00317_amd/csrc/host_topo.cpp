#include "host_topo.hpp"

#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <map>
#include <queue>
#include <tuple>
#include <string>
#include <unordered_map>

namespace nimble {

nimble_status_t validate_csr(int32_t n_links, const double *cap, int32_t n_comm,
                             const int32_t *comm_path_ptr, int32_t n_paths,
                             const int32_t *path_link_ptr, const int32_t *path_links,
                             std::string &why)
{
    if (n_links < 1 || n_comm < 1 || n_paths < 1) {
        why = "n_links, n_comm and n_paths must be >= 1";
        return NIMBLE_ERR_INVALID;
    }
    if (!comm_path_ptr || !path_link_ptr || !path_links) {
        why = "null CSR pointer";
        return NIMBLE_ERR_INVALID;
    }
    if (cap) {
        for (int32_t e = 0; e < n_links; ++e)
            if (!(cap[e] > 0.0) || !std::isfinite(cap[e])) {
                why = "capacity of link " + std::to_string(e) + " is not finite and > 0";
                return NIMBLE_ERR_INVALID;
            }
    }
    if (comm_path_ptr[0] != 0 || comm_path_ptr[n_comm] != n_paths) {
        why = "comm_path_ptr must start at 0 and end at n_paths";
        return NIMBLE_ERR_INVALID;
    }
    int32_t pmax = 0;
    for (int32_t k = 0; k < n_comm; ++k) {
        int32_t np = comm_path_ptr[k + 1] - comm_path_ptr[k];
        if (np < 1 || comm_path_ptr[k + 1] > n_paths) {
            why = "comm_path_ptr is not strictly increasing at commodity " + std::to_string(k);
            return NIMBLE_ERR_INVALID;
        }
        if (np > pmax) pmax = np;
    }
    if (path_link_ptr[0] != 0) {
        why = "path_link_ptr must start at 0";
        return NIMBLE_ERR_INVALID;
    }
    for (int32_t p = 0; p < n_paths; ++p)
        if (path_link_ptr[p + 1] <= path_link_ptr[p]) {
            why = "path_link_ptr is not strictly increasing at path " + std::to_string(p);
            return NIMBLE_ERR_INVALID;
        }
    std::vector<int32_t> stamp(n_links, -1);
    for (int32_t p = 0; p < n_paths; ++p)
        for (int32_t i = path_link_ptr[p]; i < path_link_ptr[p + 1]; ++i) {
            int32_t e = path_links[i];
            if (e < 0 || e >= n_links) {
                why = "link id out of range in path " + std::to_string(p);
                return NIMBLE_ERR_INVALID;
            }
            if (stamp[e] == p) {
                why = "link " + std::to_string(e) + " appears twice in path " + std::to_string(p);
                return NIMBLE_ERR_INVALID;
            }
            stamp[e] = p;
        }
    if (n_comm > kMaxComm) {
        why = "more than 2^24 - 2 commodities";
        return NIMBLE_ERR_RANGE;
    }
    if (pmax > kMaxPathsPerComm) {
        why = "a commodity has more than 127 candidate paths";
        return NIMBLE_ERR_RANGE;
    }
    return NIMBLE_OK;
}

void read_layout_options(HostTopo &t)
{
    auto number = [](const char *name, int lo, int hi, int32_t &out) {
        if (const char *env = std::getenv(name)) {
            const int v = std::atoi(env);
            if (v >= lo && v <= hi) out = v;
        }
    };
    number("NIMBLE_TUNE_RECORD_COMM_CAP", 1, kRecMaxComm, t.rec_comm_cap);
    number("NIMBLE_TUNE_RECORD_LANE_MAJOR", 0, 1, t.rec_lane_major);
    number("NIMBLE_TUNE_RECORD_TABLE16", 0, 1, t.rec_table16);
    number("NIMBLE_TUNE_RECORD_DICT", 0, 1, t.rec_dict);
    number("NIMBLE_TUNE_RECORD_PRODUCT_QUADS", 0, 1, t.rec_product_quads);
    number("NIMBLE_TUNE_BLOCK_PASSES", 1, 1024, t.blk_passes);
    number("NIMBLE_TUNE_TILES", 0, 1, t.tiles);
    number("NIMBLE_TUNE_TILE_MIN_ITEMS", 1, kTileIds, t.tile_min_items);
    number("NIMBLE_TUNE_LINK_GROUPS", 0, 1, t.link_groups);
    number("NIMBLE_TUNE_GROUP_BLOCKS", 1, 65536, t.grp_target);
    int32_t dense_only = 0;
    number("NIMBLE_TUNE_TILES_DENSE_ONLY", 0, 1, dense_only);
    t.tiles_dense_only = dense_only != 0;
}

// ---- quads of a two-by-two product ---------------------------------------------------------
// Candidate lists built by a product rule (rail x egress GPU x ingress GPU, two GPUs per rail)
// put four candidates into a quad that differ only in (egress, ingress): their first two links
// depend on the egress alone, the middle link on neither, the last two on the ingress alone.
// Adding +0.0 is exact wherever it happens in the left-to-right sum of a path, so the padding
// of a short path may sit anywhere among its steps: this tries to shift the links of every
// candidate of a quad (keeping their order) so that, step by step, the quad reads
//   step 0: x x y y   step 1: x x y y   step 2: x x x x   step 3: x y x y   step 4: x y x y
// The record kernel then fetches 9 prices for the quad instead of 20 and shares the partial
// sums.  q5[c][i] is the table index of step i of candidate c (kRecZeroSlot = padding); on
// success the shifted indices are written back.  Absent candidates (first index kRecInfSlot)
// are never shifted.
static bool align_product_quad(uint8_t (&q5)[4][kRecLaneSteps])
{
    int32_t len[4];
    uint8_t links[4][kRecLaneSteps];
    bool absent[4];
    for (int32_t c = 0; c < 4; ++c) {
        len[c] = 0;
        absent[c] = q5[c][0] == kRecInfSlot;
        for (int32_t i = 0; i < kRecLaneSteps; ++i)
            if (q5[c][i] != kRecZeroSlot) links[c][len[c]++] = q5[c][i];
        if (len[c] == 0) return false;
    }
    uint8_t out[4][kRecLaneSteps];
    auto place = [&](int32_t c, int32_t shift) {
        for (int32_t i = 0; i < kRecLaneSteps; ++i) out[c][i] = static_cast<uint8_t>(kRecZeroSlot);
        for (int32_t i = 0; i < len[c]; ++i) out[c][shift + i] = links[c][i];
    };
    auto fits = [&]() {
        for (int32_t i = 0; i < kRecLaneSteps; ++i) {
            const uint8_t a = out[0][i], b = out[1][i], c = out[2][i], d = out[3][i];
            const bool ok = i < 2 ? (a == b && c == d) : i == 2 ? (a == b && b == c && c == d)
                                                                : (a == c && b == d);
            if (!ok) return false;
        }
        return true;
    };
    int32_t hi[4];
    for (int32_t c = 0; c < 4; ++c) hi[c] = absent[c] ? 0 : kRecLaneSteps - len[c];
    for (int32_t s0 = 0; s0 <= hi[0]; ++s0)
        for (int32_t s1 = 0; s1 <= hi[1]; ++s1)
            for (int32_t s2 = 0; s2 <= hi[2]; ++s2)
                for (int32_t s3 = 0; s3 <= hi[3]; ++s3) {
                    place(0, s0);
                    place(1, s1);
                    place(2, s2);
                    place(3, s3);
                    if (!fits()) continue;
                    for (int32_t c = 0; c < 4; ++c)
                        for (int32_t i = 0; i < kRecLaneSteps; ++i) q5[c][i] = out[c][i];
                    return true;
                }
    return false;
}

// Brings the A quads (bit 0 of the result) and the B quads (bit 1) of all 64 lanes of a
// lane-major body into the product shape where every lane allows it; `words` holds
// kRecLaneWords words per lane and is rewritten for the quads that succeed.
static uint32_t align_product_body(std::vector<uint32_t> &words)
{
    uint32_t product = 0u;
    for (int32_t q = 0; q < 2; ++q) {
        std::vector<uint32_t> trial(words);
        bool all = true;
        for (int32_t lane = 0; lane < 64 && all; ++lane) {
            uint32_t *w = &trial[static_cast<size_t>(lane) * kRecLaneWords +
                                 static_cast<size_t>(q) * kRecLaneSteps];
            uint8_t q5[4][kRecLaneSteps];
            for (int32_t c4 = 0; c4 < 4; ++c4)
                for (int32_t i = 0; i < kRecLaneSteps; ++i)
                    q5[c4][i] = static_cast<uint8_t>((w[i] >> (8 * c4)) & 0xFFu);
            all = align_product_quad(q5);
            for (int32_t i = 0; i < kRecLaneSteps && all; ++i) {
                w[i] = 0u;
                for (int32_t c4 = 0; c4 < 4; ++c4)
                    w[i] |= static_cast<uint32_t>(q5[c4][i]) << (8 * c4);
            }
        }
        if (all) {
            words.swap(trial);
            product |= 1u << q;
        }
    }
    return product;
}

// ---- forward records ----------------------------------------------------------------------
// Repacks the forward CSR into the records the path-cost kernel streams (see host_topo.hpp).
// Needs t.pmax, t.lmax, t.nnz and t.sigma; t.rec_comm_cap, t.rec_lane_major, t.rec_table16 and
// t.rec_dict are read as options and come back as what was built.
static void build_forward_records_once(int32_t n_links, int32_t n_comm,
                                       const int32_t *comm_path_ptr, int32_t n_paths,
                                       const int32_t *path_link_ptr, const int32_t *path_links,
                                       bool want_dict, HostTopo &t)
{
    t.n_records = 0;
    t.rec_max_links = 0;
    t.records.clear();
    t.rec_stride = t.lmax;
    t.n_bodies = 0;
    t.n_bodies_product = 0;
    t.rec_price_reads = 0;
    t.rec_dict_words.clear();
    t.rec_body.clear();
    bool dict = false;
    std::unordered_map<std::string, int32_t> body_ids;
    const bool shape_ok = t.lmax <= kRecMaxStride &&
                          static_cast<double>(t.lmax) * n_paths <= 1.5 * static_cast<double>(t.nnz);
    if (shape_ok) {
        const int32_t S = t.rec_stride;
        std::vector<int32_t> stamp(n_links, -1), local(n_links, 0);
        std::vector<int32_t> links;
        std::vector<uint16_t> cp16, cq16, loc16;
        auto align4 = [](int32_t x) { return (x + 3) & ~3; };
        auto bytes_needed = [&](int32_t nl, int32_t nk, int32_t npad) {
            (void)nl;    // the link table has a fixed size
            if (t.rec_lane_major) return kRecBytes;      // a slot per commodity: always fits
            return kRecTable + kRecHeader + 4 * nk + 2 * align4(2 * (nk + 1)) + npad * S;
        };
        // lanes per commodity in the record kernel: a lane scans two quads of the largest
        // commodity; a record holds as many commodities as one round of the wave covers
        // (64 / lanes), unless the caller set the capacity
        {
            const int32_t quads = (t.pmax + 3) / 4;
            int32_t lanes = 1;
            while (2 * lanes < quads && lanes < 64) lanes <<= 1;
            t.rec_lanes = lanes;
            if (t.rec_comm_cap <= 0) t.rec_comm_cap = 64 / lanes;
            if (t.rec_comm_cap > kRecMaxComm) t.rec_comm_cap = kRecMaxComm;
            // the lane-major body needs two quads per lane to cover every commodity, paths
            // that fit five words per quad, a second lane per slot for the record's own words,
            // and 4 KiB records
            t.rec_lane_major = (t.rec_lane_major != 0 && S <= kRecLaneSteps && lanes >= 2 &&
                                lanes <= 16 && quads <= 2 * lanes && kRecBytes == 4096) ? 1 : 0;
            if (t.rec_lane_major && t.rec_comm_cap > 64 / lanes) t.rec_comm_cap = 64 / lanes;
        }
        const bool lane_major = t.rec_lane_major != 0;
        t.rec_table16 = (lane_major && t.rec_table16 != 0 && n_links <= 65535) ? 1 : 0;
        const bool table16 = t.rec_table16 != 0;
        // the dictionary format needs the lane-major body and the 16-bit table
        dict = want_dict && lane_major && table16;
        t.rec_bytes = dict ? kRecBytesDict : (table16 ? kRecBytes16 : kRecBytes);
        const int32_t table_bytes = table16 ? kRecTable16 : kRecTable;
        bool ok = true;
        int32_t k = 0;
        while (k < n_comm && ok) {
            const int32_t rec_id = t.n_records;
            const int32_t k0 = k, p0 = comm_path_ptr[k];
            links.clear();
            cp16.assign(1, 0);
            cq16.assign(1, 0);
            loc16.clear();
            int32_t np = 0, npad = 0;
            while (k < n_comm && k - k0 < t.rec_comm_cap) {
                const int32_t pa = comm_path_ptr[k], pb = comm_path_ptr[k + 1];
                // distinct links this commodity would add
                int32_t add = 0;
                for (int32_t i = path_link_ptr[pa]; i < path_link_ptr[pb]; ++i) {
                    const int32_t e = path_links[i];
                    if (stamp[e] != rec_id && stamp[e] != -2 - rec_id) {
                        stamp[e] = -2 - rec_id;
                        ++add;
                    }
                }
                const int32_t nl_new = static_cast<int32_t>(links.size()) + add;
                const bool fits = nl_new <= kRecMaxLinks &&
                                  bytes_needed(nl_new, k - k0 + 1, npad + align4(pb - pa)) <=
                                      kRecBytes;
                if (!fits) {
                    for (int32_t i = path_link_ptr[pa]; i < path_link_ptr[pb]; ++i)
                        if (stamp[path_links[i]] == -2 - rec_id) stamp[path_links[i]] = -1;
                    break;
                }
                for (int32_t p = pa; p < pb; ++p) {
                    const int32_t la = path_link_ptr[p], lb = path_link_ptr[p + 1];
                    for (int32_t i = la; i < lb; ++i) {
                        const int32_t e = path_links[i];
                        if (stamp[e] != rec_id) {
                            stamp[e] = rec_id;
                            local[e] = static_cast<int32_t>(links.size());
                            links.push_back(e);
                        }
                        loc16.push_back(static_cast<uint16_t>(local[e]));
                    }
                    for (int32_t i = lb - la; i < S; ++i) loc16.push_back(0xFFFFu);  // patched below
                }
                // candidates are padded to whole quads; a padding candidate starts at the
                // +inf price slot, so it never wins the argmin
                for (int32_t q = pb - pa; q < align4(pb - pa); ++q)
                    for (int32_t i = 0; i < S; ++i) loc16.push_back(i == 0 ? 0xFFFEu : 0xFFFFu);
                np += pb - pa;
                npad += align4(pb - pa);
                cp16.push_back(static_cast<uint16_t>(np));
                cq16.push_back(static_cast<uint16_t>(npad));
                ++k;
            }
            if (k == k0) {      // one commodity alone does not fit a record
                ok = false;
                break;
            }
            const int32_t nk = k - k0, nl = static_cast<int32_t>(links.size());
            // the link table in ascending id order: neighbouring lanes then gather neighbouring
            // prices (fewer cache lines per gather)
            {
                std::vector<int32_t> order(nl), rank(nl);
                for (int32_t i = 0; i < nl; ++i) order[i] = i;
                std::sort(order.begin(), order.end(),
                          [&](int32_t x, int32_t y) { return links[x] < links[y]; });
                std::vector<int32_t> sorted(nl);
                for (int32_t i = 0; i < nl; ++i) {
                    sorted[i] = links[order[i]];
                    rank[order[i]] = i;
                }
                links.swap(sorted);
                for (auto &v : loc16)
                    if (v < 0xFFFEu) v = static_cast<uint16_t>(rank[v]);
            }
            for (auto &v : loc16) {
                // the +0.0 and the +inf price slot
                if (v == 0xFFFFu) v = static_cast<uint16_t>(lane_major ? kRecZeroSlot : nl);
                else if (v == 0xFFFEu) v = static_cast<uint16_t>(lane_major ? kRecInfSlot : nl + 1);
            }
            t.records.resize(static_cast<size_t>(t.n_records + 1) * t.rec_bytes, 0);
            uint8_t *r = t.records.data() + static_cast<size_t>(t.n_records) * t.rec_bytes;
            const int32_t off_sig = kRecHeader;      // body offsets count from kRecTable
            const int32_t off_cp = off_sig + 4 * nk;
            const int32_t off_cq = off_cp + align4(2 * (nk + 1));
            const int32_t off_loc = off_cq + align4(2 * (nk + 1));
            const uint16_t h16[8] = {static_cast<uint16_t>(nk), static_cast<uint16_t>(np),
                                     static_cast<uint16_t>(nl), static_cast<uint16_t>(off_cp),
                                     static_cast<uint16_t>(off_loc),
                                     static_cast<uint16_t>(off_sig),
                                     static_cast<uint16_t>(off_cq),
                                     static_cast<uint16_t>(npad)};
            // gather c of lane l reads table entry 4*l + c, which is link 64*c + l; in the
            // dictionary format a lane's four 16-bit entries open its 16 bytes of the record
            {
                int32_t *tab = reinterpret_cast<int32_t *>(r);
                uint16_t *tab16 = reinterpret_cast<uint16_t *>(r);
                for (int32_t l = 0; l < 64; ++l)
                    for (int32_t c = 0; c < 4; ++c) {
                        const int32_t i = 64 * c + l;
                        const int32_t e = nl == 0 ? 0 : links[i < nl ? i : nl - 1];
                        if (dict) tab16[8 * l + c] = static_cast<uint16_t>(e);
                        else if (table16) tab16[4 * l + c] = static_cast<uint16_t>(e);
                        else tab[4 * l + c] = e;
                    }
            }
            uint8_t *body = r + table_bytes;
            if (lane_major) {
                const int32_t L = t.rec_lanes;
                std::vector<uint32_t> words(64 * kRecLaneWords, 0u);
                for (int32_t lane = 0; lane < 64; ++lane) {
                    const int32_t g = lane / L, j = lane % L;
                    uint32_t *w = &words[static_cast<size_t>(lane) * kRecLaneWords];
                    const int32_t np_g = g < nk ? cp16[g + 1] - cp16[g] : 0;
                    for (int32_t q = 0; q < 2; ++q)
                        for (int32_t i = 0; i < kRecLaneSteps; ++i) {
                            uint32_t word = 0u;
                            for (int32_t c4 = 0; c4 < 4; ++c4) {
                                const int32_t cand = 4 * (j + L * q) + c4;
                                uint32_t byte = i == 0 ? kRecInfSlot : kRecZeroSlot;
                                if (cand < np_g && i < S)
                                    byte = loc16[static_cast<size_t>(cq16[g] + cand) * S + i];
                                word |= byte << (8 * c4);
                            }
                            w[q * kRecLaneSteps + i] = word;
                        }
                    if (g < nk) {
                        w[10] = static_cast<uint32_t>(np_g) | (static_cast<uint32_t>(cp16[g]) << 8);
                        if (j == 0) w[11] = static_cast<uint32_t>(t.sigma[k0 + g]);
                    }
                }
                words[1 * kRecLaneWords + 11] =
                    static_cast<uint32_t>(k0) | (static_cast<uint32_t>(nk) << 24);
                words[static_cast<size_t>(L + 1) * kRecLaneWords + 11] = static_cast<uint32_t>(p0);
                if (dict) {
                    // words 0..10 of every lane say how the candidates index the link table and
                    // nothing about which commodities or links these are: records of the same
                    // shape share them.  The record keeps its table, word 11 and the number of
                    // its body.
                    std::string key(64 * 11 * 4, '\0');
                    for (int32_t lane = 0; lane < 64; ++lane)
                        std::memcpy(&key[static_cast<size_t>(lane) * 44],
                                    &words[static_cast<size_t>(lane) * kRecLaneWords], 44);
                    auto found = body_ids.find(key);
                    int32_t id;
                    if (found == body_ids.end()) {
                        id = t.n_bodies++;
                        body_ids.emplace(std::move(key), id);
                        const size_t at = t.rec_dict_words.size();
                        t.rec_dict_words.resize(at + 3 * 64 * 4, 0u);
                        // quads of a two-by-two product: where the A quads (or the B quads) of
                        // all 64 lanes can be brought into that shape, the body stores them so
                        // and says it in word 11 (bit 0: A quads, bit 1: B quads), the same in
                        // every lane
                        std::vector<uint32_t> stored(words);
                        const uint32_t product = (t.rec_product_quads != 0 && S == kRecLaneSteps)
                                                     ? align_product_body(stored) : 0u;
                        for (int32_t lane = 0; lane < 64; ++lane)
                            for (int32_t it = 0; it < 3; ++it)
                                for (int32_t q = 0; q < 4; ++q)
                                    t.rec_dict_words[at + (static_cast<size_t>(it) * 64 + lane) * 4 + q] =
                                        4 * it + q < 11
                                            ? stored[static_cast<size_t>(lane) * kRecLaneWords + 4 * it + q]
                                            : product;
                        if (product == 3u) t.n_bodies_product += 1;
                    } else {
                        id = found->second;
                    }
                    uint32_t *r32 = reinterpret_cast<uint32_t *>(r);
                    for (int32_t lane = 0; lane < 64; ++lane) {
                        r32[4 * lane + 2] = words[static_cast<size_t>(lane) * kRecLaneWords + 11];
                        r32[4 * lane + 3] = static_cast<uint32_t>(id);
                    }
                    {
                        const uint32_t pb = t.rec_dict_words[(static_cast<size_t>(id) * 3 + 2) * 256 + 3];
                        t.rec_price_reads += ((pb & 1u) ? 9 : 4 * kRecLaneSteps) +
                                             ((pb & 2u) ? 9 : 4 * kRecLaneSteps);
                    }
                    t.rec_body.push_back(id);
                    t.n_records += 1;
                    if (nl > t.rec_max_links) t.rec_max_links = nl;
                    continue;
                }
                // bodies kept in the record: the same product shape where the quads allow it; the
                // two bits go to word 11 of lane 2L + 1 (slot 2, second lane: no sigma, not one
                // of the record's own words)
                if (t.rec_product_quads != 0 && S == kRecLaneSteps)
                    words[static_cast<size_t>(2 * L + 1) * kRecLaneWords + 11] =
                        align_product_body(words);
                {
                    const uint32_t pb = S == kRecLaneSteps
                                            ? words[static_cast<size_t>(2 * L + 1) * kRecLaneWords + 11] : 0u;
                    t.rec_price_reads += ((pb & 1u) ? 9 : 4 * S) + ((pb & 2u) ? 9 : 4 * S);
                }
                for (int32_t lane = 0; lane < 64; ++lane)
                    for (int32_t it = 0; it < 3; ++it)
                        std::memcpy(body + 1024 * it + 16 * lane,
                                    &words[static_cast<size_t>(lane) * kRecLaneWords + 4 * it], 16);
                t.n_records += 1;
                if (nl > t.rec_max_links) t.rec_max_links = nl;
                continue;
            }
            std::memcpy(body + 0, &k0, 4);
            std::memcpy(body + 4, &p0, 4);
            std::memcpy(body + 8, h16, 16);
            std::memcpy(body + off_sig, t.sigma.data() + k0, 4 * static_cast<size_t>(nk));
            std::memcpy(body + off_cp, cp16.data(), 2 * cp16.size());
            std::memcpy(body + off_cq, cq16.data(), 2 * cq16.size());
            // step-major over the padded candidates: index i of every candidate, then index
            // i+1, ...; four consecutive candidates (a quad) are one aligned 32-bit word
            {
                std::vector<uint8_t> soa(loc16.size());
                for (int32_t p = 0; p < npad; ++p)
                    for (int32_t i = 0; i < S; ++i)
                        soa[static_cast<size_t>(i) * npad + p] =
                            static_cast<uint8_t>(loc16[static_cast<size_t>(p) * S + i]);
                std::memcpy(body + off_loc, soa.data(), soa.size());
            }
            t.n_records += 1;
            if (nl > t.rec_max_links) t.rec_max_links = nl;
        }
        if (!ok) {
            t.n_records = 0;
            t.records.clear();
        }
        if (ok && dict) {
            // records of one body next to each other (stable: ascending commodities inside a
            // body), so that a wave that walks a run of records fetches its body once
            std::vector<int32_t> order(t.n_records);
            for (int32_t i = 0; i < t.n_records; ++i) order[i] = i;
            std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
                return t.rec_body[x] < t.rec_body[y];
            });
            std::vector<uint8_t> sorted(t.records.size());
            std::vector<int32_t> body_sorted(t.n_records);
            for (int32_t i = 0; i < t.n_records; ++i) {
                std::memcpy(&sorted[static_cast<size_t>(i) * kRecBytesDict],
                            &t.records[static_cast<size_t>(order[i]) * kRecBytesDict], kRecBytesDict);
                body_sorted[i] = t.rec_body[order[i]];
            }
            t.records.swap(sorted);
            t.rec_body.swap(body_sorted);
        }
    }
    t.rec_dict = (t.n_records > 0 && dict) ? 1 : 0;
    if (t.n_records == 0) {
        t.rec_lane_major = 0;
        t.rec_table16 = 0;
    }
    if (t.rec_bytes == 0) t.rec_bytes = kRecBytes;
}

void build_forward_records(int32_t n_links, int32_t n_comm, const int32_t *comm_path_ptr,
                           int32_t n_paths, const int32_t *path_link_ptr,
                           const int32_t *path_links, HostTopo &t)
{
    // Lane-major records with 16-bit tables are first built with a dictionary of bodies (a
    // record then is 1 KiB: table, the record's own words and the number of its body).  The
    // dictionary stays when it pays -- bodies shared by four records each on average, as on
    // large fabrics built by a product rule -- or when the option asks for it; otherwise the
    // records are built again with their bodies inline (on the 16-node fabric, three records
    // per body, the dictionary changed nothing: the kernel is a latency chain there).
    const int32_t opt_cap = t.rec_comm_cap, opt_lm = t.rec_lane_major, opt_t16 = t.rec_table16;
    const int32_t opt_dict = t.rec_dict;
    if (opt_dict != 0) {
        build_forward_records_once(n_links, n_comm, comm_path_ptr, n_paths, path_link_ptr,
                                   path_links, true, t);
        if (t.rec_dict == 1 && (opt_dict == 1 || 4LL * t.n_bodies <= t.n_records)) return;
        t.rec_comm_cap = opt_cap;
        t.rec_lane_major = opt_lm;
        t.rec_table16 = opt_t16;
    }
    build_forward_records_once(n_links, n_comm, comm_path_ptr, n_paths, path_link_ptr,
                               path_links, false, t);
}

// ---- reverse CSR ---------------------------------------------------------------------------
// The (commodity, window) pairs of every link by a stable counting sort (rev_ptr, rev_pair,
// rev_rowlen, n_pairs): what the resident kernels walk, and the input of every other layout.
static void build_reverse_pairs(int32_t n_links, int32_t n_comm, const int32_t *comm_path_ptr,
                                const int32_t *path_link_ptr, const int32_t *path_links,
                                HostTopo &t)
{
    // pass 1 counts the pairs of every link: a new pair starts when the commodity or the
    // window changes with respect to the link's previous incidence (incidences are visited in
    // ascending (commodity, path) order)
    std::vector<int32_t> last_key(n_links, -1);
    t.rev_rowlen.assign(n_links, 0);
    for (int32_t k = 0; k < n_comm; ++k)
        for (int32_t p = comm_path_ptr[k]; p < comm_path_ptr[k + 1]; ++p) {
            const int32_t key = k * 4 + ((p - comm_path_ptr[k]) >> 5);
            for (int32_t i = path_link_ptr[p]; i < path_link_ptr[p + 1]; ++i) {
                const int32_t e = path_links[i];
                if (last_key[e] != key) {
                    last_key[e] = key;
                    t.rev_rowlen[e] += 1;
                }
            }
        }
    t.rev_ptr.assign(n_links + 1, 0);
    t.n_pairs = 0;
    for (int32_t e = 0; e < n_links; ++e) {
        const int32_t padded = (t.rev_rowlen[e] + kPairAlign - 1) / kPairAlign * kPairAlign;
        t.rev_ptr[e + 1] = t.rev_ptr[e] + padded;
        t.n_pairs += t.rev_rowlen[e];
    }
    t.rev_pair.assign(2 * static_cast<size_t>(t.rev_ptr[n_links]), 0u);
    for (size_t i = 0; i < t.rev_pair.size(); i += 2)
        t.rev_pair[i] = static_cast<uint32_t>(n_comm);           // padding: commodity K, mask 0
    std::vector<int32_t> fill(t.rev_ptr.begin(), t.rev_ptr.end() - 1);
    std::vector<int32_t> last_comm(n_links, -1);
    std::fill(last_key.begin(), last_key.end(), -1);
    for (int32_t k = 0; k < n_comm; ++k)
        for (int32_t p = comm_path_ptr[k]; p < comm_path_ptr[k + 1]; ++p) {
            const int32_t j = p - comm_path_ptr[k];
            const int32_t key = k * 4 + (j >> 5);
            for (int32_t i = path_link_ptr[p]; i < path_link_ptr[p + 1]; ++i) {
                const int32_t e = path_links[i];
                if (last_key[e] != key) {
                    last_key[e] = key;
                    const bool first = last_comm[e] != k;
                    last_comm[e] = k;
                    const size_t w = 2 * static_cast<size_t>(fill[e]++);
                    t.rev_pair[w] = (first ? kFirstFlag : 0u) |
                                    (static_cast<uint32_t>(j >> 5) << kWindowShift) |
                                    static_cast<uint32_t>(k);
                    t.rev_pair[w + 1] = 0u;
                }
                t.rev_pair[2 * static_cast<size_t>(fill[e] - 1) + 1] |= 1u << (j & 31);
            }
        }

}

// ---- streaming layouts of the reverse rows ---------------------------------------------------
// From the pairs: the second commodity numbering sigma, tiles and strips where rows share
// windows or octets, the flat octets with their partial-sum slots, chunked single pairs, and the
// order of the rows (link blocks).  Needs build_reverse_pairs; reads t.tiles, t.tile_min_items,
// t.tiles_dense_only and t.blk_passes as options.
static void build_streaming_layout(int32_t n_links, int32_t n_comm, const int32_t *comm_path_ptr,
                                const int32_t *path_link_ptr, const int32_t *path_links,
                                HostTopo &t)
{
    t.oct_base.clear();
    t.oct_mask.clear();
    t.pass_first_slot.clear();
    t.single_pair.clear();
    t.n_single_pairs = 0;
    t.schunk_begin.clear(); t.schunk_end.clear(); t.schunk_slot.clear();
    t.sigma.assign(n_comm, -1);
    t.n_gblocks = 0;
    t.gblk_desc.clear();
    t.gblk_max_slots = 0;
    t.gblk_max_tasks = 0;
    const int32_t sgl_chunk = kRowLanesHost * kSinglesPerLane;
    auto one_window = [&](int32_t kk) { return comm_path_ptr[kk + 1] - comm_path_ptr[kk] <= 32; };
    struct Item { int32_t key; uint32_t a, b; };       // key: commodity id or sigma, -1: single
    // greedy octet packing of items sorted by key; appends octets, returns the left-overs
    auto pack = [&](const std::vector<Item> &items, int32_t key_limit, int32_t min_fill,
                    uint32_t flags, std::vector<uint32_t> &obase, std::vector<uint32_t> &omask,
                    std::vector<Item> &left) {
        size_t i = 0;
        while (i < items.size()) {
            const int32_t base = items[i].key & ~3;
            size_t cnt = 0;
            if (items[i].key >= 0)
                while (i + cnt < items.size() && items[i + cnt].key >= 0 &&
                       items[i + cnt].key < base + 8)
                    ++cnt;
            // an octet must not read past its choice array (which has 8 spare entries when
            // indexed by commodity id): slide the window back at the end
            const int32_t b8 = base + 8 <= key_limit ? base : ((key_limit - 8) & ~3);
            const bool fits = cnt > 0 && b8 >= 0 && items[i].key >= b8 &&
                              items[i + cnt - 1].key < b8 + 8;
            if (static_cast<int32_t>(cnt) >= min_fill && fits) {
                obase.push_back(static_cast<uint32_t>(b8) | flags);
                const size_t m0 = omask.size();
                omask.resize(m0 + 8, 0u);
                for (size_t q = 0; q < cnt; ++q) omask[m0 + (items[i + q].key - b8)] = items[i + q].b;
                i += cnt;
            } else {
                left.push_back(items[i]);
                i += 1;
            }
        }
    };
    auto row_items = [&](int32_t e, std::vector<Item> &items) {
        items.clear();
        for (int32_t i = 0; i < t.rev_rowlen[e]; ++i) {
            const uint32_t a = t.rev_pair[2 * static_cast<size_t>(t.rev_ptr[e] + i)];
            const uint32_t b = t.rev_pair[2 * static_cast<size_t>(t.rev_ptr[e] + i) + 1];
            const int32_t kk = static_cast<int32_t>(a & kCommMask);
            items.push_back({one_window(kk) ? kk : -1, a, b});    // -1: never in an octet
        }
    };
    // second numbering: the commodities that octets over ids of fill >= kOctetMinFill leave
    // over, in order of first appearance, every row's new run starting at a multiple of 8
    int32_t next_sigma = 0;
    {
        std::vector<Item> items, left;
        std::vector<uint32_t> scratch_base, scratch_mask;
        for (int32_t e = 0; e < n_links; ++e) {
            row_items(e, items);
            left.clear();
            scratch_base.clear();
            scratch_mask.clear();
            pack(items, n_comm + 8, kOctetMinFill, 0u, scratch_base, scratch_mask, left);
            bool started = false;
            for (const Item &it : left) {
                if (it.key < 0) continue;
                const int32_t kk = static_cast<int32_t>(it.a & kCommMask);
                if (t.sigma[kk] < 0) {
                    if (!started) {
                        next_sigma = (next_sigma + 7) & ~7;
                        started = true;
                    }
                    t.sigma[kk] = next_sigma++;
                }
            }
        }
    }
    // the sigma-ordered copies are read in whole windows of kTileIds entries by the tile phase
    t.sigma_size = (next_sigma + 8 + kTileIds - 1) / kTileIds * kTileIds;

    // ---- tiles: dense (row, window) pieces --------------------------------------------------
    // A window is kTileIds consecutive commodity numbers (ids, or sigma numbers).  Where a row
    // holds at least tile_min_items commodities of one window, those commodities leave the
    // octet stream and become a PIECE: 64 columns x 8 masks, column c = commodities
    // window*kTileIds + 8c .. + 7, zero masks where the commodity does not use the link.
    // Pieces of the same window are grouped, up to kTileRows at a time, into one work item.
    const bool tiles_on = t.tiles > 0 || (t.tiles < 0 && t.n_pairs >= kTileAutoPairs);
    const int32_t tile_min = t.tile_min_items > 0 ? t.tile_min_items : kTileMinItems;
    struct Piece { int32_t window; int32_t sig; int32_t link; size_t mask_at; };
    std::vector<Piece> pieces;
    std::vector<uint32_t> piece_mask;                     // 512 words per piece, [column][slot]
    std::vector<std::vector<int32_t>> link_pieces(n_links);
    std::vector<std::vector<uint32_t>> row_base(n_links), row_mask(n_links);
    t.n_octets_sigma = 0;
    t.n_octets = 0;
    t.n_piece_items = 0;
    int32_t extra_slots = 0;              // slots of pieces, strip rows and single-pair chunks
    std::vector<int32_t> piece_extra;     // per piece (creation order = link order)
    std::vector<int32_t> link_chunk_first(n_links + 1, 0);
    {
        std::vector<Item> items, rest, left1, left2, left3;
        std::unordered_map<int32_t, int32_t> win_count;
        std::unordered_map<int64_t, int32_t> win_masks;
        std::unordered_map<int32_t, std::pair<int32_t, uint32_t>> win_major;
        for (int32_t e = 0; e < n_links; ++e) {
            row_items(e, items);
            rest.clear();
            if (tiles_on) {
                // id windows first, then sigma windows over what is left
                for (int sig = 0; sig < 2; ++sig) {
                    auto number = [&](const Item &it) -> int32_t {
                        if (it.key < 0) return -1;
                        return sig ? t.sigma[it.a & kCommMask] : static_cast<int32_t>(it.a & kCommMask);
                    };
                    // per window: how many of the row's commodities, and the mask value most
                    // of them share
                    win_count.clear();
                    win_masks.clear();
                    for (const Item &it : items) {
                        const int32_t nb = number(it);
                        if (nb < 0) continue;
                        win_count[nb / kTileIds] += 1;
                        win_masks[(static_cast<int64_t>(nb / kTileIds) << 32) | it.b] += 1;
                    }
                    win_major.clear();                     // window -> (count, mask) of the top value
                    for (const auto &kv : win_masks) {
                        const int32_t w = static_cast<int32_t>(kv.first >> 32);
                        const uint32_t m = static_cast<uint32_t>(kv.first & 0xFFFFFFFFll);
                        auto &top = win_major[w];
                        if (kv.second > top.first || (kv.second == top.first && m < top.second))
                            top = {kv.second, m};
                    }
                    std::unordered_map<int32_t, size_t> win_piece;
                    rest.clear();
                    for (const Item &it : items) {
                        const int32_t nb = number(it);
                        if (nb < 0 || win_count[nb / kTileIds] < tile_min) {
                            rest.push_back(it);
                            continue;
                        }
                        const int32_t w = nb / kTileIds;
                        // a window where one mask value covers most commodities becomes a
                        // uniform piece of exactly those; the few others stay octets
                        const auto &top = win_major[w];
                        const bool mostly_uniform = !t.tiles_dense_only && top.first >= tile_min &&
                                                    4 * top.first >= 3 * win_count[w];
                        if (mostly_uniform && it.b != top.second) {
                            rest.push_back(it);
                            continue;
                        }
                        auto f = win_piece.find(w);
                        if (f == win_piece.end()) {
                            f = win_piece.emplace(w, pieces.size()).first;
                            link_pieces[e].push_back(static_cast<int32_t>(pieces.size()));
                            pieces.push_back({w, sig, e, piece_mask.size()});
                            piece_mask.resize(piece_mask.size() + 512, 0u);
                        }
                        piece_mask[pieces[f->second].mask_at + static_cast<size_t>(nb % kTileIds)] = it.b;
                        t.n_piece_items += 1;
                    }
                    items.swap(rest);
                }
            }
            // what is left: octets over ids (fill >= kOctetMinFill), octets over sigma (same
            // fill), octets over ids of any fill, single pairs
            left1.clear(); left2.clear(); left3.clear();
            pack(items, n_comm + 8, kOctetMinFill, 0u, row_base[e], row_mask[e], left1);
            for (Item &x : left1) x.key = x.key < 0 ? -1 : t.sigma[x.a & kCommMask];
            std::stable_sort(left1.begin(), left1.end(), [](const Item &x, const Item &y) {
                return (x.key < 0 ? INT32_MAX : x.key) < (y.key < 0 ? INT32_MAX : y.key);
            });
            const size_t before = row_base[e].size();
            pack(left1, t.sigma_size, kOctetMinFill, kOctSigma, row_base[e], row_mask[e], left2);
            t.n_octets_sigma += static_cast<int64_t>(row_base[e].size() - before);
            // back to (commodity, window) order; eligible ones become octets of any fill
            for (Item &x : left2) x.key = x.key < 0 ? -1 : static_cast<int32_t>(x.a & kCommMask);
            std::stable_sort(left2.begin(), left2.end(), [](const Item &x, const Item &y) {
                const uint32_t kx = x.a & kCommMask, ky = y.a & kCommMask;
                return kx != ky ? kx < ky : ((x.a >> kWindowShift) & 3u) < ((y.a >> kWindowShift) & 3u);
            });
            pack(left2, n_comm + 8, 1, 0u, row_base[e], row_mask[e], left3);
            // single pairs (commodities with several windows) and their chunks, in link order
            const int32_t s_first = static_cast<int32_t>(t.single_pair.size() / 2);
            for (const Item &it : left3) {
                t.single_pair.push_back(it.a);
                t.single_pair.push_back(it.b);
                t.n_single_pairs += 1;
            }
            if ((t.single_pair.size() / 2) % kPairAlign) {       // pad the row to 16 bytes
                t.single_pair.push_back(static_cast<uint32_t>(n_comm));
                t.single_pair.push_back(0u);
            }
            const int32_t s_last = static_cast<int32_t>(t.single_pair.size() / 2);
            link_chunk_first[e] = static_cast<int32_t>(t.schunk_begin.size());
            for (int32_t b = s_first; b < s_last; b += sgl_chunk) {
                t.schunk_begin.push_back(b);
                t.schunk_end.push_back(b + sgl_chunk < s_last ? b + sgl_chunk : s_last);
            }
        }
        link_chunk_first[n_links] = static_cast<int32_t>(t.schunk_begin.size());
    }

    // ---- uniform pieces -------------------------------------------------------------------
    // A piece whose non-zero masks are all equal (the usual case when the candidates of a
    // fabric are enumerated by a product rule) is UNIFORM: it is stored as that one mask plus a
    // presence bit per commodity.
    t.n_pieces = static_cast<int32_t>(pieces.size());
    t.n_pieces_uniform = 0;
    std::vector<uint32_t> piece_umask(pieces.size(), 0u);     // 0: dense
    // which commodities of the window a uniform piece covers, hashed: pieces that cover the
    // same commodities are packed into the same items (see the shared-presence flag below)
    std::vector<uint64_t> piece_phash(pieces.size(), 0ull);
    for (size_t i = 0; i < pieces.size(); ++i) {
        uint32_t m = 0u;
        uint64_t hsh = 1469598103934665603ull;
        bool uniform = !t.tiles_dense_only;
        for (size_t q = 0; q < 512 && uniform; ++q) {
            const uint32_t v = piece_mask[pieces[i].mask_at + q];
            hsh = (hsh ^ (v != 0u ? 1u : 0u)) * 1099511628211ull;
            if (v == 0u) continue;
            if (m == 0u) m = v;
            else if (m != v) uniform = false;
        }
        if (uniform && m != 0u) {
            piece_umask[i] = m;
            piece_phash[i] = hsh;
            t.n_pieces_uniform += 1;
        }
    }

    // Tiled layouts cut the links into GROUPS whose tile items, strip units and octets belong
    // to them alone, and deal the groups to blocks: one workgroup then reduces everything a
    // block's links receive into LDS and applies their length update in the same launch.
    const bool grouped = tiles_on && t.link_groups != 0 && t.n_single_pairs == 0;

    // ---- strips: short rows that several links share ---------------------------------------
    // Rows that are left with the very same octets (the same commodities: e.g. the rail links
    // between two nodes) and one mask value each are taken out of the octet stream.  A UNIT is
    // 8 columns (octets) x up to 8 such rows and occupies 8 lanes of a strip item; lane i of
    // the unit gathers the choices and demands of column i once and uses them for all rows.
    struct UnitRef { int32_t item, group, row; };
    std::vector<std::vector<UnitRef>> link_units(n_links);
    t.strip_base.clear(); t.strip_pres.clear(); t.strip_mask.clear(); t.strip_slot.clear();
    t.n_strip_rows = 0;
    std::vector<uint32_t> row_um(n_links, 0u);            // the row's one mask value, 0: none
    std::vector<std::vector<int32_t>> clusters;
    if (tiles_on && !t.tiles_dense_only) {
        std::unordered_map<uint64_t, std::vector<int32_t>> by_hash;
        for (int32_t e = 0; e < n_links; ++e) {
            const size_t n = row_base[e].size();
            if (n < static_cast<size_t>(kStripMinCols) || n > static_cast<size_t>(kStripMaxCols))
                continue;
            // (in a grouped layout a link with pieces belongs to the group of its pieces)
            if (grouped && !link_pieces[e].empty()) continue;
            uint32_t m = 0u;
            bool uniform = true;
            for (uint32_t v : row_mask[e]) {
                if (v == 0u) continue;
                if (m == 0u) m = v;
                else if (m != v) { uniform = false; break; }
            }
            if (!uniform || m == 0u) continue;
            row_um[e] = m;
            uint64_t h = 1469598103934665603ull;
            for (uint32_t v : row_base[e]) h = (h ^ v) * 1099511628211ull;
            by_hash[h ^ (static_cast<uint64_t>(n) << 48)].push_back(e);
        }
        for (auto &kv : by_hash) {
            std::vector<int32_t> &cand = kv.second;         // ascending link ids
            std::vector<bool> used(cand.size(), false);
            for (size_t i = 0; i < cand.size(); ++i) {
                if (used[i]) continue;
                std::vector<int32_t> cl(1, cand[i]);
                for (size_t j = i + 1; j < cand.size(); ++j)
                    if (!used[j] && row_base[cand[j]] == row_base[cand[i]]) {
                        used[j] = true;
                        cl.push_back(cand[j]);
                    }
                if (static_cast<int32_t>(cl.size()) >= kStripMinRows) clusters.push_back(cl);
            }
        }
        std::sort(clusters.begin(), clusters.end());        // by first link: a fixed order
    }
    // a cluster is cut into chunks of up to 8 rows; the units of a chunk stay together
    struct StripChunk { int32_t cluster, r0, n_rows, block; };
    std::vector<StripChunk> strip_chunks;
    for (size_t ci = 0; ci < clusters.size(); ++ci)
        for (size_t r0 = 0; r0 < clusters[ci].size(); r0 += 8)
            strip_chunks.push_back({static_cast<int32_t>(ci), static_cast<int32_t>(r0),
                                    static_cast<int32_t>(std::min<size_t>(8, clusters[ci].size() - r0)),
                                    0});

    // ---- link groups and their blocks ------------------------------------------------------
    // Links whose pieces lie in the same windows with the same cover (the same "classes") would
    // share tile items, so they go into one group, up to 16 links; the links left over are
    // joined where they share a class; a chunk of strip rows is a group; any other link is a
    // group of its own.  The groups are dealt to blocks, heaviest first, each to the lightest
    // block so far.  Any assignment is correct: items and units are formed inside a block.
    std::vector<int32_t> link_block(n_links, 0);
    int32_t n_gblocks = 0;
    if (grouped) {
        struct Group { std::vector<int32_t> links; int64_t weight; };
        std::vector<Group> groups;
        std::vector<bool> placed(n_links, false);
        // classes of pieces
        std::map<std::tuple<int32_t, int32_t, int32_t, uint64_t>, int32_t> class_id;
        std::vector<int32_t> piece_class(pieces.size(), 0);
        for (size_t i = 0; i < pieces.size(); ++i) {
            const bool uni = piece_umask[i] != 0u;
            auto key = std::make_tuple(pieces[i].sig, pieces[i].window, uni ? 1 : 0,
                                       uni ? piece_phash[i] : 0ull);
            auto f = class_id.find(key);
            if (f == class_id.end())
                f = class_id.emplace(key, static_cast<int32_t>(class_id.size())).first;
            piece_class[i] = f->second;
        }
        auto tile_weight = [&](const std::vector<int32_t> &links) {
            std::map<int32_t, int32_t> per_class;
            int64_t octets = 0;
            for (int32_t e : links) {
                for (int32_t pi : link_pieces[e]) per_class[piece_class[pi]] += 1;
                octets += static_cast<int64_t>(row_base[e].size());
            }
            int64_t tasks = (octets + 63) / 64;
            for (const auto &kv : per_class) tasks += (kv.second + kTileRows - 1) / kTileRows;
            return std::make_pair(tasks, 64 * tasks + static_cast<int64_t>(links.size()));
        };
        auto add_group = [&](const std::vector<int32_t> &links, int64_t weight) {
            groups.push_back({links, weight});
            for (int32_t e : links) placed[e] = true;
        };
        // links with the same classes
        std::map<std::vector<int32_t>, std::vector<int32_t>> by_signature;
        for (int32_t e = 0; e < n_links; ++e) {
            if (link_pieces[e].empty()) continue;
            std::vector<int32_t> sgn;
            for (int32_t pi : link_pieces[e]) sgn.push_back(piece_class[pi]);
            std::sort(sgn.begin(), sgn.end());
            by_signature[sgn].push_back(e);
        }
        std::vector<int32_t> loners;
        for (const auto &kv : by_signature) {
            const std::vector<int32_t> &links = kv.second;
            if (links.size() < 2) {
                loners.push_back(links[0]);
                continue;
            }
            const size_t nc = kv.first.size();
            const size_t chunk = kTileRows * std::max<size_t>(1, 16 / nc);
            for (size_t i = 0; i < links.size();) {
                // (rows with many octets left: fewer links, so that no group outweighs a block)
                size_t take = std::min(links.size() - i, chunk);
                std::vector<int32_t> part(links.begin() + i, links.begin() + i + take);
                while (take > 1 && tile_weight(part).first > 32) {
                    take = (take + 1) / 2;
                    part.resize(take);
                }
                add_group(part, tile_weight(part).second);
                i += take;
            }
        }
        // the others, joined where they share a class
        {
            std::sort(loners.begin(), loners.end());
            std::vector<int32_t> parent(n_links);
            for (int32_t e = 0; e < n_links; ++e) parent[e] = e;
            auto find = [&](int32_t x) {
                while (parent[x] != x) x = parent[x] = parent[parent[x]];
                return x;
            };
            std::unordered_map<int32_t, int32_t> class_first;
            for (int32_t e : loners)
                for (int32_t pi : link_pieces[e]) {
                    auto f = class_first.find(piece_class[pi]);
                    if (f == class_first.end()) class_first.emplace(piece_class[pi], e);
                    else {
                        const int32_t a = find(f->second), b = find(e);
                        if (a != b) parent[std::max(a, b)] = std::min(a, b);
                    }
                }
            std::map<int32_t, std::vector<int32_t>> comps;
            for (int32_t e : loners) comps[find(e)].push_back(e);
            for (const auto &kv : comps) {
                const std::vector<int32_t> &links = kv.second;       // ascending
                const int64_t tasks = tile_weight(links).first;
                const size_t parts = static_cast<size_t>((tasks + 31) / 32);
                const size_t per = (links.size() + parts - 1) / std::max<size_t>(1, parts);
                for (size_t i = 0; i < links.size(); i += per) {
                    std::vector<int32_t> part(links.begin() + i,
                                              links.begin() + std::min(links.size(), i + per));
                    add_group(part, tile_weight(part).second);
                }
            }
        }
        // chunks of strip rows (group index remembered in the chunk)
        std::vector<int32_t> chunk_group(strip_chunks.size(), -1);
        for (size_t c = 0; c < strip_chunks.size(); ++c) {
            const StripChunk &sc = strip_chunks[c];
            const std::vector<int32_t> &cl = clusters[sc.cluster];
            std::vector<int32_t> part(cl.begin() + sc.r0, cl.begin() + sc.r0 + sc.n_rows);
            const int64_t units = (static_cast<int64_t>(row_base[cl[0]].size()) + 7) / 8;
            chunk_group[c] = static_cast<int32_t>(groups.size());
            add_group(part, 8 * units + sc.n_rows);
        }
        for (int32_t e = 0; e < n_links; ++e)
            if (!placed[e])
                add_group(std::vector<int32_t>(1, e),
                          static_cast<int64_t>(row_base[e].size()) + 1);
        // blocks
        int64_t want = t.grp_target > 0 ? t.grp_target : 256;
        if (want > static_cast<int64_t>(groups.size())) want = static_cast<int64_t>(groups.size());
        n_gblocks = static_cast<int32_t>(want);
        std::vector<int32_t> order(groups.size());
        for (size_t i = 0; i < order.size(); ++i) order[i] = static_cast<int32_t>(i);
        std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
            return groups[x].weight > groups[y].weight;
        });
        using Load = std::pair<int64_t, int32_t>;         // (weight so far, block)
        std::priority_queue<Load, std::vector<Load>, std::greater<Load>> lightest;
        for (int32_t b = 0; b < n_gblocks; ++b) lightest.push({0, b});
        std::vector<int32_t> group_block(groups.size(), 0);
        for (int32_t gi : order) {
            Load top = lightest.top();
            lightest.pop();
            group_block[gi] = top.second;
            for (int32_t e : groups[gi].links) link_block[e] = top.second;
            top.first += groups[gi].weight;
            lightest.push(top);
        }
        for (size_t c = 0; c < strip_chunks.size(); ++c)
            strip_chunks[c].block = group_block[chunk_group[c]];
        std::stable_sort(strip_chunks.begin(), strip_chunks.end(),
                         [](const StripChunk &x, const StripChunk &y) { return x.block < y.block; });
    }

    // the strip items, chunk after chunk (block after block: a block's units fill items of
    // their own)
    std::vector<int32_t> gblk_strip_ptr(static_cast<size_t>(n_gblocks) + 1, 0);
    {
        int32_t n_units = 0;
        int32_t cur_block = 0;
        for (const StripChunk &sc : strip_chunks) {
            if (grouped && sc.block != cur_block) {
                n_units = (n_units + 7) & ~7;             // the next block starts a new item
                for (int32_t b = cur_block + 1; b <= sc.block; ++b) gblk_strip_ptr[b] = n_units / 8;
                cur_block = sc.block;
            }
            const std::vector<int32_t> &cl = clusters[sc.cluster];
            const std::vector<uint32_t> &bases = row_base[cl[0]];
            const int32_t n_cols = static_cast<int32_t>(bases.size());
            const int32_t r0 = sc.r0, n_rows = sc.n_rows;
            for (int32_t c0 = 0; c0 < n_cols; c0 += 8) {
                const int32_t item = n_units / 8, group = n_units % 8;
                if (static_cast<size_t>(item) * 64 >= t.strip_base.size()) {
                    t.strip_base.resize(t.strip_base.size() + 64, 0u);
                    t.strip_pres.resize(t.strip_pres.size() + 64, 0ull);
                    t.strip_mask.resize(t.strip_mask.size() + 64, 0u);
                    t.strip_slot.resize(t.strip_slot.size() + 64, -1);
                }
                const size_t at = static_cast<size_t>(item) * 64 + static_cast<size_t>(group) * 8;
                for (int32_t i = 0; i < 8 && c0 + i < n_cols; ++i) {
                    t.strip_base[at + i] = bases[c0 + i];
                    uint64_t pres = 0;
                    for (int32_t r = 0; r < n_rows; ++r) {
                        const std::vector<uint32_t> &mk = row_mask[cl[r0 + r]];
                        for (int32_t s8 = 0; s8 < 8; ++s8)
                            if (mk[static_cast<size_t>(c0 + i) * 8 + s8] != 0u)
                                pres |= 1ull << (8 * r + s8);
                    }
                    t.strip_pres[at + i] = pres;
                }
                for (int32_t r = 0; r < n_rows; ++r) {
                    t.strip_mask[at + r] = row_um[cl[r0 + r]];
                    link_units[cl[r0 + r]].push_back({item, group, r});
                }
                n_units += 1;
            }
        }
        if (grouped) {
            n_units = (n_units + 7) & ~7;
            for (int32_t b = cur_block + 1; b <= n_gblocks; ++b) gblk_strip_ptr[b] = n_units / 8;
        }
        for (const std::vector<int32_t> &cl : clusters)
            for (int32_t e : cl) {
                t.n_strip_rows += 1;
                row_base[e].clear(); row_base[e].shrink_to_fit();
                row_mask[e].clear(); row_mask[e].shrink_to_fit();
            }
    }
    t.n_strip_items = static_cast<int32_t>(t.strip_base.size() / 64);
    t.strip_base.resize(t.strip_base.size() + 64, 0u);          // one spare item keeps the
    t.strip_pres.resize(t.strip_pres.size() + 64, 0ull);        // arrays loadable
    t.strip_mask.resize(t.strip_mask.size() + 64, 0u);
    t.strip_slot.resize(t.strip_slot.size() + 64, -1);
    for (int32_t e = 0; e < n_links; ++e) t.n_octets += static_cast<int64_t>(row_base[e].size());

    // Work items: pieces sorted by (block, numbering, window, kind, covered commodities, link),
    // up to kTileRows pieces of one block, one window, one kind and (uniform pieces) one set of
    // covered commodities per item: the rows of a uniform item have the same presence bits, so
    // the kernel clears the demands of the commodities outside once per item.  Dense pieces
    // keep their 512 masks, lane-contiguous like the masks of a pass; a uniform item stores,
    // per column, one byte of presence bits that serves all its rows.
    std::vector<int32_t> item_piece;                      // [kTileRows * n_tile_items], -1: none
    {
        std::vector<int32_t> ord(pieces.size());
        for (size_t i = 0; i < ord.size(); ++i) ord[i] = static_cast<int32_t>(i);
        auto kind = [&](int32_t x) { return piece_umask[x] != 0u ? 1 : 0; };
        std::sort(ord.begin(), ord.end(), [&](int32_t x, int32_t y) {
            const Piece &px = pieces[x], &py = pieces[y];
            if (link_block[px.link] != link_block[py.link])
                return link_block[px.link] < link_block[py.link];
            if (px.sig != py.sig) return px.sig < py.sig;
            if (px.window != py.window) return px.window < py.window;
            if (kind(x) != kind(y)) return kind(x) < kind(y);
            if (piece_phash[x] != piece_phash[y]) return piece_phash[x] < piece_phash[y];
            return px.link < py.link;
        });
        t.tile_mask.clear();
        t.tile_pres.clear();
        t.tile_desc.clear();
        int32_t n_dense = 0, n_uitems = 0;
        // do two uniform pieces cover the same commodities of their window?
        auto same_cover = [&](int32_t x, int32_t y) {
            if (piece_phash[x] != piece_phash[y]) return false;
            for (size_t q = 0; q < 512; ++q)
                if ((piece_mask[pieces[x].mask_at + q] != 0u) !=
                    (piece_mask[pieces[y].mask_at + q] != 0u))
                    return false;
            return true;
        };
        for (size_t i = 0; i < ord.size(); ++i) {
            const int32_t pi = ord[i];
            const Piece &pc = pieces[pi];
            const bool uni = kind(pi) == 1;
            const bool fresh = i == 0 || link_block[pieces[ord[i - 1]].link] != link_block[pc.link] ||
                               pieces[ord[i - 1]].sig != pc.sig ||
                               pieces[ord[i - 1]].window != pc.window ||
                               kind(ord[i - 1]) != kind(pi) ||
                               (uni && !same_cover(ord[i - 1], pi)) ||
                               t.tile_desc[t.tile_desc.size() - kTileDescInts + 2] == kTileRows;
            if (fresh) {
                t.tile_desc.resize(t.tile_desc.size() + kTileDescInts, 0);
                item_piece.resize(item_piece.size() + kTileRows, -1);
                int32_t *d = &t.tile_desc[t.tile_desc.size() - kTileDescInts];
                d[0] = pc.window * kTileIds;
                d[1] = pc.sig | (uni ? 2 : 0);
                d[2] = 0;
                d[3] = uni ? n_uitems : n_dense;
                if (uni) {
                    n_uitems += 1;
                    t.tile_pres.resize(t.tile_pres.size() + 64, 0u);
                }
            }
            int32_t *d = &t.tile_desc[t.tile_desc.size() - kTileDescInts];
            const int32_t r = d[2]++;
            item_piece[item_piece.size() - kTileRows + r] = pi;
            if (uni) {
                d[16 + r] = static_cast<int32_t>(piece_umask[pi]);
                // the same bits for every piece of the item (same_cover)
                uint8_t *pres = &t.tile_pres[t.tile_pres.size() - 64];
                for (size_t c = 0; c < 64; ++c) {
                    uint8_t bits = 0;
                    for (size_t w8 = 0; w8 < 8; ++w8)
                        if (piece_mask[pc.mask_at + c * 8 + w8] != 0u)
                            bits = static_cast<uint8_t>(bits | (1u << w8));
                    pres[c] = bits;
                }
            } else {
                const size_t at = t.tile_mask.size();
                t.tile_mask.resize(at + 512, 0u);
                for (size_t c = 0; c < 64; ++c)
                    for (size_t w8 = 0; w8 < 8; ++w8)
                        t.tile_mask[at + (w8 / 4) * 256 + c * 4 + (w8 % 4)] =
                            piece_mask[pc.mask_at + c * 8 + w8];
                n_dense += 1;
            }
        }
        t.n_tile_items = static_cast<int32_t>(t.tile_desc.size() / kTileDescInts);
        if (t.tile_desc.empty()) t.tile_desc.assign(kTileDescInts, 0);
        t.tile_mask.resize(t.tile_mask.size() + 512, 0u);      // one spare piece keeps it loadable
        t.tile_pres.resize(t.tile_pres.size() + 64, 0u);
        piece_mask.clear(); piece_mask.shrink_to_fit();
    }

    // ---- link blocks and the order of the rows in the flat array ---------------------------
    // The rows are dealt to n_blk blocks, largest row first, each to the block that is lightest
    // so far (a row weighs its octets plus a small constant for the link's update), so that all
    // blocks carry the same work within one small row.  Inside a block the links ascend by id.
    // pos_link lists the links in flat order; pos_slot_ptr gives the slots of each position.
    const int64_t kLinkWeight = 4;
    const int64_t total_passes = (t.n_octets + 63) / 64;
    int64_t blk_passes = t.blk_passes;
    if (blk_passes <= 0) {                       // default: about six blocks per compute unit
        blk_passes = (total_passes + 1535) / 1536;
        if (blk_passes < 3) blk_passes = 3;
    }
    int64_t n_blk = (total_passes + blk_passes - 1) / blk_passes;
    const int64_t by_links = (static_cast<int64_t>(n_links) + kBlkMaxLinks / 2 - 1) / (kBlkMaxLinks / 2);
    if (n_blk < by_links) n_blk = by_links;
    if (n_blk < 1) n_blk = 1;
    if (n_blk > n_links) n_blk = n_links;
    if (grouped) n_blk = n_gblocks;              // the blocks of the link groups instead
    std::vector<std::vector<int32_t>> blk_members(static_cast<size_t>(n_blk));
    if (grouped) {
        for (int32_t e = 0; e < n_links; ++e) blk_members[link_block[e]].push_back(e);
    } else {
        std::vector<int32_t> by_size(n_links);
        for (int32_t e = 0; e < n_links; ++e) by_size[e] = e;
        std::stable_sort(by_size.begin(), by_size.end(), [&](int32_t x, int32_t y) {
            return row_base[x].size() > row_base[y].size();
        });
        using Load = std::pair<int64_t, int32_t>;         // (weight so far, block)
        std::priority_queue<Load, std::vector<Load>, std::greater<Load>> lightest;
        for (int32_t b = 0; b < n_blk; ++b) lightest.push({0, b});
        for (int32_t e : by_size) {
            Load top = lightest.top();
            lightest.pop();
            blk_members[top.second].push_back(e);
            top.first += static_cast<int64_t>(row_base[e].size()) + kLinkWeight;
            lightest.push(top);
        }
    }
    bool blocks_fit = !tiles_on;          // pieces of one item belong to many links
    int32_t slot = 0;
    t.pos_link.clear();
    t.pos_slot_ptr.clear();
    t.blk_pos_ptr.assign(1, 0);
    t.blk_pass_ptr.assign(1, 0);
    for (int64_t b = 0; b < n_blk; ++b) {
        std::vector<int32_t> &members = blk_members[b];
        std::sort(members.begin(), members.end());
        const int32_t blk_slot0 = slot;
        for (int32_t e : members) {
            // append the row to the flat arrays; a new slot at the row's first octet and at
            // every pass boundary
            t.pos_link.push_back(e);
            t.pos_slot_ptr.push_back(slot);
            for (size_t q = 0; q < row_base[e].size(); ++q) {
                const size_t pos = t.oct_base.size();
                uint32_t w = row_base[e][q];
                if (q == 0 || pos % 64 == 0) {
                    w |= kOctNewSlot;
                    if (pos % 64 == 0) t.pass_first_slot.push_back(slot);
                    ++slot;
                }
                t.oct_base.push_back(w);
                t.oct_mask.insert(t.oct_mask.end(), row_mask[e].begin() + 8 * q,
                                  row_mask[e].begin() + 8 * q + 8);
            }
            row_base[e].clear(); row_base[e].shrink_to_fit();
            row_mask[e].clear(); row_mask[e].shrink_to_fit();
        }
        // the next block starts at a pass boundary: padding octets have no masks and no flags
        while (t.oct_base.size() % 64) {
            t.oct_base.push_back(0u);
            t.oct_mask.resize(t.oct_mask.size() + 8, 0u);
        }
        if (slot - blk_slot0 > kBlkMaxSlots || static_cast<int32_t>(members.size()) > kBlkMaxLinks)
            blocks_fit = false;
        t.blk_pos_ptr.push_back(static_cast<int32_t>(t.pos_link.size()));
        t.blk_pass_ptr.push_back(static_cast<int32_t>(t.oct_base.size() / 64));
    }
    t.pos_slot_ptr.push_back(slot);
    t.invcap_pos.resize(n_links);
    for (int32_t i = 0; i < n_links; ++i) t.invcap_pos[i] = t.invcap[t.pos_link[i]];
    t.n_oct_slots = slot;
    int32_t pad_slots = 0;
    if (t.oct_base.empty()) {             // keep one (empty) pass with a slot no link owns
        t.pass_first_slot.push_back(slot);
        t.oct_base.assign(64, 0u);
        t.oct_base[0] = kOctNewSlot;
        t.oct_mask.assign(8 * 64, 0u);
        pad_slots = 1;
        blocks_fit = false;
    }
    // masks lane-contiguous inside a pass: words 0..3 of the 64 octets, then words 4..7, so
    // that each of the two 16-byte loads of a lane is part of one contiguous KiB
    {
        std::vector<uint32_t> tmp(t.oct_mask.size());
        const size_t n_pass = t.oct_base.size() / 64;
        for (size_t ps = 0; ps < n_pass; ++ps)
            for (size_t ln = 0; ln < 64; ++ln)
                for (size_t w8 = 0; w8 < 8; ++w8)
                    tmp[ps * 512 + (w8 / 4) * 256 + ln * 4 + (w8 % 4)] =
                        t.oct_mask[(ps * 64 + ln) * 8 + w8];
        t.oct_mask.swap(tmp);
    }
    // The link's slots outside the octet range follow the octet slots: one per piece, per strip
    // unit it has a row in, and per single-pair chunk, link after link in the flat order of
    // the rows (so that the slots of a block's links are one range).
    const int32_t extra_slot0 = t.n_oct_slots + pad_slots;
    piece_extra.assign(pieces.size(), -1);
    t.schunk_slot.assign(t.schunk_begin.size(), -1);
    t.pos_xslot.resize(2 * static_cast<size_t>(n_links));
    for (int32_t i = 0; i < n_links; ++i) {
        const int32_t e = t.pos_link[i];
        t.pos_xslot[2 * static_cast<size_t>(i)] = extra_slot0 + extra_slots;
        for (int32_t pi : link_pieces[e]) piece_extra[pi] = extra_slots++;
        for (const UnitRef &u : link_units[e])
            t.strip_slot[static_cast<size_t>(u.item) * 64 + static_cast<size_t>(u.group) * 8 + u.row] =
                extra_slot0 + extra_slots++;
        for (int32_t c = link_chunk_first[e]; c < link_chunk_first[e + 1]; ++c)
            t.schunk_slot[c] = extra_slot0 + extra_slots++;
        t.pos_xslot[2 * static_cast<size_t>(i) + 1] = extra_slot0 + extra_slots;
    }
    t.n_slots = extra_slot0 + extra_slots;
    for (int32_t it = 0; it < t.n_tile_items; ++it) {
        int32_t *d = &t.tile_desc[static_cast<size_t>(it) * kTileDescInts];
        for (int32_t r = 0; r < kTileRows; ++r) {
            const int32_t pi = item_piece[static_cast<size_t>(it) * kTileRows + r];
            d[8 + r] = pi >= 0 ? extra_slot0 + piece_extra[pi] : -1;
        }
    }
    // what the workgroup of a block of link groups needs (kGblkDescInts int32 per block):
    //   [0] first and [1] end position   [2] first and [3] end pass
    //   [4] first octet slot, [5] octet slots   [6] first other slot, [7] other slots
    //   [8] first and [9] end tile item  [10] first and [11] end strip item
    if (grouped) {
        std::vector<int32_t> gblk_tile_ptr(static_cast<size_t>(n_gblocks) + 1, t.n_tile_items);
        {
            int32_t b_seen = -1;
            for (int32_t it = 0; it < t.n_tile_items; ++it) {
                const int32_t b = link_block[pieces[item_piece[static_cast<size_t>(it) * kTileRows]].link];
                for (int32_t q = b_seen + 1; q <= b; ++q) gblk_tile_ptr[q] = it;
                b_seen = b;
            }
        }
        bool fits = true;
        t.gblk_desc.assign(static_cast<size_t>(kGblkDescInts) * n_gblocks, 0);
        for (int32_t b = 0; b < n_gblocks; ++b) {
            int32_t *d = &t.gblk_desc[static_cast<size_t>(kGblkDescInts) * b];
            const int32_t i0 = t.blk_pos_ptr[b], i1 = t.blk_pos_ptr[b + 1];
            d[0] = i0;
            d[1] = i1;
            d[2] = t.blk_pass_ptr[b];
            d[3] = t.blk_pass_ptr[b + 1];
            d[4] = t.pos_slot_ptr[i0];
            d[5] = t.pos_slot_ptr[i1] - t.pos_slot_ptr[i0];
            d[6] = i1 > i0 ? t.pos_xslot[2 * static_cast<size_t>(i0)] : extra_slot0;
            d[7] = i1 > i0 ? t.pos_xslot[2 * static_cast<size_t>(i1 - 1) + 1] - d[6] : 0;
            d[8] = gblk_tile_ptr[b];
            d[9] = gblk_tile_ptr[b + 1];
            d[10] = gblk_strip_ptr[b];
            d[11] = gblk_strip_ptr[b + 1];
            const int32_t tasks = (d[3] - d[2]) + (d[9] - d[8]) + (d[11] - d[10]);
            t.gblk_max_slots = std::max(t.gblk_max_slots, d[5] + d[7]);
            t.gblk_max_tasks = std::max(t.gblk_max_tasks, tasks);
            if (d[5] + d[7] > kGblkMaxSlots || i1 <= i0) fits = false;
        }
        t.n_gblocks = fits ? n_gblocks : 0;
        if (!fits) t.gblk_desc.clear();
    }
    if (t.gblk_desc.empty()) t.gblk_desc.assign(kGblkDescInts, 0);
    // the fused kernel covers topologies whose reverse rows are octets only
    t.n_blocks = (blocks_fit && t.n_single_pairs == 0)
                     ? static_cast<int32_t>(t.blk_pos_ptr.size()) - 1 : 0;
    t.blk_desc.assign(8 * static_cast<size_t>(t.n_blocks > 0 ? t.n_blocks : 1), 0);
    for (int32_t b = 0; b < t.n_blocks; ++b) {
        int32_t *d = &t.blk_desc[8 * static_cast<size_t>(b)];
        d[0] = t.blk_pos_ptr[b];
        d[1] = t.blk_pos_ptr[b + 1];
        d[2] = t.blk_pass_ptr[b];
        d[3] = t.blk_pass_ptr[b + 1];
        d[4] = t.pos_slot_ptr[t.blk_pos_ptr[b]];
    }
    if (t.single_pair.empty()) {          // keep the array loadable
        for (int q = 0; q < 2; ++q) {
            t.single_pair.push_back(static_cast<uint32_t>(n_comm));
            t.single_pair.push_back(0u);
        }
    }

}

void build_host_topo(int32_t n_links, const double *cap, int32_t n_comm,
                     const int32_t *comm_path_ptr, int32_t n_paths,
                     const int32_t *path_link_ptr, const int32_t *path_links,
                     HostTopo &t)
{
    t.E = n_links;
    t.K = n_comm;
    t.P = n_paths;
    t.nnz = path_link_ptr[n_paths];
    t.invcap.resize(n_links);
    for (int32_t e = 0; e < n_links; ++e) t.invcap[e] = 1.0 / cap[e];

    t.pmax = 0;
    t.lmax = 0;
    for (int32_t k = 0; k < n_comm; ++k) {
        int32_t np = comm_path_ptr[k + 1] - comm_path_ptr[k];
        if (np > t.pmax) t.pmax = np;
    }
    for (int32_t p = 0; p < n_paths; ++p) {
        int32_t l = path_link_ptr[p + 1] - path_link_ptr[p];
        if (l > t.lmax) t.lmax = l;
    }

    build_reverse_pairs(n_links, n_comm, comm_path_ptr, path_link_ptr, path_links, t);
    build_streaming_layout(n_links, n_comm, comm_path_ptr, path_link_ptr, path_links, t);
    build_forward_records(n_links, n_comm, comm_path_ptr, n_paths, path_link_ptr, path_links, t);
}

}  // namespace nimble

extern "C" nimble_status_t nimble_host_build_reverse(int32_t n_links, int32_t n_comm,
                                                     const int32_t *comm_path_ptr,
                                                     int32_t n_paths,
                                                     const int32_t *path_link_ptr,
                                                     const int32_t *path_links,
                                                     int32_t *rev_ptr, int32_t *rev_comm,
                                                     int32_t *rev_path)
{
    std::string why;
    nimble_status_t st = nimble::validate_csr(n_links, nullptr, n_comm, comm_path_ptr, n_paths,
                                              path_link_ptr, path_links, why);
    if (st != NIMBLE_OK) return st;
    if (!rev_ptr || !rev_comm || !rev_path) return NIMBLE_ERR_INVALID;
    std::vector<double> cap(n_links, 1.0);
    nimble::HostTopo t;
    nimble::build_host_topo(n_links, cap.data(), n_comm, comm_path_ptr, n_paths, path_link_ptr,
                            path_links, t);
    // expand the (commodity, window, mask) pairs back into one entry per incidence
    int32_t w = 0;
    for (int32_t e = 0; e < n_links; ++e) {
        rev_ptr[e] = w;
        for (int32_t i = 0; i < t.rev_rowlen[e]; ++i) {
            const uint32_t a = t.rev_pair[2 * static_cast<size_t>(t.rev_ptr[e] + i)];
            const uint32_t m = t.rev_pair[2 * static_cast<size_t>(t.rev_ptr[e] + i) + 1];
            const int32_t window = static_cast<int32_t>((a >> nimble::kWindowShift) & 3u);
            for (int32_t j = 0; j < 32; ++j)
                if (m & (1u << j)) {
                    rev_comm[w] = static_cast<int32_t>(a & nimble::kCommMask);
                    rev_path[w] = window * 32 + j;
                    ++w;
                }
        }
    }
    rev_ptr[n_links] = w;
    return NIMBLE_OK;
}

extern "C" nimble_status_t nimble_host_records_roundtrip(int32_t n_links, int32_t n_comm,
                                                         const int32_t *comm_path_ptr,
                                                         int32_t n_paths,
                                                         const int32_t *path_link_ptr,
                                                         const int32_t *path_links,
                                                         int32_t *links_out, int32_t *path_record,
                                                         int32_t *n_records_out)
{
    std::string why;
    nimble_status_t st = nimble::validate_csr(n_links, nullptr, n_comm, comm_path_ptr, n_paths,
                                              path_link_ptr, path_links, why);
    if (st != NIMBLE_OK) return st;
    if (!links_out || !path_record || !n_records_out) return NIMBLE_ERR_INVALID;
    std::vector<double> cap(n_links, 1.0);
    nimble::HostTopo t;
    nimble::read_layout_options(t);
    nimble::build_host_topo(n_links, cap.data(), n_comm, comm_path_ptr, n_paths, path_link_ptr,
                            path_links, t);
    *n_records_out = t.n_records;
    if (t.n_records == 0) return NIMBLE_OK;
    // read every incidence back the way the kernel does: header -> first candidate of each
    // commodity -> `stride` local indices per candidate -> record link table; the padding
    // index n_links is skipped
    int64_t w = 0;
    int32_t next_comm = 0;
    // records in a dictionary layout are stored by body: visit them by first commodity
    std::vector<int32_t> visit(t.n_records);
    for (int32_t i = 0; i < t.n_records; ++i) visit[i] = i;
    if (t.rec_dict) {
        if (static_cast<int32_t>(t.rec_body.size()) != t.n_records) return NIMBLE_ERR_INVALID;
        auto k0_of = [&](int32_t ri) {
            uint32_t v;      // word 11 of lane 1
            std::memcpy(&v, t.records.data() + static_cast<size_t>(ri) * t.rec_bytes + 16 + 8, 4);
            return static_cast<int32_t>(v & 0xFFFFFFu);
        };
        std::sort(visit.begin(), visit.end(),
                  [&](int32_t x, int32_t y) { return k0_of(x) < k0_of(y); });
        for (int32_t i = 1; i < t.n_records; ++i)
            if (t.rec_body[i - 1] > t.rec_body[i]) return NIMBLE_ERR_INVALID;
    }
    for (int32_t vi = 0; vi < t.n_records; ++vi) {
        const int32_t ri = visit[vi];
        const uint8_t *rec = t.records.data() + static_cast<size_t>(ri) * t.rec_bytes;
        if (t.rec_lane_major) {
            const int32_t table_bytes = t.rec_table16 ? nimble::kRecTable16 : nimble::kRecTable;
            // lane-major body: word idx of lane l is in load idx / 4 of that lane; with a
            // dictionary words 0..10 come from the record's body there, word 11 and the body
            // number from the lane's 16 bytes of the record
            const int32_t L = t.rec_lanes;
            auto word = [&](int32_t lane, int32_t idx) {
                uint32_t v;
                if (t.rec_dict) {
                    if (idx == 11) {
                        std::memcpy(&v, rec + 16 * lane + 8, 4);
                        return v;
                    }
                    uint32_t body;
                    std::memcpy(&body, rec + 16 * lane + 12, 4);
                    if (static_cast<int32_t>(body) != t.rec_body[ri] ||
                        static_cast<int32_t>(body) >= t.n_bodies)
                        return 0xFFFFFFFFu;      // fails every check below
                    return t.rec_dict_words[(static_cast<size_t>(body) * 3 + idx / 4) * 256 +
                                            4 * lane + idx % 4];
                }
                std::memcpy(&v, rec + table_bytes + 1024 * (idx / 4) + 16 * lane + 4 * (idx % 4),
                            4);
                return v;
            };
            const int32_t *tab = reinterpret_cast<const int32_t *>(rec);
            const uint16_t *tab16 = reinterpret_cast<const uint16_t *>(rec);
            auto link_at = [&](int32_t i) {
                if (t.rec_dict) return static_cast<int32_t>(tab16[8 * (i % 64) + i / 64]);
                const int32_t at = 4 * (i % 64) + i / 64;
                return t.rec_table16 ? static_cast<int32_t>(tab16[at]) : tab[at];
            };
            const int32_t k0 = static_cast<int32_t>(word(1, 11) & 0xFFFFFFu);
            const int32_t nk = static_cast<int32_t>(word(1, 11) >> 24);
            const int32_t p0 = static_cast<int32_t>(word(L + 1, 11));
            if (k0 != next_comm || nk < 1 || nk > 64 / L || p0 != comm_path_ptr[k0])
                return NIMBLE_ERR_INVALID;
            next_comm = k0 + nk;
            // quads flagged as two-by-two products must have that shape in every lane: the
            // record kernel reads nine of their twenty indices and takes the rest as equal
            {
                uint32_t product = 0u;
                if (t.rec_dict)
                    product = t.rec_dict_words[(static_cast<size_t>(t.rec_body[ri]) * 3 + 2) * 256 + 3];
                else if (t.rec_stride == nimble::kRecLaneSteps)
                    product = word(2 * L + 1, 11);
                if (product > 3u) return NIMBLE_ERR_INVALID;
                for (int32_t lane = 0; lane < 64; ++lane) {
                    if (t.rec_dict &&
                        t.rec_dict_words[(static_cast<size_t>(t.rec_body[ri]) * 3 + 2) * 256 +
                                         4 * lane + 3] != product)
                        return NIMBLE_ERR_INVALID;
                    for (int32_t q = 0; q < 2; ++q) {
                        if (!((product >> q) & 1u)) continue;
                        for (int32_t i = 0; i < nimble::kRecLaneSteps; ++i) {
                            const uint32_t v = word(lane, q * nimble::kRecLaneSteps + i);
                            const uint32_t a = v & 0xFFu, b = (v >> 8) & 0xFFu,
                                           c = (v >> 16) & 0xFFu, d = v >> 24;
                            const bool ok = i < 2 ? (a == b && c == d)
                                                  : i == 2 ? (a == b && b == c && c == d)
                                                           : (a == c && b == d);
                            if (!ok) return NIMBLE_ERR_INVALID;
                        }
                    }
                }
            }
            for (int32_t g = 0; g < 64 / L; ++g) {
                const uint32_t meta = word(g * L, 10);
                for (int32_t j = 1; j < L; ++j)
                    if (word(g * L + j, 10) != meta) return NIMBLE_ERR_INVALID;
                if (g >= nk) {
                    if (meta != 0u) return NIMBLE_ERR_INVALID;
                    continue;
                }
                const int32_t np = static_cast<int32_t>(meta & 0xFFu);
                const int32_t p_lo = static_cast<int32_t>(meta >> 8);
                if (p0 + p_lo != comm_path_ptr[k0 + g] ||
                    np != comm_path_ptr[k0 + g + 1] - comm_path_ptr[k0 + g])
                    return NIMBLE_ERR_INVALID;
                if (static_cast<int32_t>(word(g * L, 11)) != t.sigma[k0 + g])
                    return NIMBLE_ERR_INVALID;
                for (int32_t cand = 0; cand < 8 * L; ++cand) {
                    const int32_t j = (cand / 4) % L, q = (cand / 4) / L, c4 = cand % 4;
                    for (int32_t i = 0; i < nimble::kRecLaneSteps; ++i) {
                        const int32_t li = static_cast<int32_t>(
                            (word(g * L + j, q * nimble::kRecLaneSteps + i) >> (8 * c4)) & 0xFFu);
                        if (cand >= np) {      // an absent candidate costs +inf
                            if (li != (i == 0 ? nimble::kRecInfSlot : nimble::kRecZeroSlot))
                                return NIMBLE_ERR_INVALID;
                            continue;
                        }
                        if (li == nimble::kRecZeroSlot) continue;
                        if (li > nimble::kRecZeroSlot || i >= t.rec_stride)
                            return NIMBLE_ERR_INVALID;
                        links_out[w++] = link_at(li);
                    }
                    if (cand < np) path_record[p0 + p_lo + cand] = vi;
                }
            }
            continue;
        }
        const uint8_t *r = rec + nimble::kRecTable;       // the body
        int32_t k0, p0;
        uint16_t h16[8];
        std::memcpy(&k0, r, 4);
        std::memcpy(&p0, r + 4, 4);
        std::memcpy(h16, r + 8, 16);
        const int32_t nk = h16[0], np = h16[1], nl = h16[2], off_cp = h16[3], off_loc = h16[4];
        const int32_t off_cq = h16[6], npad = h16[7];
        if (k0 != next_comm || p0 != comm_path_ptr[k0]) return NIMBLE_ERR_INVALID;
        next_comm = k0 + nk;
        const int32_t *tab = reinterpret_cast<const int32_t *>(rec);
        auto link_at = [&](int32_t i) { return tab[4 * (i % 64) + i / 64]; };
        for (int32_t i = nl; i < 256; ++i)      // the fill repeats the last link
            if (link_at(i) != (nl == 0 ? 0 : link_at(nl - 1))) return NIMBLE_ERR_INVALID;
        const uint16_t *cp16 = reinterpret_cast<const uint16_t *>(r + off_cp);
        const uint16_t *cq16 = reinterpret_cast<const uint16_t *>(r + off_cq);
        if (cq16[nk] != npad || npad % 4) return NIMBLE_ERR_INVALID;
        const uint8_t *loc16 = r + off_loc;
        if (cp16[nk] != np) return NIMBLE_ERR_INVALID;
        for (int32_t c = 0; c < nk; ++c) {
            if (p0 + cp16[c] != comm_path_ptr[k0 + c]) return NIMBLE_ERR_INVALID;
            if (cq16[c] % 4) return NIMBLE_ERR_INVALID;
            for (int32_t p = cp16[c]; p < cp16[c + 1]; ++p) {
                path_record[p0 + p] = ri;
                const int32_t pq = cq16[c] + (p - cp16[c]);       // padded position
                for (int32_t i = 0; i < t.rec_stride; ++i) {
                    const int32_t li = loc16[i * npad + pq];
                    if (li == nl) continue;
                    if (li > nl) return NIMBLE_ERR_INVALID;
                    links_out[w++] = link_at(li);
                }
            }
        }
    }
    return (w == t.nnz && next_comm == n_comm) ? NIMBLE_OK : NIMBLE_ERR_INVALID;
}

extern "C" nimble_status_t nimble_host_layout_stats(int32_t n_links, int32_t n_comm,
                                                    const int32_t *comm_path_ptr,
                                                    int32_t n_paths,
                                                    const int32_t *path_link_ptr,
                                                    const int32_t *path_links, int64_t *out)
{
    std::string why;
    nimble_status_t st = nimble::validate_csr(n_links, nullptr, n_comm, comm_path_ptr, n_paths,
                                              path_link_ptr, path_links, why);
    if (st != NIMBLE_OK) return st;
    if (!out) return NIMBLE_ERR_INVALID;
    std::vector<double> cap(n_links, 1.0);
    nimble::HostTopo t;
    nimble::read_layout_options(t);
    nimble::build_host_topo(n_links, cap.data(), n_comm, comm_path_ptr, n_paths, path_link_ptr,
                            path_links, t);
    out[0] = t.n_pairs;
    out[1] = t.n_octets;
    out[2] = t.n_single_pairs;
    out[3] = t.n_octets_sigma;
    out[4] = static_cast<int64_t>(t.schunk_begin.size());
    out[5] = t.n_slots;
    out[6] = t.n_records;
    out[7] = t.rec_stride;
    out[8] = t.n_blocks;
    out[9] = static_cast<int64_t>(t.oct_base.size());
    out[10] = t.n_pieces;
    out[11] = t.n_tile_items;
    out[12] = t.n_pieces_uniform;
    out[13] = t.n_strip_items;
    out[14] = t.n_strip_rows;
    out[15] = t.rec_lane_major;
    out[16] = t.rec_dict;
    out[17] = t.n_bodies;
    out[21] = t.n_bodies_product;
    out[18] = t.n_gblocks;
    out[19] = t.gblk_max_slots;
    out[20] = t.gblk_max_tasks;
    return NIMBLE_OK;
}

extern "C" nimble_status_t nimble_host_build_reverse_streaming(int32_t n_links, int32_t n_comm,
                                                               const int32_t *comm_path_ptr,
                                                               int32_t n_paths,
                                                               const int32_t *path_link_ptr,
                                                               const int32_t *path_links,
                                                               int32_t *rev_ptr,
                                                               int32_t *rev_comm,
                                                               int32_t *rev_path)
{
    std::string why;
    nimble_status_t st = nimble::validate_csr(n_links, nullptr, n_comm, comm_path_ptr, n_paths,
                                              path_link_ptr, path_links, why);
    if (st != NIMBLE_OK) return st;
    if (!rev_ptr || !rev_comm || !rev_path) return NIMBLE_ERR_INVALID;
    std::vector<double> cap(n_links, 1.0);
    nimble::HostTopo t;
    nimble::read_layout_options(t);
    nimble::build_host_topo(n_links, cap.data(), n_comm, comm_path_ptr, n_paths, path_link_ptr,
                            path_links, t);
    // decode the streaming layout the way the reduce kernel walks it: flat octets with slot
    // flags (slot -> position -> link through pos_slot_ptr and pos_link), sigma octets through the inverse numbering,
    // and chunked single pairs (chunk slot -> link through pos_xslot)
    std::vector<int32_t> inv_sigma(static_cast<size_t>(t.sigma_size), -1);
    for (int32_t k = 0; k < n_comm; ++k)
        if (t.sigma[k] >= 0) inv_sigma[t.sigma[k]] = k;
    // pos_link must list every link once
    if (static_cast<int32_t>(t.pos_link.size()) != n_links ||
        static_cast<int32_t>(t.pos_slot_ptr.size()) != n_links + 1)
        return NIMBLE_ERR_INVALID;
    std::vector<int32_t> link_pos(n_links, -1);
    for (int32_t i = 0; i < n_links; ++i) {
        const int32_t e = t.pos_link[i];
        if (e < 0 || e >= n_links || link_pos[e] >= 0) return NIMBLE_ERR_INVALID;
        link_pos[e] = i;
    }
    std::vector<int32_t> slot_link(static_cast<size_t>(t.n_slots), -1);
    for (int32_t i = 0; i < n_links; ++i)
        for (int32_t sl = t.pos_slot_ptr[i]; sl < t.pos_slot_ptr[i + 1]; ++sl)
            slot_link[sl] = t.pos_link[i];
    for (int32_t i = 0; i < n_links; ++i)
        for (int32_t sl = t.pos_xslot[2 * static_cast<size_t>(i)];
             sl < t.pos_xslot[2 * static_cast<size_t>(i) + 1]; ++sl) {
            if (sl < 0 || sl >= t.n_slots || slot_link[sl] >= 0) return NIMBLE_ERR_INVALID;
            slot_link[sl] = t.pos_link[i];
        }
    // link blocks: every pass of a block holds slots of the block's own links only, and the
    // block's slots and links fit its capacity
    std::vector<int32_t> pass_block(t.oct_base.size() / 64, -1);
    for (int32_t b = 0; b < t.n_blocks; ++b) {
        if (t.blk_pos_ptr[b] >= t.blk_pos_ptr[b + 1] || t.blk_pass_ptr[b] > t.blk_pass_ptr[b + 1])
            return NIMBLE_ERR_INVALID;
        if (t.blk_pos_ptr[b + 1] - t.blk_pos_ptr[b] > nimble::kBlkMaxLinks) return NIMBLE_ERR_INVALID;
        if (t.pos_slot_ptr[t.blk_pos_ptr[b + 1]] - t.pos_slot_ptr[t.blk_pos_ptr[b]] >
            nimble::kBlkMaxSlots)
            return NIMBLE_ERR_INVALID;
        for (int32_t ps = t.blk_pass_ptr[b]; ps < t.blk_pass_ptr[b + 1]; ++ps) pass_block[ps] = b;
    }
    if (t.n_blocks > 0 &&
        (t.blk_pos_ptr[0] != 0 || t.blk_pos_ptr[t.n_blocks] != n_links ||
         t.blk_pass_ptr[0] != 0 ||
         t.blk_pass_ptr[t.n_blocks] != static_cast<int32_t>(t.oct_base.size() / 64)))
        return NIMBLE_ERR_INVALID;
    // blocks of link groups: positions, passes, tile items and strip items are cut into
    // consecutive ranges that cover everything, and whatever a block's tasks write lies in the
    // block's own slot ranges and belongs to its own links
    std::vector<int32_t> pass_gblock(t.oct_base.size() / 64, -1);
    std::vector<int32_t> item_gblock(static_cast<size_t>(t.n_tile_items), -1);
    std::vector<int32_t> sitem_gblock(static_cast<size_t>(t.n_strip_items), -1);
    auto gdesc = [&](int32_t b) { return &t.gblk_desc[static_cast<size_t>(nimble::kGblkDescInts) * b]; };
    for (int32_t b = 0; b < t.n_gblocks; ++b) {
        const int32_t *d = gdesc(b);
        const int32_t *prev = b > 0 ? gdesc(b - 1) : nullptr;
        if (d[0] != (prev ? prev[1] : 0) || d[1] <= d[0]) return NIMBLE_ERR_INVALID;
        if (d[2] != (prev ? prev[3] : 0) || d[3] < d[2]) return NIMBLE_ERR_INVALID;
        if (d[8] != (prev ? prev[9] : 0) || d[9] < d[8]) return NIMBLE_ERR_INVALID;
        if (d[10] != (prev ? prev[11] : 0) || d[11] < d[10]) return NIMBLE_ERR_INVALID;
        if (d[4] != t.pos_slot_ptr[d[0]] || d[5] != t.pos_slot_ptr[d[1]] - d[4]) return NIMBLE_ERR_INVALID;
        if (d[5] + d[7] > nimble::kGblkMaxSlots || d[5] + d[7] > t.gblk_max_slots)
            return NIMBLE_ERR_INVALID;
        for (int32_t i = d[0]; i < d[1]; ++i)
            if (t.pos_xslot[2 * static_cast<size_t>(i)] < d[6] ||
                t.pos_xslot[2 * static_cast<size_t>(i) + 1] > d[6] + d[7])
                return NIMBLE_ERR_INVALID;
        for (int32_t ps = d[2]; ps < d[3]; ++ps) pass_gblock[ps] = b;
        for (int32_t it = d[8]; it < d[9]; ++it) item_gblock[it] = b;
        for (int32_t it = d[10]; it < d[11]; ++it) sitem_gblock[it] = b;
    }
    if (t.n_gblocks > 0) {
        const int32_t *last = gdesc(t.n_gblocks - 1);
        if (last[1] != n_links || last[9] != t.n_tile_items || last[11] != t.n_strip_items ||
            (t.n_octets > 0 && last[3] != static_cast<int32_t>(t.oct_base.size() / 64)))
            return NIMBLE_ERR_INVALID;
    }
    auto in_gblock = [&](int32_t b, int32_t e, int32_t sl, bool octet_slot) {
        if (t.n_gblocks == 0) return true;
        if (b < 0) return false;
        const int32_t *d = gdesc(b);
        if (link_pos[e] < d[0] || link_pos[e] >= d[1]) return false;
        return octet_slot ? (sl >= d[4] && sl < d[4] + d[5]) : (sl >= d[6] && sl < d[6] + d[7]);
    };
    std::vector<std::vector<int64_t>> rows(n_links);      // (commodity << 8 | path) per link
    const size_t n_flat = t.oct_base.size();
    int32_t slot = -1;
    for (size_t i = 0; i < n_flat; ++i) {
        const uint32_t w = t.oct_base[i];
        if (i % 64 == 0) slot = t.pass_first_slot[i / 64] - 1;
        if (w & nimble::kOctNewSlot) ++slot;
        const int32_t e = slot < t.n_slots ? slot_link[slot] : -1;
        if (t.n_blocks > 0 && e >= 0) {
            const int32_t b = pass_block[i / 64];
            if (b < 0 || link_pos[e] < t.blk_pos_ptr[b] || link_pos[e] >= t.blk_pos_ptr[b + 1])
                return NIMBLE_ERR_INVALID;
        }
        if (e >= 0 && t.n_octets > 0 && !in_gblock(pass_gblock[i / 64], e, slot, true))
            return NIMBLE_ERR_INVALID;
        const int32_t base = static_cast<int32_t>(w & ~3u);
        for (int32_t s8 = 0; s8 < 8; ++s8) {
            const uint32_t m = t.oct_mask[(i / 64) * 512 + (s8 / 4) * 256 + (i % 64) * 4 + (s8 % 4)];
            if (!m) continue;
            if (e < 0) return NIMBLE_ERR_INVALID;          // a mask in a padding octet
            const int32_t k = (w & nimble::kOctSigma) ? inv_sigma[base + s8] : base + s8;
            if (k < 0 || k >= n_comm) return NIMBLE_ERR_INVALID;
            for (int32_t j = 0; j < 32; ++j)
                if (m & (1u << j)) rows[e].push_back((static_cast<int64_t>(k) << 8) | j);
        }
    }
    // tile items: every piece belongs to the link that owns its slot
    for (int32_t it = 0; it < t.n_tile_items; ++it) {
        const int32_t *d = &t.tile_desc[static_cast<size_t>(it) * nimble::kTileDescInts];
        if (d[2] < 1 || d[2] > nimble::kTileRows || d[0] % nimble::kTileIds) return NIMBLE_ERR_INVALID;
        for (int32_t r = 0; r < d[2]; ++r) {
            const int32_t sl = d[8 + r];
            if (sl < 0 || sl >= t.n_slots || slot_link[sl] < 0) return NIMBLE_ERR_INVALID;
            const int32_t e = slot_link[sl];
            if (!in_gblock(item_gblock[it], e, sl, false)) return NIMBLE_ERR_INVALID;
            const bool uni = (d[1] & 2) != 0;
            const size_t at = 512 * static_cast<size_t>(d[3] + r);      // dense piece
            for (int32_t c = 0; c < 64; ++c)
                for (int32_t s8 = 0; s8 < 8; ++s8) {
                    uint32_t m;
                    if (uni)
                        m = ((t.tile_pres[64 * static_cast<size_t>(d[3]) + c] >> s8) & 1u)
                                ? static_cast<uint32_t>(d[16 + r]) : 0u;
                    else
                        m = t.tile_mask[at + (s8 / 4) * 256 + c * 4 + (s8 % 4)];
                    if (!m) continue;
                    const int32_t nb = d[0] + 8 * c + s8;
                    const int32_t k = (d[1] & 1) ? (nb < t.sigma_size ? inv_sigma[nb] : -1) : nb;
                    if (k < 0 || k >= n_comm) return NIMBLE_ERR_INVALID;
                    for (int32_t j = 0; j < 32; ++j)
                        if (m & (1u << j)) rows[e].push_back((static_cast<int64_t>(k) << 8) | j);
                }
        }
    }
    // strip items: lane = column of a unit, rows through the unit's slots
    for (int32_t it = 0; it < t.n_strip_items; ++it)
        for (int32_t lane = 0; lane < 64; ++lane) {
            const size_t at = static_cast<size_t>(it) * 64 + lane;
            const uint32_t w = t.strip_base[at];
            const int32_t base = static_cast<int32_t>(w & ~3u);
            for (int32_t r = 0; r < 8; ++r) {
                const uint32_t pb = static_cast<uint32_t>(t.strip_pres[at] >> (8 * r)) & 0xFFu;
                if (!pb) continue;
                const size_t ur = static_cast<size_t>(it) * 64 + (lane & ~7) + r;
                const int32_t sl = t.strip_slot[ur];
                if (sl < 0 || sl >= t.n_slots || slot_link[sl] < 0) return NIMBLE_ERR_INVALID;
                const int32_t e = slot_link[sl];
                if (!in_gblock(sitem_gblock[it], e, sl, false)) return NIMBLE_ERR_INVALID;
                const uint32_t m = t.strip_mask[ur];
                if (!m) return NIMBLE_ERR_INVALID;
                for (int32_t s8 = 0; s8 < 8; ++s8) {
                    if (!((pb >> s8) & 1u)) continue;
                    const int32_t k = (w & nimble::kOctSigma) ? inv_sigma[base + s8] : base + s8;
                    if (k < 0 || k >= n_comm) return NIMBLE_ERR_INVALID;
                    for (int32_t j = 0; j < 32; ++j)
                        if (m & (1u << j)) rows[e].push_back((static_cast<int64_t>(k) << 8) | j);
                }
            }
        }
    for (size_t c = 0; c < t.schunk_begin.size(); ++c) {
        const int32_t e = slot_link[t.schunk_slot[c]];
        if (e < 0) return NIMBLE_ERR_INVALID;
        for (int32_t i = t.schunk_begin[c]; i < t.schunk_end[c]; ++i) {
            const uint32_t a = t.single_pair[2 * static_cast<size_t>(i)];
            const uint32_t m = t.single_pair[2 * static_cast<size_t>(i) + 1];
            const int32_t k = static_cast<int32_t>(a & nimble::kCommMask);
            const int32_t window = static_cast<int32_t>((a >> nimble::kWindowShift) & 3u);
            for (int32_t j = 0; j < 32; ++j)
                if (m & (1u << j)) rows[e].push_back((static_cast<int64_t>(k) << 8) | (window * 32 + j));
        }
    }
    int32_t w = 0;
    for (int32_t e = 0; e < n_links; ++e) {
        std::sort(rows[e].begin(), rows[e].end());
        rev_ptr[e] = w;
        for (int64_t v : rows[e]) {
            if (w >= t.nnz) return NIMBLE_ERR_INVALID;
            rev_comm[w] = static_cast<int32_t>(v >> 8);
            rev_path[w] = static_cast<int32_t>(v & 255);
            ++w;
        }
    }
    rev_ptr[n_links] = w;
    return NIMBLE_OK;
}
