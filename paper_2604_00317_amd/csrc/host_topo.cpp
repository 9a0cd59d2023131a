#include "host_topo.hpp"

#include <cmath>
#include <cstring>

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

void build_host_topo(int32_t n_links, const double *cap, int32_t n_comm,
                     const int32_t *comm_path_ptr, int32_t n_paths,
                     const int32_t *path_link_ptr, const int32_t *path_links,
                     int32_t pairs_per_lane, HostTopo &t)
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

    // ---- reverse CSR of (commodity, window) pairs: stable counting sort by link ---------
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

    // fixed-size chunks; a link with an empty row gets no chunk (its load is 0)
    t.chunk_pairs = kRowLanesHost * pairs_per_lane;
    t.link_chunk_ptr.assign(n_links + 1, 0);
    t.chunk_begin.clear();
    t.chunk_end.clear();
    for (int32_t e = 0; e < n_links; ++e) {
        for (int32_t b = t.rev_ptr[e]; b < t.rev_ptr[e + 1]; b += t.chunk_pairs) {
            t.chunk_begin.push_back(b);
            t.chunk_end.push_back(b + t.chunk_pairs < t.rev_ptr[e + 1] ? b + t.chunk_pairs
                                                                      : t.rev_ptr[e + 1]);
        }
        t.link_chunk_ptr[e + 1] = static_cast<int32_t>(t.chunk_begin.size());
    }

    // ---- forward records ------------------------------------------------------------------
    t.n_records = 0;
    t.records.clear();
    t.rec_stride = t.lmax;
    const bool shape_ok = t.lmax <= kRecMaxStride &&
                          static_cast<double>(t.lmax) * n_paths <= 1.5 * static_cast<double>(t.nnz);
    if (shape_ok) {
        const int32_t S = t.rec_stride;
        std::vector<int32_t> stamp(n_links, -1), local(n_links, 0);
        std::vector<int32_t> links;
        std::vector<uint16_t> cp16, loc16;
        auto align4 = [](int32_t x) { return (x + 3) & ~3; };
        auto bytes_needed = [&](int32_t nl, int32_t nk, int32_t np) {
            return kRecHeader + 4 * nl + align4(2 * (nk + 1)) + 2 * np * S;
        };
        bool ok = true;
        int32_t k = 0;
        while (k < n_comm && ok) {
            const int32_t rec_id = t.n_records;
            const int32_t k0 = k, p0 = comm_path_ptr[k];
            links.clear();
            cp16.assign(1, 0);
            loc16.clear();
            int32_t np = 0;
            while (k < n_comm && k - k0 < kRecMaxComm) {
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
                                  bytes_needed(nl_new, k - k0 + 1, np + (pb - pa)) <= kRecBytes;
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
                np += pb - pa;
                cp16.push_back(static_cast<uint16_t>(np));
                ++k;
            }
            if (k == k0) {      // one commodity alone does not fit a record
                ok = false;
                break;
            }
            const int32_t nk = k - k0, nl = static_cast<int32_t>(links.size());
            for (auto &v : loc16)
                if (v == 0xFFFFu) v = static_cast<uint16_t>(nl);     // the +0.0 price slot
            t.records.resize(static_cast<size_t>(t.n_records + 1) * kRecBytes, 0);
            uint8_t *r = t.records.data() + static_cast<size_t>(t.n_records) * kRecBytes;
            const int32_t off_cp = kRecHeader + 4 * nl;
            const int32_t off_loc = off_cp + align4(2 * (nk + 1));
            const uint16_t h16[8] = {static_cast<uint16_t>(nk), static_cast<uint16_t>(np),
                                     static_cast<uint16_t>(nl), static_cast<uint16_t>(off_cp),
                                     static_cast<uint16_t>(off_loc), 0, 0, 0};
            std::memcpy(r + 0, &k0, 4);
            std::memcpy(r + 4, &p0, 4);
            std::memcpy(r + 8, h16, 16);
            std::memcpy(r + kRecHeader, links.data(), 4 * static_cast<size_t>(nl));
            std::memcpy(r + off_cp, cp16.data(), 2 * cp16.size());
            std::memcpy(r + off_loc, loc16.data(), 2 * loc16.size());
            t.n_records += 1;
        }
        if (!ok) {
            t.n_records = 0;
            t.records.clear();
        }
    }
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
                            path_links, 8, t);
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
    nimble::build_host_topo(n_links, cap.data(), n_comm, comm_path_ptr, n_paths, path_link_ptr,
                            path_links, 8, t);
    *n_records_out = t.n_records;
    if (t.n_records == 0) return NIMBLE_OK;
    // read every incidence back the way the kernel does: header -> first candidate of each
    // commodity -> `stride` local indices per candidate -> record link table; the padding
    // index n_links is skipped
    int64_t w = 0;
    int32_t next_comm = 0;
    for (int32_t ri = 0; ri < t.n_records; ++ri) {
        const uint8_t *r = t.records.data() + static_cast<size_t>(ri) * nimble::kRecBytes;
        int32_t k0, p0;
        uint16_t h16[8];
        std::memcpy(&k0, r, 4);
        std::memcpy(&p0, r + 4, 4);
        std::memcpy(h16, r + 8, 16);
        const int32_t nk = h16[0], np = h16[1], nl = h16[2], off_cp = h16[3], off_loc = h16[4];
        if (k0 != next_comm || p0 != comm_path_ptr[k0]) return NIMBLE_ERR_INVALID;
        next_comm = k0 + nk;
        const int32_t *links = reinterpret_cast<const int32_t *>(r + nimble::kRecHeader);
        const uint16_t *cp16 = reinterpret_cast<const uint16_t *>(r + off_cp);
        const uint16_t *loc16 = reinterpret_cast<const uint16_t *>(r + off_loc);
        if (cp16[nk] != np) return NIMBLE_ERR_INVALID;
        for (int32_t c = 0; c < nk; ++c) {
            if (p0 + cp16[c] != comm_path_ptr[k0 + c]) return NIMBLE_ERR_INVALID;
            for (int32_t p = cp16[c]; p < cp16[c + 1]; ++p) {
                path_record[p0 + p] = ri;
                for (int32_t i = 0; i < t.rec_stride; ++i) {
                    const int32_t li = loc16[p * t.rec_stride + i];
                    if (li == nl) continue;
                    if (li > nl) return NIMBLE_ERR_INVALID;
                    links_out[w++] = links[li];
                }
            }
        }
    }
    return (w == t.nnz && next_comm == n_comm) ? NIMBLE_OK : NIMBLE_ERR_INVALID;
}
