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
                     const int32_t *path_link_ptr, const int32_t *path_links, HostTopo &t)
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

    // stable counting sort of the incidences by link id
    t.rev_rowlen.assign(n_links, 0);
    for (int64_t i = 0; i < t.nnz; ++i) t.rev_rowlen[path_links[i]] += 1;
    t.rev_ptr.assign(n_links + 1, 0);
    for (int32_t e = 0; e < n_links; ++e) {
        int32_t padded = (t.rev_rowlen[e] + kRevAlign - 1) / kRevAlign * kRevAlign;
        t.rev_ptr[e + 1] = t.rev_ptr[e] + padded;
    }
    const uint32_t pad = pack_entry(static_cast<uint32_t>(n_comm), 0u, false);
    t.rev_entry.assign(static_cast<size_t>(t.rev_ptr[n_links]), pad);
    std::vector<int32_t> fill(t.rev_ptr.begin(), t.rev_ptr.end() - 1);
    std::vector<int32_t> last_comm(n_links, -1);
    for (int32_t k = 0; k < n_comm; ++k)
        for (int32_t p = comm_path_ptr[k]; p < comm_path_ptr[k + 1]; ++p)
            for (int32_t i = path_link_ptr[p]; i < path_link_ptr[p + 1]; ++i) {
                int32_t e = path_links[i];
                bool first = last_comm[e] != k;
                last_comm[e] = k;
                t.rev_entry[fill[e]++] = pack_entry(static_cast<uint32_t>(k),
                                                    static_cast<uint32_t>(p - comm_path_ptr[k]),
                                                    first);
            }

    // fixed-size chunks; a link with an empty row still gets no chunk (its load is 0)
    t.link_chunk_ptr.assign(n_links + 1, 0);
    t.chunk_begin.clear();
    t.chunk_end.clear();
    for (int32_t e = 0; e < n_links; ++e) {
        for (int32_t b = t.rev_ptr[e]; b < t.rev_ptr[e + 1]; b += kRevChunk) {
            t.chunk_begin.push_back(b);
            t.chunk_end.push_back(b + kRevChunk < t.rev_ptr[e + 1] ? b + kRevChunk
                                                                  : t.rev_ptr[e + 1]);
        }
        t.link_chunk_ptr[e + 1] = static_cast<int32_t>(t.chunk_begin.size());
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
                            path_links, t);
    int32_t w = 0;
    for (int32_t e = 0; e < n_links; ++e) {
        rev_ptr[e] = w;
        for (int32_t i = 0; i < t.rev_rowlen[e]; ++i) {
            uint32_t v = t.rev_entry[t.rev_ptr[e] + i];
            rev_comm[w] = static_cast<int32_t>((v >> nimble::kPathBits) & nimble::kCommMask);
            rev_path[w] = static_cast<int32_t>(v & nimble::kPathMask);
            ++w;
        }
    }
    rev_ptr[n_links] = w;
    return NIMBLE_OK;
}
