// Host-side preparation of a topology: validation of the two-level CSR, the reverse
// link -> (commodity, path) CSR, and its split into fixed-size chunks.  No HIP calls here.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/nimble_plan.h"

namespace nimble {

// Packed reverse entry: bit 31 = first entry of this commodity in this link's row,
// bits 30..7 = commodity, bits 6..0 = candidate index inside the commodity.
constexpr int kPathBits = 7;
constexpr uint32_t kPathMask = (1u << kPathBits) - 1u;
constexpr uint32_t kCommMask = (1u << 24) - 1u;
constexpr uint32_t kFirstFlag = 1u << 31;
constexpr int32_t kMaxComm = (1 << 24) - 2;   // one id is kept as the padding sentinel
constexpr int32_t kMaxPathsPerComm = 127;     // 0xFF in the choice array marks "no path"
constexpr int32_t kRevChunk = 1024;           // reverse entries per reduction chunk
constexpr int32_t kRevAlign = 4;              // rows are padded to 16 bytes

inline uint32_t pack_entry(uint32_t comm, uint32_t path, bool first)
{
    return (first ? kFirstFlag : 0u) | (comm << kPathBits) | path;
}

struct HostTopo {
    int32_t E = 0, K = 0, P = 0;
    int64_t nnz = 0;
    int32_t pmax = 0;       // most candidates of any commodity
    int32_t lmax = 0;       // most links of any path
    std::vector<double> invcap;
    // reverse CSR, rows padded to kRevAlign entries with the sentinel commodity K
    std::vector<int32_t> rev_ptr;        // [E+1], padded offsets
    std::vector<uint32_t> rev_entry;     // [rev_ptr[E]]
    std::vector<int32_t> rev_rowlen;     // [E], unpadded row lengths
    // chunks of at most kRevChunk entries, never crossing a row
    std::vector<int32_t> chunk_begin;    // [n_chunks]
    std::vector<int32_t> chunk_end;      // [n_chunks]
    std::vector<int32_t> link_chunk_ptr; // [E+1]
};

// Checks every documented precondition.  Returns NIMBLE_OK or the error; `why` gets the text.
nimble_status_t validate_csr(int32_t n_links, const double *cap, int32_t n_comm,
                             const int32_t *comm_path_ptr, int32_t n_paths,
                             const int32_t *path_link_ptr, const int32_t *path_links,
                             std::string &why);

// Builds everything in HostTopo from validated input.
void build_host_topo(int32_t n_links, const double *cap, int32_t n_comm,
                     const int32_t *comm_path_ptr, int32_t n_paths,
                     const int32_t *path_link_ptr, const int32_t *path_links, HostTopo &out);

}  // namespace nimble
