// Driver for the sanitizer run of the host-side layout code (tests/test_host_sanitizers.py builds
// it with -fsanitize=address,undefined together with csrc/host_topo.cpp; no HIP involved).
// Reads a topology from four binary files in a directory (cap.bin float64, cp.bin / lp.bin /
// pl.bin int32), runs every host-only helper of the library on it and checks the round trips:
// the streaming layout decodes to the plain reverse CSR, and every incidence reads back through
// the forward records.  Exit status 0 and a line "OK ..." on success.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../include/nimble_plan_debug.h"

template <class T>
static std::vector<T> read_all(const std::string &path)
{
    std::vector<T> v;
    FILE *f = std::fopen(path.c_str(), "rb");
    if (!f) {
        std::fprintf(stderr, "cannot open %s\n", path.c_str());
        std::exit(2);
    }
    std::fseek(f, 0, SEEK_END);
    const long n = std::ftell(f);
    std::fseek(f, 0, SEEK_SET);
    v.resize(static_cast<size_t>(n) / sizeof(T));
    if (n > 0 && std::fread(v.data(), 1, static_cast<size_t>(n), f) != static_cast<size_t>(n)) {
        std::fprintf(stderr, "short read on %s\n", path.c_str());
        std::exit(2);
    }
    std::fclose(f);
    return v;
}

int main(int argc, char **argv)
{
    if (argc < 2) return 2;
    const std::string dir = argv[1];
    const std::vector<double> cap = read_all<double>(dir + "/cap.bin");
    const std::vector<int32_t> cp = read_all<int32_t>(dir + "/cp.bin");
    const std::vector<int32_t> lp = read_all<int32_t>(dir + "/lp.bin");
    const std::vector<int32_t> pl = read_all<int32_t>(dir + "/pl.bin");
    const int32_t E = static_cast<int32_t>(cap.size());
    const int32_t K = static_cast<int32_t>(cp.size()) - 1;
    const int32_t P = static_cast<int32_t>(lp.size()) - 1;
    const size_t nnz = pl.size();

    std::vector<int32_t> rp1(E + 1), rc1(nnz + 1), rq1(nnz + 1), rp2(E + 1), rc2(nnz + 1),
        rq2(nnz + 1);
    if (nimble_host_build_reverse(E, K, cp.data(), P, lp.data(), pl.data(), rp1.data(), rc1.data(),
                                  rq1.data()) != NIMBLE_OK)
        return 3;
    if (nimble_host_build_reverse_streaming(E, K, cp.data(), P, lp.data(), pl.data(), rp2.data(),
                                            rc2.data(), rq2.data()) != NIMBLE_OK)
        return 4;
    if (rp1 != rp2 || std::memcmp(rc1.data(), rc2.data(), nnz * 4) != 0 ||
        std::memcmp(rq1.data(), rq2.data(), nnz * 4) != 0) {
        std::fprintf(stderr, "the streaming layout does not decode to the reverse CSR\n");
        return 5;
    }
    std::vector<int32_t> links(nnz + 1, -1), path_rec(static_cast<size_t>(P) + 1, -1);
    int32_t n_rec = -1;
    if (nimble_host_records_roundtrip(E, K, cp.data(), P, lp.data(), pl.data(), links.data(),
                                      path_rec.data(), &n_rec) != NIMBLE_OK)
        return 6;
    if (n_rec > 0 && std::memcmp(links.data(), pl.data(), nnz * 4) != 0) {
        std::fprintf(stderr, "the forward records do not read back the incidences\n");
        return 7;
    }
    int64_t stats[22] = {0};
    if (nimble_host_layout_stats(E, K, cp.data(), P, lp.data(), pl.data(), stats) != NIMBLE_OK)
        return 8;
    std::printf("OK records %d pairs %lld octets %lld pieces %lld blocks %lld bodies %lld groups %lld\n", n_rec,
                static_cast<long long>(stats[0]), static_cast<long long>(stats[1]),
                static_cast<long long>(stats[10]), static_cast<long long>(stats[8]),
                static_cast<long long>(stats[17]), static_cast<long long>(stats[18]));
    return 0;
}
