// CPU test program for the library's host-only code (paper_1702_05911_amd/csrc/pqt_host.cpp), built by
// tests/test_host_sanitizer.py with -fsanitize=address,undefined.  Prints one line per request.
//   load <file>                          read_index_file + check_arrays          -> "rc <code> <message>"
//   sizes D P k1 k2 M N H T C format     check_sizes                             -> "rc <code> <message>"
//   static <R> <T>                       make_static_order                       -> "Tn <n>", 9 thresholds (hex floats), 10 table rows
//   region <nA> <nB> <Tn>                region_size                             -> "n <count>"
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>

#include "../../paper_1702_05911_amd/csrc/pqt_host.hpp"

int main(int argc, char** argv) {
    if (argc < 2) return 2;
    const std::string mode = argv[1];
    std::string err;
    if (mode == "load" && argc == 3) {
        pqt_host::IndexFile f;
        int rc = pqt_host::read_index_file(argv[2], f, err);
        uint64_t nonempty = 0;
        if (rc == PQT_OK) {
            bool hashed = false;
            rc = pqt_host::check_sizes(f.D, f.P, f.k1, f.k2, f.M, f.N, f.H, f.T, f.C, f.code_format, &hashed, err);
        }
        if (rc == PQT_OK)
            rc = pqt_host::check_arrays(f.k1, f.M, f.N, f.H, f.code_format, f.offsets.data(), f.ti.data(), f.tj.data(), f.codes.data(),
                                        &nonempty, err);
        printf("rc %d %s\n", rc, rc == PQT_OK ? std::to_string(nonempty).c_str() : err.c_str());
        return 0;
    }
    if (mode == "sizes" && argc == 12) {
        unsigned long long v[10];
        for (int i = 0; i < 10; ++i) v[i] = strtoull(argv[2 + i], nullptr, 10);
        bool hashed = false;
        const int rc = pqt_host::check_sizes((uint32_t)v[0], (uint32_t)v[1], (uint32_t)v[2], (uint32_t)v[3], (uint32_t)v[4], v[5], v[6],
                                             (uint32_t)v[7], (uint32_t)v[8], (uint32_t)v[9], &hashed, err);
        printf("rc %d %s\n", rc, rc == PQT_OK ? (hashed ? "hashed" : "plain") : err.c_str());
        return 0;
    }
    if (mode == "static" && argc == 4) {
        std::vector<uint32_t> table;
        float thr[pqt_host::kSlopes - 1];
        const int Tn = pqt_host::make_static_order(atoi(argv[2]), atoi(argv[3]), table, thr);
        printf("Tn %d\n", Tn);
        for (int j = 0; j < pqt_host::kSlopes - 1; ++j) printf("%a%c", (double)thr[j], j + 2 < pqt_host::kSlopes ? ' ' : '\n');
        for (int i = 0; i < pqt_host::kSlopes; ++i) {
            for (int t = 0; t < Tn; ++t) printf("%u,%u ", table[(size_t)i * Tn + t] >> 16, table[(size_t)i * Tn + t] & 0xffffu);
            printf("\n");
        }
        return 0;
    }
    if (mode == "region" && argc == 5) {
        printf("n %ld\n", pqt_host::region_size(atoi(argv[2]), atoi(argv[3]), atoi(argv[4])));
        return 0;
    }
    return 2;
}
