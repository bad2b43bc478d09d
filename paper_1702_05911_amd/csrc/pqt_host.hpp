// Host-only parts of the library that touch no GPU: the index-file reader, the validation of index
// arrays, and the builder of the fixed traversal-order tables.  Plain C++ (no HIP header), so that this
// code also compiles into a CPU test program under the address and undefined-behaviour sanitizers.
#pragma once
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/pqt.h"

namespace pqt_host {

// First 64 bytes of the 256-byte file header.
struct FileHeader {
    char magic[8];
    uint32_t version, D, P, k1, k2, M;
    uint64_t N, H;
    uint32_t T, C, offset_bits, code_format;
};
static_assert(sizeof(FileHeader) == 64, "header prefix is 64 bytes");

// An index file in host memory (layout: see pqt_index_load in pqt.h).
struct IndexFile {
    uint32_t D = 0, P = 0, k1 = 0, k2 = 0, M = 0, T = 0, C = 0, code_format = 0;
    uint64_t N = 0, H = 0;
    std::vector<float> C1, C2, lam, cc;
    std::vector<uint8_t> ti, tj, codes;
    std::vector<uint32_t> offsets, ids;
};

// Reads and checks the header, then the nine sections.  Returns PQT_OK or PQT_EIO / PQT_EFORMAT /
// PQT_EUNSUPPORTED / PQT_ENOMEM with a message in err.  Nothing is allocated before the sizes in the
// header have passed check_sizes and are consistent with the length of the file.
int read_index_file(const char* path, IndexFile& out, std::string& err);

// Sizes and limits of an index (everything that can be said without looking at the arrays).
int check_sizes(uint32_t D, uint32_t P, uint32_t k1, uint32_t k2, uint32_t M, uint64_t N, uint64_t H, uint32_t T, uint32_t C,
                uint32_t code_format, bool* hashed, std::string& err);

// The arrays that live in host memory: the pointer array spans the ids and is monotone (also counts the
// slots that hold a vector), table entries name centroids below k1, and -- when the codes are in host
// memory (codes != null) and hold (pair, lambda) tuples -- every pair byte names a pair.
int check_arrays(uint32_t k1, uint32_t M, uint64_t N, uint64_t H, uint32_t code_format, const uint32_t* offsets,
                 const uint8_t* tbl_i, const uint8_t* tbl_j, const uint8_t* codes, uint64_t* nonempty, std::string& err);

// The fixed anisotropic traversal order (Sec. 3.2 "Bin Proposal Heuristic"): ten pre-computed orders of the
// rank pairs, one per slope 1.08^k, k = -5..4.  table receives kSlopes x Tn entries r1 << 16 | r2 with
// Tn = min(T, R^2) (returned); thr the nine boundaries 1.08^(j - 5.5), j = 1..9, between neighbouring slopes.
constexpr int kSlopes = 10;
int make_static_order(int R, int T, std::vector<uint32_t>& table, float thr[kSlopes - 1]);

// number of pairs (a, b), a < nA, b < nB, with (a+1)(b+1) <= Tn
long region_size(int nA, int nB, int Tn);

}  // namespace pqt_host
