// See pqt_host.hpp.  No GPU call in this file.
#include "pqt_host.hpp"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>

namespace pqt_host {

namespace {

constexpr size_t kAlign = 256;

struct FileCloser {
    void operator()(FILE* f) const {
        if (f) fclose(f);
    }
};

std::string format(const char* fmt, ...) __attribute__((format(printf, 1, 2)));
std::string format(const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    return buf;
}

size_t round_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

}  // namespace

int check_sizes(uint32_t D, uint32_t P, uint32_t k1, uint32_t k2, uint32_t M, uint64_t N, uint64_t H, uint32_t T, uint32_t C,
                uint32_t code_format, bool* hashed, std::string& err) {
    if (code_format != PQT_CODES_TABLE && code_format != PQT_CODES_PAIR_LAMBDA) {
        err = format("code_format %u", code_format);
        return PQT_EFORMAT;
    }
    if (D == 0 || P == 0 || k1 == 0 || k2 == 0 || M == 0 || H == 0 || D % P || D % M || M % P) {
        err = format("inconsistent sizes D=%u P=%u k1=%u k2=%u M=%u", D, P, k1, k2, M);
        return PQT_EFORMAT;
    }
    if (!(P == 1 || P == 2 || P == 4)) {
        err = format("P=%u: only 1, 2 or 4 tree parts", P);
        return PQT_EUNSUPPORTED;
    }
    if (k1 > PQT_MAX_K1 || k2 > PQT_MAX_R || M > 64 || D > 8192) {
        err = format("k1=%u k2=%u M=%u D=%u beyond the kernel limits", k1, k2, M, D);
        return PQT_EUNSUPPORTED;
    }
    if (N >= 0xffffffffull || H >= 0xffffffffull) {
        err = format("N=%llu H=%llu: 32-bit ids and slots only", (unsigned long long)N, (unsigned long long)H);
        return PQT_EUNSUPPORTED;
    }
    long double K = 1;
    for (uint32_t p = 0; p < P; ++p) K *= (long double)k1 * k2;
    if (K >= 18446744073709551616.0L) {
        err = format("(k1*k2)^P = %Lg bins do not fit 64-bit bin numbers", K);
        return PQT_EUNSUPPORTED;
    }
    if ((long double)H > K) {
        err = "H exceeds the number of bins";
        return PQT_EFORMAT;
    }
    if (T < 1 || T > PQT_MAX_T || C < 1 || C > PQT_MAX_C) {
        err = format("default budgets T=%u C=%u out of range", T, C);
        return PQT_EFORMAT;
    }
    const uint32_t npairs = k1 * (k1 - 1) / 2;
    if (code_format == PQT_CODES_PAIR_LAMBDA && (k1 < 2 || npairs > 256)) {
        err = format("k1=%u: (pair, lambda) codes number the %u centroid pairs in one byte", k1, npairs);
        return PQT_EUNSUPPORTED;
    }
    if (hashed) *hashed = (long double)H != K;
    return PQT_OK;
}

int check_arrays(uint32_t k1, uint32_t M, uint64_t N, uint64_t H, uint32_t code_format, const uint32_t* offsets,
                 const uint8_t* tbl_i, const uint8_t* tbl_j, const uint8_t* codes, uint64_t* nonempty, std::string& err) {
    if (offsets[0] != 0 || offsets[H] != N) {
        err = "offsets do not span the ids";
        return PQT_EFORMAT;
    }
    uint64_t filled = 0;
    for (size_t s = 0; s < H; ++s) {
        if (offsets[s + 1] < offsets[s]) {
            err = format("offsets not monotone at slot %zu", s);
            return PQT_EFORMAT;
        }
        filled += offsets[s + 1] > offsets[s] ? 1 : 0;
    }
    if (nonempty) *nonempty = filled;
    const bool pair_codes = code_format == PQT_CODES_PAIR_LAMBDA;
    if (!pair_codes) {
        const size_t ntab = (size_t)M * 256;
        for (size_t e = 0; e < ntab; ++e)
            if (tbl_i[e] >= k1 || tbl_j[e] >= k1) {
                err = "code table names centroid >= k1";
                return PQT_EFORMAT;
            }
    } else if (codes && N > 0) {
        const uint32_t npairs = k1 * (k1 - 1) / 2;
        const size_t code_bytes = (size_t)M * 2;
        uint32_t worst = 0;
        for (size_t v = 0; v < (size_t)N; ++v)
            for (size_t m = 0; m < M; ++m) worst = std::max<uint32_t>(worst, codes[v * code_bytes + 2 * m]);
        if (worst >= npairs) {
            err = format("a code names centroid pair %u of %u", worst, npairs);
            return PQT_EFORMAT;
        }
    }
    return PQT_OK;
}

int read_index_file(const char* path, IndexFile& out, std::string& err) {
    std::unique_ptr<FILE, FileCloser> f(fopen(path, "rb"));
    if (!f) {
        err = format("cannot open '%s'", path);
        return PQT_EIO;
    }
    unsigned char hdr[kAlign];
    if (fread(hdr, 1, kAlign, f.get()) != kAlign) {
        err = format("'%s': truncated header", path);
        return PQT_EFORMAT;
    }
    FileHeader h;
    memcpy(&h, hdr, sizeof(h));
    if (memcmp(h.magic, "PQTIDX1\0", 8) != 0) {
        err = format("'%s': bad magic", path);
        return PQT_EFORMAT;
    }
    if (h.version != 1 || h.offset_bits != 32 || h.code_format > PQT_CODES_PAIR_LAMBDA) {
        err = format("'%s': unsupported version", path);
        return PQT_EFORMAT;
    }
    std::string why;
    int rc = check_sizes(h.D, h.P, h.k1, h.k2, h.M, h.N, h.H, h.T, h.C, h.code_format, nullptr, why);
    if (rc != PQT_OK) {
        err = format("'%s': %.400s", path, why.c_str());
        return rc;
    }
    // the sections' sizes, and with them the length the file must have, before anything is allocated
    const size_t dp = h.D / h.P;
    const size_t code_bytes = (size_t)h.M * (h.code_format == PQT_CODES_PAIR_LAMBDA ? 2 : 1);
    const size_t bytes[9] = {(size_t)h.P * h.k1 * dp * 4, (size_t)h.P * h.k1 * h.k2 * dp * 4, (size_t)h.M * 256, (size_t)h.M * 256,
                             (size_t)h.M * 256 * 4, (size_t)h.M * h.k1 * h.k1 * 4, ((size_t)h.H + 1) * 4, (size_t)h.N * 4,
                             (size_t)h.N * code_bytes};
    size_t need = kAlign;
    for (int s = 0; s < 9; ++s) need = round_up(need) + bytes[s];
    if (fseek(f.get(), 0, SEEK_END) != 0) {
        err = format("'%s': cannot seek", path);
        return PQT_EIO;
    }
    const long have = ftell(f.get());
    if (have < 0 || (size_t)have < need) {
        err = format("'%s': truncated (%ld bytes, the header asks for %zu)", path, have, need);
        return PQT_EFORMAT;
    }
    try {
        out.C1.resize(bytes[0] / 4);
        out.C2.resize(bytes[1] / 4);
        out.ti.resize(bytes[2]);
        out.tj.resize(bytes[3]);
        out.lam.resize(bytes[4] / 4);
        out.cc.resize(bytes[5] / 4);
        out.offsets.resize(bytes[6] / 4);
        out.ids.resize(bytes[7] / 4);
        out.codes.resize(bytes[8]);
    } catch (const std::bad_alloc&) {
        err = format("host allocation failed while reading '%s'", path);
        return PQT_ENOMEM;
    }
    void* dst[9] = {out.C1.data(), out.C2.data(), out.ti.data(), out.tj.data(), out.lam.data(),
                    out.cc.data(), out.offsets.data(), out.ids.data(), out.codes.data()};
    size_t pos = kAlign;
    for (int s = 0; s < 9; ++s) {
        pos = round_up(pos);
        if (fseek(f.get(), (long)pos, SEEK_SET) != 0 || (bytes[s] && fread(dst[s], 1, bytes[s], f.get()) != bytes[s])) {
            err = format("'%s': truncated", path);
            return PQT_EFORMAT;
        }
        pos += bytes[s];
    }
    out.D = h.D; out.P = h.P; out.k1 = h.k1; out.k2 = h.k2; out.M = h.M; out.T = h.T; out.C = h.C;
    out.N = h.N; out.H = h.H; out.code_format = h.code_format;
    return PQT_OK;
}

long region_size(int nA, int nB, int Tn) {
    long n = 0;
    for (int a = 0; a < nA && a < Tn; ++a) {
        const int c = Tn / (a + 1);
        n += c < nB ? c : nB;
    }
    return n;
}

int make_static_order(int R, int T, std::vector<uint32_t>& table, float thr[kSlopes - 1]) {
    const long all = (long)R * R;
    const int Tn = (int)((long)T < all ? (long)T : all);
    // slopes and thresholds by repeated multiplication / division and one square root; this file is compiled
    // with floating-point contraction off, so every platform gets the same bits
    double slope[kSlopes];
    slope[5] = 1.0;
    for (int i = 6; i < kSlopes; ++i) slope[i] = slope[i - 1] * 1.08;
    for (int i = 4; i >= 0; --i) slope[i] = slope[i + 1] / 1.08;
    const double root = std::sqrt(1.08);
    for (int j = 1; j < kSlopes; ++j) thr[j - 1] = (float)(slope[j] / root);
    struct Item {
        double key;
        uint32_t ab;
    };
    // a pair can only be among the first Tn of an order that grows in both ranks if (a+1)(b+1) <= Tn
    std::vector<Item> items;
    table.assign((size_t)kSlopes * Tn, 0u);
    for (int i = 0; i < kSlopes; ++i) {
        items.clear();
        for (int a = 0; a < R && a < Tn; ++a) {
            const int c = Tn / (a + 1);
            const int nb = c < R ? c : R;
            for (int b = 0; b < nb; ++b) {
                const double x = a + 1.0;
                const double y = slope[i] * (b + 1.0);
                const double xx = x * x, yy = y * y;
                items.push_back(Item{xx + yy, ((uint32_t)a << 16) | (uint32_t)b});
            }
        }
        std::sort(items.begin(), items.end(), [](const Item& l, const Item& r) {
            return l.key != r.key ? l.key < r.key : l.ab < r.ab;           // (key, a, b)
        });
        for (int t = 0; t < Tn; ++t) table[(size_t)i * Tn + t] = items[(size_t)t].ab;
    }
    return Tn;
}

}  // namespace pqt_host
