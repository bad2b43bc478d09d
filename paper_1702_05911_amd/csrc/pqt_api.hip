// C ABI of the PQT query library: index loading, budgets, the batched query and stage timing.
// Host code only; the three kernels live in traverse.hip, rank_bins.hip and rerank.hip.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "pqt_host.hpp"
#include "pqt_index.hpp"

namespace pqt_host {

char* error_buffer() {
    static thread_local char buf[512] = "";
    return buf;
}

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 512, fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace pqt_host

using pqt_host::DeviceGuard;
using pqt_host::fail;

namespace {

constexpr int kMaxProfiledCalls = 4096;

// The entry point that allocates nothing takes its per-batch workspace from this array instead of
// hipMalloc.  Every GPU the library runs on holds its own copy at its own address (looked up once
// per device); host code only ever uses that address, never the array's name.
constexpr size_t kScratchBytes = 32u << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// address of `scratch` on the current device (which must be `device`); null on failure
unsigned char* scratch_on_device(int device) {
    if (device < 0 || device >= kMaxDevices) return nullptr;
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[device] = static_cast<unsigned char*>(ptr);
    }
    return g_scratch_ptr[device];
}

}  // namespace


namespace {

constexpr size_t kAlign = 256;

// largest byte at an even position (the pair bytes of (pair, lambda) codes); n = number of byte pairs
__global__ void max_even_byte_kernel(const uint8_t* codes, uint64_t n, uint32_t* out) {
    uint32_t worst = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        worst = max(worst, (uint32_t)codes[2 * i]);
    atomicMax(out, worst);
}

using pqt_host::FileHeader;

struct FileCloser {
    void operator()(FILE* f) const {
        if (f) fclose(f);
    }
};

template <typename Tp>
int upload(Tp** dev, const void* src, size_t bytes, hipMemcpyKind kind, uint64_t* account) {
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(dev), bytes ? bytes : 1));
    if (bytes) HIP_TRY(hipMemcpy(*dev, src, bytes, kind));
    *account += bytes;
    return PQT_OK;
}

// Workgroup size of the re-rank kernel and candidates per thread: the fewest threads that hold the
// candidate budget (a thread keeps the keys of its candidates in registers; fewer threads per query
// leave room for more queries per compute unit).
int rerank_threads(const pqt_index* ix, int* keys_per_thread = nullptr, int64_t nq = -1) {
    int t, kpt;
    pqt::rerank_shape((int)ix->C, (int)ix->M, (int)ix->code_format, &t, &kpt);
    if (keys_per_thread) *keys_per_thread = kpt;
    if (nq >= 0 && nq <= 1024) t = 1024;      // a small batch leaves the chip idle: more threads per query, answer sooner
    return t;
}

// Runs of a query the re-rank workgroup keeps in LDS: twice what the candidate budget needs at the
// index's mean run length, as a power of two (the kernel clamps it to 64..T and reads longer lists
// from memory).
int rerank_runs_in_lds(const pqt_index* ix) {
    const double mean_run = ix->nonempty_slots ? (double)ix->N / (double)ix->nonempty_slots : 1.0;
    const double want = 2.0 * (double)ix->C / (mean_run < 1.0 ? 1.0 : mean_run);
    int r = 64;
    while (r < (int)ix->T && (double)r < want) r *= 2;
    return r;
}

// Can the re-rank kernel also run the full bin ranking of the queries the head pass leaves over?
// (two tree parts; few enough tuples per thread of the re-rank workgroup; the LDS of both fits)
bool can_fuse_ranking(const pqt_index* ix, int k, int w, int64_t nq) {
    if (ix->P != 2) return false;
    const int R = w * (int)ix->k2;
    const int threads = rerank_threads(ix, nullptr, nq);
    const pqt::RankOffsets ro = pqt::rank_offsets(ix->P, R, ix->T, ix->hashed, false);
    if (ro.Tcap > pqt::rerank_fused_tuples_per_thread() * threads) return false;
    return pqt::rerank_lds_bytes(ix->M, ix->k1, ix->T, ix->C, k, threads, ro.total, (int)ix->code_format,
                                 rerank_runs_in_lds(ix)) <= ix->lds_limit;
}

int check_query_limits(const pqt_index* ix, int k, int w, int64_t nq, size_t* lds_out) {
    const int R = w * (int)ix->k2;
    const size_t l1 = pqt::traverse_lds_bytes(ix->D, ix->P, ix->k1, ix->k2, ix->M, w);
    const size_t l2 = pqt::rank_lds_bytes(ix->P, R, ix->T, ix->hashed ? 1 : 2);   // 2: room for the slots tap
    const int threads = rerank_threads(ix, nullptr, nq);
    const size_t l3 = pqt::rerank_lds_bytes(ix->M, ix->k1, ix->T, ix->C, k, threads, 0, (int)ix->code_format,
                                            rerank_runs_in_lds(ix));
    if (l1 > ix->lds_limit || l2 > ix->lds_limit || l3 > ix->lds_limit)
        return fail(PQT_EUNSUPPORTED,
                    "LDS budget exceeded (traverse %zu, rank %zu, rerank %zu bytes of %zu) for D=%u M=%u k1=%u R=%d T=%u C=%u",
                    l1, l2, l3, ix->lds_limit, ix->D, ix->M, ix->k1, R, ix->T, ix->C);
    if (lds_out) { lds_out[0] = l1; lds_out[1] = l2; lds_out[2] = l3; }
    return PQT_OK;
}

}  // namespace

int pqt_host::ensure_workspace(pqt_index* ix, int64_t nq, int R) {
    if (nq <= ix->ws_nq && R <= ix->ws_R && (int)ix->T <= ix->ws_T) return PQT_OK;
    // the new workspace covers the largest batch, list length and tuple count seen so far
    const int64_t n = nq > ix->ws_nq ? nq : ix->ws_nq;
    const int r = R > ix->ws_R ? R : ix->ws_R;
    const int t = (int)ix->T > ix->ws_T ? (int)ix->T : ix->ws_T;
    ix->free_workspace();
    ix->ws_R = ix->ws_T = 0;
    const size_t ba = sizeof(float) * (size_t)n * ix->M * ix->k1;
    const size_t bl = sizeof(float) * (size_t)n * ix->P * r;
    const size_t br = sizeof(uint2) * (size_t)n * t;
    const size_t bm = sizeof(uint2) * (size_t)n;
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->ws_a), ba));
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->ws_Ld), bl));
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->ws_Lid), bl));
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->ws_runs), br));
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->ws_meta), bm));
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->ws_counters), sizeof(uint32_t) * 2));
    HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->ws_order), sizeof(uint32_t) * (size_t)n));
    ix->ws_nq = n; ix->ws_R = r; ix->ws_T = t;
    ix->bytes_workspace = ba + 2 * bl + br + bm + sizeof(uint32_t) * ((size_t)n + 2);
    return PQT_OK;
}

extern "C" {

const char* pqt_last_error(void) { return pqt_host::error_buffer(); }

int pqt_index_from_arrays(const pqt_index_arrays* a, int location, int device, pqt_index** out) {
    if (!a || !out) return fail(PQT_EINVAL, "pqt_index_from_arrays: null argument");
    *out = nullptr;
    if (location != PQT_HOST && location != PQT_DEVICE)
        return fail(PQT_EINVAL, "pqt_index_from_arrays: location must be PQT_HOST or PQT_DEVICE");
    if (a->code_format != PQT_CODES_TABLE && a->code_format != PQT_CODES_PAIR_LAMBDA)
        return fail(PQT_EINVAL, "pqt_index_from_arrays: code_format %u", a->code_format);
    const bool pair_codes = a->code_format == PQT_CODES_PAIR_LAMBDA;   // the line table is not used then
    if (!a->C1 || !a->C2 || !a->cc || !a->offsets || (a->N > 0 && (!a->ids || !a->codes)) ||
        (!pair_codes && (!a->tbl_i || !a->tbl_j || !a->tbl_lambda)))
        return fail(PQT_EINVAL, "pqt_index_from_arrays: null array");
    const pqt_index_arrays& h = *a;
    std::string why;
    bool hashed = false;
    int vrc = pqt_host::check_sizes(h.D, h.P, h.k1, h.k2, h.M, h.N, h.H, h.T, h.C, h.code_format, &hashed, why);
    if (vrc != PQT_OK) return fail(vrc, "%s", why.c_str());
    const uint32_t npairs = h.k1 * (h.k1 - 1) / 2;

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev)
        return fail(PQT_EHIP, "GPU %d is not available (%d visible)", device, ndev);
    DeviceGuard guard(device);
    if (!guard.ok) return fail(PQT_EHIP, "cannot select GPU %d", device);

    // the pointer array must be a prefix sum that spans the ids (checked on the host)
    const size_t dp = h.D / h.P, ds = h.D / h.M;
    std::vector<uint32_t> off_copy;
    const uint32_t* off = h.offsets;
    if (location == PQT_DEVICE) {
        try {
            off_copy.resize((size_t)h.H + 1);
        } catch (const std::bad_alloc&) {
            return fail(PQT_ENOMEM, "host allocation failed");
        }
        HIP_TRY(hipMemcpy(off_copy.data(), h.offsets, off_copy.size() * 4, hipMemcpyDeviceToHost));
        off = off_copy.data();
    }
    uint64_t nonempty = 0;
    vrc = pqt_host::check_arrays(h.k1, h.M, h.N, h.H, h.code_format, off, h.tbl_i, h.tbl_j,
                                 location == PQT_HOST ? h.codes : nullptr, &nonempty, why);
    if (vrc != PQT_OK) return fail(vrc, "%s", why.c_str());
    const size_t ntab = (size_t)h.M * 256;
    const size_t code_bytes = (size_t)h.M * (pair_codes ? 2 : 1);
    if (pair_codes && h.N > 0 && location == PQT_DEVICE) {       // every pair byte must name a pair (codes on the GPU)
        uint32_t worst = 0;
        uint32_t* dmax = nullptr;
        HIP_TRY(hipMalloc(reinterpret_cast<void**>(&dmax), sizeof(uint32_t)));
        hipError_t e = hipMemset(dmax, 0, sizeof(uint32_t));
        if (e == hipSuccess) {
            hipLaunchKernelGGL(max_even_byte_kernel, dim3(1024), dim3(256), 0, 0, h.codes, (uint64_t)h.N * h.M, dmax);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipMemcpy(&worst, dmax, sizeof(uint32_t), hipMemcpyDeviceToHost);
        (void)hipFree(dmax);
        if (e != hipSuccess) return fail(PQT_EHIP, "checking the codes: %s", hipGetErrorString(e));
        if (worst >= npairs) return fail(PQT_EFORMAT, "a code names centroid pair %u of %u", worst, npairs);
    }

    // squared norms of the centroid sub-parts, and the code table with its pair distance folded in
    std::vector<float> c1n((size_t)h.M * h.k1);
    const size_t per = h.M / h.P;
    for (size_t m = 0; m < h.M; ++m) {
        const size_t p = m / per, lo = m * ds - p * dp;
        for (size_t i = 0; i < h.k1; ++i) {
            double s = 0;
            for (size_t d = 0; d < ds; ++d) {
                const double v = h.C1[(p * h.k1 + i) * dp + lo + d];
                s += v * v;
            }
            c1n[m * h.k1 + i] = (float)s;
        }
    }
    std::vector<float> c2t;
    if (dp % 4 == 0) {
        c2t.resize((size_t)h.P * h.k1 * h.k2 * dp);
        for (size_t pi = 0; pi < (size_t)h.P * h.k1; ++pi)
            for (size_t j = 0; j < h.k2; ++j)
                for (size_t d = 0; d < dp; ++d)
                    c2t[((pi * (dp / 4) + d / 4) * h.k2 + j) * 4 + d % 4] = h.C2[(pi * h.k2 + j) * dp + d];
    }
    std::vector<pqt::CodeEntry> table(ntab);
    if (pair_codes) {
        // entry = pair number of i < j in lexicographic order; kc holds ||c_i - c_j||^2 of the sub-part
        for (size_t m = 0; m < h.M; ++m) {
            size_t e = m * 256;
            for (uint32_t i = 0; i < h.k1; ++i)
                for (uint32_t j = i + 1; j < h.k1; ++j, ++e) {
                    table[e].ij = i | (j << 8);
                    table[e].lam = 0.0f;
                    table[e].kc = h.cc[(m * h.k1 + i) * h.k1 + j];
                }
            for (; e < (m + 1) * 256; ++e) table[e] = pqt::CodeEntry{0u, 0.0f, 0.0f};
        }
    }
    for (size_t m = 0; m < h.M && !pair_codes; ++m)
        for (size_t c = 0; c < 256; ++c) {
            const size_t e = m * 256 + c;
            table[e].ij = (uint32_t)h.tbl_i[e] | ((uint32_t)h.tbl_j[e] << 8);
            table[e].lam = h.tbl_lambda[e];
            const double lam = h.tbl_lambda[e];
            table[e].kc = (float)((lam * lam - lam) * (double)h.cc[(m * h.k1 + h.tbl_i[e]) * h.k1 + h.tbl_j[e]]);
        }

    // Dynamic LDS a kernel may ask for: 160 KB once the runtime has accepted that ceiling for all
    // three kernels, else the 64 KB every HIP device grants without asking.
    size_t lds_limit = pqt::kMaxLds;
    if (pqt::configure_traverse(lds_limit) != hipSuccess || pqt::configure_rank(lds_limit) != hipSuccess ||
        pqt::configure_rerank(lds_limit) != hipSuccess) {
        (void)hipGetLastError();
        lds_limit = 64 * 1024;
        HIP_TRY(pqt::configure_traverse(lds_limit));
        HIP_TRY(pqt::configure_rank(lds_limit));
        HIP_TRY(pqt::configure_rerank(lds_limit));
    }
    (void)scratch_on_device(device);       // looked up now, so that the entry point that must not allocate finds it

    pqt_index* ix = new (std::nothrow) pqt_index();
    if (!ix) return fail(PQT_ENOMEM, "host allocation failed");
    ix->D = h.D; ix->P = h.P; ix->k1 = h.k1; ix->k2 = h.k2; ix->M = h.M; ix->T = h.T; ix->C = h.C;
    ix->N = h.N; ix->H = h.H; ix->device = device;
    ix->lds_limit = lds_limit;
    ix->hashed = hashed;
    ix->code_format = h.code_format;
    ix->nonempty_slots = nonempty;
    try {
        ix->h_C1.assign(h.C1, h.C1 + (size_t)h.P * h.k1 * dp);
        ix->h_C2.assign(h.C2, h.C2 + (size_t)h.P * h.k1 * h.k2 * dp);
        if (h.tbl_i && h.tbl_j && h.tbl_lambda) {
            ix->h_ti.assign(h.tbl_i, h.tbl_i + ntab);
            ix->h_tj.assign(h.tbl_j, h.tbl_j + ntab);
            ix->h_lam.assign(h.tbl_lambda, h.tbl_lambda + ntab);
        } else {                       // (pair, lambda) codes without a line table: kept as zeros
            ix->h_ti.assign(ntab, 0);
            ix->h_tj.assign(ntab, 0);
            ix->h_lam.assign(ntab, 0.0f);
        }
        ix->h_cc.assign(h.cc, h.cc + (size_t)h.M * h.k1 * h.k1);
    } catch (const std::bad_alloc&) {
        delete ix;
        return fail(PQT_ENOMEM, "host allocation failed");
    }
    const hipMemcpyKind big = location == PQT_DEVICE ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    int rc = PQT_OK;
    if ((rc = upload(&ix->C1, h.C1, (size_t)h.P * h.k1 * dp * 4, hipMemcpyHostToDevice, &ix->bytes_index)) ||
        (rc = upload(&ix->c1n, c1n.data(), c1n.size() * 4, hipMemcpyHostToDevice, &ix->bytes_index)) ||
        (rc = upload(&ix->C2, h.C2, (size_t)h.P * h.k1 * h.k2 * dp * 4, hipMemcpyHostToDevice, &ix->bytes_index)) ||
        (c2t.size() && (rc = upload(&ix->C2t, c2t.data(), c2t.size() * 4, hipMemcpyHostToDevice, &ix->bytes_index))) ||
        (rc = upload(&ix->table, table.data(), table.size() * sizeof(pqt::CodeEntry), hipMemcpyHostToDevice,
                     &ix->bytes_index)) ||
        (rc = upload(&ix->offsets, h.offsets, ((size_t)h.H + 1) * 4, big, &ix->bytes_index)) ||
        (rc = upload(&ix->ids, h.ids, (size_t)h.N * 4, big, &ix->bytes_index)) ||
        (rc = upload(&ix->codes, h.codes, (size_t)h.N * code_bytes, big, &ix->bytes_index))) {
        pqt_index_free(ix);
        return rc;
    }
    *out = ix;
    return PQT_OK;
}

int pqt_index_load(const char* path, int device, pqt_index** out) {
    if (!path || !out) return fail(PQT_EINVAL, "pqt_index_load: null argument");
    *out = nullptr;
    pqt_host::IndexFile h;
    std::string why;
    const int frc = pqt_host::read_index_file(path, h, why);
    if (frc != PQT_OK) return fail(frc, "%s", why.c_str());
    std::vector<float>&C1 = h.C1, &C2 = h.C2, &lam = h.lam, &cc = h.cc;
    std::vector<uint8_t>&ti = h.ti, &tj = h.tj, &codes = h.codes;
    std::vector<uint32_t>&offsets = h.offsets, &ids = h.ids;
    pqt_index_arrays a = {};
    a.N = h.N; a.H = h.H; a.D = h.D; a.P = h.P; a.k1 = h.k1; a.k2 = h.k2; a.M = h.M; a.T = h.T; a.C = h.C;
    a.C1 = C1.data(); a.C2 = C2.data(); a.tbl_i = ti.data(); a.tbl_j = tj.data(); a.tbl_lambda = lam.data();
    a.cc = cc.data(); a.offsets = offsets.data(); a.ids = ids.data(); a.codes = codes.data();
    a.code_format = h.code_format;
    const int rc = pqt_index_from_arrays(&a, PQT_HOST, device, out);
    if (rc != PQT_OK) {
        char msg[512];
        snprintf(msg, sizeof(msg), "%s", pqt_host::error_buffer());
        return fail(rc, "'%s': %.400s", path, msg);
    }
    return PQT_OK;
}

int pqt_index_save(const pqt_index* ix, const char* path) {
    if (!ix || !path) return fail(PQT_EINVAL, "pqt_index_save: null argument");
    DeviceGuard guard(ix->device);
    if (!guard.ok) return fail(PQT_EHIP, "cannot select GPU %d", ix->device);
    std::unique_ptr<FILE, FileCloser> f(fopen(path, "wb"));
    if (!f) return fail(PQT_EIO, "cannot create '%s'", path);
    unsigned char hdr[kAlign] = {0};
    FileHeader h;
    memset(&h, 0, sizeof(h));
    memcpy(h.magic, "PQTIDX1\0", 8);
    h.version = 1; h.D = ix->D; h.P = ix->P; h.k1 = ix->k1; h.k2 = ix->k2; h.M = ix->M;
    h.N = ix->N; h.H = ix->H; h.T = ix->T; h.C = ix->C; h.offset_bits = 32; h.code_format = ix->code_format;
    memcpy(hdr, &h, sizeof(h));
    bool ok = fwrite(hdr, 1, kAlign, f.get()) == kAlign;
    auto put = [&](const void* src, size_t bytes) {
        static const unsigned char zeros[kAlign] = {0};
        const long pos = ftell(f.get());
        const size_t pad = (kAlign - (size_t)pos % kAlign) % kAlign;
        ok = ok && pos >= 0 && (pad == 0 || fwrite(zeros, 1, pad, f.get()) == pad) &&
             (bytes == 0 || fwrite(src, 1, bytes, f.get()) == bytes);
    };
    put(ix->h_C1.data(), ix->h_C1.size() * 4);
    put(ix->h_C2.data(), ix->h_C2.size() * 4);
    put(ix->h_ti.data(), ix->h_ti.size());
    put(ix->h_tj.data(), ix->h_tj.size());
    put(ix->h_lam.data(), ix->h_lam.size() * 4);
    put(ix->h_cc.data(), ix->h_cc.size() * 4);
    // the large arrays come back from the GPU in pieces of at most 256 MiB
    std::vector<unsigned char> stage;
    try {
        stage.resize(256u << 20);
    } catch (const std::bad_alloc&) {
        return fail(PQT_ENOMEM, "host allocation failed");
    }
    auto put_device = [&](const void* dev, size_t bytes) -> int {
        put(nullptr, 0);
        for (size_t o = 0; o < bytes && ok; o += stage.size()) {
            const size_t n = bytes - o < stage.size() ? bytes - o : stage.size();
            HIP_TRY(hipMemcpy(stage.data(), static_cast<const unsigned char*>(dev) + o, n, hipMemcpyDeviceToHost));
            ok = fwrite(stage.data(), 1, n, f.get()) == n;
        }
        return PQT_OK;
    };
    int rc;
    if ((rc = put_device(ix->offsets, ((size_t)ix->H + 1) * 4)) || (rc = put_device(ix->ids, (size_t)ix->N * 4)) ||
        (rc = put_device(ix->codes, (size_t)ix->N * ix->code_bytes())))
        return rc;
    if (!ok || fflush(f.get()) != 0) return fail(PQT_EIO, "write to '%s' failed", path);
    return PQT_OK;
}

int pqt_index_export(const pqt_index* ix, const pqt_index_arrays* dst, int location) {
    if (!ix || !dst) return fail(PQT_EINVAL, "pqt_index_export: null argument");
    if (location != PQT_HOST && location != PQT_DEVICE)
        return fail(PQT_EINVAL, "pqt_index_export: location must be PQT_HOST or PQT_DEVICE");
    DeviceGuard guard(ix->device);
    if (!guard.ok) return fail(PQT_EHIP, "cannot select GPU %d", ix->device);
    if (dst->C1) memcpy(const_cast<float*>(dst->C1), ix->h_C1.data(), ix->h_C1.size() * 4);
    if (dst->C2) memcpy(const_cast<float*>(dst->C2), ix->h_C2.data(), ix->h_C2.size() * 4);
    if (dst->tbl_i) memcpy(const_cast<uint8_t*>(dst->tbl_i), ix->h_ti.data(), ix->h_ti.size());
    if (dst->tbl_j) memcpy(const_cast<uint8_t*>(dst->tbl_j), ix->h_tj.data(), ix->h_tj.size());
    if (dst->tbl_lambda) memcpy(const_cast<float*>(dst->tbl_lambda), ix->h_lam.data(), ix->h_lam.size() * 4);
    if (dst->cc) memcpy(const_cast<float*>(dst->cc), ix->h_cc.data(), ix->h_cc.size() * 4);
    const hipMemcpyKind kind = location == PQT_DEVICE ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost;
    if (dst->offsets) HIP_TRY(hipMemcpy(const_cast<uint32_t*>(dst->offsets), ix->offsets, ((size_t)ix->H + 1) * 4, kind));
    if (dst->ids && ix->N) HIP_TRY(hipMemcpy(const_cast<uint32_t*>(dst->ids), ix->ids, (size_t)ix->N * 4, kind));
    if (dst->codes && ix->N) HIP_TRY(hipMemcpy(const_cast<uint8_t*>(dst->codes), ix->codes, (size_t)ix->N * ix->code_bytes(), kind));
    return PQT_OK;
}

void pqt_index_free(pqt_index* ix) {
    if (!ix) return;
    DeviceGuard guard(ix->device);
    (void)hipFree(ix->vectors_owned); (void)hipFree(ix->ws_short_ids); (void)hipFree(ix->ws_short_dists);
    (void)hipFree(ix->vector_norms); (void)hipFree(ix->bf_qnorm); (void)hipFree(ix->bf_dist); (void)hipFree(ix->bf_best);
    (void)hipFree(ix->C1); (void)hipFree(ix->c1n); (void)hipFree(ix->C2); (void)hipFree(ix->C2t); (void)hipFree(ix->table);
    (void)hipFree(ix->offsets); (void)hipFree(ix->ids); (void)hipFree(ix->codes); (void)hipFree(ix->static_table);
    ix->free_workspace();
    for (hipEvent_t e : ix->events) (void)hipEventDestroy(e);
    delete ix;
}

int pqt_index_info(const pqt_index* ix, pqt_info* out) {
    if (!ix || !out) return fail(PQT_EINVAL, "pqt_index_info: null argument");
    out->N = ix->N; out->H = ix->H; out->D = ix->D; out->P = ix->P; out->k1 = ix->k1; out->k2 = ix->k2;
    out->M = ix->M; out->T = ix->T; out->C = ix->C; out->device = ix->device;
    out->code_format = ix->code_format; out->code_bytes = ix->code_bytes();
    out->bytes_index = ix->bytes_index; out->bytes_workspace = ix->bytes_workspace;
    return PQT_OK;
}

int pqt_set_budget(pqt_index* ix, uint32_t T_bins, uint32_t C_candidates) {
    if (!ix) return fail(PQT_EINVAL, "pqt_set_budget: null index");
    if (T_bins < 1 || T_bins > PQT_MAX_T || C_candidates < 1 || C_candidates > PQT_MAX_C)
        return fail(PQT_EINVAL, "budget T=%u C=%u out of range (T<=%d, C<=%d)", T_bins, C_candidates, PQT_MAX_T,
                    PQT_MAX_C);
    ix->T = T_bins;
    ix->C = C_candidates;
    return PQT_OK;
}

}  // extern "C"

namespace {

// The device buffers one batch works in (see pqt_index for their shapes).
struct QueryWorkspace {
    float* a;
    float* Ld;
    uint32_t* Lid;
    uint2* runs;
    uint2* meta;
    uint32_t* counters;
    uint32_t* order;
};

// Carves the workspace of nq queries out of `base` (256-byte aligned pieces); returns the bytes used.
size_t carve_workspace(const pqt_index* ix, int64_t nq, int R, unsigned char* base, QueryWorkspace* ws) {
    size_t o = 0;
    auto take = [&](size_t bytes) {
        unsigned char* p = base ? base + o : nullptr;
        o += (bytes + kAlign - 1) / kAlign * kAlign;
        return p;
    };
    QueryWorkspace v;
    v.a = reinterpret_cast<float*>(take(sizeof(float) * (size_t)nq * ix->M * ix->k1));
    v.Ld = reinterpret_cast<float*>(take(sizeof(float) * (size_t)nq * ix->P * R));
    v.Lid = reinterpret_cast<uint32_t*>(take(sizeof(uint32_t) * (size_t)nq * ix->P * R));
    v.runs = reinterpret_cast<uint2*>(take(sizeof(uint2) * (size_t)nq * ix->T));
    v.meta = reinterpret_cast<uint2*>(take(sizeof(uint2) * (size_t)nq));
    v.counters = reinterpret_cast<uint32_t*>(take(sizeof(uint32_t) * 2));
    v.order = reinterpret_cast<uint32_t*>(take(sizeof(uint32_t) * (size_t)nq));
    if (ws) *ws = v;
    return o;
}

// The whole query path.  no_alloc: the workspace is the static scratch array and nothing may be
// allocated (no workspace growth, no events, no upload of fixed-order tables).
int run_query(pqt_index* ix, const float* queries, int64_t nq, int k, int w, int64_t* out_ids, float* out_dists,
                     void* hip_stream, const pqt_debug_taps* taps, bool no_alloc) {
    if (!ix) return fail(PQT_EINVAL, "pqt_query_batch: null index");
    if (nq < 0) return fail(PQT_EINVAL, "pqt_query_batch: nq=%lld < 0", (long long)nq);
    if (k < 1 || k > PQT_MAX_K || (uint32_t)k > ix->C)
        return fail(PQT_EINVAL, "pqt_query_batch: k=%d outside 1..min(C=%u, %d)", k, ix->C, PQT_MAX_K);
    if (w < 1 || (uint32_t)w > ix->k1) return fail(PQT_EINVAL, "pqt_query_batch: w=%d outside 1..k1=%u", w, ix->k1);
    if ((int64_t)w * ix->k2 > PQT_MAX_R)
        return fail(PQT_EINVAL, "pqt_query_batch: w*k2=%lld exceeds %d", (long long)w * ix->k2, PQT_MAX_R);
    static const pqt_debug_taps no_taps = {};
    const pqt_debug_taps& tp = taps ? *taps : no_taps;
    if (tp.lut && ix->code_format == PQT_CODES_PAIR_LAMBDA)
        return fail(PQT_EINVAL, "pqt_query_batch_debug: the lut tap is the table of the one-byte code format");
    if (nq == 0) return PQT_OK;
    if (!queries || !out_ids || !out_dists) return fail(PQT_EINVAL, "pqt_query_batch: null buffer");
    int rc = check_query_limits(ix, k, w, nq, nullptr);
    if (rc) return rc;

    DeviceGuard guard(ix->device);
    if (!guard.ok) return fail(PQT_EHIP, "cannot select GPU %d", ix->device);
    const int R = w * (int)ix->k2;
    const bool fixed_order = ix->bin_order == PQT_ORDER_STATIC_SLOPES;
    const bool tables_stale = fixed_order && (ix->static_R != R || ix->static_T != (int)ix->T);
    QueryWorkspace ws;
    if (no_alloc) {
        unsigned char* base = scratch_on_device(ix->device);
        if (!base) return fail(PQT_EHIP, "pqt_query_batch_noalloc: the scratch array of GPU %d cannot be located", ix->device);
        const size_t need = carve_workspace(ix, nq, R, nullptr, nullptr);
        if (need > kScratchBytes)
            return fail(PQT_EINVAL,
                        "pqt_query_batch_noalloc: nq=%lld needs %zu bytes of workspace (w*k2=%d, T=%u), the static scratch "
                        "array holds %zu: send fewer queries per call",
                        (long long)nq, need, R, ix->T, kScratchBytes);
        if (tables_stale)
            return fail(PQT_EUNSUPPORTED,
                        "pqt_query_batch_noalloc: the fixed bin order needs new tables for w*k2=%d, T=%u: one pqt_query_batch "
                        "call with this w builds them", R, ix->T);
        carve_workspace(ix, nq, R, base, &ws);
    } else {
        if ((rc = pqt_host::ensure_workspace(ix, nq, R))) return rc;
        ws = QueryWorkspace{ix->ws_a, ix->ws_Ld, ix->ws_Lid, ix->ws_runs, ix->ws_meta, ix->ws_counters, ix->ws_order};
    }
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);

    std::vector<uint32_t> static_host;                  // new fixed-order tables, built before anything is enqueued
    if (tables_stale) {
        try {
            ix->static_Tn = pqt::make_static_order(R, (int)ix->T, static_host, ix->static_thr);
        } catch (const std::bad_alloc&) {
            return fail(PQT_ENOMEM, "host allocation failed");
        }
    }

    hipEvent_t* ev = nullptr;
    ix->last_events = nullptr;
    if (!no_alloc && ix->profiling && ix->prof_calls < kMaxProfiledCalls) {
        while ((int)ix->events.size() < 5 * (ix->prof_calls + 1)) {
            hipEvent_t e;
            HIP_TRY(hipEventCreate(&e));
            ix->events.push_back(e);
        }
        ev = &ix->events[5 * ix->prof_calls];
    }
    // from here on every failure leaves the events of this call unused: the call is counted at the end

    pqt::TraverseArgs ta;
    ta.queries = queries; ta.nq = nq;
    ta.D = ix->D; ta.P = ix->P; ta.k1 = ix->k1; ta.k2 = ix->k2; ta.M = ix->M; ta.w = w;
    ta.C1 = ix->C1; ta.c1n = ix->c1n; ta.C2 = ix->C2; ta.C2t = ix->C2t;
    ta.a = ws.a; ta.L_d = ws.Ld; ta.L_id = ws.Lid; ta.sel_tap = tp.sel; ta.counters = ws.counters;
    if (ev) HIP_TRY(hipEventRecord(ev[0], stream));
    HIP_TRY(pqt::launch_traverse(ta, stream));
    if (ev) HIP_TRY(hipEventRecord(ev[1], stream));

    pqt::RankArgs ra;
    ra.nq = nq; ra.P = ix->P; ra.R = R; ra.T = ix->T; ra.C = ix->C;
    ra.k1k2 = ix->k1 * ix->k2; ra.H = ix->H; ra.hashed = ix->hashed ? 1 : 0;
    ra.H_inv = ix->H >= 2 ? (uint64_t)((((unsigned __int128)1) << 64) / ix->H) : 0;
    ra.offsets = ix->offsets; ra.L_d = ws.Ld; ra.L_id = ws.Lid;
    ra.runs = ws.runs; ra.meta = ws.meta; ra.counters = ws.counters; ra.order = ws.order;
    ra.n_tuples = tp.n_tuples; ra.tuples = tp.tuples; ra.tuple_keys = tp.tuple_keys; ra.slots = tp.slots;
    const bool rerank_taps = tp.n_cand || tp.cand_ids || tp.scores || tp.lut || tp.n_slots;
    const bool head = !fixed_order && pqt::rank_has_head(ra);
    // the few queries the head pass cannot finish are ranked in full by their re-rank workgroup
    const bool fuse = head && !rerank_taps && can_fuse_ranking(ix, k, w, nq);
    if (fixed_order) {
        if (tables_stale) {                                             // tables for this list length and T
            HIP_TRY(hipStreamSynchronize(stream));                      // an earlier batch may still read the old tables
            (void)hipFree(ix->static_table);
            ix->static_table = nullptr;
            ix->static_R = ix->static_T = 0;
            HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->static_table), static_host.size() * sizeof(uint32_t)));
            HIP_TRY(hipMemcpy(ix->static_table, static_host.data(), static_host.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
            ix->static_R = R;
            ix->static_T = (int)ix->T;
        }
        pqt::StaticOrder so;
        so.table = ix->static_table;
        so.Tn = ix->static_Tn;
        for (int j = 0; j < pqt::kStaticSlopes - 1; ++j) so.thr[j] = ix->static_thr[j];
        HIP_TRY(pqt::launch_rank_static(ra, so, stream));
    } else {
        HIP_TRY(pqt::launch_rank(ra, stream, fuse));
    }
    if (ev) HIP_TRY(hipEventRecord(ev[2], stream));

    pqt::RerankArgs ca;
    ca.nq = nq; ca.M = ix->M; ca.k1 = ix->k1; ca.T = ix->T; ca.C = ix->C; ca.k = k;
    ca.threads = rerank_threads(ix, &ca.keys_per_thread, nq);
    ca.code_format = (int)ix->code_format;
    ca.runs_in_lds = rerank_runs_in_lds(ix);
    ca.a = ws.a; ca.table = ix->table; ca.runs = ws.runs; ca.meta = ws.meta;
    ca.ids = ix->ids; ca.codes = ix->codes; ca.out_ids = out_ids; ca.out_dists = out_dists;
    ca.todo = ws.order; ca.todo_count = ws.counters;
    ca.early = fuse ? (int)(nq < 1024 ? nq : 1024) : 0;   // unfinished queries first: they take longest
    ca.n_cand = tp.n_cand; ca.cand_ids = tp.cand_ids; ca.scores = tp.scores; ca.lut = tp.lut;
    HIP_TRY(pqt::launch_rerank(ca, fuse ? &ra : nullptr, stream));
    if (ev) {
        HIP_TRY(hipEventRecord(ev[3], stream));
        HIP_TRY(hipEventRecord(ev[4], stream));     // moved behind the exact re-rank when that runs
        ix->last_events = ev;
        ix->prof_calls++;                           // all five events of this call are recorded
    }

    // taps that are plain copies of workspace arrays
    if (tp.a)
        HIP_TRY(hipMemcpyAsync(tp.a, ws.a, sizeof(float) * (size_t)nq * ix->M * ix->k1, hipMemcpyDeviceToDevice, stream));
    if (tp.L_d)
        HIP_TRY(hipMemcpyAsync(tp.L_d, ws.Ld, sizeof(float) * (size_t)nq * ix->P * R, hipMemcpyDeviceToDevice, stream));
    if (tp.L_id)
        HIP_TRY(hipMemcpyAsync(tp.L_id, ws.Lid, sizeof(uint32_t) * (size_t)nq * ix->P * R, hipMemcpyDeviceToDevice, stream));
    if (tp.n_slots) {
        // number of proposed slots = meta.x; strided copy of the first word of every meta pair
        HIP_TRY(hipMemcpy2DAsync(tp.n_slots, sizeof(uint32_t), ws.meta, sizeof(uint2), sizeof(uint32_t), (size_t)nq,
                                 hipMemcpyDeviceToDevice, stream));
    }
    return PQT_OK;
}

}  // namespace

extern "C" {

int pqt_query_batch_debug(pqt_index* ix, const float* queries, int64_t nq, int k, int w, int64_t* out_ids,
                          float* out_dists, void* hip_stream, const pqt_debug_taps* taps) {
    return run_query(ix, queries, nq, k, w, out_ids, out_dists, hip_stream, taps, false);
}

int pqt_query_batch_noalloc(pqt_index* ix, const float* queries, int64_t nq, int k, int w, int64_t* out_ids,
                            float* out_dists, void* hip_stream) {
    return run_query(ix, queries, nq, k, w, out_ids, out_dists, hip_stream, nullptr, true);
}

size_t pqt_noalloc_workspace_bytes(void) { return kScratchBytes; }

int pqt_set_bin_order(pqt_index* ix, int order) {
    if (!ix) return fail(PQT_EINVAL, "pqt_set_bin_order: null index");
    if (order != PQT_ORDER_SUMMED_DISTANCE && order != PQT_ORDER_STATIC_SLOPES)
        return fail(PQT_EINVAL, "pqt_set_bin_order: order %d", order);
    if (order == PQT_ORDER_STATIC_SLOPES && (ix->P != 2 || ix->hashed))
        return fail(PQT_EUNSUPPORTED, "pqt_set_bin_order: the fixed order needs two tree parts and H = (k1*k2)^2");
    ix->bin_order = order;
    return PQT_OK;
}

int pqt_query_batch(pqt_index* ix, const float* queries, int64_t nq, int k, int w, int64_t* out_ids,
                    float* out_dists, void* hip_stream) {
    return run_query(ix, queries, nq, k, w, out_ids, out_dists, hip_stream, nullptr, false);
}

int pqt_index_set_vectors(pqt_index* ix, const void* vectors, int elem_bytes, int location) {
    if (!ix) return fail(PQT_EINVAL, "pqt_index_set_vectors: null index");
    if (vectors && elem_bytes != 4 && elem_bytes != 1)
        return fail(PQT_EINVAL, "pqt_index_set_vectors: elements are 4-byte floats or 1-byte unsigned integers");
    if (vectors && location != PQT_HOST && location != PQT_DEVICE)
        return fail(PQT_EINVAL, "pqt_index_set_vectors: location must be PQT_HOST or PQT_DEVICE");
    if (vectors && ix->D % (16 / elem_bytes))
        return fail(PQT_EUNSUPPORTED, "exact re-ranking reads rows in 16-byte pieces: D=%u must be a multiple of %d",
                    ix->D, 16 / elem_bytes);
    DeviceGuard guard(ix->device);
    if (!guard.ok) return fail(PQT_EHIP, "cannot select GPU %d", ix->device);
    HIP_TRY(hipDeviceSynchronize());               // no query may still be reading the old vectors
    (void)hipFree(ix->vectors_owned);
    (void)hipFree(ix->vector_norms);
    ix->vector_norms = nullptr;
    ix->vectors_owned = nullptr;
    ix->vectors = nullptr;
    ix->vector_elem_bytes = 0;
    if (!vectors) return PQT_OK;
    if (location == PQT_HOST) {
        const size_t bytes = (size_t)ix->N * ix->D * (size_t)elem_bytes;
        HIP_TRY(hipMalloc(&ix->vectors_owned, bytes ? bytes : 1));
        if (bytes) HIP_TRY(hipMemcpy(ix->vectors_owned, vectors, bytes, hipMemcpyHostToDevice));
        ix->vectors = ix->vectors_owned;
    } else {
        ix->vectors = vectors;                     // borrowed: the caller keeps it alive
    }
    ix->vector_elem_bytes = elem_bytes;
    return PQT_OK;
}

int pqt_query_batch_exact(pqt_index* ix, const float* queries, int64_t nq, int k_short, int k, int w,
                          int64_t* out_ids, float* out_dists, void* hip_stream) {
    if (!ix) return fail(PQT_EINVAL, "pqt_query_batch_exact: null index");
    if (!ix->vectors) return fail(PQT_EINVAL, "pqt_query_batch_exact: no database vectors (pqt_index_set_vectors)");
    if (k < 1 || k > k_short) return fail(PQT_EINVAL, "pqt_query_batch_exact: k=%d outside 1..k_short=%d", k, k_short);
    if (nq < 0) return fail(PQT_EINVAL, "pqt_query_batch_exact: nq=%lld < 0", (long long)nq);
    if (nq == 0) return PQT_OK;
    if (!queries || !out_ids || !out_dists) return fail(PQT_EINVAL, "pqt_query_batch_exact: null buffer");
    if (k_short > PQT_MAX_K || (uint32_t)k_short > ix->C)
        return fail(PQT_EINVAL, "pqt_query_batch_exact: k_short=%d outside 1..min(C=%u, %d)", k_short, ix->C, PQT_MAX_K);
    if (pqt::exact_lds_bytes(ix->D, k_short) > 64 * 1024)
        return fail(PQT_EUNSUPPORTED, "pqt_query_batch_exact: D=%u with k_short=%d exceeds the LDS budget", ix->D, k_short);
    DeviceGuard guard(ix->device);
    if (!guard.ok) return fail(PQT_EHIP, "cannot select GPU %d", ix->device);
    const size_t entries = (size_t)nq * (size_t)k_short;
    if (entries > ix->ws_short_entries) {
        (void)hipFree(ix->ws_short_ids); (void)hipFree(ix->ws_short_dists);
        ix->ws_short_ids = nullptr; ix->ws_short_dists = nullptr; ix->ws_short_entries = 0;
        HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->ws_short_ids), entries * sizeof(int64_t)));
        HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->ws_short_dists), entries * sizeof(float)));
        ix->ws_short_entries = entries;
    }
    const int rc = pqt_query_batch(ix, queries, nq, k_short, w, ix->ws_short_ids, ix->ws_short_dists, hip_stream);
    if (rc) return rc;
    pqt::ExactArgs ea;
    ea.nq = nq; ea.D = ix->D; ea.k_short = k_short; ea.k = k; ea.elem_bytes = ix->vector_elem_bytes;
    ea.queries = queries; ea.vectors = ix->vectors; ea.short_ids = ix->ws_short_ids;
    ea.out_ids = out_ids; ea.out_dists = out_dists;
    HIP_TRY(pqt::launch_exact_rerank(ea, reinterpret_cast<hipStream_t>(hip_stream)));
    if (ix->last_events) HIP_TRY(hipEventRecord(ix->last_events[4], reinterpret_cast<hipStream_t>(hip_stream)));
    return PQT_OK;
}

int pqt_brute_force(pqt_index* ix, const float* queries, int64_t nq, int k, int64_t* out_ids, float* out_dists,
                    void* hip_stream) {
    if (!ix) return fail(PQT_EINVAL, "pqt_brute_force: null index");
    if (!ix->vectors) return fail(PQT_EINVAL, "pqt_brute_force: no database vectors (pqt_index_set_vectors)");
    if (k < 1 || k > 256 || (uint64_t)k > ix->N) return fail(PQT_EINVAL, "pqt_brute_force: k=%d outside 1..min(N, 256)", k);
    if (nq < 0) return fail(PQT_EINVAL, "pqt_brute_force: nq=%lld < 0", (long long)nq);
    if (nq == 0) return PQT_OK;
    if (!queries || !out_ids || !out_dists) return fail(PQT_EINVAL, "pqt_brute_force: null buffer");
    DeviceGuard guard(ix->device);
    if (!guard.ok) return fail(PQT_EHIP, "cannot select GPU %d", ix->device);
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    if (!ix->vector_norms) {
        HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->vector_norms), sizeof(float) * ix->N));
        HIP_TRY(pqt::launch_row_norms(ix->vectors, ix->vector_elem_bytes, (int64_t)ix->N, (int)ix->D, ix->vector_norms, stream));
    }
    // distance block: at most 2^30 floats (4 GiB), at most 65536 database vectors per pass
    int64_t chunk = (int64_t)(1ll << 30) / nq;
    if (chunk > 65536) chunk = 65536;
    if (chunk > (int64_t)ix->N) chunk = (int64_t)ix->N;
    chunk = chunk / 128 * 128;
    if (chunk < 128) chunk = 128;
    if (nq > ix->bf_nq || chunk > ix->bf_chunk || k > ix->bf_k) {
        (void)hipFree(ix->bf_qnorm); (void)hipFree(ix->bf_dist); (void)hipFree(ix->bf_best);
        ix->bf_qnorm = nullptr; ix->bf_dist = nullptr; ix->bf_best = nullptr; ix->bf_nq = 0;
        HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->bf_qnorm), sizeof(float) * (size_t)nq));
        HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->bf_dist), sizeof(float) * (size_t)nq * (size_t)chunk));
        HIP_TRY(hipMalloc(reinterpret_cast<void**>(&ix->bf_best), sizeof(unsigned long long) * (size_t)nq * (size_t)k));
        ix->bf_nq = nq; ix->bf_chunk = chunk; ix->bf_k = k;
    }
    HIP_TRY(pqt::launch_row_norms(queries, 4, nq, (int)ix->D, ix->bf_qnorm, stream));
    pqt::BruteArgs ba;
    ba.nq = nq; ba.D = ix->D; ba.k = k; ba.elem_bytes = ix->vector_elem_bytes; ba.chunk = chunk;
    ba.queries = queries; ba.vectors = ix->vectors; ba.qnorm = ix->bf_qnorm; ba.xnorm = ix->vector_norms;
    ba.dist = ix->bf_dist; ba.best = ix->bf_best; ba.out_ids = out_ids; ba.out_dists = out_dists;
    for (int64_t x0 = 0; x0 < (int64_t)ix->N; x0 += chunk) {
        const int64_t nx = (int64_t)ix->N - x0 < chunk ? (int64_t)ix->N - x0 : chunk;
        HIP_TRY(pqt::launch_brute_chunk(ba, x0, nx, x0 == 0, x0 + nx >= (int64_t)ix->N, stream));
    }
    return PQT_OK;
}

int pqt_set_profiling(pqt_index* ix, int enabled) {
    if (!ix) return fail(PQT_EINVAL, "pqt_set_profiling: null index");
    ix->profiling = enabled != 0;
    ix->prof_calls = 0;
    return PQT_OK;
}

int pqt_stage_times(pqt_index* ix, float ms[4], int* calls) {
    if (!ix || !ms || !calls) return fail(PQT_EINVAL, "pqt_stage_times: null argument");
    DeviceGuard guard(ix->device);
    ms[0] = ms[1] = ms[2] = ms[3] = 0.0f;
    const int n = ix->prof_calls;
    ix->prof_calls = 0;                              // also when reading an event fails below
    *calls = 0;
    for (int c = 0; c < n; ++c) {
        hipEvent_t* ev = &ix->events[5 * c];
        HIP_TRY(hipEventSynchronize(ev[4]));
        for (int s = 0; s < 4; ++s) {
            float t = 0.0f;
            HIP_TRY(hipEventElapsedTime(&t, ev[s], ev[s + 1]));
            ms[s] += t;
        }
    }
    *calls = n;
    return PQT_OK;
}

}  // extern "C"
