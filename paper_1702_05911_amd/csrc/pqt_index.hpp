// Internals shared by the host-side sources of the library: error reporting, the index object.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <vector>

#include "../../include/pqt.h"
#include "pqt_kernels.hpp"

namespace pqt_host {

char* error_buffer();          // thread-local, 512 bytes
int fail(int code, const char* fmt, ...);

#define HIP_TRY(expr)                                                                                 \
    do {                                                                                              \
        hipError_t e_ = (expr);                                                                       \
        if (e_ != hipSuccess)                                                                         \
            return pqt_host::fail(e_ == hipErrorOutOfMemory ? PQT_ENOMEM : PQT_EHIP, "%s: %s", #expr, \
                                  hipGetErrorString(e_));                                             \
    } while (0)

struct DeviceGuard {   // make the index's GPU current for the duration of a call
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(dev) == hipSuccess) ok = true;
    }
    ~DeviceGuard() {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

// grows the per-batch workspace of an index to nq queries with lists of R entries
int ensure_workspace(pqt_index* ix, int64_t nq, int R);

}  // namespace pqt_host

struct pqt_index {
    uint32_t D = 0, P = 0, k1 = 0, k2 = 0, M = 0, T = 0, C = 0;
    uint64_t N = 0, H = 0;
    int device = 0;
    size_t lds_limit = 64 * 1024;      // dynamic LDS the query kernels may ask for on this device
    bool hashed = false;
    uint64_t nonempty_slots = 0;       // slots that hold at least one vector
    uint32_t code_format = 0;          // PQT_CODES_TABLE or PQT_CODES_PAIR_LAMBDA
    uint32_t code_bytes() const { return M * (code_format == 1 ? 2u : 1u); }   // per vector
    // index arrays (device)
    float* C1 = nullptr;
    float* c1n = nullptr;
    float* C2 = nullptr;
    float* C2t = nullptr;   // children of a cluster interleaved four dimensions at a time (dp % 4 == 0)
    pqt::CodeEntry* table = nullptr;
    uint32_t* offsets = nullptr;
    uint32_t* ids = nullptr;
    uint8_t* codes = nullptr;
    uint64_t bytes_index = 0;
    // host copies of the small arrays as they were given (for pqt_index_save)
    std::vector<float> h_C1, h_C2, h_lam, h_cc;
    std::vector<uint8_t> h_ti, h_tj;
    // raw database vectors for exact re-ranking (optional)
    const void* vectors = nullptr;
    void* vectors_owned = nullptr;      // set when the library holds its own copy
    int vector_elem_bytes = 0;
    float* vector_norms = nullptr;      // squared norms of the attached vectors (made on first brute-force call)
    float* bf_qnorm = nullptr;          // brute-force workspace: query norms, distance block, running best
    float* bf_dist = nullptr;
    unsigned long long* bf_best = nullptr;
    int64_t bf_nq = 0, bf_chunk = 0;
    int bf_k = 0;
    int64_t* ws_short_ids = nullptr;    // nq x k_short results of the line-quantisation re-ranking
    float* ws_short_dists = nullptr;
    size_t ws_short_entries = 0;
    // workspace (device), sized for ws_nq queries at ws_R list entries and ws_T tuples
    int64_t ws_nq = 0;
    int ws_R = 0, ws_T = 0;
    float* ws_a = nullptr;
    float* ws_Ld = nullptr;
    uint32_t* ws_Lid = nullptr;
    uint2* ws_runs = nullptr;
    uint2* ws_meta = nullptr;
    uint32_t* ws_counters = nullptr;   // 2 words
    uint32_t* ws_order = nullptr;      // nq words
    uint64_t bytes_workspace = 0;
    // fixed traversal order (pqt_set_bin_order): tables for lists of static_R entries and static_T tuples
    int bin_order = 0;
    uint32_t* static_table = nullptr;
    int static_R = 0, static_T = 0, static_Tn = 0;
    float static_thr[pqt::kStaticSlopes - 1] = {};
    // stage timing
    bool profiling = false;
    int prof_calls = 0;
    std::vector<hipEvent_t> events;   // 5 per profiled call
    hipEvent_t* last_events = nullptr;  // events of the most recent profiled call (for the exact re-rank stage)

    void free_workspace() {
        (void)hipFree(ws_a); (void)hipFree(ws_Ld); (void)hipFree(ws_Lid);
        (void)hipFree(ws_runs); (void)hipFree(ws_meta); (void)hipFree(ws_counters); (void)hipFree(ws_order);
        ws_a = ws_Ld = nullptr; ws_Lid = nullptr; ws_runs = ws_meta = nullptr; ws_counters = ws_order = nullptr;
        ws_nq = 0; bytes_workspace = 0;
    }
};
