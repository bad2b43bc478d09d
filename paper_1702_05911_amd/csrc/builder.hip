// Offline phase on the GPU (Sec. 3.1 "bin map", Sec. 3.3 "Offline computation", Sec. 4): given the
// trained codebooks and the line-code table, database vectors are streamed through in chunks; each
// vector is sorted into its bin with the SAME traversal kernel the queries use (Sec. 4: the two
// distance kernels serve both phases) with w = 1, gets its line-quantisation code, and at the end
// the ids are ordered by (slot, id) -- a stable radix sort, so ids ascend inside a slot -- the
// pointer array is the prefix sum of the slot histogram (Sec. 4), and the codes are permuted into
// the same order.  Codebook training (Lloyd iterations on a sample) stays with the caller.
//
// The code of a vector is the nearest of the 256 code points of each sub-part.  Its distance to
// code point c is Eq. 9 evaluated on the vector's own level-1 distances -- exactly the per-query
// table of the re-ranking -- so no further distance is computed; ties go to the smaller c.
#include <hipcub/hipcub.hpp>

#include <new>

#include "pqt_device.hpp"
#include "pqt_index.hpp"

using pqt_host::DeviceGuard;
using pqt_host::fail;

namespace pqt {

constexpr int kEncodeThreads = 256;

// One wavefront per vector: for every sub-part the 256 Eq. 9 values (four per lane), the smallest
// (value, c) wins.  Lane 0 also forms the bin number from the level-2 leaves and hashes it.
__global__ __launch_bounds__(kEncodeThreads) void encode_kernel(const float* a, const uint32_t* leaf, int64_t n, int M, int k1,
                                                                int P, uint32_t k1k2, unsigned long long H,
                                                                const CodeEntry* table, uint8_t* codes, uint32_t* slots) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t v = (int64_t)blockIdx.x * (kEncodeThreads / kWave) + threadIdx.x / kWave;
    if (v >= n) return;
    const float* av = a + (size_t)v * M * k1;
    for (int m = 0; m < M; ++m) {
        unsigned long long best = ~0ull;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = u * kWave + lane;
            const CodeEntry e = table[m * 256 + c];
            const float b2 = av[m * k1 + (e.ij & 0xffu)], a2 = av[m * k1 + ((e.ij >> 8) & 0xffu)];
            const float val = fmaf(e.lam, a2 - b2, b2) + e.kc;
            const unsigned long long key = ((unsigned long long)mono_key(val) << 32) | (unsigned)c;
            best = key < best ? key : best;
        }
        // minimum over the wavefront
        for (int off = 32; off > 0; off >>= 1) {
            const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(best >> 32), off, kWave);
            const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)best, off, kWave);
            const unsigned long long o = ((unsigned long long)hi << 32) | lo;
            best = o < best ? o : best;
        }
        if (lane == 0) codes[(size_t)v * M + m] = (uint8_t)(best & 0xffu);
    }
    if (lane == 0) {
        unsigned long long lin = 0;
        for (int p = 0; p < P; ++p) lin = lin * k1k2 + leaf[(size_t)v * P + p];   // lists have one entry (w = 1, k2 children -> first)
        slots[v] = (uint32_t)(lin % H);
    }
}

// (pair, lambda) codes (Sec. 3.3 "Offline computation"; Eq. 7 stored directly).  A code stands for the
// point (1 - lambda) c_i + lambda c_j with lambda = (level - 96) / 16; a sub-vector gets the code of
// the nearest such point.  One wavefront per vector, up to four centroid pairs per lane.  With b^2, a^2
// the sub-vector's own distances to c_i, c_j and c^2 = ||c_i - c_j||^2, the projection on the line is
// at (b^2 - a^2 + c^2) / (2 c^2); the level nearest to it (clamped to a byte) is the line's nearest
// code point, whose distance is Eq. 9 on the same values.  The smallest (distance, pair number) wins;
// pairs with c^2 = 0 never do.  `table` holds the pairs (entry = pair number, kc = c^2).
__global__ __launch_bounds__(kEncodeThreads) void encode_pairs_kernel(const float* a, const uint32_t* leaf, int64_t n, int M,
                                                                      int k1, int P, uint32_t k1k2, unsigned long long H,
                                                                      const CodeEntry* table, uint8_t* codes,
                                                                      uint32_t* slots) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t v = (int64_t)blockIdx.x * (kEncodeThreads / kWave) + threadIdx.x / kWave;
    if (v >= n) return;
    const float* av = a + (size_t)v * M * k1;
    const int npairs = k1 * (k1 - 1) / 2;
    for (int m = 0; m < M; ++m) {
        unsigned long long best = ~0ull;
        uint32_t best_level = 96;                          // no usable pair: pair 0 at lambda = 0
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = u * kWave + lane;
            if (c >= npairs) continue;
            const CodeEntry e = table[m * 256 + c];
            if (!(e.kc > 0.0f)) continue;
            const float b2 = av[m * k1 + (e.ij & 0xffu)], a2 = av[m * k1 + ((e.ij >> 8) & 0xffu)];
            const float proj = ((b2 - a2) + e.kc) / (2.0f * e.kc);
            const float level = fminf(fmaxf(floorf(fmaf(proj, 16.0f, 96.5f)), 0.0f), 255.0f);
            const float lam = fmaf(level, 0.0625f, -6.0f);
            const float dist = fmaf(fmaf(lam, lam, -lam), e.kc, fmaf(lam, a2 - b2, b2));
            const unsigned long long key = ((unsigned long long)mono_key(dist) << 32) | (unsigned)c;
            if (key < best) {
                best = key;
                best_level = (uint32_t)level;
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(best >> 32), off, kWave);
            const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)best, off, kWave);
            const uint32_t ol = (uint32_t)__shfl_xor((int)best_level, off, kWave);
            const unsigned long long o = ((unsigned long long)hi << 32) | lo;
            if (o < best) {
                best = o;
                best_level = ol;
            }
        }
        if (lane == 0) {
            codes[((size_t)v * M + m) * 2] = best != ~0ull ? (uint8_t)(best & 0xffu) : (uint8_t)0;
            codes[((size_t)v * M + m) * 2 + 1] = (uint8_t)best_level;
        }
    }
    if (lane == 0) {
        unsigned long long lin = 0;
        for (int p = 0; p < P; ++p) lin = lin * k1k2 + leaf[(size_t)v * P + p];
        slots[v] = (uint32_t)(lin % H);
    }
}

__global__ void iota_kernel(uint32_t* out, uint64_t n) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = (uint32_t)i;
}

__global__ void histogram_kernel(const uint32_t* slots, uint64_t n, uint32_t* counts) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) atomicAdd(&counts[slots[i]], 1u);
}

// number of slots that hold at least one vector (one atomic per wavefront)
__global__ void count_nonempty_kernel(const uint32_t* counts, uint64_t n, unsigned long long* out) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const unsigned long long mask = __ballot(i < n && counts[i] > 0);
    if ((threadIdx.x & (kWave - 1)) == 0 && mask) atomicAdd(out, (unsigned long long)__popcll(mask));
}

// codes_out[i] = codes_in[order[i]], one thread per row of M bytes
__global__ void permute_codes_kernel(const uint8_t* in, const uint32_t* order, uint64_t n, int M, uint8_t* out) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint8_t* src = in + (size_t)order[i] * M;
    uint8_t* dst = out + (size_t)i * M;
    if (M % 4 == 0) {
        for (int j = 0; j < M / 4; ++j) reinterpret_cast<uint32_t*>(dst)[j] = reinterpret_cast<const uint32_t*>(src)[j];
    } else {
        for (int j = 0; j < M; ++j) dst[j] = src[j];
    }
}

// the first leaf of every (vector, part) list: L_id is n x P x R
__global__ void first_leaf_kernel(const uint32_t* L_id, int64_t n, int P, int R, uint32_t* leaf) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n * P) leaf[i] = L_id[i * R];
}

}  // namespace pqt

struct pqt_builder {
    pqt_index* ix = nullptr;       // codebooks and tables on the GPU; receives the lists at the end
    uint64_t N = 0, added = 0;
    uint32_t* slots = nullptr;     // N
    uint8_t* codes = nullptr;      // N x M, in id order
    uint32_t* leaf = nullptr;      // chunk x P
    int64_t chunk = 0;
};

namespace {
constexpr int64_t kChunk = 1 << 18;   // vectors per traversal launch (its workspace is 512 B per vector at M*k1 = 128)
}

extern "C" {

int pqt_builder_create(const pqt_index_arrays* params, int device, pqt_builder** out) {
    if (!params || !out) return fail(PQT_EINVAL, "pqt_builder_create: null argument");
    *out = nullptr;
    if (params->N == 0) return fail(PQT_EINVAL, "pqt_builder_create: N = 0");
    // an index without vectors: every slot empty
    std::vector<uint32_t> zeros;
    try {
        zeros.assign((size_t)params->H + 1, 0u);
    } catch (const std::bad_alloc&) {
        return fail(PQT_ENOMEM, "host allocation failed");
    }
    pqt_index_arrays empty = *params;
    empty.N = 0;
    empty.offsets = zeros.data();
    empty.ids = nullptr;
    empty.codes = nullptr;
    pqt_index* ix = nullptr;
    int rc = pqt_index_from_arrays(&empty, PQT_HOST, device, &ix);
    if (rc) return rc;
    if (params->N >= 0xffffffffull) {
        pqt_index_free(ix);
        return fail(PQT_EUNSUPPORTED, "N=%llu: 32-bit ids only", (unsigned long long)params->N);
    }
    pqt_builder* b = new (std::nothrow) pqt_builder();
    if (!b) {
        pqt_index_free(ix);
        return fail(PQT_ENOMEM, "host allocation failed");
    }
    b->ix = ix;
    b->N = params->N;
    DeviceGuard guard(device);
    b->chunk = (int64_t)(b->N < (uint64_t)kChunk ? b->N : (uint64_t)kChunk);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&b->slots), sizeof(uint32_t) * b->N);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&b->codes), (size_t)b->N * ix->code_bytes());
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&b->leaf), sizeof(uint32_t) * (size_t)b->chunk * ix->P);
    if (e != hipSuccess) {
        pqt_builder_free(b);
        return fail(e == hipErrorOutOfMemory ? PQT_ENOMEM : PQT_EHIP, "pqt_builder_create: %s", hipGetErrorString(e));
    }
    *out = b;
    return PQT_OK;
}

void pqt_builder_free(pqt_builder* b) {
    if (!b) return;
    if (b->ix) {
        DeviceGuard guard(b->ix->device);
        (void)hipFree(b->slots); (void)hipFree(b->codes); (void)hipFree(b->leaf);
        pqt_index_free(b->ix);
    }
    delete b;
}

int pqt_builder_add(pqt_builder* b, const float* vectors, int64_t n, void* hip_stream) {
    if (!b || !b->ix) return fail(PQT_EINVAL, "pqt_builder_add: null builder");
    if (n < 0 || b->added + (uint64_t)n > b->N)
        return fail(PQT_EINVAL, "pqt_builder_add: %lld more vectors after %llu exceed N=%llu", (long long)n,
                    (unsigned long long)b->added, (unsigned long long)b->N);
    if (n == 0) return PQT_OK;
    if (!vectors) return fail(PQT_EINVAL, "pqt_builder_add: null vectors");
    pqt_index* ix = b->ix;
    DeviceGuard guard(ix->device);
    if (!guard.ok) return fail(PQT_EHIP, "cannot select GPU %d", ix->device);
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    const int R = (int)ix->k2;                           // w = 1: the children of the nearest cluster
    for (int64_t s = 0; s < n; s += b->chunk) {
        const int64_t m = n - s < b->chunk ? n - s : b->chunk;
        int rc = pqt_host::ensure_workspace(ix, m, R);
        if (rc) return rc;
        pqt::TraverseArgs ta;
        ta.queries = vectors + (size_t)s * ix->D; ta.nq = m;
        ta.D = ix->D; ta.P = ix->P; ta.k1 = ix->k1; ta.k2 = ix->k2; ta.M = ix->M; ta.w = 1;
        ta.C1 = ix->C1; ta.c1n = ix->c1n; ta.C2 = ix->C2; ta.C2t = ix->C2t;
        ta.a = ix->ws_a; ta.L_d = ix->ws_Ld; ta.L_id = ix->ws_Lid; ta.sel_tap = nullptr; ta.counters = nullptr;
        if (pqt::traverse_lds_bytes(ix->D, ix->P, ix->k1, ix->k2, ix->M, 1) > pqt::kMaxLds)
            return fail(PQT_EUNSUPPORTED, "pqt_builder_add: D=%u exceeds the LDS budget of the traversal", ix->D);
        HIP_TRY(pqt::launch_traverse(ta, stream));
        const unsigned tb = 256;
        hipLaunchKernelGGL(pqt::first_leaf_kernel, dim3((unsigned)((m * ix->P + tb - 1) / tb)), dim3(tb), 0, stream,
                           ix->ws_Lid, m, (int)ix->P, R, b->leaf);
        constexpr int per = pqt::kEncodeThreads / pqt::kWave;
        hipLaunchKernelGGL(ix->code_format == PQT_CODES_PAIR_LAMBDA ? pqt::encode_pairs_kernel : pqt::encode_kernel,
                           dim3((unsigned)((m + per - 1) / per)), dim3(pqt::kEncodeThreads), 0, stream,
                           ix->ws_a, b->leaf, m, (int)ix->M, (int)ix->k1, (int)ix->P, ix->k1 * ix->k2,
                           (unsigned long long)ix->H, ix->table, b->codes + (size_t)(b->added + s) * ix->code_bytes(),
                           b->slots + b->added + s);
        HIP_TRY(hipGetLastError());
    }
    b->added += (uint64_t)n;
    return PQT_OK;
}

int pqt_builder_finish(pqt_builder* b, pqt_index** out) {
    if (!b || !b->ix || !out) return fail(PQT_EINVAL, "pqt_builder_finish: null argument");
    *out = nullptr;
    if (b->added != b->N)
        return fail(PQT_EINVAL, "pqt_builder_finish: %llu of N=%llu vectors added", (unsigned long long)b->added,
                    (unsigned long long)b->N);
    pqt_index* ix = b->ix;
    DeviceGuard guard(ix->device);
    if (!guard.ok) return fail(PQT_EHIP, "cannot select GPU %d", ix->device);
    HIP_TRY(hipDeviceSynchronize());
    const uint64_t N = b->N;
    uint32_t *ids_in = nullptr, *ids_out = nullptr, *slots_out = nullptr, *counts = nullptr, *offsets = nullptr;
    uint8_t* codes_out = nullptr;
    void* temp = nullptr;
    auto cleanup = [&]() {
        (void)hipFree(ids_in); (void)hipFree(slots_out); (void)hipFree(counts); (void)hipFree(temp);
    };
#define BUILD_TRY(expr)                                                                                          \
    do {                                                                                                         \
        hipError_t e_ = (expr);                                                                                  \
        if (e_ != hipSuccess) {                                                                                  \
            cleanup();                                                                                           \
            (void)hipFree(ids_out); (void)hipFree(offsets); (void)hipFree(codes_out);                            \
            return fail(e_ == hipErrorOutOfMemory ? PQT_ENOMEM : PQT_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
        }                                                                                                        \
    } while (0)
    BUILD_TRY(hipMalloc(reinterpret_cast<void**>(&ids_in), sizeof(uint32_t) * N));
    BUILD_TRY(hipMalloc(reinterpret_cast<void**>(&ids_out), sizeof(uint32_t) * N));
    BUILD_TRY(hipMalloc(reinterpret_cast<void**>(&slots_out), sizeof(uint32_t) * N));
    const unsigned tb = 256;
    const unsigned nb = (unsigned)((N + tb - 1) / tb);
    hipLaunchKernelGGL(pqt::iota_kernel, dim3(nb), dim3(tb), 0, 0, ids_in, N);
    // ids by (slot, id): stable sort on the slot
    int end_bit = 1;
    while (end_bit < 32 && (1ull << end_bit) < ix->H) ++end_bit;
    size_t temp_bytes = 0;
    BUILD_TRY(hipcub::DeviceRadixSort::SortPairs(nullptr, temp_bytes, b->slots, slots_out, ids_in, ids_out, N, 0, end_bit));
    BUILD_TRY(hipMalloc(&temp, temp_bytes ? temp_bytes : 1));
    BUILD_TRY(hipcub::DeviceRadixSort::SortPairs(temp, temp_bytes, b->slots, slots_out, ids_in, ids_out, N, 0, end_bit));
    (void)hipFree(temp);
    temp = nullptr;
    // pointer array = exclusive prefix sum of the slot histogram
    BUILD_TRY(hipMalloc(reinterpret_cast<void**>(&counts), sizeof(uint32_t) * ((size_t)ix->H + 1)));
    BUILD_TRY(hipMalloc(reinterpret_cast<void**>(&offsets), sizeof(uint32_t) * ((size_t)ix->H + 1)));
    BUILD_TRY(hipMemset(counts, 0, sizeof(uint32_t) * ((size_t)ix->H + 1)));
    hipLaunchKernelGGL(pqt::histogram_kernel, dim3(nb), dim3(tb), 0, 0, b->slots, N, counts);
    unsigned long long* nonempty_dev = nullptr;
    unsigned long long nonempty = 0;
    BUILD_TRY(hipMalloc(reinterpret_cast<void**>(&nonempty_dev), sizeof(unsigned long long)));
    hipError_t ce = hipMemset(nonempty_dev, 0, sizeof(unsigned long long));
    if (ce == hipSuccess) {
        hipLaunchKernelGGL(pqt::count_nonempty_kernel, dim3((unsigned)((ix->H + tb - 1) / tb)), dim3(tb), 0, 0, counts,
                           (uint64_t)ix->H, nonempty_dev);
        ce = hipMemcpy(&nonempty, nonempty_dev, sizeof(nonempty), hipMemcpyDeviceToHost);
    }
    (void)hipFree(nonempty_dev);
    BUILD_TRY(ce);
    temp_bytes = 0;
    BUILD_TRY(hipcub::DeviceScan::ExclusiveSum(nullptr, temp_bytes, counts, offsets, (size_t)ix->H + 1));
    BUILD_TRY(hipMalloc(&temp, temp_bytes ? temp_bytes : 1));
    BUILD_TRY(hipcub::DeviceScan::ExclusiveSum(temp, temp_bytes, counts, offsets, (size_t)ix->H + 1));
    // codes in the order of the ids
    BUILD_TRY(hipMalloc(reinterpret_cast<void**>(&codes_out), (size_t)N * ix->code_bytes()));
    hipLaunchKernelGGL(pqt::permute_codes_kernel, dim3(nb), dim3(tb), 0, 0, b->codes, ids_out, N, (int)ix->code_bytes(),
                       codes_out);
    BUILD_TRY(hipGetLastError());
    BUILD_TRY(hipDeviceSynchronize());
#undef BUILD_TRY
    cleanup();
    (void)hipFree(ix->offsets); (void)hipFree(ix->ids); (void)hipFree(ix->codes);
    ix->offsets = offsets;
    ix->ids = ids_out;
    ix->codes = codes_out;
    ix->bytes_index += (uint64_t)N * (4 + ix->code_bytes());
    ix->N = N;
    ix->nonempty_slots = nonempty;
    ix->free_workspace();                 // sized for the builder's chunks and w = 1
    (void)hipFree(b->slots); (void)hipFree(b->codes); (void)hipFree(b->leaf);
    b->slots = nullptr; b->codes = nullptr; b->leaf = nullptr;
    *out = ix;
    b->ix = nullptr;                      // the index now belongs to the caller
    return PQT_OK;
}

}  // extern "C"
