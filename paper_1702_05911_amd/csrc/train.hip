// Training on a sample (Sec. 3.1 "Training the codebook"; Sec. 3.3 "Offline computation"): the level-1
// product quantiser of every tree part by Lloyd iterations (Sec. 2.1), then, independently inside each
// of its cells, the level-2 quantiser of the sub-vectors that fall into the cell -- all k1 cells of a
// part are trained side by side as "groups" of one batched Lloyd run -- and the table of 256 line code
// points (i, j, lambda) per re-rank sub-part: every training sub-vector votes for the nearest line
// through two level-1 centroids (its projection error comes from its own level-1 distances, as in the
// re-ranking: b^2 - lambda^2 c^2 with lambda = (b^2 - a^2 + c^2) / (2 c^2)); lines receive code points
// in proportion to their votes, placed at the quantiles of the lambdas seen on the line.
//
// Everything per vector runs in the kernels below.  Results do not depend on the order in which the
// hardware schedules work: assignments break ties by the smaller centroid number, cell sums are taken
// over the members in ascending vector order in fixed slices (double precision), re-seeding takes the
// farthest vector with the smallest number.
#include <hipcub/hipcub.hpp>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "pqt_device.hpp"
#include "pqt_index.hpp"

using pqt_host::DeviceGuard;
using pqt_host::fail;

namespace pqt {
namespace {

constexpr int kTrainThreads = 256;

__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(v >> 32), off, kWave);
        const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)v, off, kWave);
        const unsigned long long o = ((unsigned long long)hi << 32) | lo;
        v = o < v ? o : v;
    }
    return v;
}

// Start centroids of every group (Sec. 2.1: Lloyd iterations need a start): k members at evenly spaced
// places of the group's member list.  A group with no more than k members is frozen: its members are
// centroids themselves, the remaining centroids repeat the members' mean (the parent centroid when
// the group is empty).  One workgroup per group.
__global__ __launch_bounds__(kTrainThreads) void lloyd_init_kernel(const float* X, int D, int col0, int dp,
                                                                    const uint32_t* members, const uint32_t* grp_off,
                                                                    int k, const float* parent, float* cen, float* cenT,
                                                                    uint8_t* frozen) {
    const int g = blockIdx.x, tid = threadIdx.x;
    const uint32_t lo = grp_off[g], hi = grp_off[g + 1];
    const uint32_t ng = hi - lo;
    if (tid == 0) frozen[g] = ng <= (uint32_t)k ? 1 : 0;
    for (int e = tid; e < k * dp; e += kTrainThreads) {
        const int j = e / dp, d = e - j * dp;
        float v;
        if (ng > (uint32_t)k) {
            const uint32_t at = lo + (uint32_t)(((unsigned long long)j * ng) / (unsigned)k);
            const uint32_t row = members ? members[at] : at;
            v = X[(size_t)row * D + col0 + d];
        } else if ((uint32_t)j < ng) {
            const uint32_t row = members ? members[lo + j] : lo + j;
            v = X[(size_t)row * D + col0 + d];
        } else if (ng == 0) {
            v = parent ? parent[(size_t)g * dp + d] : 0.0f;
        } else {
            double s = 0.0;
            for (uint32_t r = lo; r < hi; ++r) s += (double)X[(size_t)(members ? members[r] : r) * D + col0 + d];
            v = (float)(s / (double)ng);
        }
        cen[((size_t)g * k + j) * dp + d] = v;
        cenT[((size_t)g * dp + d) * k + j] = v;
    }
}

// Nearest centroid of every vector among the k centroids of its group: one wavefront per vector, one
// lane per centroid (several rounds when k > 64); plain sums of squared differences, dimensions in
// ascending order; ties go to the smaller centroid number.  cenT holds the centroids of a group with
// the centroid number fastest, so the lanes of a wavefront read consecutive words.
__global__ __launch_bounds__(kTrainThreads) void lloyd_assign_kernel(const float* X, int64_t n, int D, int col0, int dp,
                                                                      const float* cenT, int k, const uint32_t* group,
                                                                      uint32_t* label, float* dmin) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t nwaves = (int64_t)gridDim.x * (kTrainThreads / kWave);
    for (int64_t v = (int64_t)blockIdx.x * (kTrainThreads / kWave) + threadIdx.x / kWave; v < n; v += nwaves) {
        const uint32_t g = group ? group[v] : 0u;
        const float* xr = X + (size_t)v * D + col0;
        const float* ct = cenT + (size_t)g * dp * k;
        unsigned long long best = ~0ull;
        for (int j0 = 0; j0 < k; j0 += kWave) {
            const int j = j0 + lane;
            float acc = 0.0f;
            for (int d0 = 0; d0 < dp; d0 += kWave) {
                const float xc = (d0 + lane < dp) ? xr[d0 + lane] : 0.0f;
                const int nd = dp - d0 < kWave ? dp - d0 : kWave;
                for (int dd = 0; dd < nd; ++dd) {
                    const float xs = __shfl(xc, dd, kWave);
                    const float c = j < k ? ct[(size_t)(d0 + dd) * k + j] : 0.0f;
                    const float diff = xs - c;
                    acc = fmaf(diff, diff, acc);
                }
            }
            const unsigned long long key = j < k ? (((unsigned long long)mono_key(acc) << 32) | (unsigned)j) : ~0ull;
            best = key < best ? key : best;
        }
        best = wave_min_u64(best);
        if (lane == 0) {
            label[v] = g * (uint32_t)k + (uint32_t)best;
            dmin[v] = mono_inv((uint32_t)(best >> 32));
        }
    }
}

__global__ void iota_u32_kernel(uint32_t* out, uint32_t n) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = i;
}

__global__ void count_labels_kernel(const uint32_t* label, uint32_t n, uint32_t* counts) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) atomicAdd(&counts[label[i]], 1u);           // integer counts: the order of the additions does not matter
}

__global__ void fill_u32_kernel(uint32_t* out, uint32_t n, uint32_t value) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = value;
}

// Sum of the members of cell blockIdx.x inside slice blockIdx.y of its member list (members sorted by
// vector number), per dimension, in double precision.  Threads are laid out as (row lane, dimension):
// a row lane adds every rl-th member in ascending order, then the row lanes are added in ascending order.
__global__ __launch_bounds__(kTrainThreads) void lloyd_accumulate_kernel(const float* X, int D, int col0, int dp,
                                                                          const uint32_t* sorted_idx, const uint32_t* seg_off,
                                                                          int S, double* partial) {
    __shared__ double red[kTrainThreads];
    const int c = blockIdx.x, s = blockIdx.y, tid = threadIdx.x;
    const uint32_t lo = seg_off[c], hi = seg_off[c + 1];
    const uint32_t len = hi - lo, chunk = (len + (uint32_t)S - 1) / (uint32_t)S;
    const uint32_t a = lo + (uint32_t)s * chunk < hi ? lo + (uint32_t)s * chunk : hi;
    const uint32_t b = a + chunk < hi ? a + chunk : hi;
    int dw = 1;
    while (dw < dp && dw < kTrainThreads) dw <<= 1;        // dimensions handled side by side
    const int rl = kTrainThreads / dw, r = tid / dw, dl = tid - r * dw;
    for (int d0 = 0; d0 < dp; d0 += dw) {
        const int d = d0 + dl;
        double acc = 0.0;
        if (d < dp)
            for (uint32_t e = a + (uint32_t)r; e < b; e += (uint32_t)rl) acc += (double)X[(size_t)sorted_idx[e] * D + col0 + d];
        red[tid] = acc;
        __syncthreads();
        if (r == 0 && d < dp) {
            double t = 0.0;
            for (int rr = 0; rr < rl; ++rr) t += red[rr * dw + dl];
            partial[((size_t)c * S + s) * dp + d] = t;
        }
        __syncthreads();
    }
}

// centroid = mean of its members (the slices added in ascending order); an empty cell and the cells of a
// frozen group keep what they hold
__global__ void lloyd_finalize_kernel(const double* partial, int S, const uint32_t* seg_off, uint32_t cells, int dp, int k,
                                      const uint8_t* frozen, float* cen, float* cenT) {
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)cells * dp) return;
    const uint32_t c = (uint32_t)(e / dp);
    const int d = (int)(e - (size_t)c * dp);
    const uint32_t g = c / (uint32_t)k, j = c - g * (uint32_t)k;
    const uint32_t cnt = seg_off[c + 1] - seg_off[c];
    if (cnt == 0 || frozen[g]) return;
    double t = 0.0;
    for (int s = 0; s < S; ++s) t += partial[((size_t)c * S + s) * dp + d];
    const float v = (float)(t / (double)cnt);
    cen[e] = v;
    cenT[((size_t)g * dp + d) * k + j] = v;
}

// An empty cell is re-seeded with the member of its group that lies farthest from its centroid (ties:
// the smaller vector number); that vector then counts as at distance zero, so the next empty cell of
// the group takes another one.  One workgroup per group, its empty cells one after the other.
__global__ __launch_bounds__(kTrainThreads) void lloyd_reseed_kernel(const float* X, int D, int col0, int dp,
                                                                      const uint32_t* sorted_idx, const uint32_t* seg_off, int k,
                                                                      const uint8_t* frozen, float* dmin, float* cen, float* cenT) {
    __shared__ unsigned long long red[kTrainThreads / kWave];
    __shared__ uint32_t far_row;
    const int g = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1);
    const uint32_t glo = seg_off[(size_t)g * k], ghi = seg_off[(size_t)(g + 1) * k];
    if (frozen[g] || ghi == glo) return;
    for (int j = 0; j < k; ++j) {
        const uint32_t c = (uint32_t)g * (uint32_t)k + (uint32_t)j;
        if (seg_off[c + 1] != seg_off[c]) continue;                         // same for the whole workgroup
        unsigned long long best = 0ull;
        for (uint32_t e = glo + (uint32_t)tid; e < ghi; e += kTrainThreads) {
            const uint32_t row = sorted_idx[e];
            const unsigned long long key = ((unsigned long long)mono_key(dmin[row]) << 32) | (0xffffffffu - row);
            best = key > best ? key : best;
        }
        best = ~wave_min_u64(~best);                                        // maximum over the wavefront
        if (lane == 0) red[tid / kWave] = best;
        __syncthreads();
        if (tid == 0) {
            unsigned long long m = red[0];
            for (int w = 1; w < kTrainThreads / kWave; ++w) m = red[w] > m ? red[w] : m;
            far_row = 0xffffffffu - (uint32_t)m;
        }
        __syncthreads();
        const uint32_t row = far_row;
        for (int d = tid; d < dp; d += kTrainThreads) {
            const float v = X[(size_t)row * D + col0 + d];
            cen[(size_t)c * dp + d] = v;
            cenT[((size_t)g * dp + d) * k + j] = v;
        }
        if (tid == 0) dmin[row] = 0.0f;
        __syncthreads();                                                    // the next empty cell sees it
    }
}

// The nearest line of every training sub-vector (Sec. 3.3 "Offline computation"): one wavefront per
// vector, the centroid pairs i < j spread over the lanes.  With b^2, a^2 the vector's level-1 distances
// to c_i, c_j of sub-part m and c^2 = ||c_i - c_j||^2: the projection lies at lambda = (b^2 - a^2 + c^2) /
// (2 c^2) and misses the vector by b^2 - lambda^2 c^2.  Smallest (error, pair number) wins; pairs of
// coinciding centroids never do.  key[m][v] = pair number << 32 | ordered bits of lambda (sorting these
// orders the votes by line, then by lambda); 0xffffffff.. when the sub-part has no usable pair.
__global__ __launch_bounds__(kTrainThreads) void line_vote_kernel(const float* a, int64_t n, int M, int k1, const uint16_t* pair_ij,
                                                                   int npairs, const float* cc, unsigned long long* keys,
                                                                   int64_t key_stride, int64_t key_base) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t v = (int64_t)blockIdx.x * (kTrainThreads / kWave) + threadIdx.x / kWave;
    if (v >= n) return;
    const float* av = a + (size_t)v * M * k1;
    for (int m = 0; m < M; ++m) {
        unsigned long long best = ~0ull;
        for (int pid = lane; pid < npairs; pid += kWave) {
            const int i = pair_ij[2 * pid], j = pair_ij[2 * pid + 1];
            const float c2 = cc[((size_t)m * k1 + i) * k1 + j];
            if (!(c2 > 0.0f)) continue;
            const float b2 = av[m * k1 + i], a2 = av[m * k1 + j];
            const float lam = ((b2 - a2) + c2) / (2.0f * c2);
            const float err = fmaf(-lam * lam, c2, b2);
            const unsigned long long key = ((unsigned long long)mono_key(err) << 32) | (unsigned)pid;
            best = key < best ? key : best;
        }
        best = wave_min_u64(best);
        if (lane == 0) {
            unsigned long long out = ~0ull;
            if (best != ~0ull) {
                const int pid = (int)(uint32_t)best;
                const int i = pair_ij[2 * pid], j = pair_ij[2 * pid + 1];
                const float c2 = cc[((size_t)m * k1 + i) * k1 + j];
                const float b2 = av[m * k1 + i], a2 = av[m * k1 + j];
                const float lam = ((b2 - a2) + c2) / (2.0f * c2);
                out = ((unsigned long long)(uint32_t)pid << 32) | mono_key(lam);
            }
            keys[(size_t)m * key_stride + key_base + v] = out;
        }
    }
}

struct DeviceBuffers {      // everything pqt_train allocates on the GPU, released together
    std::vector<void*> ptrs;
    ~DeviceBuffers() {
        for (void* p : ptrs) (void)hipFree(p);
    }
    template <typename Tp>
    hipError_t alloc(Tp** out, size_t count) {
        void* p = nullptr;
        const hipError_t e = hipMalloc(&p, (count ? count : 1) * sizeof(Tp));
        if (e == hipSuccess) ptrs.push_back(p);
        *out = static_cast<Tp*>(p);
        return e;
    }
};

struct LloydScratch {
    uint32_t *label = nullptr, *label_sorted = nullptr, *idx = nullptr, *idx_sorted = nullptr, *counts = nullptr, *seg_off = nullptr;
    float* dmin = nullptr;
    double* partial = nullptr;
    uint8_t* frozen = nullptr;
    void* cub_temp = nullptr;
    size_t cub_bytes = 0;
};

int log2_ceil(uint32_t v) {
    int b = 1;
    while (b < 32 && (1ull << b) < v) ++b;
    return b;
}

// labels -> members of every cell in ascending vector order (idx_sorted) and the cells' offsets
hipError_t sort_by_label(const LloydScratch& w, uint32_t n, uint32_t cells, hipStream_t st) {
    const unsigned tb = 256;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((cells + 1 + tb - 1) / tb), dim3(tb), 0, st, w.counts, cells + 1, 0u);
    hipLaunchKernelGGL(count_labels_kernel, dim3((n + tb - 1) / tb), dim3(tb), 0, st, w.label, n, w.counts);
    size_t bytes = w.cub_bytes;
    hipError_t e = hipcub::DeviceScan::ExclusiveSum(w.cub_temp, bytes, w.counts, w.seg_off, (int)(cells + 1), st);
    if (e != hipSuccess) return e;
    bytes = w.cub_bytes;
    e = hipcub::DeviceRadixSort::SortPairs(w.cub_temp, bytes, w.label, w.label_sorted, w.idx, w.idx_sorted, (int)n, 0,
                                           log2_ceil(cells), st);
    return e == hipSuccess ? hipGetLastError() : e;
}

// Lloyd iterations for G groups of k centroids each; cen / cenT hold the start and receive the result.
hipError_t lloyd_run(const float* X, uint32_t n, int D, int col0, int dp, int G, int k, const uint32_t* group, int iters,
                     float* cen, float* cenT, const LloydScratch& w, int S, hipStream_t st) {
    const uint32_t cells = (uint32_t)G * (uint32_t)k;
    const unsigned assign_blocks = (unsigned)std::min<uint64_t>(((uint64_t)n + 3) / 4, 65536);
    for (int it = 0; it < iters; ++it) {
        hipLaunchKernelGGL(lloyd_assign_kernel, dim3(assign_blocks), dim3(kTrainThreads), 0, st, X, (int64_t)n, D, col0, dp,
                           cenT, k, group, w.label, w.dmin);
        hipError_t e = sort_by_label(w, n, cells, st);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(lloyd_accumulate_kernel, dim3(cells, S), dim3(kTrainThreads), 0, st, X, D, col0, dp, w.idx_sorted,
                           w.seg_off, S, w.partial);
        const size_t ne = (size_t)cells * dp;
        hipLaunchKernelGGL(lloyd_finalize_kernel, dim3((unsigned)((ne + 255) / 256)), dim3(256), 0, st, w.partial, S, w.seg_off,
                           cells, dp, k, w.frozen, cen, cenT);
        hipLaunchKernelGGL(lloyd_reseed_kernel, dim3(G), dim3(kTrainThreads), 0, st, X, D, col0, dp, w.idx_sorted, w.seg_off, k,
                           w.frozen, w.dmin, cen, cenT);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Code points per line by the largest-remainder method, in whole numbers: line q with use[q] of `total`
// votes gets floor(use[q] * n_codes / total), the code points left over go one each to the lines with the
// largest remainders (ties: smaller q).
std::vector<uint32_t> share_out(const std::vector<uint64_t>& use, uint64_t total, uint32_t n_codes) {
    std::vector<uint32_t> alloc(use.size(), 0);
    if (total == 0) return alloc;
    std::vector<std::pair<uint64_t, uint32_t>> rem;        // (remainder, line)
    uint64_t given = 0;
    for (uint32_t q = 0; q < use.size(); ++q) {
        const uint64_t num = use[q] * n_codes;
        alloc[q] = (uint32_t)(num / total);
        given += alloc[q];
        if (num % total) rem.emplace_back(num % total, q);
    }
    std::sort(rem.begin(), rem.end(), [](const auto& l, const auto& r) { return l.first != r.first ? l.first > r.first : l.second < r.second; });
    for (size_t t = 0; given < n_codes && t < rem.size(); ++t, ++given) alloc[rem[t].second]++;
    return alloc;
}

}  // namespace
}  // namespace pqt

extern "C" int pqt_train(const pqt_train_params* tp, const float* vectors, int device, float* C1_out, float* C2_out,
                         uint8_t* tbl_i, uint8_t* tbl_j, float* tbl_lambda, float* cc_out, void* hip_stream) {
    using namespace pqt;
    if (!tp || !vectors || !C1_out || !C2_out || !cc_out) return fail(PQT_EINVAL, "pqt_train: null argument");
    const uint32_t D = tp->D, P = tp->P, k1 = tp->k1, k2 = tp->k2, M = tp->M;
    if (D == 0 || P == 0 || k1 == 0 || k2 == 0 || M == 0 || D % P || D % M || M % P)
        return fail(PQT_EINVAL, "pqt_train: inconsistent sizes D=%u P=%u k1=%u k2=%u M=%u", D, P, k1, k2, M);
    if (!(P == 1 || P == 2 || P == 4)) return fail(PQT_EUNSUPPORTED, "P=%u: only 1, 2 or 4 tree parts", P);
    if (k1 > PQT_MAX_K1 || k2 > PQT_MAX_R || M > 64 || D > 8192)
        return fail(PQT_EUNSUPPORTED, "k1=%u k2=%u M=%u D=%u beyond the kernel limits", k1, k2, M, D);
    if (tp->n == 0 || tp->n >= 0xffffffffull) return fail(PQT_EINVAL, "pqt_train: n=%llu training vectors", (unsigned long long)tp->n);
    if (tp->n_table > tp->n) return fail(PQT_EINVAL, "pqt_train: n_table exceeds n");
    if (tp->n_table > 0 && (!tbl_i || !tbl_j || !tbl_lambda)) return fail(PQT_EINVAL, "pqt_train: null table array");
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev)
        return fail(PQT_EHIP, "GPU %d is not available (%d visible)", device, ndev);
    DeviceGuard guard(device);
    if (!guard.ok) return fail(PQT_EHIP, "cannot select GPU %d", device);
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);

    const uint32_t n = (uint32_t)tp->n;
    const int dp = (int)(D / P), ds = (int)(D / M);
    const uint32_t cells1 = k1, cells2 = k1 * k2;
    const int S1 = (int)std::max<uint32_t>(1, std::min<uint32_t>(64, 2048 / cells1));
    const int S2 = (int)std::max<uint32_t>(1, std::min<uint32_t>(64, 2048 / cells2));
    DeviceBuffers mem;
    LloydScratch w;
    float *cen1 = nullptr, *cen1T = nullptr, *cen2 = nullptr, *cen2T = nullptr;
    uint32_t *label1 = nullptr, *members1 = nullptr, *grp_off1 = nullptr, *grp_whole = nullptr;
    const size_t npartial = std::max((size_t)cells1 * S1, (size_t)cells2 * S2) * dp;
    HIP_TRY(mem.alloc(&w.label, n));
    HIP_TRY(mem.alloc(&w.label_sorted, n));
    HIP_TRY(mem.alloc(&w.idx, n));
    HIP_TRY(mem.alloc(&w.idx_sorted, n));
    HIP_TRY(mem.alloc(&w.counts, (size_t)cells2 + 1));
    HIP_TRY(mem.alloc(&w.seg_off, (size_t)cells2 + 1));
    HIP_TRY(mem.alloc(&w.dmin, n));
    HIP_TRY(mem.alloc(&w.partial, npartial));
    HIP_TRY(mem.alloc(&w.frozen, (size_t)k1 + 1));
    HIP_TRY(mem.alloc(&cen1, (size_t)k1 * dp));
    HIP_TRY(mem.alloc(&cen1T, (size_t)k1 * dp));
    HIP_TRY(mem.alloc(&cen2, (size_t)cells2 * dp));
    HIP_TRY(mem.alloc(&cen2T, (size_t)cells2 * dp));
    HIP_TRY(mem.alloc(&label1, n));
    HIP_TRY(mem.alloc(&members1, n));
    HIP_TRY(mem.alloc(&grp_off1, (size_t)k1 + 1));
    HIP_TRY(mem.alloc(&grp_whole, 2));
    {
        size_t b1 = 0, b2 = 0;
        HIP_TRY(hipcub::DeviceScan::ExclusiveSum(nullptr, b1, w.counts, w.seg_off, (int)(cells2 + 1), st));
        HIP_TRY(hipcub::DeviceRadixSort::SortPairs(nullptr, b2, w.label, w.label_sorted, w.idx, w.idx_sorted, (int)n, 0, 32, st));
        w.cub_bytes = std::max(b1, b2);
        HIP_TRY(mem.alloc(reinterpret_cast<unsigned char**>(&w.cub_temp), w.cub_bytes));
    }
    const unsigned tb = 256;
    hipLaunchKernelGGL(iota_u32_kernel, dim3((n + tb - 1) / tb), dim3(tb), 0, st, w.idx, n);
    const uint32_t whole[2] = {0u, n};
    HIP_TRY(hipMemcpyAsync(grp_whole, whole, sizeof(whole), hipMemcpyHostToDevice, st));     // one group: the whole sample
    HIP_TRY(hipStreamSynchronize(st));                   // `whole` is on this stack frame

    std::vector<float> C1((size_t)P * k1 * dp), C2((size_t)P * cells2 * dp);
    const unsigned assign_blocks = (unsigned)std::min<uint64_t>(((uint64_t)n + 3) / 4, 65536);
    for (uint32_t p = 0; p < P; ++p) {
        const int col0 = (int)p * dp;
        // ---- level 1: one group, k1 centroids ---------------------------------------------------------
        hipLaunchKernelGGL(lloyd_init_kernel, dim3(1), dim3(kTrainThreads), 0, st, vectors, (int)D, col0, dp,
                           (const uint32_t*)nullptr, grp_whole, (int)k1, (const float*)nullptr, cen1, cen1T, w.frozen);
        HIP_TRY(hipGetLastError());
        HIP_TRY(lloyd_run(vectors, n, (int)D, col0, dp, 1, (int)k1, nullptr, (int)tp->iters, cen1, cen1T, w, S1, st));
        // ---- the cells of the finished quantiser: members in ascending vector order -------------------------
        hipLaunchKernelGGL(lloyd_assign_kernel, dim3(assign_blocks), dim3(kTrainThreads), 0, st, vectors, (int64_t)n, (int)D, col0, dp,
                           cen1T, (int)k1, (const uint32_t*)nullptr, w.label, w.dmin);
        HIP_TRY(sort_by_label(w, n, cells1, st));
        HIP_TRY(hipMemcpyAsync(label1, w.label, sizeof(uint32_t) * n, hipMemcpyDeviceToDevice, st));
        HIP_TRY(hipMemcpyAsync(members1, w.idx_sorted, sizeof(uint32_t) * n, hipMemcpyDeviceToDevice, st));
        HIP_TRY(hipMemcpyAsync(grp_off1, w.seg_off, sizeof(uint32_t) * (k1 + 1), hipMemcpyDeviceToDevice, st));
        // ---- level 2: k1 groups (the cells), k2 centroids each, trained side by side ---------------------------
        hipLaunchKernelGGL(lloyd_init_kernel, dim3(k1), dim3(kTrainThreads), 0, st, vectors, (int)D, col0, dp, members1, grp_off1,
                           (int)k2, cen1, cen2, cen2T, w.frozen);
        HIP_TRY(hipGetLastError());
        HIP_TRY(lloyd_run(vectors, n, (int)D, col0, dp, (int)k1, (int)k2, label1, (int)tp->iters, cen2, cen2T, w, S2, st));
        HIP_TRY(hipMemcpyAsync(C1.data() + (size_t)p * k1 * dp, cen1, sizeof(float) * k1 * dp, hipMemcpyDeviceToHost, st));
        HIP_TRY(hipMemcpyAsync(C2.data() + (size_t)p * cells2 * dp, cen2, sizeof(float) * cells2 * dp, hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
    }
    memcpy(C1_out, C1.data(), C1.size() * sizeof(float));
    memcpy(C2_out, C2.data(), C2.size() * sizeof(float));

    // ---- distances between the level-1 centroids of every sub-part (Sec. 3.3: the table of c^2) -----------
    const size_t per = M / P;
    std::vector<float> cc((size_t)M * k1 * k1);
    for (size_t m = 0; m < M; ++m) {
        const size_t p = m / per, lo = m * ds - p * dp;
        for (size_t s = 0; s < k1; ++s)
            for (size_t t = 0; t < k1; ++t) {
                double acc = 0.0;
                for (int d = 0; d < ds; ++d) {
                    const double diff = (double)C1[(p * k1 + s) * dp + lo + d] - (double)C1[(p * k1 + t) * dp + lo + d];
                    acc += diff * diff;
                }
                cc[(m * k1 + s) * k1 + t] = (float)acc;
            }
    }
    memcpy(cc_out, cc.data(), cc.size() * sizeof(float));
    if (tbl_i) memset(tbl_i, 0, (size_t)M * 256);
    if (tbl_j) memset(tbl_j, 0, (size_t)M * 256);
    if (tbl_lambda) memset(tbl_lambda, 0, (size_t)M * 256 * sizeof(float));
    const uint32_t npairs = k1 * (k1 - 1) / 2;
    const uint32_t nt = (uint32_t)tp->n_table;
    if (nt == 0 || npairs == 0) return PQT_OK;

    // ---- line table: level-1 distances of the first n_table vectors by the query path's own traversal kernel
    // (an index without vectors carries the codebooks to the GPU), then one vote per sub-vector ---------------------
    std::vector<uint32_t> zeros(2, 0u);
    std::vector<uint8_t> zt((size_t)M * 256, 0);
    std::vector<float> zl((size_t)M * 256, 0.0f);
    pqt_index_arrays ea = {};
    ea.N = 0; ea.H = 1; ea.D = D; ea.P = P; ea.k1 = k1; ea.k2 = k2; ea.M = M; ea.T = 1; ea.C = 1;
    ea.C1 = C1.data(); ea.C2 = C2.data(); ea.tbl_i = zt.data(); ea.tbl_j = zt.data(); ea.tbl_lambda = zl.data();
    ea.cc = cc.data(); ea.offsets = zeros.data(); ea.ids = nullptr; ea.codes = nullptr; ea.code_format = PQT_CODES_TABLE;
    pqt_index* ix = nullptr;
    int rc = pqt_index_from_arrays(&ea, PQT_HOST, device, &ix);
    if (rc) return rc;
    struct IndexHolder {
        pqt_index* ix;
        ~IndexHolder() { pqt_index_free(ix); }
    } holder{ix};
    if (pqt::traverse_lds_bytes(D, P, k1, k2, M, 1) > ix->lds_limit)
        return fail(PQT_EUNSUPPORTED, "pqt_train: D=%u exceeds the LDS budget of the traversal", D);
    std::vector<uint16_t> pair_host((size_t)npairs * 2);
    {
        size_t e = 0;
        for (uint32_t i = 0; i < k1; ++i)
            for (uint32_t j = i + 1; j < k1; ++j) {
                pair_host[e++] = (uint16_t)i;
                pair_host[e++] = (uint16_t)j;
            }
    }
    uint16_t* pair_dev = nullptr;
    float* cc_dev = nullptr;
    unsigned long long *keys = nullptr, *keys_sorted = nullptr;
    HIP_TRY(mem.alloc(&pair_dev, pair_host.size()));
    HIP_TRY(mem.alloc(&cc_dev, cc.size()));
    HIP_TRY(mem.alloc(&keys, (size_t)M * nt));
    HIP_TRY(mem.alloc(&keys_sorted, (size_t)nt));
    HIP_TRY(hipMemcpyAsync(pair_dev, pair_host.data(), pair_host.size() * sizeof(uint16_t), hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(cc_dev, cc.data(), cc.size() * sizeof(float), hipMemcpyHostToDevice, st));
    const int64_t chunk = 1 << 17;
    for (int64_t s = 0; s < (int64_t)nt; s += chunk) {
        const int64_t mrows = (int64_t)nt - s < chunk ? (int64_t)nt - s : chunk;
        if ((rc = pqt_host::ensure_workspace(ix, mrows, (int)k2))) return rc;
        pqt::TraverseArgs ta;
        ta.queries = vectors + (size_t)s * D; ta.nq = mrows;
        ta.D = (int)D; ta.P = (int)P; ta.k1 = (int)k1; ta.k2 = (int)k2; ta.M = (int)M; ta.w = 1;
        ta.C1 = ix->C1; ta.c1n = ix->c1n; ta.C2 = ix->C2; ta.C2t = ix->C2t;
        ta.a = ix->ws_a; ta.L_d = ix->ws_Ld; ta.L_id = ix->ws_Lid; ta.sel_tap = nullptr; ta.counters = nullptr;
        HIP_TRY(pqt::launch_traverse(ta, st));
        constexpr int per_block = kTrainThreads / kWave;
        hipLaunchKernelGGL(line_vote_kernel, dim3((unsigned)((mrows + per_block - 1) / per_block)), dim3(kTrainThreads), 0, st,
                           ix->ws_a, mrows, (int)M, (int)k1, pair_dev, (int)npairs, cc_dev, keys, (int64_t)nt, s);
        HIP_TRY(hipGetLastError());
    }
    size_t sort_bytes = 0;
    HIP_TRY(hipcub::DeviceRadixSort::SortKeys(nullptr, sort_bytes, keys, keys_sorted, (int)nt, 0, 64, st));
    void* sort_temp = nullptr;
    HIP_TRY(mem.alloc(reinterpret_cast<unsigned char**>(&sort_temp), sort_bytes));
    std::vector<unsigned long long> votes;
    try {
        votes.resize(nt);
    } catch (const std::bad_alloc&) {
        return fail(PQT_ENOMEM, "host allocation failed");
    }
    for (uint32_t m = 0; m < M; ++m) {
        HIP_TRY(hipcub::DeviceRadixSort::SortKeys(sort_temp, sort_bytes, keys + (size_t)m * nt, keys_sorted, (int)nt, 0, 64, st));
        HIP_TRY(hipMemcpyAsync(votes.data(), keys_sorted, sizeof(unsigned long long) * nt, hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        // votes per line and where each line's lambdas start (the keys are sorted by line, then lambda)
        std::vector<uint64_t> use(npairs, 0), first(npairs, 0);
        uint64_t total = 0;
        for (uint32_t e = 0; e < nt; ++e) {
            const uint32_t q = (uint32_t)(votes[e] >> 32);
            if (q >= npairs) break;                          // sub-vectors without a usable line sort last
            if (use[q]++ == 0) first[q] = e;
            ++total;
        }
        if (total == 0) continue;
        const std::vector<uint32_t> alloc = share_out(use, total, 256);
        // a line's code points sit at the (t + 1/2) / alloc quantiles of its lambdas; lines in pair order and
        // lambdas ascending, so the entries come out ordered by (i, j, lambda)
        uint32_t c = 0;
        for (uint32_t q = 0; q < npairs && c < 256; ++q)
            for (uint32_t t = 0; t < alloc[q] && c < 256; ++t, ++c) {
                uint64_t pos = ((2ull * t + 1ull) * use[q]) / (2ull * alloc[q]);
                if (pos >= use[q]) pos = use[q] - 1;
                const uint32_t bits = (uint32_t)votes[first[q] + pos];
                const uint32_t u = (bits & 0x80000000u) ? (bits & 0x7fffffffu) : ~bits;      // ordered bits -> float
                float lam;
                memcpy(&lam, &u, sizeof(lam));
                tbl_i[(size_t)m * 256 + c] = (uint8_t)pair_host[2 * q];
                tbl_j[(size_t)m * 256 + c] = (uint8_t)pair_host[2 * q + 1];
                tbl_lambda[(size_t)m * 256 + c] = lam;
            }
        for (; c > 0 && c < 256; ++c) {                      // (cannot happen when total > 0; kept total)
            tbl_i[(size_t)m * 256 + c] = tbl_i[(size_t)m * 256 + c - 1];
            tbl_j[(size_t)m * 256 + c] = tbl_j[(size_t)m * 256 + c - 1];
            tbl_lambda[(size_t)m * 256 + c] = tbl_lambda[(size_t)m * 256 + c - 1];
        }
    }
    return PQT_OK;
}
