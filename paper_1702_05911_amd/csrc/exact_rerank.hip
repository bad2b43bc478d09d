// Exact re-ranking of a short list (step (3) of the pipelines in Sec. 1; the paper's PQT_2 of
// Table 1): the first k_short results of the line-quantisation re-ranking are scored again by their
// exact squared distance ||y - x||^2 to the raw database vectors, and the k best by (distance, id)
// are returned.
//
// One workgroup of 256 threads per query.  The query sits in LDS; a group of lanes (64, or fewer when
// the vector is short) reads one database row with consecutive 16-byte pieces per lane, so a row is a
// few fully used cache lines and the kernel is bound by HBM: k_short rows of D elements per query.
// Squared differences are summed per lane in ascending dimension, then across the group by a fixed
// xor tree, so the result does not depend on scheduling.  The (ordered distance bits, id) keys are
// sorted by the workgroup.
#include "pqt_device.hpp"
#include "pqt_kernels.hpp"

namespace pqt {

constexpr int kExactThreads = 256;

// One 16-byte piece of a row: kPiece<Elem> elements; adds their squared differences to acc in
// ascending dimension.  y points at the query's elements of the same dimensions (LDS).
template <typename Elem>
struct Piece;
template <>
struct Piece<float> {
    static constexpr int kElems = 4;
    static __device__ __forceinline__ float add(const float* row, int piece, const float* y, float acc) {
        const float4 x = reinterpret_cast<const float4*>(row)[piece];
        const float4 v = reinterpret_cast<const float4*>(y)[piece];
        float d = v.x - x.x;
        acc = fmaf(d, d, acc);
        d = v.y - x.y;
        acc = fmaf(d, d, acc);
        d = v.z - x.z;
        acc = fmaf(d, d, acc);
        d = v.w - x.w;
        return fmaf(d, d, acc);
    }
};
template <>
struct Piece<uint8_t> {
    static constexpr int kElems = 16;
    static __device__ __forceinline__ float add(const uint8_t* row, int piece, const float* y, float acc) {
        const uint4 x = reinterpret_cast<const uint4*>(row)[piece];
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 v = reinterpret_cast<const float4*>(y)[piece * 4 + j];
            float d = v.x - (float)(w[j] & 0xffu);
            acc = fmaf(d, d, acc);
            d = v.y - (float)((w[j] >> 8) & 0xffu);
            acc = fmaf(d, d, acc);
            d = v.z - (float)((w[j] >> 16) & 0xffu);
            acc = fmaf(d, d, acc);
            d = v.w - (float)(w[j] >> 24);
            acc = fmaf(d, d, acc);
        }
        return acc;
    }
};

template <typename Elem>
__global__ __launch_bounds__(kExactThreads) void exact_rerank_kernel(ExactArgs g) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int D = g.D, nd4 = D / 4, ks = g.k_short, k = g.k;
    float4* sy = reinterpret_cast<float4*>(smem);                                        // D floats
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem + sizeof(float) * D);   // next_pow2(ks), >= 64
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t q = blockIdx.x;
    const Elem* X = reinterpret_cast<const Elem*>(g.vectors);

    for (int c4 = tid; c4 < nd4; c4 += kExactThreads) sy[c4] = reinterpret_cast<const float4*>(g.queries + q * D)[c4];
    const int npad = next_pow2(ks) < 64 ? 64 : next_pow2(ks);
    for (int e = ks + tid; e < npad; e += kExactThreads) keys[e] = ~0ull;
    __syncthreads();

    // lanes per row: a power of two, at most 64, one 16-byte piece per lane and step if possible
    constexpr int pe = Piece<Elem>::kElems;
    const int npieces = D / pe;                      // D is a multiple of the piece (checked by the launcher)
    int lpr = 1;
    while (lpr < kWave && lpr < npieces) lpr <<= 1;
    const int rows_per_wave = kWave / lpr, sub = lane / lpr, l = lane & (lpr - 1);
    const int rows_per_iter = rows_per_wave * (kExactThreads / kWave);
    const float* y = reinterpret_cast<const float*>(sy);
#pragma unroll 2
    for (int c0 = 0; c0 < ks; c0 += rows_per_iter) {
        const int c = c0 + wave * rows_per_wave + sub;
        const int64_t id = c < ks ? g.short_ids[q * ks + c] : -1;
        float acc = 0.0f;
        if (id >= 0) {
            const Elem* row = X + (size_t)id * D;
            for (int piece = l; piece < npieces; piece += lpr) acc = Piece<Elem>::add(row, piece, y, acc);
        }
        for (int off = 1; off < lpr; off <<= 1) acc += __shfl_xor(acc, off, kWave);   // same order in every lane
        if (c < ks && l == 0)
            keys[c] = id >= 0 ? (((unsigned long long)mono_key(acc) << 32) | (uint32_t)id) : ~0ull;
    }
    block_sort_lds<4>(keys, npad, tid, kExactThreads);
    for (int e = tid; e < k; e += kExactThreads) {
        const unsigned long long key = keys[e];
        if (key == ~0ull) {
            g.out_ids[q * k + e] = -1;
            g.out_dists[q * k + e] = __builtin_inff();
        } else {
            g.out_ids[q * k + e] = (int64_t)(uint32_t)key;
            g.out_dists[q * k + e] = mono_inv((uint32_t)(key >> 32));
        }
    }
}

size_t exact_lds_bytes(int D, int k_short) {
    const int npad = next_pow2(k_short) < 64 ? 64 : next_pow2(k_short);
    return sizeof(float) * D + sizeof(unsigned long long) * npad;
}

hipError_t launch_exact_rerank(const ExactArgs& a, hipStream_t s) {
    if (a.nq <= 0) return hipSuccess;
    const size_t lds = exact_lds_bytes(a.D, a.k_short);
    if (a.elem_bytes == 4)
        hipLaunchKernelGGL(exact_rerank_kernel<float>, dim3((unsigned)a.nq), dim3(kExactThreads), lds, s, a);
    else
        hipLaunchKernelGGL(exact_rerank_kernel<uint8_t>, dim3((unsigned)a.nq), dim3(kExactThreads), lds, s, a);
    return hipGetLastError();
}

}  // namespace pqt
