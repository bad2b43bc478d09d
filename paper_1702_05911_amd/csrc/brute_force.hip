// Exact nearest neighbours by brute force (Eq. 1; the paper's "strong baseline" of Table 1): the
// squared distances of every query to every database vector, and per query the k smallest by
// (distance, id).  Doubles as the ground truth for recall.
//
// The database is walked in chunks.  Per chunk
//   * bf_distance_kernel: a dense contraction on the matrix cores.  A workgroup of 256 threads computes
//     a 128 x 128 tile of q.x with v_mfma_f32_16x16x4_f32 (fp32 in, fp32 accumulate), each wavefront a
//     64 x 64 quarter as 4 x 4 MFMA tiles; operands are staged through LDS sixteen dimensions at a
//     time (byte vectors are widened while staging; the next step's pieces are fetched during the MFMAs); the epilogue forms ||q||^2 + ||x||^2 - 2 q.x.
//   * bf_select_kernel: one workgroup per query scans its row of distances once (16 bytes per thread
//     and step), keeps what beats the k-th best so far in an LDS buffer, and re-selects the k best
//     whenever the buffer may fill.  Chunks
//     arrive in id order, so an equal distance that arrives later has the larger id and never wins.
#include "pqt_device.hpp"
#include "pqt_kernels.hpp"

namespace pqt {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kBfTile = 128;       // queries and database vectors per workgroup tile
constexpr int kBfKc = 16;          // dimensions staged per step
constexpr int kBfThreads = 256;
constexpr int kBfLdsStride = kBfKc + 1;

// squared norms of n rows of D elements
template <typename Elem>
__global__ void row_norms_kernel(const Elem* x, int64_t n, int D, float* out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const Elem* row = x + (size_t)i * D;
    float s = 0.0f;
    for (int d = 0; d < D; ++d) {
        const float v = (float)row[d];
        s = fmaf(v, v, s);
    }
    out[i] = s;
}

// Eight consecutive elements of a row as floats (one 8- or 32-byte piece when the row allows it).
__device__ __forceinline__ void load8(const float* p, bool aligned, float (&v)[8]) {
    if (aligned) {
        const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] = p[c];
    }
}
__device__ __forceinline__ void load8(const uint8_t* p, bool aligned, float (&v)[8]) {
    if (aligned) {
        const uint2 w = *reinterpret_cast<const uint2*>(p);
        v[0] = (float)(w.x & 0xffu); v[1] = (float)((w.x >> 8) & 0xffu); v[2] = (float)((w.x >> 16) & 0xffu); v[3] = (float)(w.x >> 24);
        v[4] = (float)(w.y & 0xffu); v[5] = (float)((w.y >> 8) & 0xffu); v[6] = (float)((w.y >> 16) & 0xffu); v[7] = (float)(w.y >> 24);
    } else {
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] = (float)p[c];
    }
}

// A thread's piece of a 128-row x 16-dimension tile: row t/2, dimensions (t%2)*8 .. +8 of step k0, as
// floats in registers; rows past nrows and dimensions past D are zero.
template <typename Elem>
__device__ __forceinline__ void fetch_piece(const Elem* base, int64_t row0, int64_t nrows, int D, int k0, int tid, float (&v)[8]) {
    const int r = tid >> 1, c0 = (tid & 1) * 8;
    const int64_t row = row0 + r;
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] = 0.0f;
    if (row < nrows) {
        const Elem* p = base + (size_t)row * D + k0 + c0;
        if (k0 + c0 + 8 <= D) {
            load8(p, D % 8 == 0, v);                  // pieces are aligned when every row is a whole number of them
        } else {
            for (int c = 0; c < 8 && k0 + c0 + c < D; ++c) v[c] = (float)p[c];
        }
    }
}
__device__ __forceinline__ void store_piece(const float (&v)[8], float* dst, int tid) {
    const int r = tid >> 1, c0 = (tid & 1) * 8;
#pragma unroll
    for (int c = 0; c < 8; ++c) dst[r * kBfLdsStride + c0 + c] = v[c];
}

template <typename Elem>
__global__ __launch_bounds__(kBfThreads) void bf_distance_kernel(BruteArgs g, int64_t x0, int64_t nx) {
    __shared__ float As[kBfTile * kBfLdsStride];
    __shared__ float Bs[kBfTile * kBfLdsStride];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t q0 = (int64_t)blockIdx.y * kBfTile;          // first query of the tile
    const int64_t c0 = (int64_t)blockIdx.x * kBfTile;          // first database vector of the tile, within the chunk
    const Elem* X = reinterpret_cast<const Elem*>(g.vectors) + (size_t)x0 * g.D;
    const int wr = (wave >> 1) * 64, wc = (wave & 1) * 64;    // this wavefront's quarter
    const int row = lane & 15, kq = lane >> 4;
    v4f acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    // the pieces of the next step are fetched into registers while the matrix cores work on this one
    float pa[8], pb[8];
    fetch_piece<float>(g.queries, q0, g.nq, g.D, 0, tid, pa);
    fetch_piece<Elem>(X, c0, nx, g.D, 0, tid, pb);
    for (int k0 = 0; k0 < g.D; k0 += kBfKc) {
        __syncthreads();                                        // the tiles of the step before are no longer read
        store_piece(pa, As, tid);
        store_piece(pb, Bs, tid);
        __syncthreads();
        if (k0 + kBfKc < g.D) {
            fetch_piece<float>(g.queries, q0, g.nq, g.D, k0 + kBfKc, tid, pa);
            fetch_piece<Elem>(X, c0, nx, g.D, k0 + kBfKc, tid, pb);
        }
#pragma unroll
        for (int kk = 0; kk < kBfKc; kk += 4) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[(wr + i * 16 + row) * kBfLdsStride + kk + kq];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[(wc + j * 16 + row) * kBfLdsStride + kk + kq];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }
    // D[row = 4*(lane/16) + r][col = lane%16] of every 16 x 16 tile
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = c0 + wc + j * 16 + row;
            if (col >= nx) continue;
            const float xn = g.xnorm[x0 + col];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t q = q0 + wr + i * 16 + 4 * kq + r;
                if (q < g.nq) g.dist[(size_t)q * g.chunk + col] = (g.qnorm[q] + xn) - 2.0f * acc[i][j][r];
            }
        }
}

constexpr int kBfSelThreads = 512;
constexpr int kBfBuf = 3840;       // pending entries the LDS buffer holds besides the k best (k <= 256:
                                   // together at most 4096 keys, eight per thread of the sort)

// best: nq x k keys (ordered distance bits << 32 | id), ascending, ~0 = none yet
__global__ __launch_bounds__(kBfSelThreads) void bf_select_kernel(BruteArgs g, int64_t x0, int64_t nx, int first, int last) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem);       // next_pow2(k + kBfBuf)
    uint32_t* counter = reinterpret_cast<uint32_t*>(keys + next_pow2(g.k + kBfBuf));
    const int tid = threadIdx.x, lane = tid & (kWave - 1), k = g.k;
    const int64_t q = blockIdx.x;
    const float* row = g.dist + (size_t)q * g.chunk;
    for (int e = tid; e < k; e += kBfSelThreads) keys[e] = first ? ~0ull : g.best[(size_t)q * k + e];
    if (tid == 0) counter[0] = 0;
    __syncthreads();
    uint32_t tau = (uint32_t)(keys[k - 1] >> 32);             // distance bits of the k-th best (all ones: none)
    auto reselect = [&](uint32_t pending) {                     // keep the k smallest of the k best and the pending entries
        const int n = k + (int)pending, npad = next_pow2(n) < 64 ? 64 : next_pow2(n);
        for (int e = n + tid; e < npad; e += kBfSelThreads) keys[e] = ~0ull;
        block_sort_lds<8>(keys, npad, tid, kBfSelThreads);
        tau = (uint32_t)(keys[k - 1] >> 32);
        if (tid == 0) counter[0] = 0;
        __syncthreads();
    };
    if (g.chunk % 4 == 0) {
        // rows are 16-byte aligned: four distances per thread and step, the next piece in flight while this
        // one is examined; one barrier per 2048 distances
        const float4* row4 = reinterpret_cast<const float4*>(row);
        const int64_t n4 = (nx + 3) / 4;                       // a last partial piece stays inside the row
        float4 next = tid < n4 ? row4[tid] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        for (int64_t b4 = 0; b4 < n4; b4 += kBfSelThreads) {
            const int64_t i4 = b4 + tid;
            const float4 v = next;
            if (i4 + kBfSelThreads < n4) next = row4[i4 + kBfSelThreads];
            const float vals[4] = {v.x, v.y, v.z, v.w};
            uint32_t kb[4], cnt = 0;
            bool tk[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                kb[c] = mono_key(vals[c]);
                tk[c] = i4 < n4 && i4 * 4 + c < nx && kb[c] < tau;
                cnt += tk[c] ? 1u : 0u;
            }
            const uint32_t incl = wave_inclusive_sum(cnt, lane);
            const uint32_t total = (uint32_t)__shfl((int)incl, kWave - 1, kWave);
            if (total) {                                        // same for the whole wavefront
                uint32_t at = 0;
                if (lane == kWave - 1) at = atomicAdd(counter, total);
                at = (uint32_t)__shfl((int)at, kWave - 1, kWave) + incl - cnt;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (tk[c]) keys[k + at++] = ((unsigned long long)kb[c] << 32) | (uint32_t)(x0 + i4 * 4 + c);
            }
            __syncthreads();
            const uint32_t pending = counter[0];
            if (pending + 4 * kBfSelThreads > (uint32_t)kBfBuf || b4 + kBfSelThreads >= n4) reselect(pending);
        }
    } else
    for (int64_t base = 0; base < nx; base += kBfSelThreads) {
        const int64_t c = base + tid;
        bool take = false;
        unsigned long long key = 0;
        if (c < nx) {
            const uint32_t kb = mono_key(row[c]);
            take = kb < tau;
            key = ((unsigned long long)kb << 32) | (uint32_t)(x0 + c);
        }
        const unsigned long long m = __ballot(take);
        if (take) {
            const int leader = __ffsll((long long)m) - 1;
            uint32_t at = 0;
            if (lane == leader) at = atomicAdd(counter, (uint32_t)__popcll(m));
            at = (uint32_t)__shfl((int)at, leader, kWave);
            keys[k + at + (uint32_t)__popcll(m & ((1ull << lane) - 1ull))] = key;
        }
        __syncthreads();
        const uint32_t pending = counter[0];
        if (pending + kBfSelThreads > (uint32_t)kBfBuf || base + kBfSelThreads >= nx) reselect(pending);
    }
    if (last) {
        for (int e = tid; e < k; e += kBfSelThreads) {
            const unsigned long long key = keys[e];
            g.out_ids[(size_t)q * k + e] = key == ~0ull ? -1 : (int64_t)(uint32_t)key;
            g.out_dists[(size_t)q * k + e] = key == ~0ull ? __builtin_inff() : mono_inv((uint32_t)(key >> 32));
        }
    } else {
        for (int e = tid; e < k; e += kBfSelThreads) g.best[(size_t)q * k + e] = keys[e];
    }
}

hipError_t launch_row_norms(const void* x, int elem_bytes, int64_t n, int D, float* out, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    const unsigned tb = 256, nb = (unsigned)((n + tb - 1) / tb);
    if (elem_bytes == 4) hipLaunchKernelGGL(row_norms_kernel<float>, dim3(nb), dim3(tb), 0, s, static_cast<const float*>(x), n, D, out);
    else hipLaunchKernelGGL(row_norms_kernel<uint8_t>, dim3(nb), dim3(tb), 0, s, static_cast<const uint8_t*>(x), n, D, out);
    return hipGetLastError();
}

size_t brute_select_lds_bytes(int k) { return sizeof(unsigned long long) * next_pow2(k + kBfBuf) + 16; }

hipError_t launch_brute_chunk(const BruteArgs& a, int64_t x0, int64_t nx, bool first, bool last, hipStream_t s) {
    const dim3 grid((unsigned)((nx + kBfTile - 1) / kBfTile), (unsigned)((a.nq + kBfTile - 1) / kBfTile));
    if (a.elem_bytes == 4) hipLaunchKernelGGL(bf_distance_kernel<float>, grid, dim3(kBfThreads), 0, s, a, x0, nx);
    else hipLaunchKernelGGL(bf_distance_kernel<uint8_t>, grid, dim3(kBfThreads), 0, s, a, x0, nx);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bf_select_kernel, dim3((unsigned)a.nq), dim3(kBfSelThreads), brute_select_lds_bytes(a.k), s, a, x0, nx,
                       first ? 1 : 0, last ? 1 : 0);
    return hipGetLastError();
}

}  // namespace pqt
