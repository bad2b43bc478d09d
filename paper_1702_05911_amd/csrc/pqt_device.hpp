// Device-side helpers shared by the PQT query kernels (gfx950, 64-lane wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pqt {

constexpr int kWave = 64;

// Order-preserving map float -> uint32 (ascending floats give ascending keys).
// Adding +0.0f first turns -0.0 into +0.0 so that equal floats get equal keys.
__device__ __forceinline__ uint32_t mono_key(float f) {
    const uint32_t u = __float_as_uint(f + 0.0f);
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);   // negative: ~u, else u | sign bit
}
__device__ __forceinline__ float mono_inv(uint32_t k) {
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

// Orders the LDS accesses of ONE wavefront: LDS instructions of a wave execute in program order,
// so only the compiler has to be kept from moving them across this point.
__device__ __forceinline__ void wave_lds_order() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// In-place ascending bitonic sort of n (a power of two) keys in LDS by the `nthreads` threads of
// the workgroup (tid = threadIdx.x; nthreads a power-of-two multiple of 64).  Every thread must
// call it with the same arguments.  Each wavefront owns a contiguous chunk of n / (nthreads/64)
// keys: compare-exchange steps whose stride stays inside a chunk need no workgroup barrier, only
// the steps that cross chunks do.
template <typename K>
__device__ __forceinline__ void bitonic_sort_lds(K* keys, int n, int tid, int nthreads) {
    const int nwaves = nthreads / kWave, wave = tid / kWave, lane = tid & (kWave - 1);
    const int chunk = n / nwaves;                 // 0 or 1 when n is small: every step is a workgroup step
    bool crossed = true;                          // the previous step touched other wavefronts' keys
    for (int size = 2; size <= n; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            if (stride < chunk) {
                if (crossed) __syncthreads(); else wave_lds_order();
                crossed = false;
                for (int e = wave * (chunk >> 1) + lane; e < (wave + 1) * (chunk >> 1); e += kWave) {
                    const int i = 2 * e - (e & (stride - 1));
                    const int j = i + stride;
                    const bool asc = (i & size) == 0;
                    const K x = keys[i], y = keys[j];
                    if ((x > y) == asc) {
                        keys[i] = y;
                        keys[j] = x;
                    }
                }
            } else {
                __syncthreads();
                crossed = true;
                for (int e = tid; e < (n >> 1); e += nthreads) {
                    const int i = 2 * e - (e & (stride - 1));
                    const int j = i + stride;
                    const bool asc = (i & size) == 0;
                    const K x = keys[i], y = keys[j];
                    if ((x > y) == asc) {
                        keys[i] = y;
                        keys[j] = x;
                    }
                }
            }
        }
    }
    __syncthreads();
}

// ---- cross-lane helpers on the data-parallel-primitive path (no LDS traffic) ---------------------
// dpp_ctrl codes: quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E, row_half_mirror = 0x141,
// row_mirror = 0x140, row_bcast15 = 0x142 (lane 15 of a row to the next row), row_bcast31 = 0x143.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_take(uint32_t keep, uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)keep, (int)v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ uint32_t quad_swap1(uint32_t v) { return dpp_take<0xB1, 0xf>(v, v); }   // lane ^ 1
__device__ __forceinline__ uint32_t quad_swap2(uint32_t v) { return dpp_take<0x4E, 0xf>(v, v); }   // lane ^ 2

// Minimum / maximum over the 64 lanes of a wavefront, returned in every lane.
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    v = min(v, dpp_take<0xB1, 0xf>(v, v));
    v = min(v, dpp_take<0x4E, 0xf>(v, v));
    v = min(v, dpp_take<0x141, 0xf>(v, v));
    v = min(v, dpp_take<0x140, 0xf>(v, v));      // every lane of a row holds the row minimum
    v = min(v, dpp_take<0x142, 0xa>(v, v));      // rows 1 and 3 fold in rows 0 and 2
    v = min(v, dpp_take<0x143, 0xc>(v, v));      // rows 2 and 3 fold in rows 0-1: lane 63 has all
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = max(v, dpp_take<0xB1, 0xf>(v, v));
    v = max(v, dpp_take<0x4E, 0xf>(v, v));
    v = max(v, dpp_take<0x141, 0xf>(v, v));
    v = max(v, dpp_take<0x140, 0xf>(v, v));
    v = max(v, dpp_take<0x142, 0xa>(v, v));
    v = max(v, dpp_take<0x143, 0xc>(v, v));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Inclusive prefix sum across the 64 lanes of a wavefront.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v, int lane) {
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t n = __shfl_up(v, off, kWave);
        if (lane >= off) v += n;
    }
    return v;
}

// In a 1024-bin histogram held in LDS, find the bin that holds the item of 1-based rank `need`
// (need <= total count): digit = that bin, before = items in lower bins, count = items in it.
// Read-only and wave-local: every wavefront may call it at the same time and all lanes of all
// callers get the same answer.
__device__ __forceinline__ void hist_locate(const uint32_t* hist, uint32_t need, int lane, uint32_t& digit,
                                            uint32_t& before, uint32_t& count) {
    constexpr int cb = 1024 / kWave;                         // bins per lane
    uint32_t s = 0;
#pragma unroll
    for (int j = 0; j < cb; ++j) s += hist[lane * cb + ((j + lane) & (cb - 1))];   // rotated: no bank conflicts
    const uint32_t incl = wave_inclusive_sum(s, lane);
    uint32_t c = incl - s;
    const bool mine = c < need && need <= incl;              // exactly one lane
    uint32_t d = 0, bf = 0, ct = 0;
    if (mine) {
        int b = lane * cb;
        while (c + hist[b] < need) c += hist[b++];
        d = (uint32_t)b;
        bf = c;
        ct = hist[b];
    }
    const unsigned long long who = __ballot(mine);
    const int owner = who ? __ffsll((long long)who) - 1 : 0;
    digit = (uint32_t)__shfl((int)d, owner, kWave);
    before = (uint32_t)__shfl((int)bf, owner, kWave);
    count = (uint32_t)__shfl((int)ct, owner, kWave);
}

// Ascending bitonic sort of n (a power of two) keys in LDS by the 64 lanes of one wavefront;
// no workgroup barrier, other wavefronts may do anything else meanwhile.
template <typename K>
__device__ __forceinline__ void wave_bitonic_sort_lds(K* keys, int n, int lane) {
    wave_lds_order();
    for (int size = 2; size <= n; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int e = lane; e < (n >> 1); e += kWave) {
                const int i = 2 * e - (e & (stride - 1));
                const int j = i + stride;
                const bool asc = (i & size) == 0;
                const K x = keys[i], y = keys[j];
                if ((x > y) == asc) {
                    keys[i] = y;
                    keys[j] = x;
                }
            }
            wave_lds_order();
        }
    }
}

// Exclusive prefix sum over data[0..n) in LDS, in place, by the whole workgroup.
// part needs blockDim.x + 1 entries.  Returns the total.  Ends with a barrier.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t* data, int n, uint32_t* part) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & (kWave - 1);
    const int chunk = (n + nt - 1) / nt;
    const int lo = min(tid * chunk, n), hi = min(lo + chunk, n);
    uint32_t s = 0;
    for (int e = lo; e < hi; ++e) s += data[e];
    part[tid] = s;
    __syncthreads();
    if (tid < kWave) {                            // the first wavefront scans the per-thread sums
        const int per = nt / kWave;
        uint32_t ls = 0;
        for (int i = 0; i < per; ++i) ls += part[lane * per + i];
        const uint32_t incl = wave_inclusive_sum(ls, lane);
        uint32_t run = incl - ls;
        for (int i = 0; i < per; ++i) {
            const uint32_t v = part[lane * per + i];
            part[lane * per + i] = run;           // exclusive prefix of thread lane*per+i
            run += v;
        }
        if (lane == kWave - 1) part[nt] = incl;   // grand total
    }
    __syncthreads();
    s = part[tid];
    const uint32_t total = part[nt];
    for (int e = lo; e < hi; ++e) {
        const uint32_t v = data[e];
        data[e] = s;
        s += v;
    }
    __syncthreads();
    return total;
}

__host__ __device__ inline int next_pow2(int v) {
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

}  // namespace pqt
