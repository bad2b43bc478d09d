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

// Inclusive prefix sum across the 64 lanes of a wavefront (all lanes must be active): shifts inside
// each row of 16 lanes, then the totals of rows 0 and 2 into rows 1 and 3, then the total of the
// first 32 lanes into the last 32.  dpp_ctrl row_shr:n = 0x110 + n; lanes without a source add 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v, int lane) {
    (void)lane;
    v += dpp_or_zero<0x111, 0xf>(v);
    v += dpp_or_zero<0x112, 0xf>(v);
    v += dpp_or_zero<0x114, 0xf>(v);
    v += dpp_or_zero<0x118, 0xf>(v);
    v += dpp_or_zero<0x142, 0xa>(v);
    v += dpp_or_zero<0x143, 0xc>(v);
    return v;
}

// Exclusive prefix of v over the threads of the workgroup in thread order; total = sum over all
// threads.  part: one word of LDS per wavefront.  One barrier inside; every thread must call it.
// part may be written again only after a later barrier.
__device__ __forceinline__ uint32_t block_exclusive_sum(uint32_t v, uint32_t* part, uint32_t& total) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave, nw = blockDim.x / kWave;
    const uint32_t incl = wave_inclusive_sum(v, lane);
    if (lane == kWave - 1) part[wave] = incl;
    __syncthreads();
    const uint32_t p = lane < nw ? part[lane] : 0u;
    const uint32_t pin = wave_inclusive_sum(p, lane);
    const uint32_t base = (uint32_t)__shfl((int)(pin - p), wave, kWave);
    total = (uint32_t)__shfl((int)pin, nw - 1, kWave);
    return base + incl - v;
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

// ---- bitonic sorting of 64-bit keys held in registers ---------------------------------------------
// A wavefront holds a chunk of 64*E keys, E per lane: element r*64 + lane of the chunk is k[r] of
// that lane.  The chunk is elements gbase .. gbase + 64*E - 1 of a longer sequence (gbase a
// multiple of 64*E, wave-uniform), whose bitonic network decides every direction: at merge level
// `size` the block containing element g ascends iff (g & size) == 0.  Compare-exchange steps with a
// stride below 64 exchange keys between lanes (DPP for strides 1 and 2, ds_swizzle for 4..16,
// ds_bpermute for 32: no LDS memory is touched); larger strides exchange registers of one lane.
// Equal keys are only ever padding, for which either choice is the same.

// lanes l of a wavefront with (l & bit) == 0, as a mask
__host__ __device__ constexpr unsigned long long lanes_with_bit_clear(int bit) {
    unsigned long long m = 0;
    for (int l = 0; l < 64; ++l)
        if ((l & bit) == 0) m |= 1ull << l;
    return m;
}

template <int STRIDE>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v, int lane) {
    if constexpr (STRIDE == 1) return dpp_take<0xB1, 0xf>(v, v);
    else if constexpr (STRIDE == 2) return dpp_take<0x4E, 0xf>(v, v);
    else if constexpr (STRIDE < 32) return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, (STRIDE << 10) | 0x1f);
    else return (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, (int)v);
}

// One compare-exchange step with partner lane ^ STRIDE; keep_min[r]: lanes that keep the smaller key.
template <int E, int STRIDE>
__device__ __forceinline__ void xlane_step(unsigned long long (&k)[E], int lane, const unsigned long long (&keep_min)[E]) {
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const uint32_t ohi = lane_xor<STRIDE>((uint32_t)(k[r] >> 32), lane);
        const uint32_t olo = lane_xor<STRIDE>((uint32_t)k[r], lane);
        const unsigned long long o = ((unsigned long long)ohi << 32) | olo;
        const bool km = __builtin_amdgcn_inverse_ballot_w64(keep_min[r]);
        k[r] = ((o < k[r]) == km) ? o : k[r];
    }
}

// Strides STRIDE, STRIDE/2, .., 1 of the merge level SIZE <= 32 (directions depend on lane bits only).
template <int E, int SIZE, int STRIDE>
__device__ __forceinline__ void merge_small(unsigned long long (&k)[E], int lane) {
    constexpr unsigned long long km = ~(lanes_with_bit_clear(STRIDE) ^ lanes_with_bit_clear(SIZE));
    unsigned long long keep[E];
#pragma unroll
    for (int r = 0; r < E; ++r) keep[r] = km;
    xlane_step<E, STRIDE>(k, lane, keep);
    if constexpr (STRIDE > 1) merge_small<E, SIZE, STRIDE / 2>(k, lane);
}

// Strides STRIDE, .., 1 (STRIDE < 64*E) of a merge level size >= 64: the direction is uniform per register.
template <int E, int STRIDE>
__device__ __forceinline__ void merge_large(unsigned long long (&k)[E], int lane, uint32_t gbase, uint32_t size) {
    if constexpr (STRIDE >= 64) {
        constexpr int dr = STRIDE / 64;
#pragma unroll
        for (int r = 0; r < E; ++r) {
            if ((r & dr) != 0) continue;
            const bool asc = ((gbase + (uint32_t)r * 64u) & size) == 0;
            const unsigned long long x = k[r], y = k[r + dr];
            const bool swap = (x > y) == asc;
            k[r] = swap ? y : x;
            k[r + dr] = swap ? x : y;
        }
    } else {
        constexpr unsigned long long lower = lanes_with_bit_clear(STRIDE);
        unsigned long long keep[E];
#pragma unroll
        for (int r = 0; r < E; ++r) keep[r] = (((gbase + (uint32_t)r * 64u) & size) == 0) ? lower : ~lower;
        xlane_step<E, STRIDE>(k, lane, keep);
    }
    if constexpr (STRIDE > 1) merge_large<E, STRIDE / 2>(k, lane, gbase, size);
}

template <int E, int SIZE>
__device__ __forceinline__ void sort_levels_large(unsigned long long (&k)[E], int lane, uint32_t gbase) {
    if constexpr (SIZE <= 64 * E) {
        merge_large<E, SIZE / 2>(k, lane, gbase, (uint32_t)SIZE);
        sort_levels_large<E, SIZE * 2>(k, lane, gbase);
    }
}

// Sorts the chunk (all merge levels 2 .. 64*E); gbase must be wave-uniform.
template <int E>
__device__ __forceinline__ void wave_sort_chunk(unsigned long long (&k)[E], int lane, uint32_t gbase) {
    merge_small<E, 2, 1>(k, lane);
    merge_small<E, 4, 2>(k, lane);
    merge_small<E, 8, 4>(k, lane);
    merge_small<E, 16, 8>(k, lane);
    merge_small<E, 32, 16>(k, lane);
    sort_levels_large<E, 64>(k, lane, gbase);
}

// The strides below 64*E of merge level `size` (>= 128*E): finishes a merge whose longer strides
// were done through LDS.
template <int E>
__device__ __forceinline__ void wave_merge_chunk(unsigned long long (&k)[E], int lane, uint32_t gbase, uint32_t size) {
    merge_large<E, 32 * E>(k, lane, gbase, size);
}

// Ascending sort of n keys in LDS (n a power of two, 64 <= n <= 64 * E * number of wavefronts) by the
// whole workgroup: every wavefront sorts a chunk of 64*E keys in registers; merge levels beyond a
// chunk do their long strides in LDS (one barrier each) and their short strides in registers again.
template <int E>
__device__ __forceinline__ void block_sort_chunks(unsigned long long* keys, int n, int tid, int nthreads) {
    constexpr int chunk = 64 * E;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const bool active = wave * chunk < n;
    const uint32_t gbase = (uint32_t)(wave * chunk);
    unsigned long long k[E];
    __syncthreads();
    if (active) {
#pragma unroll
        for (int r = 0; r < E; ++r) k[r] = keys[gbase + r * 64 + lane];
        wave_sort_chunk<E>(k, lane, gbase);
#pragma unroll
        for (int r = 0; r < E; ++r) keys[gbase + r * 64 + lane] = k[r];
    }
    __syncthreads();
    for (int size = 2 * chunk; size <= n; size <<= 1) {
        for (int stride = size >> 1; stride >= chunk; stride >>= 1) {
            for (int e = tid; e < (n >> 1); e += nthreads) {
                const int i = 2 * e - (e & (stride - 1));
                const int j = i + stride;
                const bool asc = (i & size) == 0;
                const unsigned long long x = keys[i], y = keys[j];
                if ((x > y) == asc) {
                    keys[i] = y;
                    keys[j] = x;
                }
            }
            __syncthreads();
        }
        if (active) {
#pragma unroll
            for (int r = 0; r < E; ++r) k[r] = keys[gbase + r * 64 + lane];
            wave_merge_chunk<E>(k, lane, gbase, (uint32_t)size);
#pragma unroll
            for (int r = 0; r < E; ++r) keys[gbase + r * 64 + lane] = k[r];
        }
        __syncthreads();
    }
}

// Ascending sort of n (a power of two) keys in LDS by the workgroup; every thread calls it with the
// same arguments; nthreads a power-of-two multiple of 64 with n <= MAXE * nthreads (MAXE = 2, 4 or 8
// keys per thread at most: fewer keeps the register count of the calling kernel down).  Ends with a barrier.
template <int MAXE = 8>
__device__ __forceinline__ void block_sort_lds(unsigned long long* keys, int n, int tid, int nthreads) {
    if (n < 64) {
        __syncthreads();
        bitonic_sort_lds(keys, n, tid, nthreads);
        return;
    }
    const int per = n / nthreads;
    if (per <= 1) block_sort_chunks<1>(keys, n, tid, nthreads);
    else if (per == 2 || MAXE == 2) block_sort_chunks<2>(keys, n, tid, nthreads);
    else if (per == 4 || MAXE == 4) block_sort_chunks<4>(keys, n, tid, nthreads);
    else block_sort_chunks<8>(keys, n, tid, nthreads);
}

// bin mod H (Sec. 4: the bin number is hashed into the pointer array) without a 64-bit division:
// q' = floor(bin * floor(2^64 / H) / 2^64) is the quotient or one less, so one conditional subtraction
// gives the exact remainder.  H_inv = 0 stands for H = 1.
__device__ __forceinline__ unsigned long long slot_of_bin(unsigned long long bin, unsigned long long H,
                                                          unsigned long long H_inv) {
    if (H_inv == 0) return 0;
    unsigned long long r = bin - __umul64hi(bin, H_inv) * H;
    return r >= H ? r - H : r;
}

__host__ __device__ inline int next_pow2(int v) {
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

}  // namespace pqt
