// Tree traversal (Sec. 3.2 "Tree Traversal"): level-1 distances of every query sub-part to
// all k1 centroids (Eq. 6, kept per re-rank sub-part as Sec. 3.3's last paragraph asks),
// the w closest clusters per part, the level-2 distances to their children, and the sorted
// (distance, leaf) lists per part.
//
// One workgroup (256, 512 or 1024 threads for 1, 2 or 4 tree parts) handles a tile of 16 queries.
//   * level 1 is a dense contraction [16 x ds] . [ds x k1] per sub-part on the matrix cores
//     (v_mfma_f32_16x16x4_f32, fp32 in, fp32 accumulate) with ||q||^2 + ||c||^2 - 2 q.c;
//   * the per-part distance is the sum of its sub-part distances in ascending sub-part order;
//   * cluster selection ranks the k1 keys (distance, id) by counting;
//   * level 2 is a gathered set of small matrix-vector products (every query picks its own
//     w clusters), done on the vector ALU with direct squared differences: one wavefront
//     per (query, part), one lane per child;
//   * each list is sorted as 64-bit keys (ordered distance bits, leaf id) by a bitonic
//     network in registers (in LDS for lists of more than 256 entries or part dimensions that
//     are not a multiple of four).
#include "pqt_device.hpp"
#include "pqt_kernels.hpp"

namespace pqt {

typedef float v4f __attribute__((ext_vector_type(4)));

struct TraverseLds {
    int qs;          // row stride of the query tile (floats)
    int k1p;         // k1 rounded up to a multiple of 16
    int Rpad;        // R rounded up to a power of two
    size_t off_q, off_a, off_d1, off_qn, off_sel, off_key, total;
};

// lists_in_lds: the general level-2 path sorts its lists in LDS; the register paths need no room for them
// (16 KB at lists of 128 that would cost the large codebooks a resident workgroup)
__host__ __device__ inline TraverseLds traverse_layout(int D, int P, int k1, int k2, int M, int w, bool lists_in_lds) {
    TraverseLds L;
    L.qs = (D + 4) & ~3;       // rows 16-byte aligned, stride not a multiple of 32 words when D is
    L.k1p = (k1 + 15) & ~15;
    L.Rpad = next_pow2(w * k2);
    size_t o = 0;
    L.off_q = o;   o += sizeof(float) * kQueryTile * L.qs;
    L.off_a = o;   o += sizeof(float) * kQueryTile * M * k1;
    L.off_d1 = o;  o += sizeof(float) * kQueryTile * P * k1;
    L.off_qn = o;  o += sizeof(float) * kQueryTile * M;
    L.off_sel = o; o += sizeof(int) * kQueryTile * P * w;
    o = (o + 7) & ~size_t(7);
    L.off_key = o; o += lists_in_lds ? sizeof(unsigned long long) * (kTraverseMaxThreads / kWave) * L.Rpad : 0;
    L.total = o;
    return L;
}

size_t traverse_lds_bytes(int D, int P, int k1, int k2, int M, int w) {
    return traverse_layout(D, P, k1, k2, M, w, true).total;      // the larger of the two layouts
}

// Level-2 lists of the tile's queries, E list entries per lane (R <= 64 * E), from the interleaved
// codebook.  The distance is the plain sum of squared differences, dimensions in ascending order.
template <int E>
__device__ __forceinline__ void level2_lists(const TraverseArgs& g, int64_t q0, const float* sq, int qs, const int* ssel,
                                             int pbase, int np) {
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int nwaves = (int)blockDim.x / kWave;
    const int P = g.P, k1 = g.k1, k2 = g.k2, w = g.w;
    const int dp = g.D / P, R = w * k2, nd4 = dp / 4;
    const float4* C2t = reinterpret_cast<const float4*>(g.C2t);
    for (int job = wave; job < kQueryTile * np; job += nwaves) {
        const int q = job / np, p = pbase + (job - q * np);
        if (q0 + q >= g.nq) continue;                              // uniform per wavefront
        const float4* yp = reinterpret_cast<const float4*>(sq + q * qs + (p - pbase) * dp);   // 16-byte aligned rows
        unsigned long long key[E];
        const float4* row[E];
        uint32_t leaf[E];
        float acc[E];
#pragma unroll
        for (int r = 0; r < E; ++r) {
            const int e = lane + r * kWave;
            const int ee = e < R ? e : 0;
            const int s = ee / k2, j = ee - s * k2;
            const int i = ssel[(q * P + p) * w + s];
            leaf[r] = (uint32_t)(i * k2 + j);
            row[r] = C2t + ((size_t)p * k1 + i) * nd4 * k2 + j;
            acc[r] = 0.0f;
        }
        if constexpr (E >= 2) {
            // the pieces of four steps are requested together and are operands of one empty statement, which
            // keeps the compiler's scheduler from moving every load down to its use: left alone it waited for
            // each 16-byte piece before it asked for the next, one request in flight per wavefront
            for (int d0 = 0; d0 < nd4; d0 += 4) {
                v4f c[E][4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int r = 0; r < E; ++r)
                        c[r][u] = *reinterpret_cast<const v4f*>(row[r] + (size_t)(d0 + u < nd4 ? d0 + u : nd4 - 1) * k2);
                if constexpr (E == 2)
                    asm volatile("" : "+v"(c[0][0]), "+v"(c[0][1]), "+v"(c[0][2]), "+v"(c[0][3]),
                                      "+v"(c[1][0]), "+v"(c[1][1]), "+v"(c[1][2]), "+v"(c[1][3]));
                else
                    asm volatile("" : "+v"(c[0][0]), "+v"(c[0][1]), "+v"(c[0][2]), "+v"(c[0][3]),
                                      "+v"(c[1][0]), "+v"(c[1][1]), "+v"(c[1][2]), "+v"(c[1][3]),
                                      "+v"(c[2][0]), "+v"(c[2][1]), "+v"(c[2][2]), "+v"(c[2][3]),
                                      "+v"(c[3][0]), "+v"(c[3][1]), "+v"(c[3][2]), "+v"(c[3][3]));
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (d0 + u < nd4) {                                // uniform
                        const float4 y = yp[d0 + u];
#pragma unroll
                        for (int r = 0; r < E; ++r) {
                            float diff = y.x - c[r][u][0];
                            acc[r] = fmaf(diff, diff, acc[r]);
                            diff = y.y - c[r][u][1];
                            acc[r] = fmaf(diff, diff, acc[r]);
                            diff = y.z - c[r][u][2];
                            acc[r] = fmaf(diff, diff, acc[r]);
                            diff = y.w - c[r][u][3];
                            acc[r] = fmaf(diff, diff, acc[r]);
                        }
                    }
                }
            }
        } else {
#pragma unroll 4
            for (int d4 = 0; d4 < nd4; ++d4) {
                const float4 y = yp[d4];
                const float4 c = row[0][(size_t)d4 * k2];
                float diff = y.x - c.x;
                acc[0] = fmaf(diff, diff, acc[0]);
                diff = y.y - c.y;
                acc[0] = fmaf(diff, diff, acc[0]);
                diff = y.z - c.z;
                acc[0] = fmaf(diff, diff, acc[0]);
                diff = y.w - c.w;
                acc[0] = fmaf(diff, diff, acc[0]);
            }
        }
#pragma unroll
        for (int r = 0; r < E; ++r)
            key[r] = (lane + r * kWave < R) ? (((unsigned long long)mono_key(acc[r]) << 32) | leaf[r]) : ~0ull;
        wave_sort_chunk<E>(key, lane, 0u);
        const int64_t gq = q0 + q;
#pragma unroll
        for (int r = 0; r < E; ++r) {
            const int e = lane + r * kWave;
            if (e < R) {
                g.L_d[(gq * P + p) * R + e] = mono_inv((uint32_t)(key[r] >> 32));
                g.L_id[(gq * P + p) * R + e] = (uint32_t)key[r];
            }
        }
    }
}

// E: level-2 list entries per lane on the register path (lists of at most 64 * E entries from the
// interleaved codebook), 0: the general path.  One kernel per E, so that the short-list kernels are not
// held to the register count -- and with it the number of resident tiles -- of the long-list code.
template <int E>
__global__ __launch_bounds__(kTraverseMaxThreads, E == 1 ? 8 : (E == 2 ? 6 : 4)) void traverse_kernel(TraverseArgs g) {
    extern __shared__ __align__(16) unsigned char smem[];
    // A grid with P rows splits every tile by tree part (small batches: see launch_traverse): the workgroup
    // then stages, ranks and lists only part blockIdx.y; nothing in this kernel crosses parts.
    const int np = gridDim.y > 1 ? 1 : g.P;                 // parts this workgroup handles ...
    const int pbase = gridDim.y > 1 ? (int)blockIdx.y : 0;  // ... starting with this one
    const int Dl = np * (g.D / g.P), dbase = pbase * (g.D / g.P);   // the dimensions it stages
    const TraverseLds L = traverse_layout(Dl, g.P, g.k1, g.k2, g.M, g.w, E == 0);
    float* sq = reinterpret_cast<float*>(smem + L.off_q);
    float* sa = reinterpret_cast<float*>(smem + L.off_a);
    float* sd1 = reinterpret_cast<float*>(smem + L.off_d1);
    float* sqn = reinterpret_cast<float*>(smem + L.off_qn);
    int* ssel = reinterpret_cast<int*>(smem + L.off_sel);
    unsigned long long* skey = reinterpret_cast<unsigned long long*>(smem + L.off_key);

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int nthreads = blockDim.x, nwaves = nthreads / kWave;
    const int D = g.D, P = g.P, k1 = g.k1, k2 = g.k2, M = g.M, w = g.w;
    const int dp = D / P, ds = D / M, per = M / P, R = w * k2;
    const int64_t q0 = (int64_t)blockIdx.x * kQueryTile;
    if (g.counters && blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) g.counters[0] = g.counters[1] = 0u;   // used by the bin ranking

    // ---- stage the query tile in LDS (rows past nq are zero) -------------------------------
    for (int e = tid; e < kQueryTile * Dl; e += nthreads) {
        int q = e / Dl, d = e - q * Dl;
        int64_t gq = q0 + q;
        sq[q * L.qs + d] = (gq < g.nq) ? g.queries[gq * D + dbase + d] : 0.0f;
    }
    __syncthreads();
    const int Ml = np * per, mbase = pbase * per;           // the sub-parts of those parts
    for (int e = tid; e < kQueryTile * Ml; e += nthreads) {
        int q = e / Ml, m = mbase + (e - q * Ml);
        const float* row = sq + q * L.qs + (m * ds - dbase);
        float s = 0.0f;
        for (int d = 0; d < ds; ++d) s = fmaf(row[d], row[d], s);
        sqn[q * M + m] = s;
    }
    __syncthreads();

    // ---- level 1 on the matrix cores: one job = (sub-part m, tile of 16 centroids) -------------
    // A operand: lane holds A[row = lane%16][k = lane/16]; B operand: B[k = lane/16][col = lane%16];
    // result: lane holds D[row = 4*(lane/16) + r][col = lane%16] in register r.
    {
        const int ntiles = L.k1p / 16;
        const int row = lane & 15, kq = lane >> 4;
        for (int job = wave; job < Ml * ntiles; job += nwaves) {
            const int m = mbase + job / ntiles, nt = job % ntiles;
            const int p = m / per, lo = m * ds - p * dp;
            const int col = nt * 16 + row;            // centroid this lane feeds as B column
            const float* arow = sq + row * L.qs + (m * ds - dbase);
            const float* brow = g.C1 + ((size_t)p * k1 + (col < k1 ? col : 0)) * dp + lo;
            v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
            // the centroid values of eight k-steps are fetched together, so that their latencies overlap
            for (int k0 = 0; k0 < ds; k0 += 32) {
                float bv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int kd = k0 + 4 * u + kq;
                    bv[u] = (kd < ds && col < k1) ? brow[kd] : 0.0f;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int kd = k0 + 4 * u + kq;
                    if (k0 + 4 * u < ds) {                               // uniform
                        const float av = (kd < ds) ? arow[kd] : 0.0f;
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv[u], acc, 0, 0, 0);
                    }
                }
            }
            if (col < k1) {
                const float cn = g.c1n[m * k1 + col];
                for (int r = 0; r < 4; ++r) {
                    const int q = 4 * kq + r;
                    const float v = (sqn[q * M + m] + cn) - 2.0f * acc[r];
                    sa[(q * M + m) * k1 + col] = v;
                    const int64_t gq = q0 + q;
                    if (gq < g.nq) g.a[(gq * M + m) * k1 + col] = v;
                }
            }
        }
    }
    __syncthreads();

    // ---- per-part distances and the w closest clusters ------------------------------------------
    for (int e = tid; e < kQueryTile * np * k1; e += nthreads) {
        const int i = e % k1, ql = e / k1, p = pbase + ql % np, q = ql / np;
        float s = sa[(q * M + p * per) * k1 + i];
        for (int m = p * per + 1; m < (p + 1) * per; ++m) s += sa[(q * M + m) * k1 + i];
        sd1[(q * P + p) * k1 + i] = s;
    }
    __syncthreads();
    for (int e = tid; e < kQueryTile * np * k1; e += nthreads) {
        const int i = e % k1, ql = e / k1;
        const int qp = (ql / np) * P + pbase + ql % np;
        const float* row = sd1 + qp * k1;
        const unsigned long long me = ((unsigned long long)mono_key(row[i]) << 32) | (unsigned)i;
        int rank = 0;
        for (int j = 0; j < k1; ++j) {
            const unsigned long long other = ((unsigned long long)mono_key(row[j]) << 32) | (unsigned)j;
            rank += (other < me) ? 1 : 0;
        }
        if (rank < w) {
            ssel[qp * w + rank] = i;
            const int64_t gq = q0 + qp / P;
            if (g.sel_tap && gq < g.nq) g.sel_tap[(gq * P + (qp % P)) * w + rank] = i;
        }
    }
    __syncthreads();

    // ---- level 2: one wavefront per (query, part), one lane per child ---------------------------
    if constexpr (E > 0) {
        // children of one cluster interleaved four dimensions at a time (C2t[p][i][d/4][j][4]): the
        // lanes of one cluster read consecutive 16-byte pieces; lists sorted in registers
        level2_lists<E>(g, q0, sq, L.qs, ssel, pbase, np);
        return;
    }
    unsigned long long* mykeys = skey + (size_t)wave * L.Rpad;
    for (int job = wave; job < kQueryTile * np; job += nwaves) {   // same trip count for every wave
        const int q = job / np, p = pbase + (job - q * np);
        const float* yp = sq + q * L.qs + (p - pbase) * dp;
        for (int e = lane; e < L.Rpad; e += kWave) {
            unsigned long long key = ~0ull;
            if (e < R) {
                const int s = e / k2, j = e - s * k2;
                const int i = ssel[(q * P + p) * w + s];
                const float* c = g.C2 + (((size_t)p * k1 + i) * k2 + j) * dp;
                float acc = 0.0f;
                for (int d = 0; d < dp; ++d) {
                    const float diff = yp[d] - c[d];
                    acc = fmaf(diff, diff, acc);
                }
                key = ((unsigned long long)mono_key(acc) << 32) | (unsigned)(i * k2 + j);
            }
            mykeys[e] = key;
        }
        wave_bitonic_sort_lds(mykeys, L.Rpad, lane);
        const int64_t gq = q0 + q;
        if (gq < g.nq) {
            for (int e = lane; e < R; e += kWave) {
                const unsigned long long key = mykeys[e];
                g.L_d[(gq * P + p) * R + e] = mono_inv((uint32_t)(key >> 32));
                g.L_id[(gq * P + p) * R + e] = (uint32_t)key;
            }
        }
        wave_lds_order();
    }
}

// One wavefront per four (query, part) lists of the tile when the batch fills the chip.  A small batch (at
// most one tile per compute unit) gets the largest workgroup and one workgroup per (tile, tree part), so
// that more compute units take part, a wavefront has one list to work through and the call returns
// sooner (1,000 queries of 960 dimensions with four parts: 63 tiles became 252 workgroups).
static bool traverse_small_batch(int64_t nq) { return nq <= 256 * kQueryTile; }
static int traverse_threads(int P, int64_t nq) {
    if (traverse_small_batch(nq)) return kTraverseMaxThreads;
    return P >= 4 ? 1024 : (P == 2 ? 512 : 256);
}

hipError_t launch_traverse(const TraverseArgs& a, hipStream_t s) {
    if (a.nq <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)((a.nq + kQueryTile - 1) / kQueryTile);
    const bool by_part = traverse_small_batch(a.nq) && a.P > 1;
    const dim3 grid(blocks, by_part ? a.P : 1), block(traverse_threads(a.P, a.nq));
    const int R = a.w * a.k2;
    const bool general = a.C2t == nullptr || R > 4 * kWave;
    const size_t lds = traverse_layout(by_part ? a.D / a.P : a.D, a.P, a.k1, a.k2, a.M, a.w, general).total;
    if (general) hipLaunchKernelGGL(traverse_kernel<0>, grid, block, lds, s, a);
    else if (R <= kWave) hipLaunchKernelGGL(traverse_kernel<1>, grid, block, lds, s, a);
    else if (R <= 2 * kWave) hipLaunchKernelGGL(traverse_kernel<2>, grid, block, lds, s, a);
    else hipLaunchKernelGGL(traverse_kernel<4>, grid, block, lds, s, a);
    return hipGetLastError();
}

hipError_t configure_traverse(size_t max_dynamic_lds) {
    const void* kernels[] = {reinterpret_cast<const void*>(traverse_kernel<0>), reinterpret_cast<const void*>(traverse_kernel<1>),
                             reinterpret_cast<const void*>(traverse_kernel<2>), reinterpret_cast<const void*>(traverse_kernel<4>)};
    for (const void* kfn : kernels) {
        const hipError_t e = hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_dynamic_lds);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace pqt
