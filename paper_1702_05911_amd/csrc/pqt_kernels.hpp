// Launch interface of the three query kernels.  Host code fills the argument structs,
// checks sizes against the kernels' limits and calls launch_*; nothing here allocates.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

namespace pqt {

constexpr int kQueryTile = 16;          // queries per workgroup of the traversal kernel (MFMA rows)
constexpr int kTraverseMaxThreads = 1024; // workgroup size grows with the number of tree parts
constexpr int kRankThreads = 1024;        // full ranking pass: one workgroup per query
constexpr int kRankThreadsFourParts = 512;  // the same for four tree parts (up to 4096 tuples)
constexpr int kRankHeadThreads = 256;     // head pass: one wavefront per query
constexpr size_t kMaxLds = 160 * 1024;  // LDS per workgroup on gfx950

// One entry of the folded line-code table: centroid numbers i | j<<8, lambda, and
// (lambda^2 - lambda) ||c_i - c_j||^2 of the sub-part (the pair table of Sec. 3.3 gathered per
// code value; Eq. 9 reads b^2 + lambda (a^2 - b^2) + that constant).
struct CodeEntry {
    uint32_t ij;
    float lam;
    float kc;
};

struct TraverseArgs {
    const float* queries;   // nq x D
    int64_t nq;
    int D, P, k1, k2, M, w;
    const float* C1;        // P x k1 x dp
    const float* c1n;       // M x k1   squared norms of the centroid sub-parts
    const float* C2;        // P x k1 x k2 x dp
    const float* C2t;       // the same, children interleaved: P x k1 x dp/4 x k2 x 4 (null unless dp % 4 == 0)
    float* a;               // nq x M x k1
    float* L_d;             // nq x P x R
    uint32_t* L_id;         // nq x P x R
    int32_t* sel_tap;       // nq x P x w or null
    uint32_t* counters;     // [0], [1]: the bin ranking's query counters, reset here (null: nothing to reset)
};
size_t traverse_lds_bytes(int D, int P, int k1, int k2, int M, int w);
hipError_t launch_traverse(const TraverseArgs& a, hipStream_t s);

struct RankArgs {
    int64_t nq;
    int P, R, T, C;
    uint32_t k1k2;
    uint64_t H;
    uint64_t H_inv;           // floor(2^64 / H) for H >= 2 (slot_of_bin divides by multiplying), else 0
    int hashed;               // H != (k1*k2)^P: slots may repeat within a query
    const uint32_t* offsets;  // H+1
    const float* L_d;
    const uint32_t* L_id;
    uint2* runs;              // nq x T   (.x = first position in ids/codes, .y = start in candidate list)
    uint2* meta;              // nq       (.x = number of runs, .y = number of candidates; or .x = kMetaTodo:
                              //           the head pass left the query to the full pass, .y = its place in order[])
    uint32_t* counters;       // [0] = number of queries the head pass left to the full pass
    uint32_t* order;          // nq: those queries
    // taps (nullable)
    uint32_t* n_tuples;
    uint16_t* tuples;         // nq x T x 4
    float* tuple_keys;        // nq x T
    uint64_t* slots;          // nq x T
};
constexpr uint32_t kMetaTodo = 0xffffffffu;

struct RankOffsets {   // LDS layout of the full ranking pass (computed once on the host)
    int Tcap, cap, npair, nreg, nreg_pair, Tmid, nreg_mid;
    int force;             // 1: rank every query (taps wanted, or no head pass ran)
    uint32_t keys, hist, Ld, Lid, ps, pt, len, slot, part, misc;
    uint32_t total;        // bytes
};
// number of (r1, r2) pairs that can be among the first T of an R x R sum table
int rank_region_size(int R, int T);
// LDS of the stand-alone ranking kernel / layout of a ranking (place: with the room the stand-alone kernels
// use for placing keys by bin; without: the ranking inside the re-rank kernel)
size_t rank_lds_bytes(int P, int R, int T, int hashed);
RankOffsets rank_offsets(int P, int R, int T, int hashed, bool place);
// does a head pass exist for these arguments (two tree parts, no taps of the ranking)?
bool rank_has_head(const RankArgs& a);
// defer_full: only the head pass is launched; the caller runs the full pass of the unfinished
// queries elsewhere (inside the re-rank kernel).  Needs rank_has_head(a).
hipError_t launch_rank(const RankArgs& a, hipStream_t s, bool defer_full);

// The fixed anisotropic traversal order (Sec. 3.2 "Bin Proposal Heuristic"): ten pre-computed orders of
// the rank pairs, one per slope 1.08^k, k = -5..4; a query takes the one whose slope matches how fast
// its two lists rise.  Two tree parts, unhashed bins.
constexpr int kStaticSlopes = 10;
struct StaticOrder {
    const uint32_t* table;     // kStaticSlopes x Tn entries r1 << 16 | r2 (device)
    int Tn;                    // min(T, R^2)
    float thr[kStaticSlopes - 1];   // 1.08^(j - 5.5), j = 1..9: boundaries between neighbouring slopes
};
// host: the tables for lists of R entries and T tuples; returns Tn
int make_static_order(int R, int T, std::vector<uint32_t>& table, float thr[kStaticSlopes - 1]);
hipError_t launch_rank_static(const RankArgs& a, const StaticOrder& so, hipStream_t s);

struct RerankArgs {
    int64_t nq;
    int M, k1, T, C, k;
    int threads;              // workgroup size (multiple of 64)
    int keys_per_thread;      // candidates a thread scores; both from rerank_shape
    const float* a;           // nq x M x k1
    const CodeEntry* table;   // M x 256
    int code_format;          // 0: codes are entries of the table, one byte per sub-part;
                              // 1: two bytes per sub-part, (centroid pair, lambda level); the table is then
                              //    indexed by pair number and its kc field holds ||c_i - c_j||^2
    int pair_shift;           // code format 1: log2 of the LDS table's entries per sub-part (set by launch_rerank)
    int runs_in_lds;          // runs of a query the workgroup keeps in LDS (at least 64, at most T); a longer list
                              // is read from memory past that.  Sized from the index's mean run length so that
                              // the common case fits without spending LDS (and thus resident queries) on it.
    const uint2* runs;
    const uint2* meta;
    const uint32_t* ids;
    const uint8_t* codes;     // N x M (N x 2M for code format 1)
    // Queries the ranking head pass left unfinished take longest, so they go first: the first
    // `early` workgroups take entries of todo[0 .. *todo_count) (the rest of them exit at once), then
    // workgroup early + q takes query q unless one of the first did.  early = 0: workgroup q, query q.
    const uint32_t* todo;
    const uint32_t* todo_count;
    int early;
    // set by launch_rerank when the kernel ranks left-over queries: their first wavefront tries this many
    // tuples (the pairs of the head-pass table up to mid_npairs) before the workgroup ranks in full
    int mid_T1 = 0, mid_npairs = 0;
    int64_t* out_ids;         // nq x k
    float* out_dists;         // nq x k
    // taps (nullable)
    uint32_t* n_cand;
    int64_t* cand_ids;        // nq x C
    float* scores;            // nq x C
    float* lut;               // nq x M x 256
};
// rank_lds: LDS bytes of the full ranking pass when the kernel also runs it (0: it does not)
size_t rerank_lds_bytes(int M, int k1, int T, int C, int k, int threads, size_t rank_lds, int code_format,
                        int runs_in_lds);
// tuples per thread the in-kernel ranking can hold: fusing needs min(T, R^2) <= that * threads
int rerank_fused_tuples_per_thread();
// workgroup size and candidates per thread of the re-rank kernel for a candidate budget C
// (C <= threads * keys_per_thread; the fewest threads that hold the budget)
void rerank_shape(int C, int M, int code_format, int* threads, int* keys_per_thread);
// fused: the full ranking pass of the queries whose meta.x is kMetaTodo runs inside the kernel
hipError_t launch_rerank(const RerankArgs& a, const RankArgs* fused, hipStream_t s);

struct ExactArgs {
    int64_t nq;
    int D, k_short, k;
    int elem_bytes;            // 4: fp32 vectors, 1: uint8 vectors
    const float* queries;      // nq x D
    const void* vectors;       // N x D, row id = database id
    const int64_t* short_ids;  // nq x k_short, -1 = no entry
    int64_t* out_ids;          // nq x k
    float* out_dists;          // nq x k
};
size_t exact_lds_bytes(int D, int k_short);
hipError_t launch_exact_rerank(const ExactArgs& a, hipStream_t s);

struct BruteArgs {
    int64_t nq;
    int D, k;
    int elem_bytes;               // 4: fp32 vectors, 1: uint8 vectors
    int64_t chunk;                // database vectors per pass = row stride of dist
    const float* queries;         // nq x D
    const void* vectors;          // N x D
    const float* qnorm;           // nq
    const float* xnorm;           // N
    float* dist;                  // nq x chunk
    unsigned long long* best;     // nq x k running result between passes
    int64_t* out_ids;             // nq x k
    float* out_dists;             // nq x k
};
hipError_t launch_row_norms(const void* x, int elem_bytes, int64_t n, int D, float* out, hipStream_t s);
size_t brute_select_lds_bytes(int k);
// distances of all queries to database vectors x0 .. x0+nx-1, then the running k best
hipError_t launch_brute_chunk(const BruteArgs& a, int64_t x0, int64_t nx, bool first, bool last, hipStream_t s);

// raise the dynamic-LDS ceiling of each kernel (once per device)
hipError_t configure_traverse(size_t max_dynamic_lds);
hipError_t configure_rank(size_t max_dynamic_lds);
hipError_t configure_rerank(size_t max_dynamic_lds);

}  // namespace pqt
