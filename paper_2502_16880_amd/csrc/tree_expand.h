// One level of draft-tree expansion (sections 2.1 and 4.1: tree drafting with several
// candidates per node and a fixed number of nodes kept per level): the score of candidate i
// of node m is the node's cumulative log-probability plus the candidate's, and the n_next
// best scores of all M*k candidates become the next level.  The candidate lists arrive
// sorted (the head's top-k output), so a candidate's global rank is the sum over the M lists
// of a binary search; a candidate at position i >= n_next of its own list cannot be kept and
// is skipped.  One wave per node: it ranks its own node's candidates against a table of the
// keys of all M*k <= 4096 candidates in LDS.  The stand-alone kernel gives every node a
// workgroup of one wave that builds the whole table itself (32 KB at most; cheaper than a
// hand-over between workgroups); the single-launch head's log-probability mode calls the
// same ranking from the workgroup that has just written the lists.  Latency-bound by
// construction: it is here so that a draft level needs no host round trip, not for bandwidth.
#pragma once
#include "device_utils.h"

namespace {

constexpr int kTreeMaxCand = kMaxM * kMaxK;      // 4096

// Key of candidate e = m*k + i of the table: equal scores rank by lower node, then lower
// position, which is the lower flat index; an empty slot has key 0.
__device__ __forceinline__ unsigned long long tree_key(float parent, float logp, int id, int e) {
    return id >= 0 ? cand_key(parent + logp, e) : 0ull;
}

// Ranks node m's candidates among all M*k of the key table (list l at keys[l*k .. l*k + k),
// descending).  Lane = (candidate i of this node, part): only the first min(k, n_next)
// candidates of a list can be kept (n_next of its own list beat a later one), so when those
// are fewer than 64 the lists are split over 64 / C lanes per candidate and the partial
// ranks added.  Returns the rank (the number of candidates above) of candidate e_out, with
// keep = this lane writes it (first part, a real candidate, rank < n_next).
__device__ __forceinline__ int tree_rank_node(const unsigned long long* keys, int M, int k, int n_next,
                                              int m, int lane, int& e_out, bool& keep) {
    const int cmax = k < n_next ? k : n_next;
    int C = 1;                                             // power of two >= cmax, <= 64
    while (C < cmax) C *= 2;
    const int lpc = kWave / C;
    const int i = lane & (C - 1), part = lane / C;
    int top = 1;                                           // largest power of two <= k
    while (top * 2 <= k) top *= 2;
    const int e = m * k + (i < cmax ? i : 0);
    const unsigned long long key = i < cmax ? keys[e] : 0ull;
    // entries of list l above key = first position of the (descending) list whose key is not
    // above it: branchless binary search, four lists at a time so that their LDS reads overlap
    int rank = 0;
    for (int l0 = part; l0 < M; l0 += 4 * lpc) {           // (lanes of one part run the same trips)
        int pos[4] = {0, 0, 0, 0};
        const unsigned long long* L[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) L[u] = keys + (l0 + u * lpc < M ? l0 + u * lpc : M - 1) * k - 1;
        for (int step = top; step >= 1; step >>= 1) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int at = pos[u] + step;
                if (at <= k && L[u][at] > key) pos[u] = at;
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) rank += l0 + u * lpc < M ? pos[u] : 0;
    }
    for (int off = C; off < kWave; off <<= 1) rank += __shfl_xor(rank, off);   // wave-uniform trips
    e_out = e;
    keep = part == 0 && key != 0ull && rank < n_next;
    return rank;
}

// Slots of the next level beyond the number of real candidates: (-1, -1, -inf).
__device__ __forceinline__ void tree_pad(int n_real, int n_next, int lane, int32_t* next_parent,
                                         int32_t* next_token, float* next_score) {
    const int filled = n_real < n_next ? n_real : n_next;
    for (int r = filled + lane; r < n_next; r += kWave) {
        next_parent[r] = -1;
        next_token[r] = -1;
        next_score[r] = -INFINITY;
    }
}

__global__ __launch_bounds__(kWave) void k_tree_expand(
    const float* __restrict__ parent_score, const int32_t* __restrict__ cand_ids,
    const float* __restrict__ cand_logp, int M, int k, int n_next, int32_t* __restrict__ next_parent,
    int32_t* __restrict__ next_token, float* __restrict__ next_score) {
    extern __shared__ unsigned long long tree_keys[];    // list m at [m*k, m*k + k), descending
    unsigned long long* keys = tree_keys;
    const int lane = threadIdx.x;
    const int N = M * k;
    int n_real = 0;
    for (int base = 0; base < N; base += kWave * 8) {      // wave-uniform; eight loads of each array in flight
        int id[8];
        float lp[8], ps[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int e = base + u * kWave + lane;
            id[u] = -1;
            lp[u] = 0.f;
            ps[u] = 0.f;
            if (e < N) {
                id[u] = cand_ids[e];
                lp[u] = cand_logp[e];
                if (parent_score) ps[u] = parent_score[e / k];
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int e = base + u * kWave + lane;
            const unsigned long long key = tree_key(ps[u], lp[u], id[u], e);
            if (e < N) keys[e] = key;
            n_real += __popcll(__ballot(key != 0ull));
        }
    }
    // (a wave's LDS accesses complete in order: no barrier in a one-wave workgroup)
    const int m = blockIdx.x;
    int e;
    bool keep;
    const int rank = tree_rank_node(keys, M, k, n_next, m, lane, e, keep);
    if (keep) {
        next_parent[rank] = m;
        next_token[rank] = cand_ids[e];
        next_score[rank] = (parent_score ? parent_score[m] : 0.f) + cand_logp[e];
    }
    if (blockIdx.x == 0) tree_pad(n_real, n_next, lane, next_parent, next_token, next_score);
}

}  // namespace
