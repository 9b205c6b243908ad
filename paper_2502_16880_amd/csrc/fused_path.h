// Single-launch path of the grouped / dense LM head.
//
// One persistent workgroup of 16 waves per compute unit.  Every workgroup
//   1. stages the M hidden vectors in LDS,
//   2. computes the whole gate s[M,G] itself from the L2-resident gate matrix (Eq. 7's
//      W2 projection; redundant per workgroup, which costs less than a grid-wide
//      synchronisation would), selects the g best groups per token and builds the list
//      of activated groups with their token masks,
//   3. streams its share of the activated rows: global wave w takes row pairs w,
//      w + #waves, ... of the concatenated activated groups, each row as eight 1 KB
//      non-temporal wave loads, and dots it with the hidden vectors of the tokens that
//      selected the row's group (v_dot2c_f32_bf16, fp32 accumulation),
//   4. keeps per (wave, token) a sorted list of the k best logits in LDS, touched only
//      when a logit beats the wave's current k-th,
//   5. merges its waves' lists and publishes one list per token; the workgroup that
//      arrives last merges all workgroups' lists and writes the result.
// The logits row never exists in memory.  No workgroup ever waits for another.
//
// Log-probability mode (LP, Eq. 8: log p(x) = log p_router(n) + z[x] - lse_n, the softmax
// taken inside each selected group): a workgroup streams rows of one group only, the
// workgroups shared out among the activated groups by cost; beside the lists, lane t of
// every wave notes the (max, sum of exp) of every row pair for token t, and the workgroup
// sums these pieces in pair order (the result then does not depend on which wave drew
// which pair); the last workgroup of each group finishes the group (lse_n, offset, the
// group's k best per token) and the last group merges every token's g lists.  A draft-level
// call also expands the tree level in that last workgroup (tree_expand.h).
#pragma once
#include "control_words.h"
#include "device_utils.h"
#include "tree_expand.h"

namespace {

constexpr int kFusedWaves = 16;
constexpr int kFusedBlock = kFusedWaves * kWave;
constexpr int kFusedRows = 2;          // rows a wave loads together
constexpr int kFusedSegs = 8;          // 1 KB segments of a row held in registers
constexpr int kLdsLimit = 160 * 1024;
// Log-probability mode: a row pair's cost in a workgroup's time is its load latency plus
// the dot products of every token that selected its group; measured in units of one
// token's dot products the latency is about this much.
constexpr int kLpBaseCost = 10;
constexpr int kLpPiecesMax = 16 * 1024;    // LDS for a workgroup's log-sum-exp pieces, at most
// Collected candidates: where a workgroup meets few rows per token (the configured shapes:
// g * v / 256, about 63), the waves append every logit to one buffer per token instead of
// keeping sorted lists, and one wave per token ranks the buffer at the end.
constexpr int kCollectCap = 128;       // entries per token
constexpr int kLpGroupCounters = coral_ctrl::kLpGroupArrival - coral_ctrl::kFusedArrival;   // from p.counter
// How the gate (step 2a) is computed: on the vector units, or on the matrix cores (16-bit
// storage, four tokens or more).
enum GateMode { kGateVector = 0, kGateMfma = 1 };
constexpr int kGateTileFloats = 256;          // a wave's partial 16 x 16 tile
// Wave-private LDS scratch of the merges: ranking keys, gathered candidates, list tags.
struct WaveScratch {
    unsigned long long keys[kWave];
    unsigned keys32[kWave];
    Cand cand[kWave];
    int tags[kWave];
};
constexpr int kMergeAreaBytes = sizeof(WaveScratch);

struct FusedParams {
    const uint4* hidden;        // [M, n_vec]   what the LM head sees
    const uint4* gate_hidden;   // [M, n_vec]   what the router sees (grouped; may equal hidden)
    const uint4* gate_W;        // [G, n_vec]   (grouped)
    const float* bias;          // [G] or null  (grouped)
    const uint4* lm_W;          // [V, n_vec]
    const int32_t* offsets;     // [G+1]        (grouped)
    const int32_t* rows;        // [V]          (grouped)
    int32_t* sel_out;           // [M, g] or null
    Cand* part;                 // [M, k, gridDim.x] per-workgroup lists, entry-major
    unsigned long long* lse_part;   // [M, gridDim.x] (max, sum of exp) pairs (log-probability mode)
    Cand* glist;                // [M, g, k] a token's list per selected group (log-probability mode)
    unsigned long long* pair_lse;   // (max, sum of exp) of every (row pair, token) (same mode)
    // Draft-level call (log-probability mode): the tokens are the nodes of a tree level and
    // the workgroup that writes the result also expands the level (tree_expand.h).
    const float* parent_score;  // [M] cumulative log-probabilities of the nodes, or null (zero)
    int32_t* next_parent;       // [n_next], or null: no expansion
    int32_t* next_token;        // [n_next]
    float* next_score;          // [n_next]
    int n_next;
    unsigned int* counter;      // arrival counter, zero between calls; the log-probability
                                // mode also uses words kLpGroupCounters .. + 63, zero as well
    int32_t* topk_ids;          // [M, k]
    float* topk_logits;         // [M, k]
    int M, V, G, g, k;
    int n_vec, jp;
    int collect;                // candidates are collected per token (see kCollectCap) instead of listed per wave
    int stream_waves;           // waves of a workgroup that stream weight rows (1..16)
};

struct FusedLds {
    int o_hidden, o_lists, o_s, o_mask, o_ugroup, o_ustart, o_uend, o_uprefix, o_umask, o_flags, o_count;
    int o_keys, o_offsets, o_bias;
    int o_sel, o_wgstart;       // log-probability mode only
    int o_pieces, pieces_bytes; // same mode: the log-sum-exp pieces of a workgroup's pairs, if they fit
    int total;
};

// 16-byte vectors between consecutive hidden vectors in LDS: the row length plus one, so
// that the matrix-core gate, which reads a column of 16 rows at a time, meets no bank conflicts.
__host__ __device__ inline int hidden_lds_stride(int jp) { return jp * kWave + 1; }

// Byte offsets of the kernel's regions in dynamic LDS (the host sizes the launch with the
// same function the kernel lays its pointers out with).
__host__ __device__ inline FusedLds fused_lds_layout(int M, int G, int g, int k, int jp, bool dense,
                                                     int gate_mode, bool logprob = false,
                                                     bool collect = false) {
    FusedLds L;
    int off = 0;
    auto take = [&](size_t bytes) {
        int at = off;
        off = (int)((off + bytes + 15) / 16 * 16);
        return at;
    };
    long long um = (long long)M * g < G ? (long long)M * g : G;   // activated groups at most
    if (dense || um < 1) um = 1;
    size_t hidden_bytes = (size_t)M * hidden_lds_stride(jp) * sizeof(uint4);
    const size_t scratch_bytes = (size_t)kFusedWaves * kMergeAreaBytes;
    if (hidden_bytes < scratch_bytes) hidden_bytes = scratch_bytes;   // reused by the merges
    L.o_hidden = take(hidden_bytes);
    size_t lists_bytes = collect ? (size_t)M * kCollectCap * sizeof(unsigned long long)
                                 : (size_t)kFusedWaves * M * k * sizeof(Cand);
    // the MFMA gate parks its per-wave partial tiles here before the lists are initialised
    const size_t gate_part_bytes =
        (!dense && gate_mode != kGateVector)
            ? (size_t)kFusedWaves * ((M + 15) / 16) * kGateTileFloats * sizeof(float)
            : 0;
    if (lists_bytes < gate_part_bytes) lists_bytes = gate_part_bytes;
    L.o_lists = take(lists_bytes);
    L.o_s = take(dense ? 16 : (size_t)M * G * sizeof(float));
    L.o_mask = take(dense ? 16 : (size_t)G * sizeof(unsigned long long));
    L.o_ugroup = take((size_t)um * sizeof(int));
    L.o_ustart = take((size_t)um * sizeof(int));
    L.o_uend = take((size_t)um * sizeof(int));
    L.o_uprefix = take((size_t)(um + 1) * sizeof(int));
    L.o_umask = take((size_t)um * sizeof(unsigned long long));
    L.o_flags = take(16);
    L.o_count = take(collect ? (size_t)M * sizeof(int) : 0);      // collected candidates per token
    L.o_keys = take(dense ? 16 : (size_t)kFusedWaves * kWave * sizeof(unsigned long long));
    L.o_offsets = take(dense ? 16 : (size_t)(G + 1) * sizeof(int));
    L.o_bias = take(dense ? 16 : (size_t)G * sizeof(float));
    L.o_sel = take(logprob ? (size_t)M * g * sizeof(int) : 0);
    L.o_wgstart = take(logprob ? (size_t)(um + 1) * sizeof(int) : 0);
    L.o_pieces = off;
    L.pieces_bytes = 0;
    if (logprob) {                                     // what is left, up to kLpPiecesMax
        const int left = (kLdsLimit - off) / 16 * 16;
        L.pieces_bytes = left < 0 ? 0 : left < kLpPiecesMax ? left : kLpPiecesMax;
        off += L.pieces_bytes;
    }
    L.total = off;
    return L;
}

__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ unsigned long long uni64(unsigned long long x) {
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)x);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(x >> 32));
    return ((unsigned long long)hi << 32) | lo;
}

__device__ __forceinline__ Cand sentinel() {
    Cand c;
    c.v = -INFINITY;
    c.id = INT_MAX;
    return c;
}

// Insert the wave-uniform candidate (z, id) of token t into that token's LDS list if it
// beats the list's k-th entry.  thr_v / thr_i cache the k-th entry of every token's list
// of this wave, token t in lane t.
__device__ __forceinline__ void lds_list_insert(Cand* list, int k, int lane, float z, int id,
                                                float& thr_v, int& thr_i, int t) {
    const float tv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(thr_v), t));
    const int ti = __builtin_amdgcn_readlane(thr_i, t);
    if (!better(z, id, tv, ti)) return;                // wave-uniform
    Cand c = sentinel();
    if (lane < k) c = list[lane];
    const unsigned long long b = __ballot(better(z, id, c.v, c.id));
    const int pos = __ffsll(b) - 1;                    // <= k-1: the k-th entry is beaten
    const float sv = lane_below(c.v);
    const int si = lane_below(c.id);
    if (lane == pos) {
        c.v = z;
        c.id = id;
    } else if (lane > pos) {
        c.v = sv;
        c.id = si;
    }
    if (lane < k) list[lane] = c;
    const float nv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(c.v), k - 1));
    const int ni = __builtin_amdgcn_readlane(c.id, k - 1);
    if (lane == t) {
        thr_v = nv;
        thr_i = ni;
    }
}

// Candidate lists that cross workgroups are written and read with agent-scope atomic
// accesses (they go through to memory, past the per-XCD L2), so that publishing needs
// no L2 write-back fence.
__device__ __forceinline__ void publish_cand(Cand* dst, float v, int id) {
    const unsigned long long bits =
        ((unsigned long long)(unsigned)id << 32) | (unsigned long long)(unsigned)__float_as_int(v);
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(dst), bits, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ Cand fetch_cand(const Cand* src) {
    const unsigned long long bits = __hip_atomic_load(
        reinterpret_cast<const unsigned long long*>(src), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    Cand c;
    c.v = __int_as_float((int)(unsigned)(bits & 0xffffffffull));
    c.id = (int)(unsigned)(bits >> 32);
    return c;
}

// One step of a streamed top-k: every lane offers one candidate; those that beat the
// current k-th entry of the register list (lane i = rank i) are inserted one by one.
__device__ __forceinline__ void offer_candidates(float& lv, int& li, Cand c, int k, int lane) {
    const float tv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(lv), k - 1));
    const int ti = __builtin_amdgcn_readlane(li, k - 1);
    unsigned long long pass = __ballot(better(c.v, c.id, tv, ti));
    while (pass) {                                     // wave-uniform
        const int src = __ffsll(pass) - 1;
        pass &= pass - 1ull;
        const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(c.v), src));
        const int id = __builtin_amdgcn_readlane(c.id, src);
        list_insert(lv, li, v, id, lane, k);
    }
}

// ---------------------------------------------------------------- merging sorted lists
// Number of keys[0, n) above `key`.  keys is LDS that this wave wrote itself (a wave's LDS
// accesses complete in order); every lane reads the same address, which LDS broadcasts.
__device__ __forceinline__ int count_above(const unsigned long long* keys, int n, unsigned long long key) {
    int r = 0;
#pragma unroll 8
    for (int j = 0; j < n; ++j) r += keys[j] > key ? 1 : 0;    // wave-uniform trip count
    return r;
}

// Rank of this lane's candidate among the candidates of lanes [0, n), n <= 64: the number
// of those that beat it.  Candidates are distinct under the total order (distinct ids).
__device__ __forceinline__ int wave_rank(unsigned long long* keys, float v, int id, int n, int lane) {
    const unsigned long long key = cand_key(v, id);
    keys[lane] = key;
    return count_above(keys, n, key);
}

__device__ __forceinline__ bool is_real(Cand c) { return c.id != INT_MAX; }

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_max(float x) {
    const int moved = __builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
    return fmaxf(x, __int_as_float(moved));
}
// Maximum over the 64 lanes (no NaN among the inputs), wave-uniform.
__device__ __forceinline__ float wave_max(float x) {
    x = dpp_max<0x111, 0xf>(x);   // row_shr:1
    x = dpp_max<0x112, 0xf>(x);   // row_shr:2
    x = dpp_max<0x114, 0xf>(x);   // row_shr:4
    x = dpp_max<0x118, 0xf>(x);   // row_shr:8
    x = dpp_max<0x142, 0xa>(x);   // row_bcast:15
    x = dpp_max<0x143, 0xc>(x);   // row_bcast:31
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// Order-preserving 32-bit key of a logit (0 is below every logit, used for padding).
__device__ __forceinline__ unsigned ord32(float v) {
    const unsigned u = __float_as_uint(v + 0.0f);
    return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}
__device__ __forceinline__ unsigned cand_ord(Cand c) { return is_real(c) ? ord32(c.v) : 0u; }

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ unsigned dpp_min(unsigned x) {
    const unsigned moved = (unsigned)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, ROW_MASK, 0xf, false);
    return x < moved ? x : moved;
}
__device__ __forceinline__ unsigned wave_min_u32(unsigned x) {
    x = dpp_min<0x111, 0xf>(x);   // row_shr:1
    x = dpp_min<0x112, 0xf>(x);   // row_shr:2
    x = dpp_min<0x114, 0xf>(x);   // row_shr:4
    x = dpp_min<0x118, 0xf>(x);   // row_shr:8
    x = dpp_min<0x142, 0xa>(x);   // row_bcast:15
    x = dpp_min<0x143, 0xc>(x);   // row_bcast:31
    return (unsigned)__builtin_amdgcn_readlane((int)x, 63);
}

// k-th largest of the keys in lanes [0, n), or 0 if there are fewer than k keys.
// Wave-uniform.  Used as a bound only: candidates are kept if their key reaches it, ties
// included.  A key is among the k largest values exactly when fewer than k keys exceed it;
// the smallest such key is the k-th largest.  keys32: 64 wave-private LDS words.
__device__ __forceinline__ unsigned wave_kth_key(unsigned* keys32, unsigned key, int n, int k, int lane) {
    if (n < k) return 0u;
    if (lane >= n) key = 0u;
    keys32[lane] = key;
    int above = 0;
#pragma unroll 16
    for (int j = 0; j < n; ++j) above += keys32[j] > key ? 1 : 0;   // wave-uniform trip count
    return wave_min_u32(lane < n && above < k ? key : 0xffffffffu);
}

// e / k for 0 <= e < 4096 and 1 <= k <= 64 without an integer division.
__device__ __forceinline__ int div_small(int e, int inv_k) { return (int)(((unsigned)e * (unsigned)inv_k) >> 20); }
__device__ __forceinline__ int inv_small(int k) { return (1 << 20) / k + 1; }

// Appends the candidates flagged `keep` to scratch[cnt...] in lane order; returns the
// new count (entries past `cap` are dropped, the caller checks the count).
__device__ __forceinline__ int wave_append(Cand* scratch, int* tag_scratch, int cnt, int cap,
                                           bool keep, Cand c, int tag, int lane) {
    const unsigned long long b = __ballot(keep);
    if (keep) {
        const int pos = cnt + __popcll(b & ((1ull << lane) - 1ull));
        if (pos < cap) {
            scratch[pos] = c;
            if (tag_scratch) tag_scratch[pos] = tag;
        }
    }
    return cnt + __popcll(b);
}

// One wave merges n_lists sorted lists of k candidates (get(list, i), padding entries are
// sentinels) into the k best, put(rank, candidate) for every rank < k.
// Fast path: a value that k lists' first entries reach is a lower bound of the result's
// k-th value, so only lists whose first entry reaches it can contribute, and of those only
// entries that reach it (ties kept); the few survivors are ranked by counting.  If a bound
// does not exist (fewer than k lists, more than 256 lists) or too many survive (64), the
// lists are streamed through a sorted register list instead.  No more than 64 candidates in
// all are ranked directly; DIRECT > 0 (lists that are far away, in memory): no more than
// DIRECT per lane are fetched in one trip, bounded by a sample of themselves, and ranked.
template <int DIRECT = 0, class Get, class Put>
__device__ __forceinline__ void wave_merge_topk(int n_lists, int k, int lane, WaveScratch* ws,
                                                Get get, Put put) {
    constexpr int kCap = kWave;
    Cand* scratch = ws->cand;
    int* tags = ws->tags;
    const int inv_k = inv_small(k);
    if (n_lists * k <= kWave) {
        // one candidate per lane: ranked by counting at once
        const int n_e = n_lists * k;
        Cand c = sentinel();
        if (lane < n_e) {
            const int l = div_small(lane, inv_k);
            c = get(l, lane - l * k);
        }
        const int n_real = __popcll(__ballot(is_real(c)));
        const int r = wave_rank(ws->keys, c.v, c.id, n_e, lane);   // real ones are distinct
        if (is_real(c) && r < k) put(r, c);
        if (lane >= n_real && lane < k) put(lane, sentinel());
        return;
    }
    if (DIRECT && n_lists * k <= DIRECT * kWave) {
        // up to DIRECT candidates per lane, all requested at once; the k-th largest of the
        // lanes' best candidates (k lanes reach it) bounds the result's k-th entry, and what
        // reaches the bound is ranked by counting
        constexpr int kPerLane = DIRECT > 0 ? DIRECT : 1;
        const int n_e = n_lists * k;
        Cand cd[kPerLane];
        unsigned sample = 0u;
#pragma unroll
        for (int u = 0; u < kPerLane; ++u) {
            const int e = u * kWave + lane;
            cd[u] = sentinel();
            if (e < n_e) {
                const int l = div_small(e, inv_k);
                cd[u] = get(l, e - l * k);
            }
            const unsigned o = cand_ord(cd[u]);
            sample = o > sample ? o : sample;
        }
        const unsigned bound = wave_kth_key(ws->keys32, sample, kWave, k, lane);
        int cnt = 0;
#pragma unroll
        for (int u = 0; u < kPerLane; ++u)
            if (u * kWave < n_e)                       // uniform
                cnt = wave_append(scratch, nullptr, cnt, kCap, is_real(cd[u]) && ord32(cd[u].v) >= bound,
                                  cd[u], 0, lane);
        if (cnt <= kCap) {
            Cand s = sentinel();
            if (lane < cnt) s = scratch[lane];
            const int r = wave_rank(ws->keys, s.v, s.id, cnt, lane);
            if (lane < cnt && r < k) put(r, s);
            if (lane >= cnt && lane < k) put(lane, sentinel());
            return;
        }
    }
    bool fast = n_lists >= k && n_lists <= 4 * kWave;
    int n_s = 0;
    unsigned tau = 0u;
    if (fast) {
        Cand mx[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int l = c * kWave + lane;
            mx[c] = sentinel();
            if (c * kWave < n_lists && l < n_lists) mx[c] = get(l, 0);
        }
        // bound: the k-th largest of the lanes' best first entries (k lanes reach it, so k
        // lists do); if more than 64 lists reach it, the 64 kept so far are the next,
        // tighter sample
        unsigned sample = cand_ord(mx[0]);
#pragma unroll
        for (int c = 1; c < 4; ++c) {
            const unsigned o = cand_ord(mx[c]);
            sample = o > sample ? o : sample;
        }
        int n_sample = n_lists < kWave ? n_lists : kWave;
        int cnt = 0;
#pragma unroll
        for (int round = 0; round < 3; ++round) {              // wave-uniform
            tau = wave_kth_key(ws->keys32, sample, n_sample, k, lane);
            cnt = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (c * kWave < n_lists)
                    cnt = wave_append(scratch, tags, cnt, kCap,
                                      is_real(mx[c]) && ord32(mx[c].v) >= tau, mx[c],
                                      c * kWave + lane, lane);
            if (cnt <= kCap) break;
            sample = cand_ord(scratch[lane]);
            n_sample = kCap;
        }
        if (cnt > kCap) {
            fast = false;                                      // no usable bound (ties)
        } else {
            n_s = cnt;                                         // the lists that reach the bound
        }
    }
    if (fast) {
        int cnt = 0;
        const int n_e = n_s * k;
        for (int base = 0; base < n_e; base += 2 * kWave) {    // wave-uniform; two loads in flight
            Cand c2[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int e = base + u * kWave + lane;
                c2[u] = sentinel();
                if (e < n_e) {
                    const int sl = div_small(e, inv_k);
                    c2[u] = get(tags[sl], e - sl * k);
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
                cnt = wave_append(scratch, nullptr, cnt, kCap,
                                  is_real(c2[u]) && ord32(c2[u].v) >= tau, c2[u], 0, lane);
        }
        if (cnt <= kCap) {
            Cand s = sentinel();
            if (lane < cnt) s = scratch[lane];
            const int r = wave_rank(ws->keys, s.v, s.id, cnt, lane);
            if (lane < cnt && r < k) put(r, s);
            if (lane >= cnt && lane < k) put(lane, sentinel());
            return;
        }
    }
    // general path: the candidates stream through a sorted register list (lane i = rank i),
    // 256 at a time so that their loads are in flight together; the first list, sorted
    // already, seeds the register list
    float lv = -INFINITY;
    int li = INT_MAX;
    const int n_e = n_lists * k;
    const bool small = n_e <= 4096;                    // div_small's range
    for (int base = 0; base < n_e; base += 4 * kWave) {    // wave-uniform
        Cand c4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = base + u * kWave + lane;
            c4[u] = sentinel();
            if (e < n_e) {
                const int l = small ? div_small(e, inv_k) : e / k;
                c4[u] = get(l, e - l * k);
            }
        }
        if (base == 0) {
            if (lane < k) {
                lv = c4[0].v;
                li = c4[0].id;
                c4[0] = sentinel();
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (base + u * kWave < n_e) offer_candidates(lv, li, c4[u], k, lane);
    }
    if (lane < k) {
        Cand o;
        o.v = lv;
        o.id = li;
        put(lane, o);
    }
}

// (max, sum of exp(z - max)) of the one or two logits of a row pair (z1 = -inf: absent).
__device__ __forceinline__ void pair_lse(float& m, float& s, float z0, float z1) {
    m = fmaxf(z0, z1);
    s = m > -INFINITY ? expf(z0 - m) + expf(z1 - m) : 0.f;
}
__device__ __forceinline__ unsigned long long pack_lse(float m, float s) {
    return ((unsigned long long)__float_as_uint(s) << 32) | __float_as_uint(m);
}
// Takes a packed (max, sum) piece into the running state (m, s).
__device__ __forceinline__ void lse_take(float& m, float& s, unsigned long long piece) {
    const float pm = __uint_as_float((unsigned)(piece & 0xffffffffull));
    const float ps = __uint_as_float((unsigned)(piece >> 32));
    const float nm = fmaxf(m, pm);
    if (nm > -INFINITY) s = s * expf(m - nm) + ps * expf(pm - nm);
    m = nm;
}

// Combines the (max, sum) states of all lanes (absent: (-inf, 0)) into log(sum of exp); -inf
// if there is nothing to sum.
__device__ __forceinline__ float lse_finish(float m, float s) {
    float wm = m;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) wm = fmaxf(wm, __shfl_xor(wm, off));
    const float ws = wave_sum(wm > -INFINITY ? s * expf(m - wm) : 0.f);
    return wm + logf(ws);
}

template <int DT, int NT, bool LP>
__device__ __forceinline__ void fused_tokens(const FusedParams& p, const uint4* hs, Cand* my_lists,
                                             unsigned long long* collect_keys, int* collect_count,
                                             const uint4 (&w0)[kFusedSegs],
                                             const uint4 (&w1)[kFusedSegs],
                                             unsigned long long& rem, int rid0, int rid1, bool has1,
                                             float& thr_v, int& thr_i, float& lse_m, float& lse_s) {
    const int lane = threadIdx.x & (kWave - 1);
    const int hs_stride = hidden_lds_stride(p.jp);
    int tok[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        tok[i] = __ffsll(rem) - 1;
        rem &= rem - 1ull;
    }
    float a0[NT], a1[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) a0[i] = a1[i] = 0.f;
#pragma unroll
    for (int j = 0; j < kFusedSegs; ++j) {
        if (j < p.jp) {                                // uniform
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                const uint4 h = hs[tok[i] * hs_stride + j * kWave + lane];
                a0[i] = dot_vec<DT>(w0[j], h, a0[i]);
                a1[i] = dot_vec<DT>(w1[j], h, a1[i]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        const float z0 = wave_sum(a0[i]);
        float z1 = -INFINITY;
        if (has1) z1 = wave_sum(a1[i]);                // uniform
        if (!LP && p.collect) {                        // uniform: the token's buffer takes every logit
            if (lane == 0) {
                const int at = atomicAdd(&collect_count[tok[i]], has1 ? 2 : 1);
                unsigned long long* dst = collect_keys + (size_t)tok[i] * kCollectCap + at;
                if (at + 1 < kCollectCap) {            // holds by the host's bound on rows per token
                    dst[0] = cand_key(z0, rid0);
                    if (has1) dst[1] = cand_key(z1, rid1);
                }
            }
            continue;
        }
        lds_list_insert(my_lists + tok[i] * p.k, p.k, lane, z0, rid0, thr_v, thr_i, tok[i]);
        if (has1) lds_list_insert(my_lists + tok[i] * p.k, p.k, lane, z1, rid1, thr_v, thr_i, tok[i]);
        if (LP && lane == tok[i]) pair_lse(lse_m, lse_s, z0, z1);   // lane t: token t's piece
    }
}

template <int DT, bool DENSE, int GATE, bool ROUTED = false, bool LP = false>
__global__ __launch_bounds__(kFusedBlock) void k_fused(FusedParams p) {
    static_assert(!(LP && DENSE), "the log-probability mode belongs to the grouped head");
    extern __shared__ uint4 smem[];
    char* lds = reinterpret_cast<char*>(smem);
    const FusedLds lay = fused_lds_layout(p.M, p.G, p.g, p.k, p.jp, DENSE, GATE, LP, p.collect != 0);
    uint4* hs = reinterpret_cast<uint4*>(lds + lay.o_hidden);
    Cand* lists = reinterpret_cast<Cand*>(lds + lay.o_lists);
    float* s_lds = reinterpret_cast<float*>(lds + lay.o_s);
    unsigned long long* mask_lds = reinterpret_cast<unsigned long long*>(lds + lay.o_mask);
    int* ugroup = reinterpret_cast<int*>(lds + lay.o_ugroup);
    int* ustart = reinterpret_cast<int*>(lds + lay.o_ustart);
    int* uend = reinterpret_cast<int*>(lds + lay.o_uend);
    int* uprefix = reinterpret_cast<int*>(lds + lay.o_uprefix);
    unsigned long long* umask = reinterpret_cast<unsigned long long*>(lds + lay.o_umask);
    int* flags = reinterpret_cast<int*>(lds + lay.o_flags);
    int* collect_count = reinterpret_cast<int*>(lds + lay.o_count);                  // [M], collect mode only
    unsigned long long* collect_keys = reinterpret_cast<unsigned long long*>(lds + lay.o_lists);   // [M][kCollectCap]
    int* off_lds = reinterpret_cast<int*>(lds + lay.o_offsets);
    float* bias_lds = reinterpret_cast<float*>(lds + lay.o_bias);
    int* sel_lds = reinterpret_cast<int*>(lds + lay.o_sel);          // LP: [M, g] selections
    int* wgstart = reinterpret_cast<int*>(lds + lay.o_wgstart);      // LP: first workgroup of a group

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int hs_stride = hidden_lds_stride(p.jp);
    const int M = p.M, k = p.k;

    // row-pair counter, see step 3: a wave's first pair is fixed (i = wave), the others are drawn
    if (threadIdx.x == 0) flags[2] = LP ? 0 : p.stream_waves;
    if (p.collect && (int)threadIdx.x < p.M) collect_count[threadIdx.x] = 0;     // (seen by all after the gate's barriers)
    // ---- 1. hidden vectors: requested first, written to LDS only after the grouped
    // variants have requested their first gate rows as well (loads return in order, so the
    // wait for the hidden vectors does not wait for the gate rows behind them)
    constexpr int kHU = 4;
    const int row_vecs = p.jp * kWave;                     // <= 512: at least 2 rows a pass
    int h_mm = threadIdx.x / row_vecs;
    int h_vec = threadIdx.x - h_mm * row_vecs;
    const int rows_per_pass = kFusedBlock / row_vecs;
    uint4 htmp[kHU];
    // The router may see another vector than the LM head (Eq. 7: W2 is applied to
    // act(W1 h) + h): then the gate's vectors are staged first and the LM head's replace
    // them after the gate, their loads in flight during the selection (ROUTED, compiled
    // apart: the kernel has no registers to spare).
    const uint4* h_src = ROUTED ? p.gate_hidden : p.hidden;
    auto hidden_request = [&](int m0) {
#pragma unroll
        for (int u = 0; u < kHU; ++u) {
            const int m = m0 + u * rows_per_pass + h_mm;
            htmp[u] = make_uint4(0, 0, 0, 0);
            if (h_mm < rows_per_pass && m < M && h_vec < p.n_vec)
                htmp[u] = h_src[(size_t)m * p.n_vec + h_vec];
        }
    };
    auto hidden_commit = [&](int m0) {                     // then the passes that remain
#pragma unroll
        for (int u = 0; u < kHU; ++u) {
            const int m = m0 + u * rows_per_pass + h_mm;
            if (h_mm < rows_per_pass && m < M) hs[m * hs_stride + h_vec] = htmp[u];
        }
    };
    auto hidden_rest = [&]() {
        for (int m0 = rows_per_pass * kHU; m0 < M; m0 += rows_per_pass * kHU) {
            hidden_request(m0);
            hidden_commit(m0);
        }
    };
    hidden_request(0);
    // group offsets and bias travel with them (G <= 1024 = the workgroup's size), so that
    // no later step waits for memory
    int off_r0 = 0, off_r1 = 0;
    float bias_r = 0.f;
    if (!DENSE) {
        if ((int)threadIdx.x <= p.G) off_r0 = p.offsets[threadIdx.x];
        if ((int)threadIdx.x + kFusedBlock <= p.G) off_r1 = p.offsets[threadIdx.x + kFusedBlock];
        if ((int)threadIdx.x < p.G && p.bias) bias_r = p.bias[threadIdx.x];
    }
    auto small_commit = [&]() {
        if ((int)threadIdx.x <= p.G) off_lds[threadIdx.x] = off_r0;
        if ((int)threadIdx.x + kFusedBlock <= p.G) off_lds[threadIdx.x + kFusedBlock] = off_r1;
        if ((int)threadIdx.x < p.G) bias_lds[threadIdx.x] = bias_r;
    };
    Cand* my_lists = lists + (size_t)wave * M * k;
    float thr_v = -INFINITY;
    int thr_i = INT_MAX;

    int total_batches;
    if (DENSE) {
        hidden_commit(0);
        hidden_rest();
        total_batches = (p.V + kFusedRows - 1) / kFusedRows;
        __syncthreads();
    } else {
        for (int n = threadIdx.x; n < p.G; n += kFusedBlock) mask_lds[n] = 0ull;
        if (GATE != kGateVector) {
            // ---- 2a. gate on the matrix cores: s[16 groups x 16 tokens] tiles, the H
            // columns split over the 16 waves in steps of 32 (v_mfma_f32_16x16x32_bf16:
            // lane l feeds row l%16, columns 8*(l/16)..+8 of both operands and receives
            // rows 4*(l/16)..+4, column l%16 of the tile); the waves' partial tiles are
            // summed in wave order.
            const int r16 = lane & 15, q4 = lane >> 4;
            const int n_gt = (p.G + 15) / 16, n_tt = (M + 15) / 16;
            constexpr int kSlice = kGateTileFloats;
            float* gpart = reinterpret_cast<float*>(lds + lay.o_lists);   // [wave][n_tt][kSlice]
            // waves 0-7 work on the even tile of a pair of group tiles, waves 8-15 on the odd
            // one; wave kw of either half takes the 256-byte blocks kw, kw + 8, kw + 16, kw + 24
            // of the gate rows (jp <= 8: a row has at most 32).  A block is four wave loads of
            // four rows x 256 contiguous bytes, transposed in registers to the operands of four
            // 32-column steps (mfma_operands_from_quad_rows in device_utils.h): register
            // 4 B + c then feeds rows 0..15, 16-byte chunks {c, 4 + c, 8 + c, 12 + c} of block
            // 8 B + kw, and the hidden vectors are read from LDS with the same choice.
            const int half = wave >> 3, kw = wave & 7;
            constexpr int kSteps = 2 * kFusedSegs;
            uint4 ga[kSteps];
            // (every workgroup sums the columns in the same order: the scores, and with them
            // the selection, must come out bit-identical in all of them)
            auto load_gate_tile = [&](int gt) {
#pragma unroll
                for (int i = 0; i < kSteps; ++i) {
                    const int n = gt * 16 + ((lane >> 2) & 3) * 4 + (i & 3);
                    const int vec = ((i >> 2) * 8 + kw) * 16 + q4 * 4 + (lane & 3);
                    ga[i] = make_uint4(0, 0, 0, 0);
                    if (vec < p.n_vec && n < p.G) ga[i] = p.gate_W[(size_t)n * p.n_vec + vec];
                }
            };
            auto to_operand_layout = [&]() {
#pragma unroll
                for (int i = 0; i < kSteps; i += 4)
                    mfma_operands_from_quad_rows(ga[i], ga[i + 1], ga[i + 2], ga[i + 3], lane);
            };
            load_gate_tile(half);
            hidden_commit(0);
            small_commit();
            hidden_rest();
            // The first tile's rows are transposed before the barrier, while the workgroup
            // waits for its last wave's hidden vectors (1.6 us at 8 tokens).
            to_operand_layout();
            __syncthreads();
            for (int pair = 0; pair * 2 < n_gt; ++pair) {
                if (pair) {
                    load_gate_tile(pair * 2 + half);
                    to_operand_layout();
                }
                for (int tt = 0; tt < n_tt; ++tt) {            // uniform
                    f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
                    const int m = tt * 16 + r16;
                    const int mc = m < M ? m : M - 1;          // clamped: the load is unconditional
#pragma unroll
                    for (int i0 = 0; i0 < kSteps; i0 += 2) {
                        uint4 hb[2];
#pragma unroll
                        for (int u = 0; u < 2; ++u) {
                            const int vec = (((i0 + u) >> 2) * 8 + kw) * 16 + q4 * 4 + ((i0 + u) & 3);
                            const bool in = vec < p.n_vec;
                            hb[u] = hs[mc * hs_stride + (in ? vec : 0)];
                            if (m >= M || !in) hb[u] = make_uint4(0, 0, 0, 0);
                        }
#pragma unroll
                        for (int u = 0; u < 2; ++u)
                            acc = mfma_tile<DT>(ga[i0 + u], hb[u], acc);
                    }
                    *reinterpret_cast<f32x4_t*>(gpart + ((size_t)wave * n_tt + tt) * kSlice + lane * 4) = acc;
                }
                __syncthreads();
                for (int idx = threadIdx.x; idx < 2 * n_tt * 256; idx += kFusedBlock) {
                    const int hh = idx / (n_tt * 256);
                    const int rest = idx - hh * n_tt * 256;
                    const int tt = rest >> 8, e = rest & 255;
                    const int l = e >> 2, i = e & 3;
                    const int n = (pair * 2 + hh) * 16 + (l >> 4) * 4 + i;
                    const int m = tt * 16 + (l & 15);
                    float sum = 0.f;
                    for (int w = hh * 8; w < hh * 8 + 8; ++w)
                        sum += gpart[((size_t)w * n_tt + tt) * kSlice + e];
                    if (n < p.G && m < M) s_lds[m * p.G + n] = sum + bias_lds[n];
                }
                __syncthreads();
            }
        } else {
            // ---- 2a. gate on the vector units (fp32 storage, or few tokens): each wave takes
            // rows n0 and n0 + 16 per pass
            uint4 ga[kFusedSegs], gb[kFusedSegs];
            auto load_gate_rows = [&](int n0) {
                const int n1 = n0 + kFusedWaves;
#pragma unroll
                for (int j = 0; j < kFusedSegs; ++j) {
                    const int vec = j * kWave + lane;
                    ga[j] = make_uint4(0, 0, 0, 0);
                    gb[j] = make_uint4(0, 0, 0, 0);
                    if (j < p.jp && vec < p.n_vec) {
                        if (n0 < p.G) ga[j] = p.gate_W[(size_t)n0 * p.n_vec + vec];
                        if (n1 < p.G) gb[j] = p.gate_W[(size_t)n1 * p.n_vec + vec];
                    }
                }
            };
            load_gate_rows(wave);
            hidden_commit(0);
            small_commit();
            hidden_rest();
            __syncthreads();
            for (int n0 = wave; n0 < p.G; n0 += 2 * kFusedWaves) {
                if (n0 != wave) load_gate_rows(n0);
                const int n1 = n0 + kFusedWaves;
                for (int m = 0; m + 1 < M; m += 2) {           // two tokens per pass
                    const int m1 = m + 1;
                    float a0 = 0.f, b0 = 0.f, a1 = 0.f, b1 = 0.f;
#pragma unroll
                    for (int j = 0; j < kFusedSegs; ++j)
                        if (j < p.jp) {
                            const uint4 h0 = hs[m * hs_stride + j * kWave + lane];
                            const uint4 h1 = hs[m1 * hs_stride + j * kWave + lane];
                            a0 = dot_vec<DT>(ga[j], h0, a0);
                            b0 = dot_vec<DT>(gb[j], h0, b0);
                            a1 = dot_vec<DT>(ga[j], h1, a1);
                            b1 = dot_vec<DT>(gb[j], h1, b1);
                        }
                    a0 = wave_sum(a0);
                    b0 = wave_sum(b0);
                    a1 = wave_sum(a1);
                    b1 = wave_sum(b1);
                    if (lane == 0) {
                        const float bias0 = bias_lds[n0];
                        const float bias1 = n1 < p.G ? bias_lds[n1] : 0.f;
                        s_lds[m * p.G + n0] = a0 + bias0;
                        s_lds[m1 * p.G + n0] = a1 + bias0;
                        if (n1 < p.G) {
                            s_lds[m * p.G + n1] = b0 + bias1;
                            s_lds[m1 * p.G + n1] = b1 + bias1;
                        }
                    }
                }
                if (M & 1) {                                   // the last of an odd number of tokens
                    const int m = M - 1;                       // (the dot instructions bound this step)
                    float a0 = 0.f, b0 = 0.f;
#pragma unroll
                    for (int j = 0; j < kFusedSegs; ++j)
                        if (j < p.jp) {
                            const uint4 h0 = hs[m * hs_stride + j * kWave + lane];
                            a0 = dot_vec<DT>(ga[j], h0, a0);
                            b0 = dot_vec<DT>(gb[j], h0, b0);
                        }
                    a0 = wave_sum(a0);
                    b0 = wave_sum(b0);
                    if (lane == 0) {
                        s_lds[m * p.G + n0] = a0 + bias_lds[n0];
                        if (n1 < p.G) s_lds[m * p.G + n1] = b0 + bias_lds[n1];
                    }
                }
            }
            __syncthreads();
        }
        if (ROUTED) {                                  // the gate's last read of hs is behind a barrier
            h_src = p.hidden;
            // (recomputed behind a compiler barrier: the first staging's addresses would
            // otherwise be kept through the gate, where there are no registers to spare)
            int tid = threadIdx.x;
            asm volatile("" : "+v"(tid));
            h_mm = tid / row_vecs;
            h_vec = tid - h_mm * row_vecs;
            hidden_request(0);
        }
        // Log-probability mode: every workgroup streams rows of one group only (it keeps one
        // list and one log-sum-exp state per token, Eq. 8 normalises per group), so the
        // workgroups are shared out among the count <= 64 activated groups in proportion to
        // their cost, row pairs x (kLpBaseCost + tokens that selected the group): one each,
        // the rest by the groups' shares rounded down, what is then left one more each to the
        // groups with the highest cost per workgroup.  The numbers add up to gridDim.x.
        // One wave's work (activated group u in lane u), after it has written the tables of 2c.
        auto share_out_workgroups = [&](int count, int all_pairs) {
            const int P = gridDim.x;
            const int nb_u = lane < count ? uprefix[lane + 1] - uprefix[lane] : 0;
            // (row pairs scaled to 16 bits so that the products below stay in 31)
            const int shift = max(0, 16 - __clz(all_pairs));
            const unsigned cost =
                lane < count ? (unsigned)(nb_u >> shift) * (unsigned)(kLpBaseCost + __popcll(umask[lane])) : 0u;
            const unsigned total = (unsigned)__builtin_amdgcn_readlane(wave_scan_inclusive((int)cost), 63);
            int n_wg = lane < count ? 1 + (int)(cost * (unsigned)(P - count) / (total ? total : 1u)) : 0;
            const int left = P - __builtin_amdgcn_readlane(wave_scan_inclusive(n_wg), 63);
            if (left > 0) {                            // wave-uniform
                unsigned long long* rank_keys =
                    reinterpret_cast<unsigned long long*>(lds + lay.o_keys) + (size_t)wave * kWave;
                const int rank = wave_rank(rank_keys, lane < count ? (float)cost / (float)n_wg : -INFINITY,
                                           lane, kWave, lane);
                if (lane < count && rank < left) ++n_wg;
            }
            const int incl_wg = wave_scan_inclusive(n_wg);
            if (lane < count) wgstart[lane] = incl_wg - n_wg;
            if (lane == 0) wgstart[count] = P;
        };
        // ---- 2b. per-token top-g by rank counting: group n of token m is selected iff
        // fewer than g groups beat it (larger score first, then lower group id); its rank
        // is its position in the selection
        if (p.G <= kWave) {
            // group n in lane n.  gm: the tokens that selected this lane's group.
            unsigned long long gm = 0ull;
            unsigned long long* sel_keys =
                reinterpret_cast<unsigned long long*>(lds + lay.o_keys) + (size_t)wave * kWave;
            for (int m = wave; m < M; m += kFusedWaves) {  // one wave per token
                float v = lane < p.G ? s_lds[m * p.G + lane] : -INFINITY;
                if (!(v == v)) v = -INFINITY;              // NaN: unspecified, but keep a total order
                const int rank = wave_rank(sel_keys, v, lane, p.G, lane);
                if (lane < p.G && rank < p.g) {
                    atomicOr(&mask_lds[lane], 1ull << m);
                    if (p.sel_out && blockIdx.x == 0) p.sel_out[m * p.g + rank] = lane;
                    if (LP) sel_lds[m * p.g + rank] = lane;
                }
            }
            __syncthreads();
            if (lane < p.G) gm = mask_lds[lane];
            // ---- 2c. activated groups in ascending id order, their row ranges and the row
            // pairs before each.  Every wave builds the same tables and writes them to the
            // same LDS words (equal values), then reads back only what it wrote itself: no
            // barrier, no wave waits for another.
            const unsigned long long act = __ballot(gm != 0ull);
            const int count = __popcll(act);
            const int at = __popcll(act & ((1ull << lane) - 1ull));
            int lo = 0, hi = 0;
            if (gm != 0ull) {
                lo = off_lds[lane];
                hi = off_lds[lane + 1];
            }
            const int nb = (hi - lo + kFusedRows - 1) / kFusedRows;       // 0 for the others
            const int incl = wave_scan_inclusive(nb);
            if (gm != 0ull) {
                ugroup[at] = lane;
                umask[at] = gm;
                ustart[at] = lo;
                uend[at] = hi;
                uprefix[at] = incl - nb;
            }
            const int all_pairs = __builtin_amdgcn_readlane(incl, 63);
            if (lane == 0) {
                uprefix[count] = all_pairs;
                flags[0] = count;
            }
            if (LP) share_out_workgroups(count, all_pairs);
            if (ROUTED) {
                hidden_commit(0);
                hidden_rest();
                __syncthreads();
            }
            total_batches = all_pairs;
        } else {
            // more groups than lanes
            for (int idx = threadIdx.x; idx < M * p.G; idx += kFusedBlock) {
                const int m = idx / p.G;
                const int n = idx - m * p.G;
                const float* row = s_lds + m * p.G;
                float v = row[n];
                if (!(v == v)) v = -INFINITY;
                int rank = 0;
                for (int o = 0; o < p.G; ++o) {
                    float ov = row[o];
                    if (!(ov == ov)) ov = -INFINITY;
                    rank += better(ov, o, v, n) ? 1 : 0;
                }
                if (rank < p.g) {
                    atomicOr(&mask_lds[n], 1ull << m);
                    if (p.sel_out && blockIdx.x == 0) p.sel_out[m * p.g + rank] = n;
                    if (LP) sel_lds[m * p.g + rank] = n;
                }
            }
            __syncthreads();
            if (wave == 0) {
                int count = 0;
                for (int base = 0; base < p.G; base += kWave) {
                    const int n = base + lane;
                    const unsigned long long gm = n < p.G ? mask_lds[n] : 0ull;
                    const unsigned long long b = __ballot(gm != 0ull);
                    if (gm != 0ull) {
                        const int u = count + __popcll(b & ((1ull << lane) - 1ull));
                        ugroup[u] = n;
                        umask[u] = gm;
                        ustart[u] = off_lds[n];
                        uend[u] = off_lds[n + 1];
                    }
                    count += __popcll(b);
                }
                int carry = 0;                             // row pairs before each activated group
                for (int base = 0; base < count; base += kWave) {
                    const int u = base + lane;
                    const int nb = u < count ? (uend[u] - ustart[u] + kFusedRows - 1) / kFusedRows : 0;
                    const int incl = wave_scan_inclusive(nb);
                    if (u < count) uprefix[u] = carry + incl - nb;
                    carry += __builtin_amdgcn_readlane(incl, 63);
                }
                if (lane == 0) {
                    uprefix[count] = carry;
                    flags[0] = count;
                }
                if (LP) share_out_workgroups(count, carry);
            }
            if (ROUTED) {
                hidden_commit(0);
                hidden_rest();
            }
            __syncthreads();
            total_batches = uni(uprefix[uni(flags[0])]);
        }
    }

    // ---- 3./4. stream row pairs (the lists share LDS with the gate's partial tiles, so
    // they are emptied only now; each wave touches its own lists only)
    if (LP || !p.collect)
        for (int i = lane; i < M * k; i += kWave) my_lists[i] = sentinel();
    // The workgroup's row pairs are b(i) = (i / 16) * 16 * #workgroups + 16 * blockIdx + i % 16
    // for i = 0, 1, ...; its waves draw i from an LDS counter, so a wave that the memory
    // system serves faster takes more of them and all waves finish together.
    // (Log-probability mode: the workgroup's share is a contiguous range of one group's row
    // pairs instead, the j-th of the equal parts its group's workgroups cut the group into.)
    const int stride_batches = gridDim.x * kFusedWaves;
    int u = 0;
    int lp_lo = 0, lp_nwg = 0;
    // lane t: (max, sum of exp) of the current row pair for token t.  The pieces go to memory
    // per pair and are summed in pair order at the end: a running state per wave would make
    // the sum depend on which wave drew which pair, and the result would not repeat bit for bit
    float lse_m = -INFINITY, lse_s = 0.f;
    unsigned long long* lp_pieces = nullptr;           // piece of (token slot j, pair b) at
    int lp_stride = 0, lp_origin = 0;                  // lp_pieces[j * lp_stride + b - lp_origin],
    bool lp_in_lds = false;                            // in memory, or in lds_pieces likewise
    unsigned long long* lds_pieces = reinterpret_cast<unsigned long long*>(lds + lay.o_pieces);
    if (LP) {
        const int count = uni(flags[0]);
        const int nxt = lane < count ? wgstart[lane + 1] : INT_MAX;
        u = __popcll(__ballot(nxt <= (int)blockIdx.x));    // wgstart[u] <= blockIdx.x < wgstart[u + 1]
        const int j = blockIdx.x - uni(wgstart[u]);
        lp_nwg = uni(wgstart[u + 1]) - uni(wgstart[u]);
        const int nb = uni(uprefix[u + 1]) - uni(uprefix[u]);
        const int per = (nb + lp_nwg - 1) / lp_nwg;
        lp_lo = uni(uprefix[u]) + min(j * per, nb);
        total_batches = uni(uprefix[u]) + min((j + 1) * per, nb);  // the end of this workgroup's range
        // The pieces stay in LDS if this workgroup's fit there; else they go through memory,
        // this group's behind those of the activated groups before it.
        const int n_mine = total_batches - lp_lo;
        if ((size_t)n_mine * __popcll(uni64(umask[u])) * sizeof(unsigned long long) <= (size_t)lay.pieces_bytes) {
            lp_in_lds = true;
            lp_stride = n_mine;
            lp_origin = lp_lo;
        } else {
            const int before = lane < u ? (uprefix[lane + 1] - uprefix[lane]) * __popcll(umask[lane]) : 0;
            lp_pieces = p.pair_lse + (size_t)__builtin_amdgcn_readlane(wave_scan_inclusive(before), 63);
            lp_stride = nb;
            lp_origin = uni(uprefix[u]);
        }
    }
    auto draw_batch = [&]() {
        int i = 0;
        if (lane == 0) i = atomicAdd(&flags[2], 1);
        i = uni(i);
        if (LP) return lp_lo + i;
        return (int)((i / kFusedWaves) * stride_batches + blockIdx.x * kFusedWaves + (i % kFusedWaves));
    };
    const unsigned long long all_tokens = M >= 64 ? ~0ull : ((1ull << M) - 1ull);
    auto describe = [&](int b, int& rid0, int& rid1, bool& has1, unsigned long long& bm) {
        if (DENSE) {
            rid0 = b * kFusedRows;
            has1 = rid0 + 1 < p.V;
            rid1 = has1 ? rid0 + 1 : rid0;
            bm = all_tokens;
        } else {
            while (b >= uni(uprefix[u + 1])) ++u;      // b < total_batches = uprefix[count]
            const int r0 = uni(ustart[u]) + (b - uni(uprefix[u])) * kFusedRows;
            has1 = r0 + 1 < uni(uend[u]);
            rid0 = p.rows[r0];
            rid1 = has1 ? p.rows[r0 + 1] : rid0;
            bm = uni64(umask[u]);
        }
    };
    // the first pair is fixed (i = wave), the others are drawn from the LDS counter
    // (With few tokens the dense head's consecutive rows stream fastest with 64 to 160 KB in
    // flight per compute unit rather than 256 KB: its waves beyond p.stream_waves sit out.)
    int b = LP ? draw_batch() : wave < p.stream_waves ? (int)(blockIdx.x * kFusedWaves + wave) : total_batches;
    int rid0 = 0, rid1 = 0;
    bool has1 = false;
    unsigned long long bm = 0ull;
    if (b < total_batches) describe(b, rid0, rid1, has1, bm);
    while (b < total_batches) {                        // wave-uniform
        rid0 = __builtin_amdgcn_readfirstlane(rid0);
        rid1 = __builtin_amdgcn_readfirstlane(rid1);
        uint4 w0[kFusedSegs], w1[kFusedSegs];
        const uint4* p0 = p.lm_W + (size_t)rid0 * p.n_vec;
        const uint4* p1 = p.lm_W + (size_t)rid1 * p.n_vec;
#pragma unroll
        for (int j = 0; j < kFusedSegs; ++j) {
            const int vec = j * kWave + lane;
            w0[j] = make_uint4(0, 0, 0, 0);
            w1[j] = make_uint4(0, 0, 0, 0);
            if (j < p.jp && vec < p.n_vec) {
                w0[j] = load_stream(p0 + vec);
                w1[j] = load_stream(p1 + vec);
            }
        }
        const int nb = draw_batch();
        int nrid0 = 0, nrid1 = 0;
        bool nhas1 = false;
        unsigned long long nbm = 0ull;
        if (nb < total_batches) describe(nb, nrid0, nrid1, nhas1, nbm);

        unsigned long long rem = bm;
        while (rem) {                                  // wave-uniform
            const int cnt = __popcll(rem);
            if (cnt >= 4)
                fused_tokens<DT, 4, LP>(p, hs, my_lists, collect_keys, collect_count, w0, w1, rem, rid0, rid1, has1, thr_v, thr_i,
                                        lse_m, lse_s);
            else if (cnt >= 2)
                fused_tokens<DT, 2, LP>(p, hs, my_lists, collect_keys, collect_count, w0, w1, rem, rid0, rid1, has1, thr_v, thr_i,
                                        lse_m, lse_s);
            else
                fused_tokens<DT, 1, LP>(p, hs, my_lists, collect_keys, collect_count, w0, w1, rem, rid0, rid1, has1, thr_v, thr_i,
                                        lse_m, lse_s);
        }
        if (LP && ((bm >> lane) & 1ull)) {             // token slot j of the group, pair b
            const int j = __popcll(bm & ((1ull << lane) - 1ull));
            const int at = j * lp_stride + (b - lp_origin);
            if (lp_in_lds)                             // uniform
                lds_pieces[at] = pack_lse(lse_m, lse_s);
            else
                __hip_atomic_store(lp_pieces + at, pack_lse(lse_m, lse_s), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        b = nb;
        rid0 = nrid0;
        rid1 = nrid1;
        has1 = nhas1;
        bm = nbm;
    }

    // ---- 5. merge the waves' lists, publish, last workgroup merges all
    __syncthreads();
    // the hidden vectors are no longer needed: their LDS is the merge scratch
    WaveScratch* ws = reinterpret_cast<WaveScratch*>(lds + lay.o_hidden) + wave;
    const int P = gridDim.x;
    // published lists are entry-major, part[(t*k + i)*P + workgroup]: the first entries of
    // all workgroups, which bound the result, are contiguous
    if (!LP && p.collect) {
        // The token's collected logits are ranked by counting (keys are distinct: distinct
        // ids; a key of zero is below every logit) and the k best published.  With fewer
        // tokens than waves, S waves share a token: each counts over a slice of the keys and
        // the token's first wave adds the counts up.
        const int S = M <= 1 ? 16 : M <= 2 ? 8 : M <= 4 ? 4 : M <= 8 ? 2 : 1;
        unsigned short* partial = reinterpret_cast<unsigned short*>(lds + lay.o_hidden);   // [wave][2][64]
        for (int base = 0; base < M; base += kFusedWaves / S) {    // block-uniform; one round if S > 1
            const int t = base + wave / S, slice = wave % S;
            const unsigned long long* keys = collect_keys + (size_t)(t < M ? t : 0) * kCollectCap;
            const int n = t < M ? min(uni(collect_count[t]), kCollectCap) : 0;
            const unsigned long long c0 = lane < n ? keys[lane] : 0ull;
            const unsigned long long c1 = lane + kWave < n ? keys[lane + kWave] : 0ull;
            const int per = (n + S - 1) / S;
            const int j1 = min(n, (slice + 1) * per);
            int r0 = 0, r1 = 0;
            if (n <= kWave) {                          // wave-uniform
#pragma unroll 8
                for (int j = slice * per; j < j1; ++j) r0 += keys[j] > c0 ? 1 : 0;
            } else {
#pragma unroll 8
                for (int j = slice * per; j < j1; ++j) {
                    const unsigned long long o = keys[j];
                    r0 += o > c0 ? 1 : 0;
                    r1 += o > c1 ? 1 : 0;
                }
            }
            if (S > 1) {                               // block-uniform
                partial[wave * 2 * kWave + lane] = (unsigned short)r0;
                partial[wave * 2 * kWave + kWave + lane] = (unsigned short)r1;
                __syncthreads();
                if (slice == 0)
                    for (int q = 1; q < S; ++q) {
                        r0 += partial[(wave + q) * 2 * kWave + lane];
                        r1 += partial[(wave + q) * 2 * kWave + kWave + lane];
                    }
            }
            if (t < M && slice == 0) {
                Cand* dst = p.part + (size_t)t * k * P + blockIdx.x;
                if (c0 != 0ull && r0 < k) publish_cand(dst + (size_t)r0 * P, key_value(c0), key_id(c0));
                if (c1 != 0ull && r1 < k) publish_cand(dst + (size_t)r1 * P, key_value(c1), key_id(c1));
                if (lane >= n && lane < k) publish_cand(dst + (size_t)lane * P, -INFINITY, INT_MAX);
            }
        }
    } else if (!LP) {
        for (int t = wave; t < M; t += kFusedWaves) {
            Cand* dst = p.part + (size_t)t * k * P + blockIdx.x;
            wave_merge_topk(
                kFusedWaves, k, lane, ws,
                [&](int l, int i) { return lists[((size_t)l * M + t) * k + i]; },
                [&](int r, Cand c) { publish_cand(dst + (size_t)r * P, c.v, c.id); });
        }
    } else {
        // the tokens of this workgroup's group only: their lists, ranked by logit (inside
        // a group that is the order of log p as well), and their log-sum-exp pieces
        unsigned long long rem = uni64(umask[u]);
        for (int idx = 0; rem; ++idx, rem &= rem - 1ull) {     // block-uniform
            if ((idx & (kFusedWaves - 1)) != wave) continue;
            const int t = __ffsll(rem) - 1;
            // the pieces of this workgroup's pairs for token slot idx, summed in pair order;
            // the first 256 are requested before the merge, which hides their latency
            const int q0 = idx * lp_stride + lp_lo - lp_origin + lane;
            const int q_end = idx * lp_stride + total_batches - lp_origin;
            auto piece_at = [&](int q) {
                return lp_in_lds ? lds_pieces[q]
                                 : __hip_atomic_load(lp_pieces + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            };
            unsigned long long early[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                early[c] = 0xff800000ull;              // (-inf, 0)
                if (q0 + c * kWave < q_end) early[c] = piece_at(q0 + c * kWave);
            }
            Cand* dst = p.part + (size_t)t * k * P + blockIdx.x;
            wave_merge_topk(
                kFusedWaves, k, lane, ws,
                [&](int l, int i) { return lists[((size_t)l * M + t) * k + i]; },
                [&](int r, Cand c) { publish_cand(dst + (size_t)r * P, c.v, c.id); });
            // (the maximum first, then every piece scaled to it: independent exponentials)
            float late_m = -INFINITY, late_s = 0.f;    // pairs beyond the first 256, if any
            for (int q = q0 + 4 * kWave; q < q_end; q += kWave) lse_take(late_m, late_s, piece_at(q));
            float wm = late_m;
#pragma unroll
            for (int c = 0; c < 4; ++c) wm = fmaxf(wm, __uint_as_float((unsigned)(early[c] & 0xffffffffull)));
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) wm = fmaxf(wm, __shfl_xor(wm, off));
            float mine_s = 0.f;
            if (wm > -INFINITY) {
#pragma unroll
                for (int c = 0; c < 4; ++c)            // ascending pair order
                    mine_s += __uint_as_float((unsigned)(early[c] >> 32)) *
                              expf(__uint_as_float((unsigned)(early[c] & 0xffffffffull)) - wm);
                mine_s += late_s * expf(late_m - wm);
            }
            const float tot = wave_sum(mine_s);
            if (lane == 0)
                __hip_atomic_store(p.lse_part + (size_t)t * P + blockIdx.x,
                                   pack_lse(wm, tot), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0): the published lists are out
    __syncthreads();
    if (LP) {
        // Eq. 8: log p(x) = log p_router(n) + z[x] - lse_n.  finish(t, gu) is one wave's work
        // for token t and its selected group ugroup[gu]: it combines the log-sum-exp pieces
        // of the group's workgroups, takes the router's log-softmax over all G scores, merges
        // the group's published lists by logit and leaves the k best, offset added, in its
        // lanes (lane r = rank r).
        Cand* mine = lists + (size_t)wave * M * k;     // the waves' lists are merged: free
        auto finish = [&](int t, int gu) {
            const int n = uni(ugroup[gu]);
            const int w0 = uni(wgstart[gu]);
            const int n_wg = uni(wgstart[gu + 1]) - w0;
            // the pieces are requested first and used after the merge, whose own loads
            // then share their trip to memory
            unsigned long long piece[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int l = c * kWave + lane;
                piece[c] = 0xff800000ull;              // (-inf, 0)
                if (l < n_wg)
                    piece[c] = __hip_atomic_load(p.lse_part + (size_t)t * P + w0 + l, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
            }
            const Cand* src = p.part + (size_t)t * k * P + w0;
            wave_merge_topk<4>(
                n_wg, k, lane, ws, [&](int l, int e) { return fetch_cand(src + (size_t)e * P + l); },
                [&](int r, Cand c) { mine[r] = c; });
            float bm = -INFINITY, bs = 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c) lse_take(bm, bs, piece[c]);   // ascending workgroup order
            const float lse_n = lse_finish(bm, bs);
            float rm = -INFINITY, rs = 0.f, s_n = 0.f;
            for (int o = lane; o < p.G; o += kWave) {
                float v = s_lds[t * p.G + o];
                if (!(v == v)) v = -INFINITY;
                if (o == n) s_n = v;
                const float nm = fmaxf(rm, v);
                if (nm > -INFINITY) rs = rs * expf(rm - nm) + expf(v - nm);
                rm = nm;
            }
            s_n = wave_sum(s_n);                       // one lane holds it, the others zero
            const float shift = (s_n - lse_finish(rm, rs)) - lse_n;
            Cand c = sentinel();
            if (lane < k) c = mine[lane];
            if (is_real(c)) c.v += shift;
            return c;
        };
        // Draft-level call: the results also go to a table of tree keys in LDS (the waves'
        // lists are no longer needed), from which the level is expanded below.
        const bool expand = p.next_parent != nullptr;  // uniform
        unsigned long long* tree_keys = reinterpret_cast<unsigned long long*>(lists);   // [M * k]
        int* tree_ids = reinterpret_cast<int*>(tree_keys + M * k);
        float* tree_scores = reinterpret_cast<float*>(tree_ids + M * k);
        auto write_result = [&](int t, int r, Cand c) {
            p.topk_ids[(size_t)t * k + r] = c.id;
            p.topk_logits[(size_t)t * k + r] = c.v;
            if (expand) {
                const int e = t * k + r;
                const float parent = p.parent_score ? p.parent_score[t] : 0.f;
                tree_keys[e] = tree_key(parent, c.v, is_real(c) ? c.id : -1, e);
                tree_ids[e] = c.id;
                tree_scores[e] = parent + c.v;
            }
        };
        auto expand_level = [&]() {                    // called by every thread of the workgroup
            if (!expand) return;
            __syncthreads();
            for (int m = wave; m < M; m += kFusedWaves) {
                int e;
                bool keep;
                const int rank = tree_rank_node(tree_keys, M, k, p.n_next, m, lane, e, keep);
                if (keep) {
                    p.next_parent[rank] = m;
                    p.next_token[rank] = tree_ids[e];
                    p.next_score[rank] = tree_scores[e];
                }
            }
            if (wave == 0) {
                int n_real = 0;
                for (int e = lane; e < M * k; e += kWave) n_real += tree_keys[e] != 0ull ? 1 : 0;
                n_real = wave_scan_inclusive(n_real);
                n_real = __builtin_amdgcn_readlane(n_real, 63);
                tree_pad(n_real, p.n_next, lane, p.next_parent, p.next_token, p.next_score);
            }
        };
        if (2 * M * p.g <= kFusedWaves) {
            // Few (token, group) pairs: the workgroup that arrives last takes them all, one
            // wave each, and merges every token's g lists through LDS (two hand-overs through
            // memory fewer than below; from about 16 pairs on the scheme below is faster).
            if (threadIdx.x == 0) {
                const unsigned int old = __hip_atomic_fetch_add(p.counter, 1u, __ATOMIC_RELAXED,
                                                                __HIP_MEMORY_SCOPE_AGENT);
                flags[1] = old == gridDim.x - 1 ? 1 : 0;
            }
            __syncthreads();
            if (!uni(flags[1])) return;                // block-uniform
            const int count = uni(flags[0]);
            Cand* glists = reinterpret_cast<Cand*>(lds + lay.o_keys);   // [M * g, k], <= 16 x 64 entries
            if (wave < M * p.g) {
                const int n = uni(sel_lds[wave]);
                const int gu = __ffsll(__ballot(lane < count && ugroup[lane] == n)) - 1;
                const Cand c = finish(wave / p.g, gu);
                if (lane < k) glists[wave * k + lane] = c;
            }
            __syncthreads();
            if (wave < M) {
                const Cand* src = glists + (size_t)wave * p.g * k;
                wave_merge_topk(
                    p.g, k, lane, ws, [&](int l, int e) { return src[l * k + e]; },
                    [&](int r, Cand c) { write_result(wave, r, c); });
            }
            expand_level();
            if (threadIdx.x == 0)                      // ready for the next call
                __hip_atomic_store(p.counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        // More pairs than waves: the workgroup of a group that arrives last (a counter per
        // activated group) finishes the group, one wave per token that selected it, and
        // publishes the lists; the group that finishes last (one more counter) merges every
        // token's g lists.  The groups' last workgroups work side by side, most of them
        // while other groups still stream.
        unsigned int* group_counter = p.counter + kLpGroupCounters + u;
        if (threadIdx.x == 0) {
            const unsigned int old = __hip_atomic_fetch_add(group_counter, 1u, __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT);
            flags[1] = old == (unsigned)lp_nwg - 1u ? 1 : 0;
        }
        __syncthreads();
        if (!uni(flags[1])) return;                    // block-uniform
        if (threadIdx.x == 0)                          // ready for the next call
            __hip_atomic_store(group_counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int n = uni(ugroup[u]);
        unsigned long long rem = uni64(umask[u]);
        for (int idx = 0; rem; ++idx, rem &= rem - 1ull) {     // block-uniform
            if ((idx & (kFusedWaves - 1)) != wave) continue;
            const int t = __ffsll(rem) - 1;
            const int i = __ffsll(__ballot(lane < p.g && sel_lds[t * p.g + lane] == n)) - 1;
            const Cand c = finish(t, u);
            if (lane < k) publish_cand(p.glist + ((size_t)t * p.g + i) * k + lane, c.v, c.id);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): the group's lists are out
        __syncthreads();
        if (threadIdx.x == 0) {
            const unsigned int old = __hip_atomic_fetch_add(p.counter, 1u, __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT);
            flags[1] = old == (unsigned)uni(flags[0]) - 1u ? 1 : 0;
        }
        __syncthreads();
        if (!uni(flags[1])) return;                    // block-uniform
        for (int t = wave; t < M; t += kFusedWaves) {
            const Cand* src = p.glist + (size_t)t * p.g * k;
            wave_merge_topk(
                p.g, k, lane, ws, [&](int l, int e) { return fetch_cand(src + l * k + e); },
                [&](int r, Cand c) { write_result(t, r, c); });
        }
        expand_level();
        if (threadIdx.x == 0)
            __hip_atomic_store(p.counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    if (threadIdx.x == 0) {
        const unsigned int old = __hip_atomic_fetch_add(p.counter, 1u, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
        flags[1] = old == gridDim.x - 1 ? 1 : 0;
    }
    __syncthreads();
    if (!uni(flags[1])) return;                        // block-uniform

    // Last workgroup: one wave per token merges the P published lists.
    for (int t = wave; t < M; t += kFusedWaves) {
        const Cand* src = p.part + (size_t)t * k * P;
        wave_merge_topk(
            P, k, lane, ws,
            [&](int l, int i) { return fetch_cand(src + (size_t)i * P + l); },
            [&](int r, Cand c) {
                p.topk_ids[(size_t)t * k + r] = c.id;
                p.topk_logits[(size_t)t * k + r] = c.v;
            });
    }
    if (threadIdx.x == 0)                              // ready for the next call
        __hip_atomic_store(p.counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void k_zero_words(unsigned int* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

}  // namespace
