// Matrix-core path for groups that many tokens selected (wide draft-tree steps) and for
// the dense head with many tokens: the logits of a block of 128 weight rows for up to 64
// tokens are 16x16 tiles of v_mfma_f32_16x16x32_bf16.
//
// One persistent workgroup of 8 waves per compute unit; wave = (row group rg = wave/2: 32
// rows = two row tiles, half kq = wave%2 of every 512-column chunk).  Per block of 128
// rows of one group:
//   - the weight rows go from HBM into registers in whole 128-byte lines (a wave load
//     covers 8 rows x 128 B), and pairs of such registers go through a wave-private LDS
//     slice into the MFMA A operands of two 32-column steps; 16 KB per wave in flight,
//     the next block's first 16 loads issued before this block's epilogue;
//   - the hidden vectors of the tokens that selected the group are staged chunk by chunk
//     (512 columns, double buffered) in LDS and read as B operands, each fragment used for
//     both row tiles of the wave;
//   - the two half sums of each tile are added in a fixed order through LDS, which
//     leaves, per token, the block's 128 logits two per lane of a wave; those that beat the
//     token's current k-th are merged into the workgroup's running list by rank counting.
// Each workgroup publishes its lists; a second small kernel merges them per token.
// The logits row is never written to memory.
#pragma once
#include "device_utils.h"
#include "fused_path.h"
#include <type_traits>

namespace {

constexpr int kTileWaves = 8;
constexpr int kTileSplit = 2;                    // waves that share a row group (split of a chunk)
constexpr int kTileBlock = kTileWaves * kWave;
constexpr int kTileRows = 128;                   // weight rows per block (4 row groups of 32)
constexpr int kChunkVecs = 64;                   // 16-byte vectors per 512-column chunk
constexpr int kHbStride = kChunkVecs + 1;        // LDS row stride in vectors (pad: no bank conflicts)
constexpr int kHbBufVecs = 64 * kHbStride;       // one staging buffer: 64 token slots
constexpr int kTileMaxK = 64;                    // a list occupies the lanes of one wave
constexpr int kRing = 16;                        // weight loads of a wave per chunk = ring size
// Strides (floats) of the accumulator tiles parked in LDS for the epilogue: token tile,
// row tile of a wave, wave.  Modulo the 64 banks they are 16, 16 and 48.
constexpr int kRedCt = 272, kRedTile = 4 * kRedCt + 16, kRedWave = 2 * kRedTile + 16;
static_assert(kTileWaves * kRedWave * 4 <= 2 * kHbBufVecs * 16, "the parked tiles fit the staging buffers");
// Compiler-only barrier: no memory access is moved across it.  Keeps global loads at the
// place in the instruction stream where the source puts them (the compiler would otherwise
// sink them to their first use, which defeats prefetching).
__device__ __forceinline__ void keep_memory_order() { asm volatile("" ::: "memory"); }

// One activated group as the gate kernel hands it to the tile kernel: a single read per
// group instead of a chain of dependent ones (list -> masks and offsets -> prefix).
struct TileGroup {
    int32_t group, start, end;              // rows group_rows[start, end)
    int32_t first_block;                    // blocks of the groups before it
    unsigned long long mask;                // tokens that selected it
};

struct TileParams {
    const uint4* hidden;                    // [M, n_vec]
    const uint4* lm_W;                      // [V, n_vec]
    const int32_t* offsets;                 // [G+1]   (grouped)
    const int32_t* rows;                    // [V]     (grouped)
    const struct TileGroup* table;          // [G]     (grouped) activated groups in working order
    const int32_t* n_union;                 // [1]     (grouped) how many
    Cand* part;                             // [M, k, gridDim.x] published lists, entry-major
    unsigned int* next_block;               // block queue: zero before the launch
    int M, V, G, k;
    int n_vec, n_chunks;
    int u_max;                              // capacity of the activated-group arrays
    // Log-probability mode (Eq. 8 normalises per group, and a block is rows of one group):
    // every block leaves, per token that selected its group, the k best of its rows by logit
    // and the (max, sum of exp) of its logits, slot = the block's number in the working order.
    Cand* blk_part;                         // [M, blk_stride, k]
    float* blk_lse;                         // [M, blk_stride, 2]
    int blk_stride;
};

struct TileLds {
    int o_hbuf, o_lists, o_rowid, o_tokslot, o_scratch, o_ugroup, o_ustart, o_uend, o_uprefix,
        o_umask, o_flags, total;
};

__host__ __device__ inline TileLds tile_lds_layout(int M, int k, int u_max) {
    TileLds L;
    int off = 0;
    auto take = [&](size_t bytes) {
        int at = off;
        off = (int)((off + bytes + 15) / 16 * 16);
        return at;
    };
    L.o_hbuf = take((size_t)2 * kHbBufVecs * sizeof(uint4));
    L.o_lists = take((size_t)M * k * sizeof(Cand));
    L.o_rowid = take(kTileRows * sizeof(int));
    L.o_tokslot = take(64 * sizeof(int));
    L.o_scratch = take((size_t)kTileWaves * kLinePairSlots * sizeof(uint4));
    L.o_ugroup = take((size_t)u_max * sizeof(int));
    L.o_ustart = take((size_t)u_max * sizeof(int));
    L.o_uend = take((size_t)u_max * sizeof(int));
    L.o_uprefix = take((size_t)(u_max + 1) * sizeof(int));
    L.o_umask = take((size_t)u_max * sizeof(unsigned long long));
    L.o_flags = take(16);
    L.total = off;
    return L;
}

// Merges a block's logits of one token (one per lane, padding = sentinel) into the
// token's sorted list in LDS.  Only candidates that beat the list's k-th entry take part.
// Every participant's new rank is counted directly: a candidate's rank is the number of
// list entries and of other candidates that beat it, a list entry moves down by the number
// of candidates that beat it.  Ranks are distinct, so all writes go to distinct slots.
// keys: 128 wave-private 64-bit LDS words (ordering keys of the passing candidates, then of the list).
__device__ __forceinline__ void tile_merge_token(Cand* list, int k, int lane, Cand c,
                                                 unsigned long long* keys) {
    const Cand tail = list[k - 1];                     // one address for all lanes: a broadcast
    const bool pass = is_real(c) && better(c.v, c.id, tail.v, tail.id);
    const unsigned long long b = __ballot(pass);
    if (b == 0ull) return;                             // wave-uniform, the common case
    Cand e = sentinel();
    if (lane < k) e = list[lane];
    const int np = __popcll(b);
    const int kr = __popcll(__ballot(lane < k && is_real(e)));   // real entries are a prefix
    const unsigned long long ckey = cand_key(c.v, c.id), ekey = cand_key(e.v, e.id);
    unsigned long long* ckeys = keys;
    unsigned long long* lkeys = keys + kWave;
    if (pass) ckeys[__popcll(b & ((1ull << lane) - 1ull))] = ckey;
    if (lane < kr) lkeys[lane] = ekey;
    int rc = count_above(lkeys, kr, ckey), re = lane;
#pragma unroll 4
    for (int j = 0; j < np; ++j) {                     // wave-uniform
        const unsigned long long o = ckeys[j];
        rc += o > ckey ? 1 : 0;
        re += o > ekey ? 1 : 0;
    }
    if (pass && rc < k) list[rc] = c;
    if (lane < kr && re < k) list[re] = e;
}

// The candidate an ordering key was made from (cand_key's inverse; -0.0 comes back as +0.0).
__device__ __forceinline__ Cand cand_from_key(unsigned long long key) {
    const unsigned o = (unsigned)(key >> 32);
    Cand c;
    c.v = __uint_as_float((o >> 31) ? (o ^ 0x80000000u) : ~o);
    c.id = (int)~(unsigned)key;
    return c;
}

// The two halves of a block's logits of one token (two candidates per lane) go into the
// token's sorted list in LDS.  Candidates that do not beat the list's k-th entry drop out
// first (the common case: none is left).  While the list is short, or early in the stream,
// most candidates pass; the k-th largest of the lanes' better candidates then bounds the
// result from below (k candidates reach it), and only candidates that reach it (ties kept)
// stay.  The survivors' keys are compacted, one per lane; then one pass over them gives
// every survivor its final position (list entries above it + survivors above it, two
// ballots) and moves every list entry down by the number of survivors above it.
// keys: 128 wave-private 64-bit LDS words, keys32: 64 more 32-bit words.
__device__ __forceinline__ void tile_merge_pair(Cand* list, int k, int lane, Cand c0, Cand c1,
                                                unsigned long long* keys, unsigned* keys32) {
    const Cand tail = list[k - 1];                     // a broadcast
    bool p0 = is_real(c0) && better(c0.v, c0.id, tail.v, tail.id);
    bool p1 = is_real(c1) && better(c1.v, c1.id, tail.v, tail.id);
    unsigned long long b0 = __ballot(p0), b1 = __ballot(p1);
    if ((b0 | b1) == 0ull) return;                     // wave-uniform, the common case
    if ((int)(__popcll(b0) + __popcll(b1)) > k + (k >> 1)) {  // wave-uniform
        const unsigned o0 = p0 ? ord32(c0.v) : 0u, o1 = p1 ? ord32(c1.v) : 0u;
        const unsigned tau = wave_kth_key(keys32, o0 > o1 ? o0 : o1, kWave, k, lane);
        p0 = p0 && o0 >= tau;
        p1 = p1 && o1 >= tau;
        b0 = __ballot(p0);
        b1 = __ballot(p1);
    }
    const int n0 = __popcll(b0), np = n0 + __popcll(b1);
    if (np > kWave) {                                  // ties at the bound: one half at a time
        if (!p0) c0 = sentinel();
        if (!p1) c1 = sentinel();
        tile_merge_token(list, k, lane, c0, keys);
        tile_merge_token(list, k, lane, c1, keys);
        return;
    }
    const unsigned long long below = (1ull << lane) - 1ull;
    if (p0) keys[__popcll(b0 & below)] = cand_key(c0.v, c0.id);
    if (p1) keys[n0 + __popcll(b1 & below)] = cand_key(c1.v, c1.id);
    Cand e = sentinel();
    if (lane < k) e = list[lane];
    const int kr = __popcll(__ballot(lane < k && is_real(e)));   // real entries are a prefix
    const bool is_e = lane < kr;
    // lanes without an entry (a survivor) hold key 0, which is above nothing
    const unsigned long long ekey = is_e ? cand_key(e.v, e.id) : 0ull;
    const unsigned long long ckey = lane < np ? keys[lane] : 0ull;
    int re = lane;
    unsigned long long placed = 0ull;
    for (int j = 0; j < np; ++j) {                     // wave-uniform
        const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)ckey, j);
        const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(ckey >> 32), j);
        const unsigned long long kj = ((unsigned long long)hi << 32) | lo;
        const bool e_above = ekey > kj;
        const int rank = __popcll(__ballot(e_above)) + __popcll(__ballot(ckey > kj));
        re += (is_e && !e_above) ? 1 : 0;              // keys are distinct
        if (lane == rank) placed = kj;
    }
    if (is_e && re != lane && re < k) list[re] = e;
    if (placed != 0ull && lane < k) list[lane] = cand_from_key(placed);
}

// One 512-column chunk of a block's K loop for NCT token tiles (a compile-time count: no
// branch inside a chunk, so that LDS reads, matrix instructions and loads of neighbouring
// steps interleave).  REFILL: a next chunk exists; its weight lines refill the ring slots as
// they are consumed.  Its hidden vectors are requested at the top of the chunk, before those
// refills, and written to the other staging buffer only in the chunk's last step pair: loads
// complete in order, and the requests are younger than all 16 weight lines of this chunk, so
// an earlier write would wait for lines that are not needed yet (and were requested least
// long ago), while by the last step pair all of them have been consumed anyway.
struct TileStage {                                     // staging registers, 2 NCT in use
    uint4 r0, r1, r2, r3, r4, r5, r6, r7;
};

template <int NCT>
__device__ __forceinline__ void tile_fetch_hidden(const TileParams& p, const int* tokslot, int n_t,
                                                  TileStage& hst, int c, int lane, int wave) {
    constexpr int kN = 2 * NCT;
    const uint4* src = p.hidden + c * kChunkVecs + lane;
    // token of slot wave + 8 i (wave-uniform); slots past the group's tokens repeat its last
    auto tok = [&](int i) {
        const int s = wave + i * kTileWaves;
        return (size_t)uni(tokslot[s < n_t ? s : n_t - 1]);
    };
    if (kN > 0) hst.r0 = load_vec(src + tok(0) * p.n_vec);
    if (kN > 1) hst.r1 = load_vec(src + tok(1) * p.n_vec);
    if (kN > 2) hst.r2 = load_vec(src + tok(2) * p.n_vec);
    if (kN > 3) hst.r3 = load_vec(src + tok(3) * p.n_vec);
    if (kN > 4) hst.r4 = load_vec(src + tok(4) * p.n_vec);
    if (kN > 5) hst.r5 = load_vec(src + tok(5) * p.n_vec);
    if (kN > 6) hst.r6 = load_vec(src + tok(6) * p.n_vec);
    if (kN > 7) hst.r7 = load_vec(src + tok(7) * p.n_vec);
}
template <int NCT>
__device__ __forceinline__ void tile_store_hidden(const TileStage& hst, uint4* hbuf, int c, int lane,
                                                  int wave) {
    constexpr int kN = 2 * NCT;
    uint4* dst = hbuf + (size_t)(c & 1) * kHbBufVecs + (size_t)wave * kHbStride + lane;
    if (kN > 0) store_vec(dst + 0 * kTileWaves * kHbStride, hst.r0);
    if (kN > 1) store_vec(dst + 1 * kTileWaves * kHbStride, hst.r1);
    if (kN > 2) store_vec(dst + 2 * kTileWaves * kHbStride, hst.r2);
    if (kN > 3) store_vec(dst + 3 * kTileWaves * kHbStride, hst.r3);
    if (kN > 4) store_vec(dst + 4 * kTileWaves * kHbStride, hst.r4);
    if (kN > 5) store_vec(dst + 5 * kTileWaves * kHbStride, hst.r5);
    if (kN > 6) store_vec(dst + 6 * kTileWaves * kHbStride, hst.r6);
    if (kN > 7) store_vec(dst + 7 * kTileWaves * kHbStride, hst.r7);
}

// The 128-byte line of step pair sp of chunk c in the lane's row at byte offset `row` of
// the weight matrix (offsets are 32-bit: the path takes matrices below 4 GiB).
__device__ __forceinline__ uint4 tile_load_w(const TileParams& p, unsigned row, int c, int sp) {
    const unsigned off = row + (unsigned)(c * kChunkVecs + sp * 8) * 16u;
    return load_stream(reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(p.lm_W) + off));
}

// Step pair SP of a chunk: the two 32-column steps whose weight lines sit in ring slots
// 4 SP .. 4 SP + 3.
template <int DT, int NCT, bool REFILL, int SP>
__device__ __forceinline__ void tile_step_pair(const TileParams& p, int c, uint4 (&a)[kRing],
                                               f32x4_t (&acc)[2][4], const unsigned (&wrow)[4],
                                               uint4* hbuf, TileStage& hst, uint4* my_slice) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int r16 = lane & 15, q4 = lane >> 4;
    const int kq = wave % kTileSplit;
    const uint4* hb = hbuf + (size_t)(c & 1) * kHbBufVecs;
    uint4 op[2][2];                                    // [row tile][step of the pair]
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        mfma_operands_from_lines(a[SP * 4 + 2 * t], a[SP * 4 + 2 * t + 1], lane, my_slice, op[t][0],
                                 op[t][1]);
        if (REFILL) {                                  // refill the two slots just consumed
            a[SP * 4 + 2 * t] = tile_load_w(p, wrow[2 * t], c + 1, SP);
            a[SP * 4 + 2 * t + 1] = tile_load_w(p, wrow[2 * t + 1], c + 1, SP);
        }
    }
    if (REFILL) keep_memory_order();
    if (REFILL && SP == 3) {                           // the other buffer is free since the last barrier
        tile_store_hidden<NCT>(hst, hbuf, c + 1, lane, wave);
        keep_memory_order();
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
        const int off = (kq * 8 + 2 * SP + s2) * 4 + q4;
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            const uint4 hv = hb[(ct * 16 + r16) * kHbStride + off];
#pragma unroll
            for (int t = 0; t < 2; ++t)
                acc[t][ct] = mfma_tile<DT>(op[t][s2], hv, acc[t][ct]);
        }
    }
}

template <int DT, int NCT, bool REFILL>
__device__ __forceinline__ void tile_chunk(const TileParams& p, int c, uint4 (&a)[kRing],
                                           f32x4_t (&acc)[2][4], const unsigned (&wrow)[4],
                                           uint4* hbuf, const int* tokslot, int n_t, uint4* my_slice) {
    TileStage hst;
    // (the scheduling barriers keep the compiler from sinking the loads to where their
    // registers are first needed, which would undo the ordering)
    if (REFILL) {
        tile_fetch_hidden<NCT>(p, tokslot, n_t, hst, c + 1, threadIdx.x & (kWave - 1),
                               __builtin_amdgcn_readfirstlane(threadIdx.x / kWave));
        keep_memory_order();
    }
    tile_step_pair<DT, NCT, REFILL, 0>(p, c, a, acc, wrow, hbuf, hst, my_slice);
    tile_step_pair<DT, NCT, REFILL, 1>(p, c, a, acc, wrow, hbuf, hst, my_slice);
    tile_step_pair<DT, NCT, REFILL, 2>(p, c, a, acc, wrow, hbuf, hst, my_slice);
    tile_step_pair<DT, NCT, REFILL, 3>(p, c, a, acc, wrow, hbuf, hst, my_slice);
    __syncthreads();
}

// The K loop of one block.  Hidden chunk staging: slots wave, wave + 8, ... below 16 NCT;
// lane = vector inside the chunk; slots past the group's tokens repeat its last token
// (their columns of the tiles are never read back).
template <int DT, int NCT>
__device__ __forceinline__ void tile_k_loop(const TileParams& p, uint4 (&a)[kRing], f32x4_t (&acc)[2][4],
                                            const unsigned (&wrow)[4], uint4* hbuf,
                                            const int* tokslot, uint4* my_slice, int n_t) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    {
        TileStage hst;
        tile_fetch_hidden<NCT>(p, tokslot, n_t, hst, 0, lane, wave);
        tile_store_hidden<NCT>(hst, hbuf, 0, lane, wave);
    }
    __syncthreads();
    for (int c = 0; c + 1 < p.n_chunks; ++c)
        tile_chunk<DT, NCT, true>(p, c, a, acc, wrow, hbuf, tokslot, n_t, my_slice);
    tile_chunk<DT, NCT, false>(p, p.n_chunks - 1, a, acc, wrow, hbuf, tokslot, n_t, my_slice);
}

template <int DT, bool LP = false>
__global__ __launch_bounds__(kTileBlock) void k_tiles(TileParams p, int dense) {
    extern __shared__ uint4 smem[];
    char* lds = reinterpret_cast<char*>(smem);
    const TileLds lay = tile_lds_layout(p.M, p.k, p.u_max);
    uint4* hbuf = reinterpret_cast<uint4*>(lds + lay.o_hbuf);
    Cand* lists = reinterpret_cast<Cand*>(lds + lay.o_lists);
    int* rowid = reinterpret_cast<int*>(lds + lay.o_rowid);
    int* tokslot = reinterpret_cast<int*>(lds + lay.o_tokslot);
    int* ugroup = reinterpret_cast<int*>(lds + lay.o_ugroup);
    int* ustart = reinterpret_cast<int*>(lds + lay.o_ustart);
    int* uend = reinterpret_cast<int*>(lds + lay.o_uend);
    int* uprefix = reinterpret_cast<int*>(lds + lay.o_uprefix);
    unsigned long long* umask = reinterpret_cast<unsigned long long*>(lds + lay.o_umask);
    int* flags = reinterpret_cast<int*>(lds + lay.o_flags);

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int rg = wave / kTileSplit, kq = wave % kTileSplit;
    const int M = p.M, k = p.k;
    uint4* my_slice = reinterpret_cast<uint4*>(lds + lay.o_scratch) + (size_t)wave * kLinePairSlots;

    // Blocks cost very different amounts (one to four token tiles), so they are handed
    // out from a queue, most expensive groups first, rather than dealt round robin.
    unsigned int drawn = 0u;
    if (threadIdx.x == 0)
        drawn = __hip_atomic_fetch_add(p.next_block, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int i = threadIdx.x; i < M * k; i += kTileBlock) lists[i] = sentinel();
    int total_blocks;
    if (dense) {
        total_blocks = (p.V + kTileRows - 1) / kTileRows;
        if (threadIdx.x == 0) flags[1] = (int)drawn;
        __syncthreads();
    } else {
        if (wave == 0) {
            // the count and the table rows are requested together (rows past the count are
            // stale but inside the table, which has u_max rows)
            const int count = *p.n_union;
            for (int u = lane; u < p.u_max; u += kWave) {
                const TileGroup tg = p.table[u];
                if (u < count) {
                    ugroup[u] = tg.group;
                    umask[u] = tg.mask;
                    ustart[u] = tg.start;
                    uend[u] = tg.end;
                    uprefix[u] = tg.first_block;
                    if (u == count - 1)
                        uprefix[count] = tg.first_block + (tg.end - tg.start + kTileRows - 1) / kTileRows;
                }
            }
            if (lane == 0) {                           // LDS is in order within a wave
                if (count == 0) uprefix[0] = 0;
                flags[0] = count;
                flags[1] = (int)drawn;
            }
        }
        __syncthreads();
        total_blocks = uni(uprefix[uni(flags[0])]);
    }

    const unsigned long long all_tokens = M >= 64 ? ~0ull : ((1ull << M) - 1ull);
    int u = 0;
    // first row and end of the block's group (row indices into p.rows, or vocabulary ids)
    auto locate = [&](int b, int& first, int& end, unsigned long long& bm) {
        if (dense) {
            first = b * kTileRows;
            end = p.V;
            bm = all_tokens;
        } else {
            while (b >= uni(uprefix[u + 1])) ++u;      // blocks come in increasing order
            first = uni(ustart[u]) + (b - uni(uprefix[u])) * kTileRows;
            end = uni(uend[u]);
            bm = uni64(umask[u]);
        }
    };
    // This lane's four weight rows: row (lane / 8) of each 8-row octet o of the wave's 32
    // rows (clamped inside the group; the duplicates are dropped when the candidates are
    // formed).
    auto my_rows = [&](int first, int end, int (&rid)[4]) {
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            int idx = first + rg * 32 + o * 8 + line_load_row(lane);
            if (idx >= end) idx = end - 1;
            rid[o] = dense ? idx : p.rows[idx];
        }
    };
    // Ring slot sp * 4 + o holds, of the current chunk, octet o's 128-byte line of the step
    // pair sp (steps kq * 8 + 2 sp and + 1 of the chunk).  H is a multiple of 512 on this
    // path, so every chunk is whole and the loads need no guards.
    uint4 a[kRing];
    unsigned wrow[4];                                  // byte offsets of this lane's rows at its place in a chunk
    auto set_rows = [&](const int (&rid)[4]) {
#pragma unroll
        for (int o = 0; o < 4; ++o)
            wrow[o] = ((unsigned)rid[o] * (unsigned)p.n_vec + kq * 32 + line_load_chunk(lane)) * 16u;
    };
    auto load_a = [&](int c, int sp, int o) { a[sp * 4 + o] = tile_load_w(p, wrow[o], c, sp); };

    int b = uni(flags[1]);
    int first = 0, end = 0;
    unsigned long long bm = 0ull;
    int rid[4] = {0, 0, 0, 0};
    if (b < total_blocks) {
        locate(b, first, end, bm);
        my_rows(first, end, rid);
        set_rows(rid);
#pragma unroll
        for (int sp = 0; sp < 4; ++sp)
#pragma unroll
            for (int o = 0; o < 4; ++o) load_a(0, sp, o);
    }
    while (b < total_blocks) {                         // block-uniform
        if (threadIdx.x == 0)                          // the draw returns long before the K loop ends
            drawn = __hip_atomic_fetch_add(p.next_block, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int n_t = __popcll(bm);
        const int n_ct = (n_t + 15) >> 4;
        // token of every slot, and the vocabulary id of every row of the block
        if (wave == 0) {
            const bool on = (bm >> lane) & 1ull;
            if (on) tokslot[__popcll(bm & ((1ull << lane) - 1ull))] = lane;
        }
        if (wave == 1 || wave == 2) {
            const int j = (wave - 1) * kWave + lane;
            const int idx = first + j;
            rowid[j] = idx < end ? (dense ? idx : p.rows[idx]) : -1;
        }
        __syncthreads();

        f32x4_t acc[2][4];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) acc[t][ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        switch (n_ct) {                                    // block-uniform
            case 1: tile_k_loop<DT, 1>(p, a, acc, wrow, hbuf, tokslot, my_slice, n_t); break;
            case 2: tile_k_loop<DT, 2>(p, a, acc, wrow, hbuf, tokslot, my_slice, n_t); break;
            case 3: tile_k_loop<DT, 3>(p, a, acc, wrow, hbuf, tokslot, my_slice, n_t); break;
            default: tile_k_loop<DT, 4>(p, a, acc, wrow, hbuf, tokslot, my_slice, n_t); break;
        }

        // next block: locate it and start its first 16 weight loads before the epilogue
        // (flags[1] was last read before this block's barriers)
        if (threadIdx.x == 0) flags[1] = (int)drawn;
        __syncthreads();
        const int nb = uni(flags[1]);
        int nfirst = 0, nend = 0;
        unsigned long long nbm = 0ull;
        if (nb < total_blocks) {
            locate(nb, nfirst, nend, nbm);
            my_rows(nfirst, nend, rid);
            set_rows(rid);
#pragma unroll
            for (int sp = 0; sp < 4; ++sp)
#pragma unroll
                for (int o = 0; o < 4; ++o) load_a(0, sp, o);
        }

        // half sums -> LDS (over the staging buffers, free after the last barrier).  A
        // tile's accumulators sit at lane * 4 plus 4 floats of padding per 16 lanes, and the
        // strides between tiles are chosen so that the reads below, whose 64 lanes want one
        // column of four different tiles, fall on 64 different banks.
        float* red = reinterpret_cast<float*>(hbuf);
        const int red_lane = lane * 4 + (lane >> 4) * 4;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int ct = 0; ct < 4; ++ct)
                if (ct < n_ct)
                    *reinterpret_cast<f32x4_t*>(red + wave * kRedWave + t * kRedTile + ct * kRedCt + red_lane) =
                        acc[t][ct];
        __syncthreads();
        // one wave per token slot, the block's rows in two halves of 64: lane = (row tile,
        // row) -> 64 logits of the token
        auto slot_logits = [&](int s, Cand (&cand)[2]) {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int tile = hf * 4 + (lane >> 4), row = lane & 15;   // row tile 0..7 of the block
                const int e = (row >> 2) * 68 + (s & 15) * 4 + (row & 3);
                const int w0 = (tile >> 1) * kTileSplit;                  // the row group's first wave
                float z = 0.f;
#pragma unroll
                for (int q = 0; q < kTileSplit; ++q)
                    z += red[(w0 + q) * kRedWave + (tile & 1) * kRedTile + (s >> 4) * kRedCt + e];
                cand[hf].v = z;
                cand[hf].id = rowid[hf * kWave + lane];
                if (cand[hf].id < 0) cand[hf] = sentinel();
            }
        };
        if (LP) {
            // this block's share of the group's log-sum-exp for every token (a pass of its own:
            // the merge below has no registers to spare), and fresh lists: the block's k best
            // are its own (the tokens' LDS lists are scratch here)
            for (int s = wave; s < n_t; s += kTileWaves) {
                const int tok = tokslot[s];
                Cand cand[2];
                slot_logits(s, cand);
                const float z0 = is_real(cand[0]) ? cand[0].v : -INFINITY;
                const float z1 = is_real(cand[1]) ? cand[1].v : -INFINITY;
                float wm = fmaxf(z0, z1);
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) wm = fmaxf(wm, __shfl_xor(wm, off));
                const float tot = wave_sum(wm > -INFINITY ? expf(z0 - wm) + expf(z1 - wm) : 0.f);
                if (lane < 2) p.blk_lse[uni(tok * p.blk_stride + b) * 2 + lane] = lane ? tot : wm;
                if (lane < k) lists[tok * k + lane] = sentinel();
            }
        }
        for (int s = wave; s < n_t; s += kTileWaves) {
            const int tok = tokslot[s];
            Cand cand[2];
            slot_logits(s, cand);
            tile_merge_pair(lists + (size_t)tok * k, k, lane, cand[0], cand[1],
                            reinterpret_cast<unsigned long long*>(my_slice),
                            reinterpret_cast<unsigned*>(my_slice) + 4 * kWave);
            if (LP && lane < k)
                p.blk_part[uni(tok * p.blk_stride + b) * k + lane] = lists[tok * k + lane];
        }
        __syncthreads();
        b = nb;
        first = nfirst;
        end = nend;
        bm = nbm;
    }

    if (LP) return;                                    // (every block has left its own lists)
    // publish the workgroup's lists (all tokens; untouched ones are padding)
    const int P = gridDim.x;
    for (int i = threadIdx.x; i < M * k; i += kTileBlock) {
        const Cand c = lists[i];
        p.part[(size_t)i * P + blockIdx.x] = c;        // i = t*k + entry
    }
}

// Gate and selection for the tile path (Eq. 7's W2 projection, then top-g): one workgroup
// per tile of 16 groups x 16 tokens, the columns split over its 16 waves in steps of 32
// (MFMA operands straight from memory: lane l feeds row l%16, 8 columns at 8*(l/16));
// the partial tiles are summed in wave order.  The workgroup that finishes last ranks
// every token's scores by counting and writes the selection, the token mask of every
// group and the ascending list of activated groups.
struct GateSelParams {
    const uint4* hidden;                    // [M, n_vec]
    const uint4* gate_W;                    // [G, n_vec]
    const float* bias;                      // [G] or null
    float* s;                               // [M, G] scores (workspace)
    int32_t* sel;                           // [M, g]
    unsigned long long* group_mask;         // [G]
    const int32_t* offsets;                 // [G+1] row ranges of the groups
    TileGroup* table;                       // [G] out: activated groups in working order
    int32_t* n_union;                       // [1]
    unsigned int* counter;                  // arrival counter, zero between calls
    int M, G, g, n_vec;
    // log-probability mode (G <= 64, M * g <= kGateSelMaxPairs), else null:
    int32_t* first_block;                   // [M, g] out: first block of the selected group
    int32_t* block_count;                   // [M, g] out: how many blocks it has
    float* logp_sel;                        // [M, g] out: log p_router of the selected group
};
constexpr int kGateSelMaxPairs = 1024;

__device__ __forceinline__ float load_score(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int DT>
__global__ __launch_bounds__(kFusedBlock) void k_gate_select(GateSelParams p) {
    __shared__ __attribute__((aligned(16))) float part[kFusedWaves][kGateSlice];
    __shared__ unsigned long long mask[kMaxG];
    __shared__ unsigned long long sel_keys[kFusedWaves][kWave];
    __shared__ int ulist[kMaxG];
    __shared__ int order[kMaxG], nblk[kMaxG];
    __shared__ int is_last, ucount;
    __shared__ int off_lds[kMaxG + 1];
    __shared__ int rank_of[kMaxG];
    __shared__ int sel_lds[kGateSelMaxPairs];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    // the groups' row ranges travel with the first operand loads (requested here, put into LDS
    // after the contraction): the workgroup that ends up building the table then has them
    // without two more dependent trips to memory
    int off_r0 = 0, off_r1 = 0;
    if ((int)threadIdx.x <= p.G) off_r0 = p.offsets[threadIdx.x];
    if ((int)threadIdx.x + kFusedBlock <= p.G) off_r1 = p.offsets[threadIdx.x + kFusedBlock];
    const int n_tt = (p.M + 15) / 16;
    const int gt = blockIdx.x / n_tt, tt = blockIdx.x - gt * n_tt;
    float bias_r = 0.f;                                // (likewise: the bias of the score this thread will sum)
    if (threadIdx.x < 256 && p.bias) {
        const int gn = gt * 16 + ((threadIdx.x >> 2) >> 4) * 4 + (threadIdx.x & 3);
        if (gn < p.G) bias_r = p.bias[gn];
    }
    const int n_ks = (p.n_vec + 3) / 4;
    const int n = gt * 16 + mfma_load_row(lane), m = tt * 16 + mfma_load_row(lane);
    f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int ks0 = wave; ks0 < n_ks; ks0 += kFusedWaves * 8) {      // wave-uniform
        uint4 a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int ks = ks0 + kFusedWaves * i;
            const int vec = ks * 4 + mfma_load_chunk(lane);
            a[i] = make_uint4(0, 0, 0, 0);
            b[i] = make_uint4(0, 0, 0, 0);
            if (ks < n_ks && vec < p.n_vec) {
                if (n < p.G) a[i] = p.gate_W[(size_t)n * p.n_vec + vec];
                if (m < p.M) b[i] = p.hidden[(size_t)m * p.n_vec + vec];
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc = mfma_tile<DT>(mfma_operand_from_quads(a[i], lane, reinterpret_cast<uint4*>(part[wave])),
                                mfma_operand_from_quads(b[i], lane, reinterpret_cast<uint4*>(part[wave])), acc);
    }
    *reinterpret_cast<f32x4_t*>(&part[wave][lane * 4]) = acc;
    if ((int)threadIdx.x <= p.G) off_lds[threadIdx.x] = off_r0;
    if ((int)threadIdx.x + kFusedBlock <= p.G) off_lds[threadIdx.x + kFusedBlock] = off_r1;
    __syncthreads();
    if (threadIdx.x < 256) {
        const int e = threadIdx.x, l = e >> 2, i = e & 3;
        const int gn = gt * 16 + (l >> 4) * 4 + i;
        const int tm = tt * 16 + (l & 15);
        float sum = 0.f;
        for (int w = 0; w < kFusedWaves; ++w) sum += part[w][e];
        if (gn < p.G && tm < p.M)
            __hip_atomic_store(p.s + (size_t)tm * p.G + gn, sum + bias_r,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0): the scores are out
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int old = __hip_atomic_fetch_add(p.counter, 1u, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
        is_last = old == gridDim.x - 1 ? 1 : 0;
    }
    __syncthreads();
    if (!uni(is_last)) return;                         // block-uniform

    for (int g0 = threadIdx.x; g0 < p.G; g0 += kFusedBlock) mask[g0] = 0ull;
    __syncthreads();
    if (p.G <= kWave) {
        // one wave per token, group in lane; the scores of all the wave's tokens (up to four:
        // M <= 64) are requested together, so that the selection costs one trip to memory
        float sv[kMaxM / kFusedWaves];
#pragma unroll
        for (int j = 0; j < kMaxM / kFusedWaves; ++j) {
            const int tm = wave + j * kFusedWaves;
            sv[j] = (tm < p.M && lane < p.G) ? load_score(p.s + (size_t)tm * p.G + lane) : -INFINITY;
        }
#pragma unroll
        for (int j = 0; j < kMaxM / kFusedWaves; ++j) {
            const int tm = wave + j * kFusedWaves;
            if (tm >= p.M) break;                           // wave-uniform
            float v = sv[j];
            if (!(v == v)) v = -INFINITY;
            const int rank = wave_rank(sel_keys[wave], v, lane, p.G, lane);
            float lse_s = 0.f;
            if (p.logp_sel) {                               // the router's softmax over all G scores (Eq. 7)
                const float smax = wave_max(v);
                lse_s = smax + logf(wave_sum(lane < p.G ? expf(v - smax) : 0.f));
            }
            if (lane < p.G && rank < p.g) {
                atomicOr(&mask[lane], 1ull << tm);
                p.sel[tm * p.g + rank] = lane;
                if (p.logp_sel) {
                    p.logp_sel[tm * p.g + rank] = v - lse_s;
                    sel_lds[tm * p.g + rank] = lane;
                }
            }
        }
    } else {
        for (int idx = threadIdx.x; idx < p.M * p.G; idx += kFusedBlock) {
            const int tm = idx / p.G;
            const int gn = idx - tm * p.G;
            const float* row = p.s + (size_t)tm * p.G;
            float v = load_score(row + gn);
            if (!(v == v)) v = -INFINITY;
            int rank = 0;
            for (int o = 0; o < p.G; ++o) {
                float ov = load_score(row + o);
                if (!(ov == ov)) ov = -INFINITY;
                rank += better(ov, o, v, gn) ? 1 : 0;
            }
            if (rank < p.g) {
                atomicOr(&mask[gn], 1ull << tm);
                p.sel[tm * p.g + rank] = gn;
            }
        }
    }
    __syncthreads();
    for (int g0 = threadIdx.x; g0 < p.G; g0 += kFusedBlock) p.group_mask[g0] = mask[g0];
    if (wave == 0) {
        int count = 0;
        for (int base = 0; base < p.G; base += kWave) {
            const int g0 = base + lane;
            const bool on = g0 < p.G && mask[g0] != 0ull;
            const unsigned long long b = __ballot(on);
            if (on) ulist[count + __popcll(b & ((1ull << lane) - 1ull))] = g0;
            count += __popcll(b);
        }
        if (lane == 0) {
            ucount = count;
            *p.n_union = count;
            __hip_atomic_store(p.counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
    // The activated groups in the order the tile kernel works through them: most token
    // tiles (16 tokens each) first, then ascending group id; placed by rank counting.  The
    // table row of each carries its row range, token mask and the number of blocks before it.
    const int count = uni(ucount);
    if (count <= kWave) {
        // a group has one to four token tiles (M <= 64): four ballots place it
        if (wave == 0) {
            const int g0 = lane < count ? ulist[lane] : 0;
            const int w0 = lane < count ? (__popcll(mask[g0]) + 15) >> 4 : 0;
            int rank = 0;
#pragma unroll
            for (int w = 4; w >= 1; --w) {
                const unsigned long long b = __ballot(w0 == w);
                if (w0 < w) rank += __popcll(b);
                if (w0 == w) rank += __popcll(b & ((1ull << lane) - 1ull));
            }
            if (lane < count) {
                order[rank] = g0;
                rank_of[g0] = rank;
                nblk[rank] = (off_lds[g0 + 1] - off_lds[g0] + kTileRows - 1) / kTileRows;
            }
        }
    } else {
        for (int u0 = threadIdx.x; u0 < count; u0 += kFusedBlock) {
            const int g0 = ulist[u0];
            const int w0 = (__popcll(mask[g0]) + 15) >> 4;
            int rank = 0;
            for (int v = 0; v < count; ++v) {
                const int wv = (__popcll(mask[ulist[v]]) + 15) >> 4;
                rank += (wv > w0 || (wv == w0 && v < u0)) ? 1 : 0;
            }
            order[rank] = g0;
            rank_of[g0] = rank;
            nblk[rank] = (off_lds[g0 + 1] - off_lds[g0] + kTileRows - 1) / kTileRows;
        }
    }
    __syncthreads();
    if (wave == 0) {
        int carry = 0;
        for (int base = 0; base < count; base += kWave) {  // wave-uniform
            const int r = base + lane;
            const int nb = r < count ? nblk[r] : 0;
            const int incl = wave_scan_inclusive(nb);
            if (r < count) {
                const int g0 = order[r];
                TileGroup tg;
                tg.group = g0;
                tg.start = off_lds[g0];
                tg.end = off_lds[g0 + 1];
                tg.first_block = carry + incl - nb;
                tg.mask = mask[g0];
                p.table[r] = tg;
            }
            if (p.first_block && r < count) {
                nblk[r] = carry + incl - nb;            // (now: blocks before it)
                ulist[r] = nb;                          // (the list of activated groups is spent)
            }
            carry += __builtin_amdgcn_readlane(incl, 63);
        }
    }
    if (p.first_block) {                               // block-uniform
        __syncthreads();
        for (int idx = threadIdx.x; idx < p.M * p.g; idx += kFusedBlock)
        {
            const int r = rank_of[sel_lds[idx]];
            p.first_block[idx] = nblk[r];
            p.block_count[idx] = ulist[r];
        }
    }
}

// Per token, merges the P published lists part[(t*k + i)*P + w] into the result.
__global__ __launch_bounds__(256) void k_merge_published(const Cand* __restrict__ part, int P, int M,
                                                         int k, int32_t* __restrict__ topk_ids,
                                                         float* __restrict__ topk_logits,
                                                         unsigned int* next_block) {
    if (blockIdx.x == 0 && threadIdx.x == 0)           // the tile kernel's queue, for the next call
        __hip_atomic_store(next_block, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __shared__ WaveScratch scratch_all[4];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int t = blockIdx.x * 4 + wave;
    if (t >= M) return;                                // wave-uniform, no barriers below
    const Cand* src = part + (size_t)t * k * P;
    wave_merge_topk(
        P, k, lane, scratch_all + wave,
        [&](int l, int i) { return src[(size_t)i * P + l]; },
        [&](int r, Cand c) {
            topk_ids[(size_t)t * k + r] = c.id;
            topk_logits[(size_t)t * k + r] = c.v;
        });
}

}  // namespace
