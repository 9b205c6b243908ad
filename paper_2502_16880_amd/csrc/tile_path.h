// Matrix-core path for groups that many tokens selected (wide draft-tree steps) and for
// the dense head with many tokens: the logits of a block of 128 weight rows for up to 64
// tokens are 16x16 tiles of v_mfma_f32_16x16x32_bf16.
//
// k_tiles: one persistent workgroup of 8 waves per compute unit; wave = (row group rg =
// wave/2: 32 rows = two row tiles, half kq = wave%2 of every 512-column chunk).  Per block of
// 128 rows of one group:
//   - the weight rows go from HBM into registers in whole 128-byte lines (a wave load
//     covers 8 rows x 128 B), and pairs of such registers go through a wave-private LDS
//     slice into the MFMA A operands of two 32-column steps; 16 KB per wave in flight,
//     the next block's first 16 loads issued before this block's epilogue;
//   - the hidden vectors of the tokens that selected the group are staged chunk by chunk
//     (512 columns, double buffered) in LDS and read as B operands, each fragment used for
//     both row tiles of the wave;
//   - the two half sums of each tile are added in a fixed order through LDS, which
//     leaves, per token, the block's 128 logits two per lane of a wave; they go to memory as
//     they are, 512 bytes per (block, token), with the largest of them (and the sum of exp in
//     the log-probability mode): a few MB per step against the hundreds of MB of weight rows,
//     and the workgroup is back in its next block's K loop within a few microseconds.
// k_gate_select in front of it: gate and selection per tile of 16 tokens.  k_tile_select behind
// it: one workgroup per token bounds the token's k-th logit by the k-th largest block maximum,
// reads the logits of the blocks that reach the bound and ranks them (Eq. 8's offsets added
// per group in the log-probability mode).
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
constexpr int kRing = 16;                        // weight loads of a wave per chunk = ring size
constexpr int kGateParts = 2;                    // workgroups that share the columns of a gate tile
// Strides (floats) of the accumulator tiles parked in LDS for the epilogue: token tile,
// row tile of a wave, wave.  Modulo the 64 banks they are 16, 16 and 48.
constexpr int kRedCt = 272, kRedTile = 4 * kRedCt + 16, kRedWave = 2 * kRedTile + 16;
static_assert(kTileWaves * kRedWave * 4 <= 2 * kHbBufVecs * 16, "the parked tiles fit the staging buffers");
// Compiler-only barrier: no memory access is moved across it.  Keeps global loads at the
// place in the instruction stream where the source puts them (the compiler would otherwise
// sink them to their first use, which defeats prefetching).
__device__ __forceinline__ void keep_memory_order() { asm volatile("" ::: "memory"); }

struct TileParams {
    const uint4* hidden;                    // [M, n_vec]
    const uint4* lm_W;                      // [V, n_vec]
    const int32_t* rows;                    // [V]     (grouped)
    const int32_t* offsets;                 // [G+1]   (grouped)
    const unsigned long long* tile_mask;    // [token tiles, G] (grouped) what k_gate_select left
    unsigned long long* group_mask;         // [G] out (grouped): tokens that selected the group
    int32_t* group_first_block;             // [G] out (grouped): first block of an activated group
    float* z;                               // [blocks, M, 128] out: logits of (block, token slot)
    float2* stat;                           // [blocks, M] out: the slot's largest logit, and in the
                                            // log-probability mode the sum of exp(z - largest)
    int want_lse;
    unsigned int* next_block;               // block queue: zero before the launch
    int M, V, G;
    int n_vec, n_chunks;
    int u_max;                              // capacity of the activated-group arrays
};

struct TileLds {
    int o_hbuf, o_tokslot, o_scratch, o_ustart, o_uend, o_uprefix, o_umask, o_flags, total;
};

__host__ __device__ inline TileLds tile_lds_layout(int u_max) {
    TileLds L;
    int off = 0;
    auto take = [&](size_t bytes) {
        int at = off;
        off = (int)((off + bytes + 15) / 16 * 16);
        return at;
    };
    L.o_hbuf = take((size_t)2 * kHbBufVecs * sizeof(uint4));
    L.o_tokslot = take(64 * sizeof(int));
    L.o_scratch = take((size_t)kTileWaves * kLinePairSlots * sizeof(uint4));
    L.o_ustart = take((size_t)u_max * sizeof(int));
    L.o_uend = take((size_t)u_max * sizeof(int));
    L.o_uprefix = take((size_t)(u_max + 1) * sizeof(int));
    L.o_umask = take((size_t)u_max * sizeof(unsigned long long));
    L.o_flags = take(16);
    L.total = off;
    return L;
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

template <int DT>
__global__ __launch_bounds__(kTileBlock) void k_tiles(TileParams p, int dense) {
    extern __shared__ uint4 smem[];
    char* lds = reinterpret_cast<char*>(smem);
    const TileLds lay = tile_lds_layout(p.u_max);
    uint4* hbuf = reinterpret_cast<uint4*>(lds + lay.o_hbuf);
    int* tokslot = reinterpret_cast<int*>(lds + lay.o_tokslot);
    int* ustart = reinterpret_cast<int*>(lds + lay.o_ustart);
    int* uend = reinterpret_cast<int*>(lds + lay.o_uend);
    int* uprefix = reinterpret_cast<int*>(lds + lay.o_uprefix);
    unsigned long long* umask = reinterpret_cast<unsigned long long*>(lds + lay.o_umask);
    int* flags = reinterpret_cast<int*>(lds + lay.o_flags);

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int rg = wave / kTileSplit, kq = wave % kTileSplit;
    const int M = p.M;
    uint4* my_slice = reinterpret_cast<uint4*>(lds + lay.o_scratch) + (size_t)wave * kLinePairSlots;

    // Blocks cost different amounts (one to four token tiles), so they are handed out from
    // a queue, most expensive groups first, rather than dealt round robin.
    unsigned int drawn = 0u;
    if (threadIdx.x == 0)
        drawn = __hip_atomic_fetch_add(p.next_block, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int total_blocks;
    if (dense) {
        total_blocks = (p.V + kTileRows - 1) / kTileRows;
        if (threadIdx.x == 0) flags[1] = (int)drawn;
        __syncthreads();
    } else {
        // The activated groups in the order the workgroups go through them: most token
        // tiles first (a block costs more the more tokens it serves), then ascending group id;
        // each with its row range, token mask and the number of blocks before it.  Every
        // workgroup builds the same table; the scratch arrays lie over the staging buffers,
        // which are free until the first K loop.
        unsigned long long* gmask = reinterpret_cast<unsigned long long*>(hbuf);      // [G]
        int* off_lds = reinterpret_cast<int*>(gmask + p.G);                            // [G + 1]
        int* ulist = off_lds + p.G + 1;                                                // [G]
        int* order = ulist + p.G;                                                      // [G]
        const int n_tt = (M + 15) / 16;
        for (int g0 = threadIdx.x; g0 <= p.G; g0 += kTileBlock) {
            off_lds[g0] = p.offsets[g0];
            if (g0 < p.G) {
                unsigned long long mk = 0ull;
                for (int c = 0; c < n_tt; ++c) mk |= p.tile_mask[(size_t)c * p.G + g0];
                gmask[g0] = mk;
                if (blockIdx.x == 0) p.group_mask[g0] = mk;
            }
        }
        __syncthreads();
        if (wave == 0) {
            int count = 0;
            for (int base = 0; base < p.G; base += kWave) {    // wave-uniform
                const int g0 = base + lane;
                const bool on = g0 < p.G && gmask[g0] != 0ull;
                const unsigned long long bal = __ballot(on);
                if (on) ulist[count + __popcll(bal & ((1ull << lane) - 1ull))] = g0;
                count += __popcll(bal);
            }
            if (count <= kWave) {
                // a group has one to four token tiles (M <= 64): four ballots place it
                const int g0 = lane < count ? ulist[lane] : 0;
                const int w0 = lane < count ? (__popcll(gmask[g0]) + 15) >> 4 : 0;
                int rank = 0;
#pragma unroll
                for (int w = 4; w >= 1; --w) {
                    const unsigned long long bal = __ballot(w0 == w);
                    if (w0 < w) rank += __popcll(bal);
                    if (w0 == w) rank += __popcll(bal & ((1ull << lane) - 1ull));
                }
                if (lane < count) order[rank] = g0;
            } else {
                // (many groups: ascending id; the order only balances the load)
                for (int r = lane; r < count; r += kWave) order[r] = ulist[r];
            }
            int carry = 0;
            for (int base = 0; base < count; base += kWave) {  // wave-uniform
                const int r = base + lane;
                const int g0 = r < count ? order[r] : 0;
                const int nb = r < count ? (off_lds[g0 + 1] - off_lds[g0] + kTileRows - 1) / kTileRows : 0;
                const int incl = wave_scan_inclusive(nb);
                if (r < count) {
                    ustart[r] = off_lds[g0];
                    uend[r] = off_lds[g0 + 1];
                    uprefix[r] = carry + incl - nb;
                    umask[r] = gmask[g0];
                    if (blockIdx.x == 0) p.group_first_block[g0] = carry + incl - nb;
                }
                carry += __builtin_amdgcn_readlane(incl, 63);
            }
            if (lane == 0) {                           // LDS is in order within a wave
                uprefix[count] = carry;
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
    // rows (clamped inside the group; the logits of the duplicates are never read).
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
        if (wave == 0) {                               // token of every slot
            const bool on = (bm >> lane) & 1ull;
            if (on) tokslot[__popcll(bm & ((1ull << lane) - 1ull))] = lane;
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
        // row) -> 64 logits of the slot, 256 consecutive bytes of the block's logits
        // and the slot's largest logit (rows past the group's end do not count): the ranking
        // kernel reads the logits only of blocks whose largest can matter.  Log-probability
        // mode: the sum of exp(z - largest) as well, the block's piece of the group's lse.
        for (int s = wave; s < n_t; s += kTileWaves) {
            float* dst = p.z + ((size_t)b * M + s) * kTileRows + lane;
            float zs[2];
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int tile = hf * 4 + (lane >> 4), row = lane & 15;   // row tile 0..7 of the block
                const int e = (row >> 2) * 68 + (s & 15) * 4 + (row & 3);
                const int w0 = (tile >> 1) * kTileSplit;                  // the row group's first wave
                float z = 0.f;
#pragma unroll
                for (int q = 0; q < kTileSplit; ++q)
                    z += red[(w0 + q) * kRedWave + (tile & 1) * kRedTile + (s >> 4) * kRedCt + e];
                dst[hf * kWave] = z;
                zs[hf] = first + hf * kWave + lane < end ? z : -INFINITY;
            }
            const float wm = wave_max(fmaxf(zs[0], zs[1]));
            float sum = 0.f;
            if (p.want_lse)                            // block-uniform
                sum = wave_sum(wm > -INFINITY ? expf(zs[0] - wm) + expf(zs[1] - wm) : 0.f);
            if (lane == 0) p.stat[(size_t)b * M + s] = make_float2(wm, sum);
        }
        __syncthreads();
        b = nb;
        first = nfirst;
        end = nend;
        bm = nbm;
    }
}

// Gate and selection for the tile path (Eq. 7's W2 projection, then top-g): one workgroup
// per tile of 16 groups x 16 tokens and half of the columns (two workgroups share a tile: 32
// compute units pull the operands instead of 16), the columns split over its 16 waves in
// blocks of 128 (256 bytes of a row: both operands are loaded four rows x 256 bytes per wave
// load and transposed in registers); the partial tiles are summed in wave order and the two workgroups' sums by
// whoever reads the scores, in a fixed order.  The workgroups of one token tile count
// themselves in on that tile's counter; the one that arrives last has all scores of its 16
// tokens and ranks them by counting, one wave per token, writes the selection and, per
// group, the mask of those of its tokens that selected it.  The tile kernel combines the
// token tiles' masks itself, so the token tiles finish independently of each other.
struct GateSelParams {
    const uint4* hidden;                    // [M, n_vec]
    const uint4* gate_W;                    // [G, n_vec]
    const float* bias;                      // [G] or null
    float* s;                               // [parts, M, G] scores (workspace)
    int32_t* sel;                           // [M, g]
    unsigned long long* tile_mask;          // [token tiles, G] out: tokens of the tile that selected the group
    unsigned int* counters;                 // [token tiles] arrival counters, zero between calls
    int M, G, g, n_vec;
    float* logp_sel;                        // [M, g] out: log p_router of the selected group
                                            // (log-probability mode, G <= 64), else null
};

__device__ __forceinline__ float load_score(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int DT>
__global__ __launch_bounds__(kFusedBlock) void k_gate_select(GateSelParams p) {
    __shared__ __attribute__((aligned(16))) float part[kFusedWaves][kGateTileFloats];
    __shared__ unsigned long long mask[kMaxG];
    __shared__ unsigned long long sel_keys[kFusedWaves][kWave];
    __shared__ int is_last;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int n_tt = (p.M + 15) / 16, n_gt = (p.G + 15) / 16;
    const int gt = blockIdx.x / n_tt, tt = blockIdx.x - gt * n_tt;
    float bias_r = 0.f;                                // the bias of the score this thread will sum
    if (threadIdx.x < 256 && p.bias) {
        const int gn = gt * 16 + ((threadIdx.x >> 2) >> 4) * 4 + (threadIdx.x & 3);
        if (gn < p.G) bias_r = p.bias[gn];
    }
    // A wave takes 256-byte blocks of the columns (every kFusedWaves * n_parts-th), two per
    // pass with all loads requested before the first is used: per block four wave loads of
    // four rows x 256 contiguous bytes for each operand, transposed in registers to the
    // operands of four 32-column steps (mfma_operands_from_quad_rows).
    const int q4 = lane >> 4, a4 = (lane >> 2) & 3, c4 = lane & 3;
    f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const int cpart = blockIdx.y, n_parts = gridDim.y;              // the columns are split over n_parts workgroups
    const int n_blk = (p.n_vec + 15) / 16, bstride = kFusedWaves * n_parts;
    for (int blk0 = cpart * kFusedWaves + wave; blk0 < n_blk; blk0 += 2 * bstride) {     // wave-uniform
        uint4 a[2][4], b[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int vec = (blk0 + u * bstride) * 16 + q4 * 4 + c4;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int n = gt * 16 + a4 * 4 + t, m = tt * 16 + a4 * 4 + t;
                a[u][t] = make_uint4(0, 0, 0, 0);
                b[u][t] = make_uint4(0, 0, 0, 0);
                if (vec < p.n_vec) {
                    if (n < p.G) a[u][t] = p.gate_W[(size_t)n * p.n_vec + vec];
                    if (m < p.M) b[u][t] = p.hidden[(size_t)m * p.n_vec + vec];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (blk0 + u * bstride >= n_blk) break;        // wave-uniform
            mfma_operands_from_quad_rows(a[u][0], a[u][1], a[u][2], a[u][3], lane);
            mfma_operands_from_quad_rows(b[u][0], b[u][1], b[u][2], b[u][3], lane);
#pragma unroll
            for (int c = 0; c < 4; ++c) acc = mfma_tile<DT>(a[u][c], b[u][c], acc);
        }
    }
    *reinterpret_cast<f32x4_t*>(&part[wave][lane * 4]) = acc;
    __syncthreads();
    if (threadIdx.x < 256) {
        const int e = threadIdx.x, l = e >> 2, i = e & 3;
        const int gn = gt * 16 + (l >> 4) * 4 + i;
        const int tm = tt * 16 + (l & 15);
        float sum = 0.f;
        for (int w = 0; w < kFusedWaves; ++w) sum += part[w][e];
        if (gn < p.G && tm < p.M)
            __hip_atomic_store(p.s + ((size_t)cpart * p.M + tm) * p.G + gn, cpart == 0 ? sum + bias_r : sum,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0): the scores are out
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int old = __hip_atomic_fetch_add(p.counters + tt, 1u, __ATOMIC_RELAXED,
                                                        __HIP_MEMORY_SCOPE_AGENT);
        is_last = old == (unsigned)(n_gt * n_parts - 1) ? 1 : 0;
    }
    __syncthreads();
    if (!uni(is_last)) return;                         // block-uniform

    // the token tile is complete: its tokens tt * 16 .. + 15; a score is the sum of its parts in order
    auto score = [&](int tm, int gn) {
        float v = load_score(p.s + (size_t)tm * p.G + gn);
        for (int q = 1; q < n_parts; ++q) v += load_score(p.s + ((size_t)q * p.M + tm) * p.G + gn);
        return v;
    };
    for (int g0 = threadIdx.x; g0 < p.G; g0 += kFusedBlock) mask[g0] = 0ull;
    __syncthreads();
    if (p.G <= kWave) {
        // one wave per token, group in lane
        const int tm = tt * 16 + wave;
        if (wave < 16 && tm < p.M) {                   // wave-uniform
            float v = lane < p.G ? score(tm, lane) : -INFINITY;
            if (!(v == v)) v = -INFINITY;
            const int rank = wave_rank(sel_keys[wave], v, lane, p.G, lane);
            float lse_s = 0.f;
            if (p.logp_sel) {                          // the router's softmax over all G scores (Eq. 7)
                const float smax = wave_max(v);
                lse_s = smax + logf(wave_sum(lane < p.G ? expf(v - smax) : 0.f));
            }
            if (lane < p.G && rank < p.g) {
                atomicOr(&mask[lane], 1ull << tm);
                p.sel[tm * p.g + rank] = lane;
                if (p.logp_sel) p.logp_sel[tm * p.g + rank] = v - lse_s;
            }
        }
    } else {
        const int n_tok = p.M - tt * 16 < 16 ? p.M - tt * 16 : 16;
        for (int idx = threadIdx.x; idx < n_tok * p.G; idx += kFusedBlock) {
            const int tm = tt * 16 + idx / p.G;
            const int gn = idx - (idx / p.G) * p.G;
            float v = score(tm, gn);
            if (!(v == v)) v = -INFINITY;
            int rank = 0;
            for (int o = 0; o < p.G; ++o) {
                float ov = score(tm, o);
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
    for (int g0 = threadIdx.x; g0 < p.G; g0 += kFusedBlock) p.tile_mask[(size_t)tt * p.G + g0] = mask[g0];
    if (threadIdx.x == 0)
        __hip_atomic_store(p.counters + tt, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Ranking behind k_tiles: one workgroup per token.  Its blocks are those of the groups it
// selected (dense: all), and k_tiles left every block's largest logit.  The k-th largest of
// these block maxima is a lower bound of the token's k-th logit (k blocks hold a logit that
// reaches it), so only blocks whose largest reaches it can hold a result: about k of them,
// out of 128 (wide draft tree) or a thousand (dense).  Their logits, 32 blocks (4096
// candidates, eight per thread) at a time, are filtered by the bound and by the k-th entry
// of the list so far, collected in LDS with the list, and ranked by counting (64-bit
// ordering keys, all distinct).  Should more than 512 pass (equal logits, adversarial
// inputs), the k-th largest of each wave's lanes' best keys and the largest of these eight
// is a second bound that leaves at most 8 (8 (k - 1) + 1).
// Log-probability mode (Eq. 8): log p(x) = log p_router(n) + z[x] - lse_n; lse_n comes from
// the (largest, sum of exp) pieces k_tiles left per block, combined in block order, and
// bounds and keys are formed from z + (log p_router(n) - lse_n).
struct TileSelectParams {
    const float* z;                         // [blocks, M, 128] what k_tiles left
    const float2* stat;                     // [blocks, M]
    const int32_t* sel;                     // [M, g] selected groups (grouped)
    const int32_t* offsets;                 // [G+1]
    const int32_t* rows;                    // [V]
    const int32_t* group_first_block;       // [G] first block of an activated group
    const unsigned long long* group_mask;   // [G] tokens that selected it
    const float* logp_sel;                  // [M, g] log p_router (log-probability mode)
    unsigned int* next_block;               // k_tiles' queue: left at zero for the next call
    int32_t* topk_ids;                      // [M, k]
    float* topk_out;                        // [M, k]
    int M, V, g, k;
    int max_blocks;                         // capacity of the per-block arrays in LDS
};

constexpr int kSelectThreads = 512;
constexpr int kSelectWaves = kSelectThreads / kWave;
constexpr int kSelectKeys = 8;                   // candidates per thread and chunk
constexpr int kSelectChunkBlocks = kSelectKeys * kSelectThreads / kTileRows;
constexpr int kKeptMax = kSelectKeys * kSelectThreads + kMaxK;   // a chunk's candidates and the list

struct TileSelectLds {
    int o_buf, o_list, o_wkeys, o_start, o_rows, o_fb, o_slot, o_nb, o_pre, o_shift, o_bst, o_binfo,
        o_bval, o_qblk, o_qval, total;
};
__host__ __device__ inline TileSelectLds tile_select_lds_layout(int n_groups, int max_blocks) {
    TileSelectLds L;
    int off = 0;
    auto take = [&](size_t bytes) {
        int at = off;
        off = (int)((off + bytes + 15) / 16 * 16);
        return at;
    };
    L.o_buf = take((size_t)kKeptMax * sizeof(unsigned long long));
    L.o_list = take((size_t)kMaxK * sizeof(unsigned long long));
    L.o_wkeys = take((size_t)kSelectThreads * sizeof(unsigned long long));
    L.o_start = take((size_t)n_groups * sizeof(int));
    L.o_rows = take((size_t)n_groups * sizeof(int));
    L.o_fb = take((size_t)n_groups * sizeof(int));
    L.o_slot = take((size_t)n_groups * sizeof(int));
    L.o_nb = take((size_t)n_groups * sizeof(int));
    L.o_pre = take((size_t)(n_groups + 1) * sizeof(int));
    L.o_shift = take((size_t)n_groups * sizeof(float));
    L.o_bst = take((size_t)max_blocks * sizeof(float2));
    L.o_binfo = take((size_t)max_blocks * sizeof(int));
    L.o_bval = take((size_t)max_blocks * sizeof(unsigned));
    L.o_qblk = take((size_t)max_blocks * sizeof(int));
    L.o_qval = take((size_t)max_blocks * sizeof(unsigned));
    L.total = off;
    return L;
}

// wave_kth_key for all 64 lanes with the keys read four at a time (keys32 16-byte aligned).
__device__ __forceinline__ unsigned wave_kth_key4(unsigned* keys32, unsigned key, int k, int lane) {
    keys32[lane] = key;
    int above = 0;
#pragma unroll 4
    for (int j = 0; j < kWave / 4; ++j) {
        const uint4 q = reinterpret_cast<const uint4*>(keys32)[j];
        above += (q.x > key ? 1 : 0) + (q.y > key ? 1 : 0) + (q.z > key ? 1 : 0) + (q.w > key ? 1 : 0);
    }
    return wave_min_u32(above < k ? key : 0xffffffffu);
}

template <bool DENSE, bool LP>
__global__ __launch_bounds__(kSelectThreads) void k_tile_select(TileSelectParams p) {
    extern __shared__ uint4 smem[];
    char* lds = reinterpret_cast<char*>(smem);
    const int n_groups = DENSE ? 1 : p.g;
    const TileSelectLds lay = tile_select_lds_layout(n_groups, p.max_blocks);
    unsigned long long* buf = reinterpret_cast<unsigned long long*>(lds + lay.o_buf);
    unsigned long long* list = reinterpret_cast<unsigned long long*>(lds + lay.o_list);
    unsigned long long* wkeys = reinterpret_cast<unsigned long long*>(lds + lay.o_wkeys);
    int* g_start = reinterpret_cast<int*>(lds + lay.o_start);
    int* g_rows = reinterpret_cast<int*>(lds + lay.o_rows);
    int* g_fb = reinterpret_cast<int*>(lds + lay.o_fb);
    int* g_slot = reinterpret_cast<int*>(lds + lay.o_slot);
    int* g_nb = reinterpret_cast<int*>(lds + lay.o_nb);
    int* g_pre = reinterpret_cast<int*>(lds + lay.o_pre);
    float* g_shift = reinterpret_cast<float*>(lds + lay.o_shift);
    float2* bst = reinterpret_cast<float2*>(lds + lay.o_bst);
    int* binfo = reinterpret_cast<int*>(lds + lay.o_binfo);
    int* qblk = reinterpret_cast<int*>(lds + lay.o_qblk);
    unsigned* bval = reinterpret_cast<unsigned*>(lds + lay.o_bval);
    unsigned* qval = reinterpret_cast<unsigned*>(lds + lay.o_qval);
    __shared__ unsigned long long bound_w[kSelectWaves];
    __shared__ unsigned tau_w[kSelectWaves];
    __shared__ int n_kept, n_qual;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int t = blockIdx.x, k = p.k;
    if (blockIdx.x == 0 && threadIdx.x == 0)
        __hip_atomic_store(p.next_block, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (threadIdx.x == 0) {
        n_kept = 0;
        n_qual = 0;
    }

    // 1. the token's groups: row range, first block, the token's slot in the group's blocks
    if (DENSE) {
        if (threadIdx.x == 0) {
            g_start[0] = 0;
            g_rows[0] = p.V;
            g_fb[0] = 0;
            g_slot[0] = t;
            g_nb[0] = (p.V + kTileRows - 1) / kTileRows;
            g_shift[0] = 0.f;
        }
    } else {
        for (int j = threadIdx.x; j < p.g; j += kSelectThreads) {
            const int grp = p.sel[t * p.g + j];
            const int lo = p.offsets[grp], hi = p.offsets[grp + 1];
            const unsigned long long mk = p.group_mask[grp];
            g_start[j] = lo;
            g_rows[j] = hi - lo;
            g_fb[j] = p.group_first_block[grp];
            g_slot[j] = __popcll(mk & ((1ull << t) - 1ull));
            g_nb[j] = (hi - lo + kTileRows - 1) / kTileRows;
            g_shift[j] = 0.f;
        }
    }
    __syncthreads();
    if (wave == 0) {                                   // blocks before each group, in the token's order
        int carry = 0;
        for (int base = 0; base < n_groups; base += kWave) {   // wave-uniform
            const int j = base + lane;
            const int nb = j < n_groups ? g_nb[j] : 0;
            const int incl = wave_scan_inclusive(nb);
            if (j < n_groups) g_pre[j] = carry + incl - nb;
            carry += __builtin_amdgcn_readlane(incl, kWave - 1);
        }
        if (lane == 0) g_pre[n_groups] = carry;
    }
    __syncthreads();
    const int n_blocks = uni(g_pre[n_groups]);         // <= max_blocks: the groups are distinct

    // 2. the blocks' statistics, one block per thread and trip
    for (int i = threadIdx.x; i < n_blocks; i += kSelectThreads) {
        int lo = 0, hi = n_groups;                     // the group j with g_pre[j] <= i < g_pre[j + 1]
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (g_pre[mid] <= i) lo = mid; else hi = mid;
        }
        const int lb = i - g_pre[lo];
        binfo[i] = (lo << 16) | lb;
        const float2 st = p.stat[(size_t)(g_fb[lo] + lb) * p.M + g_slot[lo]];
        if (LP) bst[i] = st;
        else bval[i] = ord32(st.x);                    // (no offsets: the block's largest logit as it is)
    }
    __syncthreads();
    if (LP) {
        // lse of every group from its blocks' pieces, a wave per group (block in lane); the
        // offset log p_router(n) - lse_n of its entries
        for (int j = wave; j < n_groups; j += kSelectWaves) {          // wave-uniform
            float m = -INFINITY, sum = 0.f;
            for (int i = g_pre[j] + lane; i < g_pre[j + 1]; i += kWave) {
                const float2 st = bst[i];
                const float nm = fmaxf(m, st.x);
                if (nm > -INFINITY) sum = sum * expf(m - nm) + st.y * expf(st.x - nm);
                m = nm;
            }
            const float wm = wave_max(m);
            const float wsum = wave_sum(wm > -INFINITY ? sum * expf(m - wm) : 0.f);
            if (lane == 0) g_shift[j] = p.logp_sel[t * p.g + j] - (wm + logf(wsum));
        }
        __syncthreads();
    }

    // 3. the bound: a value that k block maxima reach.  A thread's best over its candidates
    // (every 256th), the k-th largest of a wave's 64 bests (k threads, so k blocks reach it;
    // 0 if fewer than k threads have one), the largest of the waves' values; blocks that
    // reach it are the next round's candidates.  With one candidate per thread the bound
    // leaves between k and 4 k blocks; with more (the dense head's thousand blocks) a second
    // and third round tighten it.
    if (LP) {
        for (int i = threadIdx.x; i < n_blocks; i += kSelectThreads)
            bval[i] = ord32(bst[i].x + g_shift[binfo[i] >> 16]);
        __syncthreads();
    }
    unsigned* keys32 = reinterpret_cast<unsigned*>(wkeys) + wave * kWave;
    unsigned tau = 0u;
    int n_q = n_blocks;
    {
        int* src_i = binfo;
        unsigned* src_v = bval;
        int* dst_i = qblk;
        unsigned* dst_v = qval;
        for (int round = 0; round < 3; ++round) {      // block-uniform
            unsigned best = 0u;
            for (int i = threadIdx.x; i < n_q; i += kSelectThreads) best = src_v[i] > best ? src_v[i] : best;
            const unsigned kth = wave_kth_key4(keys32, best, k, lane);
            if (lane == 0) tau_w[wave] = kth;
            __syncthreads();
            tau = tau_w[0];
#pragma unroll
            for (int w = 1; w < kSelectWaves; ++w) tau = tau_w[w] > tau ? tau_w[w] : tau;
            for (int base = 0; base < n_q; base += kSelectThreads) {   // block-uniform
                const int i = base + threadIdx.x;
                const bool on = i < n_q && src_v[i] >= tau;
                const unsigned long long bal = __ballot(on);
                int at = 0;
                if (lane == 0 && bal) at = atomicAdd(&n_qual, __popcll(bal));
                at = __builtin_amdgcn_readfirstlane(at) + __popcll(bal & ((1ull << lane) - 1ull));
                if (on) {
                    dst_i[at] = src_i[i];
                    dst_v[at] = src_v[i];
                }
            }
            __syncthreads();
            const bool tight = n_q <= kSelectThreads;
            n_q = uni(n_qual);
            int* ti = src_i; src_i = dst_i; dst_i = ti;
            unsigned* tv = src_v; src_v = dst_v; dst_v = tv;
            if (tight && n_q <= kSelectChunkBlocks) break;     // (else once more: the candidates of one chunk)
            __syncthreads();                           // (everyone has the count)
            if (threadIdx.x == 0) n_qual = 0;
        }
        qblk = src_i;                                  // the blocks whose largest reaches the bound
    }

    // 5. their candidates, 16 blocks at a time, merged with the list so far (buf[0, have))
    int have = 0;                                      // entries of the list so far
    unsigned long long list_kth = 0ull;                // its k-th key once it has k entries
    for (int base = 0; base < n_q; base += kSelectChunkBlocks) {       // block-uniform
        unsigned long long key[kSelectKeys];
        {
            float zv[kSelectKeys];
            int idv[kSelectKeys], grp[kSelectKeys];
            bool valid[kSelectKeys];
#pragma unroll
            for (int q = 0; q < kSelectKeys; ++q) {
                const int e = q * kSelectThreads + threadIdx.x;
                const int qb = base + (e >> 7), r = e & (kTileRows - 1);
                const int info = qblk[qb < n_q ? qb : n_q - 1];
                const int j = info >> 16, lb = info & 0xffff;
                const int row = lb * kTileRows + r, n_rows = g_rows[j];
                valid[q] = qb < n_q && row < n_rows;
                grp[q] = j;
                zv[q] = p.z[((size_t)(g_fb[j] + lb) * p.M + g_slot[j]) * kTileRows + r];
                idv[q] = DENSE ? row : p.rows[g_start[j] + (row < n_rows ? row : n_rows - 1)];
            }
#pragma unroll
            for (int q = 0; q < kSelectKeys; ++q) {
                const float v = LP ? zv[q] + g_shift[grp[q]] : zv[q];
                const unsigned long long kk = cand_key(v, idv[q]);
                key[q] = valid[q] && ord32(v) >= tau && kk > list_kth ? kk : 0ull;
            }
        }
        unsigned long long pass[kSelectKeys];
        auto reserve = [&](unsigned long long bnd) {
            int mine = 0;
#pragma unroll
            for (int q = 0; q < kSelectKeys; ++q) {
                pass[q] = __ballot(key[q] != 0ull && key[q] >= bnd);
                mine += __popcll(pass[q]);
            }
            int at = 0;
            if (lane == 0 && mine) at = atomicAdd(&n_kept, mine);
            return __builtin_amdgcn_readfirstlane(at);
        };
        int at = reserve(0ull);                        // (n_kept = have: the list comes first)
        __syncthreads();
        const int passed = uni(n_kept) - have;
        if (passed > kSelectThreads) {                 // block-uniform: too many for one key per thread
            unsigned long long best = key[0];
#pragma unroll
            for (int q = 1; q < kSelectKeys; ++q) best = key[q] > best ? key[q] : best;
            unsigned long long* wk = wkeys + wave * kWave;
            wk[lane] = best;
            const int above = count_above(wk, kWave, best);
            const unsigned long long hit = __ballot(best != 0ull && above == k - 1);   // one lane or none
            unsigned long long bnd = 0ull;
            if (hit) {
                const int src = __ffsll((long long)hit) - 1;
                bnd = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)(unsigned)(best >> 32), src) << 32) |
                      (unsigned)__builtin_amdgcn_readlane((int)(unsigned)best, src);
            }
            if (lane == 0) bound_w[wave] = bnd;
            __syncthreads();                           // (every wave has read the count by now)
            if (threadIdx.x == 0) n_kept = have;
            __syncthreads();
            bnd = bound_w[0];
#pragma unroll
            for (int w = 1; w < kSelectWaves; ++w) bnd = bound_w[w] > bnd ? bound_w[w] : bnd;
            at = reserve(bnd);
            __syncthreads();
        }
#pragma unroll
        for (int q = 0; q < kSelectKeys; ++q) {
            if ((pass[q] >> lane) & 1ull) buf[at + __popcll(pass[q] & ((1ull << lane) - 1ull))] = key[q];
            at += __popcll(pass[q]);
        }
        __syncthreads();
        const int kept = uni(n_kept);
        for (int i = threadIdx.x; i < kept; i += kSelectThreads) {
            const unsigned long long mine = buf[i];
            const int r = count_above(buf, kept, mine);
            if (r < k) list[r] = mine;
        }
        __syncthreads();
        have = kept < k ? kept : k;
        if (base + kSelectChunkBlocks >= n_q) break;   // block-uniform: that was the last chunk
        if ((int)threadIdx.x < have) buf[threadIdx.x] = list[threadIdx.x];
        if (threadIdx.x == 0) n_kept = have;
        list_kth = have == k ? list[k - 1] : 0ull;
        __syncthreads();
    }
    if ((int)threadIdx.x < k) {
        Cand c = sentinel();
        if ((int)threadIdx.x < have) {
            c.v = key_value(list[threadIdx.x]);
            c.id = key_id(list[threadIdx.x]);
        }
        p.topk_ids[(size_t)t * k + threadIdx.x] = c.id;
        p.topk_out[(size_t)t * k + threadIdx.x] = c.v;
    }
}

}  // namespace
