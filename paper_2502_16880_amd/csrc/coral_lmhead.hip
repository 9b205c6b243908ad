// Weight-grouped LM head of a speculative-decoding draft model, gfx950 (MI355X).
//
// Paper section 3.3 ("LM Head Router"): the router's W2 projection scores G
// vocabulary groups per draft token, the g best groups are activated, logits are
// computed over the rows of those groups only and the k best candidates per token
// go to tree expansion (appendix "Discussion on LM Head Router").  The paper gives
// no kernel; this design is for CDNA4: the path is bound by streaming the active
// weight rows from HBM once, so
//   - one wavefront reads one weight row as consecutive 1 KB segments (64 lanes x
//     16 B), several rows in flight, non-temporal so the stream does not evict the
//     small reused operands from L2;
//   - the hidden vectors of the tokens that selected the group sit in LDS and are
//     re-used for every row of the chunk; bf16 pairs go through v_dot2c_f32_bf16
//     with fp32 accumulation;
//   - each wavefront keeps its running k best per token in registers (lane i holds
//     rank i), so the logits row never leaves the chip; workgroup partial lists are
//     merged by rank counting, then a last small kernel merges per token.
// A group selected by several tokens is read once for all of them (the "activate
// all the involved groups" of the appendix's tree-decoding paragraph).
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>
#include <stdlib.h>

#include "coral_lmhead.h"

namespace {

constexpr int kWave = 64;
constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kRowsPerWave = 8;
constexpr int kChunkRows = kRowsPerWave * kWavesPerBlock;   // rows one workgroup streams
constexpr int kRowsInFlight = 2;                            // rows a wave loads together
constexpr int kTokBatch = 8;                                // tokens staged in LDS at once
constexpr int kMaxM = 64;
constexpr int kMaxK = 64;
constexpr int kMaxG = 1024;
constexpr int kSelRegs = kMaxG / kWave;

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

struct Cand {
    float v;
    int id;
};

__device__ __forceinline__ bool better(float av, int aid, float bv, int bid) {
    return av > bv || (av == bv && aid < bid);
}

// ---------------------------------------------------------------- loads / dots
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
    u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <bool BF16>
__device__ __forceinline__ float dot_vec(uint4 w, uint4 h, float acc) {
    if (BF16) {
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.x),
                                              __builtin_bit_cast(bf16x2_t, h.x), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.y),
                                              __builtin_bit_cast(bf16x2_t, h.y), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.z),
                                              __builtin_bit_cast(bf16x2_t, h.z), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.w),
                                              __builtin_bit_cast(bf16x2_t, h.w), acc, false);
    } else {
        acc = fmaf(__uint_as_float(w.x), __uint_as_float(h.x), acc);
        acc = fmaf(__uint_as_float(w.y), __uint_as_float(h.y), acc);
        acc = fmaf(__uint_as_float(w.z), __uint_as_float(h.z), acc);
        acc = fmaf(__uint_as_float(w.w), __uint_as_float(h.w), acc);
    }
    return acc;
}

// ---------------------------------------------------------------- wave helpers
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float x) {
    int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
    return x + __int_as_float(moved);
}

// Sum over the 64 lanes, returned to every lane (wave-uniform).  Fixed order:
// inclusive scan inside each row of 16 lanes, then rows 0+1, 2+3, then halves.
__device__ __forceinline__ float wave_sum(float x) {
    x = dpp_add<0x111, 0xf>(x);   // row_shr:1
    x = dpp_add<0x112, 0xf>(x);   // row_shr:2
    x = dpp_add<0x114, 0xf>(x);   // row_shr:4
    x = dpp_add<0x118, 0xf>(x);   // row_shr:8  -> lane 15 of each row holds the row total
    x = dpp_add<0x142, 0xa>(x);   // row_bcast:15 into rows 1 and 3
    x = dpp_add<0x143, 0xc>(x);   // row_bcast:31 into rows 2 and 3 -> lane 63 holds the total
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// Sorted list of the best candidates seen so far, lane i holding rank i.
// (v, id) is wave-uniform.  Lanes past the wanted k simply hold further ranks.
__device__ __forceinline__ void list_insert(float& lv, int& li, float v, int id, int lane, int k) {
    const float tv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(lv), k - 1));
    const int ti = __builtin_amdgcn_readlane(li, k - 1);
    if (!better(v, id, tv, ti)) return;                // does not reach the k best: wave-uniform
    const bool beats = better(v, id, lv, li);
    const unsigned long long b = __ballot(beats);
    if (b == 0) return;
    const int pos = __ffsll(b) - 1;
    const float sv = __shfl_up(lv, 1);
    const int si = __shfl_up(li, 1);
    if (lane == pos) {
        lv = v;
        li = id;
    } else if (lane > pos) {
        lv = sv;
        li = si;
    }
}

// Workgroup merge of n_lists sorted lists of k candidates held in `buf`
// (n_lists*k <= blockDim.x): the rank of a candidate is the number of candidates
// that beat it (slot index breaks full ties between padding entries), the k best
// are written to dst in rank order.  Both barriers are reached by every thread.
__device__ __forceinline__ void block_rank_merge(const Cand* buf, int n, int k, Cand* dst) {
    __syncthreads();
    const int tid = threadIdx.x;
    if (tid < n) {
        const Cand c = buf[tid];
        int rank = 0;
        for (int j = 0; j < n; ++j) {
            const Cand o = buf[j];
            rank += (better(o.v, o.id, c.v, c.id) || (o.v == c.v && o.id == c.id && j < tid)) ? 1 : 0;
        }
        if (rank < k) dst[rank] = c;
    }
    __syncthreads();
}

// ---------------------------------------------------------------- parameters
struct LogitsParams {
    const uint4* hidden;        // [M, n_vec]
    const uint4* lm_W;          // [V, n_vec]
    const int32_t* offsets;     // [G+1]            (grouped)
    const int32_t* rows;        // [V]              (grouped)
    const int32_t* sel;         // [M, g]           (grouped)
    const unsigned long long* group_mask;   // [G]  (grouped)
    const int32_t* union_list;  // [G]              (grouped)
    const int32_t* n_union;     // [1]              (grouped)
    const int32_t* chunk_base;  // [M, g] first partial slot of (token, selected group)
    Cand* part;                 // [M, part_stride, k]
    int M, V, G, g, k;
    int n_vec;                  // 16-byte vectors per row
    int jp;                     // ceil(n_vec / 64)
    int tb_max;                 // tokens the LDS staging area holds
    int part_stride;            // partial lists reserved per token
};

// Streams the rows [row_begin, row_end) of one chunk for the nt tokens staged in
// LDS and leaves each wave's best candidates per token in (lv, li).
template <bool BF16, bool DENSE, int TB>
__device__ __forceinline__ void stream_chunk(const LogitsParams& p, const uint4* hs, int nt,
                                             int row_begin, int row_end, float (&lv)[TB],
                                             int (&li)[TB]) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int hs_stride = p.jp * kWave;
    constexpr int R = kRowsInFlight;
    constexpr int JU = 4;
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        lv[t] = -INFINITY;
        li[t] = INT_MAX;
    }
    for (int rr = 0; rr < kRowsPerWave; rr += R) {
        const int r0 = row_begin + wave * kRowsPerWave + rr;
        if (r0 >= row_end) break;                      // wave-uniform
        int row_id[R];
        bool valid[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            valid[r] = r0 + r < row_end;
            const int idx = valid[r] ? r0 + r : row_end - 1;
            row_id[r] = DENSE ? idx : __builtin_amdgcn_readfirstlane(p.rows[idx]);
        }
        float acc[R][TB];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int t = 0; t < TB; ++t) acc[r][t] = 0.f;

        for (int j0 = 0; j0 < p.jp; j0 += JU) {
            uint4 w[JU][R];
#pragma unroll
            for (int ju = 0; ju < JU; ++ju) {
                const int vec = (j0 + ju) * kWave + lane;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    w[ju][r] = make_uint4(0, 0, 0, 0);
                    if (vec < p.n_vec)
                        w[ju][r] = load_stream(p.lm_W + (size_t)row_id[r] * p.n_vec + vec);
                }
            }
#pragma unroll
            for (int ju = 0; ju < JU; ++ju) {
                if (j0 + ju < p.jp) {                  // wave-uniform; LDS is padded to jp*64
                    const int vec = (j0 + ju) * kWave + lane;
#pragma unroll
                    for (int t = 0; t < TB; ++t) {
                        const int tt = t < nt ? t : nt - 1;
                        const uint4 h = hs[tt * hs_stride + vec];
#pragma unroll
                        for (int r = 0; r < R; ++r) acc[r][t] = dot_vec<BF16>(w[ju][r], h, acc[r][t]);
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (!valid[r]) continue;                   // wave-uniform
#pragma unroll
            for (int t = 0; t < TB; ++t) {
                const float z = wave_sum(acc[r][t]);
                if (t < nt) list_insert(lv[t], li[t], z, row_id[r], lane, p.k);
            }
        }
    }
}

__device__ __forceinline__ int nth_set_bit(unsigned long long m, int n) {
    for (int i = 0; i < n; ++i) m &= m - 1;
    return __ffsll(m) - 1;
}

template <bool BF16, bool DENSE, int TB>
__device__ __forceinline__ void chunk_tokens(const LogitsParams& p, const uint4* hs, Cand* mbuf,
                                             unsigned long long batch, int nt, int group,
                                             int chunk, int row_begin, int row_end) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    float lv[TB];
    int li[TB];
    stream_chunk<BF16, DENSE, TB>(p, hs, nt, row_begin, row_end, lv, li);
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        if (t >= nt) break;                            // block-uniform
        const int m = nth_set_bit(batch, t);
        int slot;
        if (DENSE) {
            slot = chunk;
        } else {
            int i = 0;
            while (i < p.g - 1 && p.sel[m * p.g + i] != group) ++i;
            slot = p.chunk_base[m * p.g + i] + chunk;
        }
        if (lane < p.k) {
            mbuf[wave * p.k + lane].v = lv[t];
            mbuf[wave * p.k + lane].id = li[t];
        }
        block_rank_merge(mbuf, kWavesPerBlock * p.k, p.k,
                         p.part + ((size_t)m * p.part_stride + slot) * p.k);
    }
}

// One workgroup per (chunk of kChunkRows rows, activated group).  Dense: per chunk.
template <bool BF16, bool DENSE>
__global__ __launch_bounds__(kBlock) void k_logits(LogitsParams p) {
    extern __shared__ uint4 smem[];
    uint4* hs = smem;
    Cand* mbuf = reinterpret_cast<Cand*>(smem + (size_t)p.tb_max * p.jp * kWave);

    const int chunk = blockIdx.x;
    unsigned long long mask;
    int row_begin, row_end, group = 0;
    if (DENSE) {
        mask = p.M >= 64 ? ~0ull : ((1ull << p.M) - 1ull);
        row_begin = chunk * kChunkRows;
        if (row_begin >= p.V) return;
        row_end = min(p.V, row_begin + kChunkRows);
    } else {
        const int u = blockIdx.y;
        if (u >= *p.n_union) return;
        group = p.union_list[u];
        mask = p.group_mask[group];
        const int off0 = p.offsets[group], off1 = p.offsets[group + 1];
        row_begin = off0 + chunk * kChunkRows;
        if (row_begin >= off1) return;
        row_end = min(off1, row_begin + kChunkRows);
    }

    const int hs_stride = p.jp * kWave;
    unsigned long long rem = mask;
    while (rem) {                                      // block-uniform
        unsigned long long batch = 0;
        int nt = 0;
        while (rem && nt < p.tb_max) {
            const unsigned long long low = rem & (~rem + 1ull);
            batch |= low;
            rem ^= low;
            ++nt;
        }
        for (int t = 0; t < nt; ++t) {
            const int m = nth_set_bit(batch, t);
            for (int vec = threadIdx.x; vec < hs_stride; vec += kBlock)
                hs[t * hs_stride + vec] = vec < p.n_vec ? p.hidden[(size_t)m * p.n_vec + vec]
                                                        : make_uint4(0, 0, 0, 0);
        }
        __syncthreads();
        if (nt == 1)
            chunk_tokens<BF16, DENSE, 1>(p, hs, mbuf, batch, nt, group, chunk, row_begin, row_end);
        else if (nt == 2)
            chunk_tokens<BF16, DENSE, 2>(p, hs, mbuf, batch, nt, group, chunk, row_begin, row_end);
        else if (nt <= 4)
            chunk_tokens<BF16, DENSE, 4>(p, hs, mbuf, batch, nt, group, chunk, row_begin, row_end);
        else
            chunk_tokens<BF16, DENSE, kTokBatch>(p, hs, mbuf, batch, nt, group, chunk, row_begin, row_end);
        // chunk_tokens ends on a barrier, so hs may be overwritten now
    }
}

// ---------------------------------------------------------------- gate
// s[m,n] = sum_j gate_W[n,j] hidden[m,j] + bias[n]   (Eq. 7, W2 projection).
// One workgroup per group n.
template <bool BF16>
__global__ __launch_bounds__(kBlock) void k_gate(const uint4* __restrict__ hidden,
                                                 const uint4* __restrict__ gate_W,
                                                 const float* __restrict__ bias, int M, int G,
                                                 int n_vec, float* __restrict__ s) {
    __shared__ float red[kWavesPerBlock];
    const int n = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    for (int m = 0; m < M; ++m) {
        float acc = 0.f;
        for (int vec = threadIdx.x; vec < n_vec; vec += kBlock)
            acc = dot_vec<BF16>(gate_W[(size_t)n * n_vec + vec], hidden[(size_t)m * n_vec + vec], acc);
        acc = wave_sum(acc);
        __syncthreads();
        if (lane == 0) red[wave] = acc;
        __syncthreads();
        if (threadIdx.x == 0) {
            float tot = red[0];
            for (int w = 1; w < kWavesPerBlock; ++w) tot += red[w];
            s[(size_t)m * G + n] = tot + (bias ? bias[n] : 0.f);
        }
    }
}

// Per-token top-g of the gate scores (larger first, then lower group id), the
// token mask of every group, the list of activated groups and, per (token,
// selected group), the first partial-list slot its chunks write to.
__global__ __launch_bounds__(kBlock) void k_select(const float* __restrict__ s,
                                                   const int32_t* __restrict__ offsets, int M,
                                                   int G, int g, int32_t* __restrict__ sel,
                                                   unsigned long long* __restrict__ group_mask,
                                                   int32_t* __restrict__ union_list,
                                                   int32_t* __restrict__ n_union,
                                                   int32_t* __restrict__ chunk_base) {
    __shared__ unsigned long long mask[kMaxG];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    for (int n = threadIdx.x; n < G; n += kBlock) mask[n] = 0ull;
    __syncthreads();

    for (int m = wave; m < M; m += kWavesPerBlock) {
        float sc[kSelRegs];
        unsigned taken = 0;
#pragma unroll
        for (int i = 0; i < kSelRegs; ++i) {
            const int n = i * kWave + lane;
            sc[i] = n < G ? s[(size_t)m * G + n] : -INFINITY;
            if (n >= G) taken |= 1u << i;
        }
        for (int round = 0; round < g; ++round) {
            float bv = -INFINITY;
            int bi = INT_MAX;
#pragma unroll
            for (int i = 0; i < kSelRegs; ++i) {
                const int n = i * kWave + lane;
                if (!((taken >> i) & 1u) && better(sc[i], n, bv, bi)) {
                    bv = sc[i];
                    bi = n;
                }
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const float ov = __shfl_xor(bv, off);
                const int oi = __shfl_xor(bi, off);
                if (better(ov, oi, bv, bi)) {
                    bv = ov;
                    bi = oi;
                }
            }
            // every lane now holds the same winner (g <= G guarantees one exists)
            if ((bi & (kWave - 1)) == lane) taken |= 1u << (bi / kWave);
            if (lane == 0) {
                sel[m * g + round] = bi;
                atomicOr(&mask[bi], 1ull << m);
            }
        }
    }
    __syncthreads();
    for (int n = threadIdx.x; n < G; n += kBlock) group_mask[n] = mask[n];
    if (wave == 0) {
        int count = 0;
        for (int base = 0; base < G; base += kWave) {
            const int n = base + lane;
            const bool on = n < G && mask[n] != 0ull;
            const unsigned long long b = __ballot(on);
            if (on) union_list[count + __popcll(b & ((1ull << lane) - 1ull))] = n;
            count += __popcll(b);
        }
        if (lane == 0) *n_union = count;
    }
    for (int m = threadIdx.x; m < M; m += kBlock) {
        int base = 0;
        for (int i = 0; i < g; ++i) {
            chunk_base[m * g + i] = base;
            // sel was written by lane 0 of this block's waves before the barrier above
            const int n = sel[m * g + i];
            base += (offsets[n + 1] - offsets[n] + kChunkRows - 1) / kChunkRows;
        }
    }
}

// ---------------------------------------------------------------- final merge
// One workgroup per token: streams the token's partial lists through per-wave
// sorted lists (64 candidates per step, only those beating the current k-th are
// inserted), merges the four waves and writes the sorted result.
__global__ __launch_bounds__(kBlock) void k_merge(const Cand* __restrict__ part, int part_stride,
                                                  const int32_t* __restrict__ sel,
                                                  const int32_t* __restrict__ offsets, int g,
                                                  int dense_chunks, int k,
                                                  int32_t* __restrict__ topk_ids,
                                                  float* __restrict__ topk_logits) {
    __shared__ Cand mbuf[kWavesPerBlock * kMaxK];
    __shared__ Cand outbuf[kMaxK];
    const int m = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    int lists = dense_chunks;
    if (sel) {
        lists = 0;
        for (int i = 0; i < g; ++i) {
            const int n = sel[m * g + i];
            lists += (offsets[n + 1] - offsets[n] + kChunkRows - 1) / kChunkRows;
        }
    }
    const int n_cand = lists * k;
    const Cand* src = part + (size_t)m * part_stride * k;
    float lv = -INFINITY;
    int li = INT_MAX;
    for (int base = wave * kWave; base < n_cand; base += kBlock) {   // wave-uniform
        const int i = base + lane;
        Cand c;
        c.v = -INFINITY;
        c.id = INT_MAX;
        if (i < n_cand) c = src[i];
        const float tv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(lv), k - 1));
        const int ti = __builtin_amdgcn_readlane(li, k - 1);
        unsigned long long pass = __ballot(better(c.v, c.id, tv, ti));
        while (pass) {
            const int srcl = __ffsll(pass) - 1;
            pass &= pass - 1ull;
            const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(c.v), srcl));
            const int id = __builtin_amdgcn_readlane(c.id, srcl);
            list_insert(lv, li, v, id, lane, k);
        }
    }
    if (lane < k) {
        mbuf[wave * k + lane].v = lv;
        mbuf[wave * k + lane].id = li;
    }
    block_rank_merge(mbuf, kWavesPerBlock * k, k, outbuf);
    if (threadIdx.x < k) {
        topk_ids[(size_t)m * k + threadIdx.x] = outbuf[threadIdx.x].id;
        topk_logits[(size_t)m * k + threadIdx.x] = outbuf[threadIdx.x].v;
    }
}

// ---------------------------------------------------------------- host side
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
    size_t s, sel, mask, union_list, n_union, chunk_base, part, total;
    int part_stride;
};

bool sizes_ok(int M, int H, int V, int G, int g, int k) {
    if (M < 1 || H < 1 || V < 1 || k < 1) return false;
    if (G < 0 || g < 0 || (G == 0) != (g == 0) || g > G) return false;
    return true;
}

Layout make_layout(int M, int V, int G, int g, int k) {
    Layout L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    L.s = take((size_t)M * (G ? G : 1) * sizeof(float));
    L.sel = take((size_t)M * (g ? g : 1) * sizeof(int32_t));
    L.mask = take((size_t)(G ? G : 1) * sizeof(unsigned long long));
    L.union_list = take((size_t)(G ? G : 1) * sizeof(int32_t));
    L.n_union = take(sizeof(int32_t));
    L.chunk_base = take((size_t)M * (g ? g : 1) * sizeof(int32_t));
    L.part_stride = (V + kChunkRows - 1) / kChunkRows + g;
    L.part = take((size_t)M * L.part_stride * k * sizeof(Cand));
    L.total = off;
    return L;
}

coral_status check_common(const void* hidden, const void* lm_W, int M, int H, int V, int k,
                          coral_dtype dt, const int32_t* topk_ids, const float* topk_logits) {
    if (!hidden || !lm_W || !topk_ids || !topk_logits) return CORAL_ERR_NULL;
    if (dt != CORAL_F32 && dt != CORAL_BF16) return CORAL_ERR_SHAPE;
    if (M < 1 || H < 1 || V < 1 || k < 1) return CORAL_ERR_SHAPE;
    if (M > kMaxM || k > kMaxK) return CORAL_ERR_UNSUPPORTED;
    if (H % (dt == CORAL_BF16 ? 8 : 4) != 0) return CORAL_ERR_UNSUPPORTED;
    if (((uintptr_t)hidden | (uintptr_t)lm_W) & 15u) return CORAL_ERR_UNSUPPORTED;
    return CORAL_OK;
}

coral_status check_workspace(const void* ws, size_t have, size_t need) {
    if (!ws) return CORAL_ERR_WORKSPACE;
    if ((uintptr_t)ws & 255u) return CORAL_ERR_WORKSPACE;
    if (have < need) return CORAL_ERR_WORKSPACE;
    return CORAL_OK;
}

size_t logits_lds_bytes(int tb_max, int jp, int k) {
    return (size_t)tb_max * jp * kWave * sizeof(uint4) + (size_t)kWavesPerBlock * k * sizeof(Cand);
}

inline coral_status launch_status() {
    return hipGetLastError() == hipSuccess ? CORAL_OK : CORAL_ERR_HIP;
}

}  // namespace

extern "C" const char* coral_status_string(coral_status st) {
    switch (st) {
        case CORAL_OK: return "ok";
        case CORAL_ERR_NULL: return "a required pointer is NULL";
        case CORAL_ERR_SHAPE: return "a size is out of range or inconsistent";
        case CORAL_ERR_GROUP_INDEX: return "the group index is not a partition of the vocabulary";
        case CORAL_ERR_UNSUPPORTED: return "request outside the kernels' stated limits";
        case CORAL_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case CORAL_ERR_HIP: return "the HIP runtime refused a launch";
    }
    return "unknown status";
}

extern "C" coral_status coral_group_index_validate(const int32_t* host_offsets,
                                                   const int32_t* host_rows, int G, int V) {
    if (!host_offsets || !host_rows) return CORAL_ERR_NULL;
    if (G < 1 || V < 1) return CORAL_ERR_SHAPE;
    if (host_offsets[0] != 0 || host_offsets[G] != V) return CORAL_ERR_GROUP_INDEX;
    for (int n = 0; n < G; ++n)
        if (host_offsets[n + 1] < host_offsets[n]) return CORAL_ERR_GROUP_INDEX;
    unsigned char* seen = static_cast<unsigned char*>(calloc((size_t)V, 1));
    if (!seen) return CORAL_ERR_SHAPE;
    coral_status st = CORAL_OK;
    for (int i = 0; i < V; ++i) {
        const int32_t r = host_rows[i];
        if (r < 0 || r >= V || seen[r]) {
            st = CORAL_ERR_GROUP_INDEX;
            break;
        }
        seen[r] = 1;
    }
    free(seen);
    return st;
}

extern "C" size_t coral_lmhead_workspace_bytes(int M, int H, int V, int G, int g, int k,
                                               coral_dtype dt) {
    (void)dt;
    if (!sizes_ok(M, H, V, G, g, k)) return 0;
    return make_layout(M, V, G, g, k).total;
}

namespace {

coral_status record(void* ev, hipStream_t stream) {
    if (!ev) return CORAL_OK;
    return hipEventRecord(static_cast<hipEvent_t>(ev), stream) == hipSuccess ? CORAL_OK
                                                                             : CORAL_ERR_HIP;
}

coral_status grouped_impl(const void* hidden, const void* gate_W, const float* gate_bias,
                          const void* lm_W, const coral_group_index* gi, int M, int H, int V,
                          int g, int k, coral_dtype dt, int32_t* topk_ids, float* topk_logits,
                          int32_t* sel_groups, void* workspace, size_t workspace_bytes,
                          void* hip_stream, void* ev_before, void* ev_after) {
    if (!gate_W || !gi) return CORAL_ERR_NULL;
    coral_status st = check_common(hidden, lm_W, M, H, V, k, dt, topk_ids, topk_logits);
    if (st != CORAL_OK) return st;
    if (!gi->group_offsets_host || !gi->group_offsets || !gi->group_rows) return CORAL_ERR_NULL;
    const int G = gi->G;
    if (G < 1 || g < 1 || g > G) return CORAL_ERR_SHAPE;
    if (G > kMaxG) return CORAL_ERR_UNSUPPORTED;
    if ((uintptr_t)gate_W & 15u) return CORAL_ERR_UNSUPPORTED;
    const int32_t* off = gi->group_offsets_host;
    if (off[0] != 0 || off[G] != V) return CORAL_ERR_GROUP_INDEX;
    int max_rows = 0;
    // the g smallest groups bound the number of candidates a token can have
    int smallest[kMaxG];
    for (int n = 0; n < G; ++n) {
        const int len = off[n + 1] - off[n];
        if (len < 0) return CORAL_ERR_GROUP_INDEX;
        if (len > max_rows) max_rows = len;
        smallest[n] = len;
    }
    long long min_cand = 0;
    for (int i = 0; i < g; ++i) {           // partial selection sort, g <= G <= 1024
        int best = i;
        for (int n = i + 1; n < G; ++n)
            if (smallest[n] < smallest[best]) best = n;
        const int tmp = smallest[i];
        smallest[i] = smallest[best];
        smallest[best] = tmp;
        min_cand += smallest[i];
    }
    if ((long long)k > min_cand) return CORAL_ERR_SHAPE;
    const Layout L = make_layout(M, V, G, g, k);
    st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != CORAL_OK) return st;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    float* s = reinterpret_cast<float*>(ws + L.s);
    int32_t* sel = sel_groups ? sel_groups : reinterpret_cast<int32_t*>(ws + L.sel);
    unsigned long long* mask = reinterpret_cast<unsigned long long*>(ws + L.mask);
    int32_t* union_list = reinterpret_cast<int32_t*>(ws + L.union_list);
    int32_t* n_union = reinterpret_cast<int32_t*>(ws + L.n_union);
    int32_t* chunk_base = reinterpret_cast<int32_t*>(ws + L.chunk_base);
    Cand* part = reinterpret_cast<Cand*>(ws + L.part);

    const bool bf16 = dt == CORAL_BF16;
    const int n_vec = H / (bf16 ? 8 : 4);
    const uint4* hid = static_cast<const uint4*>(hidden);
    const uint4* gw = static_cast<const uint4*>(gate_W);
    if (bf16)
        hipLaunchKernelGGL(k_gate<true>, dim3(G), dim3(kBlock), 0, stream, hid, gw, gate_bias, M, G,
                           n_vec, s);
    else
        hipLaunchKernelGGL(k_gate<false>, dim3(G), dim3(kBlock), 0, stream, hid, gw, gate_bias, M, G,
                           n_vec, s);
    if ((st = launch_status()) != CORAL_OK) return st;
    hipLaunchKernelGGL(k_select, dim3(1), dim3(kBlock), 0, stream, s, gi->group_offsets, M, G, g, sel,
                       mask, union_list, n_union, chunk_base);
    if ((st = launch_status()) != CORAL_OK) return st;

    LogitsParams p;
    p.hidden = hid;
    p.lm_W = static_cast<const uint4*>(lm_W);
    p.offsets = gi->group_offsets;
    p.rows = gi->group_rows;
    p.sel = sel;
    p.group_mask = mask;
    p.union_list = union_list;
    p.n_union = n_union;
    p.chunk_base = chunk_base;
    p.part = part;
    p.M = M; p.V = V; p.G = G; p.g = g; p.k = k;
    p.n_vec = n_vec;
    p.jp = (n_vec + kWave - 1) / kWave;
    p.tb_max = M < kTokBatch ? M : kTokBatch;
    p.part_stride = L.part_stride;
    const size_t lds = logits_lds_bytes(p.tb_max, p.jp, k);
    if (lds > 160 * 1024) return CORAL_ERR_UNSUPPORTED;
    const int chunks = (max_rows + kChunkRows - 1) / kChunkRows;
    const long long max_union = (long long)M * g < G ? (long long)M * g : G;
    if (chunks < 1) return CORAL_ERR_SHAPE;
    dim3 grid(chunks, (unsigned)max_union);
    if ((st = record(ev_before, stream)) != CORAL_OK) return st;
    if (bf16) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(k_logits<true, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return CORAL_ERR_HIP;
        hipLaunchKernelGGL((k_logits<true, false>), grid, dim3(kBlock), lds, stream, p);
    } else {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(k_logits<false, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return CORAL_ERR_HIP;
        hipLaunchKernelGGL((k_logits<false, false>), grid, dim3(kBlock), lds, stream, p);
    }
    if ((st = launch_status()) != CORAL_OK) return st;
    if ((st = record(ev_after, stream)) != CORAL_OK) return st;
    hipLaunchKernelGGL(k_merge, dim3(M), dim3(kBlock), 0, stream, part, L.part_stride, sel,
                       gi->group_offsets, g, 0, k, topk_ids, topk_logits);
    return launch_status();
}

coral_status dense_impl(const void* hidden, const void* lm_W, int M, int H, int V, int k,
                        coral_dtype dt, int32_t* topk_ids, float* topk_logits, void* workspace,
                        size_t workspace_bytes, void* hip_stream, void* ev_before,
                        void* ev_after) {
    coral_status st = check_common(hidden, lm_W, M, H, V, k, dt, topk_ids, topk_logits);
    if (st != CORAL_OK) return st;
    if (k > V) return CORAL_ERR_SHAPE;
    const Layout L = make_layout(M, V, 0, 0, k);
    st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != CORAL_OK) return st;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    const bool bf16 = dt == CORAL_BF16;
    LogitsParams p = {};
    p.hidden = static_cast<const uint4*>(hidden);
    p.lm_W = static_cast<const uint4*>(lm_W);
    p.part = reinterpret_cast<Cand*>(ws + L.part);
    p.M = M; p.V = V; p.G = 0; p.g = 0; p.k = k;
    p.n_vec = H / (bf16 ? 8 : 4);
    p.jp = (p.n_vec + kWave - 1) / kWave;
    p.tb_max = M < kTokBatch ? M : kTokBatch;
    p.part_stride = L.part_stride;
    const size_t lds = logits_lds_bytes(p.tb_max, p.jp, k);
    if (lds > 160 * 1024) return CORAL_ERR_UNSUPPORTED;
    const int chunks = (V + kChunkRows - 1) / kChunkRows;
    if ((st = record(ev_before, stream)) != CORAL_OK) return st;
    if (bf16) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(k_logits<true, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return CORAL_ERR_HIP;
        hipLaunchKernelGGL((k_logits<true, true>), dim3(chunks), dim3(kBlock), lds, stream, p);
    } else {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(k_logits<false, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return CORAL_ERR_HIP;
        hipLaunchKernelGGL((k_logits<false, true>), dim3(chunks), dim3(kBlock), lds, stream, p);
    }
    if ((st = launch_status()) != CORAL_OK) return st;
    if ((st = record(ev_after, stream)) != CORAL_OK) return st;
    hipLaunchKernelGGL(k_merge, dim3(M), dim3(kBlock), 0, stream, p.part, L.part_stride,
                       (const int32_t*)nullptr, (const int32_t*)nullptr, 0, chunks, k, topk_ids,
                       topk_logits);
    return launch_status();
}

}  // namespace

extern "C" coral_status coral_lmhead_grouped(const void* hidden, const void* gate_W,
                                             const float* gate_bias, const void* lm_W,
                                             const coral_group_index* gi, int M, int H, int V,
                                             int g, int k, coral_dtype dt, int32_t* topk_ids,
                                             float* topk_logits, int32_t* sel_groups,
                                             void* workspace, size_t workspace_bytes,
                                             void* hip_stream) {
    return grouped_impl(hidden, gate_W, gate_bias, lm_W, gi, M, H, V, g, k, dt, topk_ids,
                        topk_logits, sel_groups, workspace, workspace_bytes, hip_stream, nullptr,
                        nullptr);
}

extern "C" coral_status coral_lmhead_grouped_profiled(
    const void* hidden, const void* gate_W, const float* gate_bias, const void* lm_W,
    const coral_group_index* gi, int M, int H, int V, int g, int k, coral_dtype dt,
    int32_t* topk_ids, float* topk_logits, int32_t* sel_groups, void* workspace,
    size_t workspace_bytes, void* hip_stream, void* ev_before, void* ev_after) {
    if (!ev_before || !ev_after) return CORAL_ERR_NULL;
    return grouped_impl(hidden, gate_W, gate_bias, lm_W, gi, M, H, V, g, k, dt, topk_ids,
                        topk_logits, sel_groups, workspace, workspace_bytes, hip_stream, ev_before,
                        ev_after);
}

extern "C" coral_status coral_lmhead_dense(const void* hidden, const void* lm_W, int M, int H,
                                           int V, int k, coral_dtype dt, int32_t* topk_ids,
                                           float* topk_logits, void* workspace,
                                           size_t workspace_bytes, void* hip_stream) {
    return dense_impl(hidden, lm_W, M, H, V, k, dt, topk_ids, topk_logits, workspace,
                      workspace_bytes, hip_stream, nullptr, nullptr);
}

extern "C" coral_status coral_lmhead_dense_profiled(const void* hidden, const void* lm_W, int M,
                                                    int H, int V, int k, coral_dtype dt,
                                                    int32_t* topk_ids, float* topk_logits,
                                                    void* workspace, size_t workspace_bytes,
                                                    void* hip_stream, void* ev_before,
                                                    void* ev_after) {
    if (!ev_before || !ev_after) return CORAL_ERR_NULL;
    return dense_impl(hidden, lm_W, M, H, V, k, dt, topk_ids, topk_logits, workspace,
                      workspace_bytes, hip_stream, ev_before, ev_after);
}
