// General path: one launch per stage (gate, selection, chunked weight streaming with
// per-workgroup partial top-k, per-token merge).  Handles every supported shape; used
// when the single-launch path's LDS budget does not fit.
#pragma once
#include "device_utils.h"
#include "fused_path.h"

namespace {

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
    float* lse_part;            // [M, part_stride, 2] (max, sum of exp) of a slot's logits; log-prob mode
    int M, V, G, g, k;
    int n_vec;                  // 16-byte vectors per row
    int jp;                     // ceil(n_vec / 64)
    int tb_max;                 // tokens the LDS staging area holds
    int part_stride;            // partial lists reserved per token
};

// Streams the rows [row_begin, row_end) of one chunk for the nt tokens staged in
// LDS and leaves each wave's best candidates per token in (lv, li).
// LP: also keep, per token, the running maximum and the sum of exp(logit - maximum) over the
// wave's rows (the pieces of Eq. 8's softmax inside a group).
template <int DT, bool DENSE, int TB, bool LP>
__device__ __forceinline__ void stream_chunk(const LogitsParams& p, const uint4* hs, int nt,
                                             int row_begin, int row_end, float (&lv)[TB],
                                             int (&li)[TB], float (&mx)[TB], float (&sm)[TB]) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int hs_stride = p.jp * kWave;
    constexpr int R = kRowsInFlight;
    constexpr int JU = 8;
#pragma unroll
    for (int t = 0; t < TB; ++t) {
        lv[t] = -INFINITY;
        li[t] = INT_MAX;
        mx[t] = -INFINITY;
        sm[t] = 0.f;
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
                        for (int r = 0; r < R; ++r) acc[r][t] = dot_vec<DT>(w[ju][r], h, acc[r][t]);
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
                if (LP) {                              // wave-uniform values
                    const float nm = fmaxf(mx[t], z);
                    sm[t] = sm[t] * expf(mx[t] - nm) + expf(z - nm);
                    mx[t] = nm;
                }
            }
        }
    }
}

__device__ __forceinline__ int nth_set_bit(unsigned long long m, int n) {
    for (int i = 0; i < n; ++i) m &= m - 1;
    return __ffsll(m) - 1;
}

template <int DT, bool DENSE, int TB, bool LP>
__device__ __forceinline__ void chunk_tokens(const LogitsParams& p, const uint4* hs, Cand* mbuf,
                                             unsigned long long batch, int nt, int group,
                                             int chunk, int row_begin, int row_end) {
    __shared__ float lse_red[kWavesPerBlock][2];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    float lv[TB], mx[TB], sm[TB];
    int li[TB];
    stream_chunk<DT, DENSE, TB, LP>(p, hs, nt, row_begin, row_end, lv, li, mx, sm);
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
        if (LP && lane == 0) {
            lse_red[wave][0] = mx[t];
            lse_red[wave][1] = sm[t];
        }
        block_rank_merge(mbuf, kWavesPerBlock * p.k, p.k,
                         p.part + ((size_t)m * p.part_stride + slot) * p.k);
        if (LP && threadIdx.x == 0) {                  // the waves' pieces, combined in wave order
            float bm = -INFINITY, bs = 0.f;
            for (int w = 0; w < kWavesPerBlock; ++w) {
                const float nm = fmaxf(bm, lse_red[w][0]);
                if (nm > -INFINITY) bs = bs * expf(bm - nm) + lse_red[w][1] * expf(lse_red[w][0] - nm);
                bm = nm;
            }
            float* dst = p.lse_part + ((size_t)m * p.part_stride + slot) * 2;
            dst[0] = bm;
            dst[1] = bs;
        }
        if (LP) __syncthreads();                       // lse_red is rewritten for the next token
    }
}

// One workgroup per (chunk of kChunkRows rows, activated group).  Dense: per chunk.
template <int DT, bool DENSE, bool LP = false>
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
            chunk_tokens<DT, DENSE, 1, LP>(p, hs, mbuf, batch, nt, group, chunk, row_begin, row_end);
        else if (nt == 2)
            chunk_tokens<DT, DENSE, 2, LP>(p, hs, mbuf, batch, nt, group, chunk, row_begin, row_end);
        else if (nt <= 4)
            chunk_tokens<DT, DENSE, 4, LP>(p, hs, mbuf, batch, nt, group, chunk, row_begin, row_end);
        else
            chunk_tokens<DT, DENSE, kTokBatch, LP>(p, hs, mbuf, batch, nt, group, chunk, row_begin, row_end);
        // chunk_tokens ends on a barrier, so hs may be overwritten now
    }
}

// ---------------------------------------------------------------- gate
// s[m,n] = sum_j gate_W[n,j] hidden[m,j] + bias[n]   (Eq. 7, W2 projection).
// One workgroup per group n.
template <int DT>
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
            acc = dot_vec<DT>(gate_W[(size_t)n * n_vec + vec], hidden[(size_t)m * n_vec + vec], acc);
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
                                                   int32_t* __restrict__ chunk_base,
                                                   float* __restrict__ logp_sel,
                                                   int32_t* __restrict__ slot_count) {
    __shared__ unsigned long long mask[kMaxG];
    __shared__ int off_lds[kMaxG + 1];                 // group offsets: no dependent loads later
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    for (int n = threadIdx.x; n < G; n += kBlock) mask[n] = 0ull;
    for (int n = threadIdx.x; n <= G; n += kBlock) off_lds[n] = offsets[n];
    __syncthreads();

    __shared__ unsigned long long rank_keys[kWavesPerBlock][kWave];
    if (G <= kWave) {
        // one score per lane: rank by counting (larger score first, then lower group id)
        for (int m = wave; m < M; m += kWavesPerBlock) {
            float v = lane < G ? s[(size_t)m * G + lane] : -INFINITY;
            if (!(v == v)) v = -INFINITY;                   // NaN: unspecified, keep a total order
            float lse_s = 0.f;
            if (logp_sel) {
                float smax = v;
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) smax = fmaxf(smax, __shfl_xor(smax, off));
                lse_s = smax + logf(wave_sum(lane < G ? expf(v - smax) : 0.f));
            }
            const int rank = wave_rank(rank_keys[wave], v, lane, G, lane);
            const bool chosen = lane < G && rank < g;
            const int nch = lane < G ? (off_lds[lane + 1] - off_lds[lane] + kChunkRows - 1) / kChunkRows : 0;
            if (chosen) {
                sel[m * g + rank] = lane;
                if (logp_sel) logp_sel[m * g + rank] = v - lse_s;
                atomicOr(&mask[lane], 1ull << m);
            }
            int slot_base = 0;                              // slots in rank order
            for (int r = 0; r < g; ++r) {                   // wave-uniform
                const int src = __ffsll(__ballot(chosen && rank == r)) - 1;
                if (lane == src) {
                    chunk_base[m * g + r] = slot_base;
                    if (slot_count) slot_count[m * g + r] = nch;
                }
                slot_base += __builtin_amdgcn_readlane(nch, src);
            }
        }
    } else
    for (int m = wave; m < M; m += kWavesPerBlock) {
        float sc[kSelRegs];
        unsigned taken = 0;
#pragma unroll
        for (int i = 0; i < kSelRegs; ++i) {
            const int n = i * kWave + lane;
            sc[i] = n < G ? s[(size_t)m * G + n] : -INFINITY;
            if (!(sc[i] == sc[i])) sc[i] = -INFINITY;       // NaN: keeps every round a winner
            if (n >= G) taken |= 1u << i;
        }
        // log of the router's softmax denominator over all G groups (Eq. 7), log-prob mode
        float lse_s = 0.f;
        if (logp_sel) {
            float smax = -INFINITY;
#pragma unroll
            for (int i = 0; i < kSelRegs; ++i) smax = fmaxf(smax, sc[i]);
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) smax = fmaxf(smax, __shfl_xor(smax, off));
            float ssum = 0.f;
#pragma unroll
            for (int i = 0; i < kSelRegs; ++i)
                if (i * kWave + lane < G) ssum += expf(sc[i] - smax);
            ssum = wave_sum(ssum);
            lse_s = smax + logf(ssum);
        }
        int slot_base = 0;                             // first partial-list slot of the next group
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
                chunk_base[m * g + round] = slot_base;
                if (slot_count)
                    slot_count[m * g + round] = (off_lds[bi + 1] - off_lds[bi] + kChunkRows - 1) / kChunkRows;
                if (logp_sel) logp_sel[m * g + round] = bv - lse_s;
                atomicOr(&mask[bi], 1ull << m);
            }
            slot_base += (off_lds[bi + 1] - off_lds[bi] + kChunkRows - 1) / kChunkRows;
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
    if ((int)threadIdx.x < k) {
        topk_ids[(size_t)m * k + threadIdx.x] = outbuf[threadIdx.x].id;
        topk_logits[(size_t)m * k + threadIdx.x] = outbuf[threadIdx.x].v;
    }
}


// Final merge of the log-probability mode behind k_logits (a slot = a chunk of kChunkRows
// rows): slot_count[m, i] slots from chunk_base[m, i] on belong to token m's i-th selected
// group.
// Eq. 8: log p(x) = log p_router(n) + z[x] - lse_n
// for x in the selected group n, where lse_n is the log of the sum of exp(z) over the
// group's rows.  One workgroup per token; wave w takes the token's selected groups w, w + WAVES,
// ...: it combines the (max, sum) pieces of the group's slots into lse_n, merges the group's
// partial lists (sorted by logit, which inside a group is the order of log p as well) into
// the group's k best, adds the offset log p_router(n) - lse_n and merges that list into its
// running list.  The waves' running lists are merged at the end; equal values: lower id first.
template <int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void k_merge_logprob(const Cand* __restrict__ part,
                                                          const float* __restrict__ lse_part,
                                                          int part_stride,
                                                          const int32_t* __restrict__ slot_count,
                                                          const int32_t* __restrict__ chunk_base,
                                                          const float* __restrict__ logp_sel, int g,
                                                          int k, int32_t* __restrict__ topk_ids,
                                                          float* __restrict__ topk_logprob) {
    __shared__ Cand mbuf[WAVES * kMaxK];      // the waves' running lists
    __shared__ Cand fresh[WAVES * kMaxK];     // a group's k best, then the merged list
    __shared__ Cand outbuf[kMaxK];
    __shared__ WaveScratch scratch[WAVES];
    const int m = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    Cand* mine = mbuf + wave * k;
    Cand* grp = fresh + wave * k;
    if (lane < k) mine[lane] = sentinel();
    const Cand* src = part + (size_t)m * part_stride * k;
    for (int i = wave; i < g; i += WAVES) {   // wave-uniform
        const int s0 = chunk_base[m * g + i];          // (three loads that do not wait for each other)
        const int n_slots = slot_count[m * g + i];
        // lse_n from the slots' pieces: per lane in ascending slot order, then across lanes
        float bm = -INFINITY, bs = 0.f;
        for (int s = lane; s < n_slots; s += kWave) {
            const float pm = lse_part[((size_t)m * part_stride + s0 + s) * 2];
            const float ps = lse_part[((size_t)m * part_stride + s0 + s) * 2 + 1];
            const float nm = fmaxf(bm, pm);
            if (nm > -INFINITY) bs = bs * expf(bm - nm) + ps * expf(pm - nm);
            bm = nm;
        }
        float wm = bm;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) wm = fmaxf(wm, __shfl_xor(wm, off));
        const float ws = wave_sum(wm > -INFINITY ? bs * expf(bm - wm) : 0.f);
        const float shift = logp_sel[m * g + i] - (wm + logf(ws));
        // the group's k best by logit, offset added
        wave_merge_topk<4>(                          // (few slots: all candidates in one trip)
            n_slots, k, lane, &scratch[wave],
            [&](int l, int e) { return src[(size_t)(s0 + l) * k + e]; },
            [&](int r, Cand c) {
                if (is_real(c)) c.v += shift;
                grp[r] = c;
            });
        // merge with the running list (two sorted lists of k): ranks by counting
        Cand a = sentinel(), b = sentinel();
        if (lane < k) {
            a = mine[lane];
            b = grp[lane];
        }
        const unsigned long long ka = cand_key(a.v, a.id), kb = cand_key(b.v, b.id);
        scratch[wave].keys[lane] = lane < k ? ka : 0ull;
        int ra = lane, rb = lane;                       // rank inside the own list
        unsigned long long* keys = scratch[wave].keys;
        rb += count_above(keys, k, kb);
        // (LDS accesses of a wave complete in order: the reads above precede this write)
        keys[lane] = lane < k ? kb : 0ull;
        ra += count_above(keys, k, ka);
        if (lane < k && is_real(a) && ra < k) grp[ra] = a;     // grp is free: b sits in registers
        if (lane < k && is_real(b) && rb < k) grp[rb] = b;
        const int n_real = __popcll(__ballot(lane < k && is_real(a))) + __popcll(__ballot(lane < k && is_real(b)));
        if (lane < k && lane >= n_real) grp[lane] = sentinel();
        if (lane < k) mine[lane] = grp[lane];
    }
    block_rank_merge(mbuf, WAVES * k, k, outbuf);
    if ((int)threadIdx.x < k) {
        topk_ids[(size_t)m * k + threadIdx.x] = outbuf[threadIdx.x].id;
        topk_logprob[(size_t)m * k + threadIdx.x] = outbuf[threadIdx.x].v;
    }
}

}  // namespace
