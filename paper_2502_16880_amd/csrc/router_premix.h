// Router pre-mix (section 3.3, Eq. 7): the router's second projection W2 is applied to
// u = act(W1 h) + h, with W1 [d,d] one row per output feature.  A d x d matrix read once per
// step for all tokens: HBM-bound like the LM head itself (33.6 MB at d = 4096 in bf16).
// One wave computes two output features at a time for up to eight tokens whose hidden
// vectors sit in LDS: both weight rows are requested whole (non-temporal, 16 KB per wave in
// flight at d = 4096), dotted with every token's vector (fp32 accumulation), and lane t
// finishes token t: activation, residual, rounding to the storage type.
//
// From four tokens on the vector units would bound the kernel (a bf16 dot instruction per two
// products of every token), so the contraction goes to the matrix cores: a workgroup owns 16
// output features, its four waves split their columns, and each wave holds 16 whole 128-byte
// lines of each of the 16 rows (32 loads, 32 KB) in registers at once.
#pragma once
#include "device_utils.h"
#include "fused_path.h"

namespace {

constexpr int kPremixTok = 8;                    // tokens of a workgroup (LDS residents)
constexpr int kPremixSegs = 8;                   // 1 KB segments of a row requested together
constexpr int kPremixStage = 8;                  // 16-byte vectors a thread stages through registers

struct PremixParams {
    const uint4* hidden;        // [M, n_vec]
    const uint4* W1;            // [H, n_vec]
    void* out;                  // [M, H] storage type
    int M, H, n_vec, act, tok_per_wg;
};

__device__ __forceinline__ float premix_act(float y, int act) {
    if (act == CORAL_ACT_SILU) return y / (1.0f + expf(-y));
    if (act == CORAL_ACT_RELU) return y > 0.f ? y : 0.f;
    return y;
}

template <int DT>
__global__ __launch_bounds__(kBlock) void k_premix(PremixParams p) {
    extern __shared__ uint4 smem[];                                // [tb][n_vec]
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int m0 = blockIdx.y * p.tok_per_wg;
    const int tb = p.M - m0 < p.tok_per_wg ? p.M - m0 : p.tok_per_wg;
    // The tokens' vectors are requested first and written to LDS only after the first weight
    // rows have been requested too: loads complete in order, so the wait for the tokens does
    // not wait for the weights behind them (what does not fit the registers goes directly).
    const int total = tb * p.n_vec;                                // consecutive rows: one block
    const uint4* hsrc = p.hidden + (size_t)m0 * p.n_vec;
    uint4 st[kPremixStage];
#pragma unroll
    for (int j = 0; j < kPremixStage; ++j) {
        const int i = threadIdx.x + j * kBlock;
        if (i < total) st[j] = load_vec(hsrc + i);
    }
    for (int i = threadIdx.x + kPremixStage * kBlock; i < total; i += kBlock) smem[i] = hsrc[i];
    const int n_waves = gridDim.x * kWavesPerBlock;
    const int r_first = (blockIdx.x * kWavesPerBlock + wave) * 2;
    auto commit_tokens = [&]() {                                   // every wave exactly once
        asm volatile("" ::: "memory");
#pragma unroll
        for (int j = 0; j < kPremixStage; ++j) {
            const int i = threadIdx.x + j * kBlock;
            if (i < total) store_vec(smem + i, st[j]);
        }
        __syncthreads();
    };
    bool staged = false;
    if (r_first >= p.H) commit_tokens();                           // a wave without rows (wave-uniform)
    for (int r0 = r_first; r0 < p.H; r0 += n_waves * 2) {          // wave-uniform
        const int r1 = r0 + 1 < p.H ? r0 + 1 : r0;
        float a0[kPremixTok], a1[kPremixTok];
#pragma unroll
        for (int t = 0; t < kPremixTok; ++t) a0[t] = a1[t] = 0.f;
        const uint4* w0p = p.W1 + (size_t)r0 * p.n_vec;
        const uint4* w1p = p.W1 + (size_t)r1 * p.n_vec;
        for (int base = 0; base < p.n_vec; base += kWave * kPremixSegs) {
            uint4 w0[kPremixSegs], w1[kPremixSegs];
#pragma unroll
            for (int j = 0; j < kPremixSegs; ++j) {
                const int vec = base + j * kWave + lane;
                w0[j] = make_uint4(0, 0, 0, 0);
                w1[j] = make_uint4(0, 0, 0, 0);
                if (vec < p.n_vec) {
                    w0[j] = load_stream(w0p + vec);
                    w1[j] = load_stream(w1p + vec);
                }
            }
            if (!staged) {                                         // wave-uniform: the wave's first pass
                commit_tokens();
                staged = true;
            }
#pragma unroll
            for (int j = 0; j < kPremixSegs; ++j) {
                const int vec = base + j * kWave + lane;
                const int hv = vec < p.n_vec ? vec : 0;            // the weights there are zero
#pragma unroll
                for (int t = 0; t < kPremixTok; ++t)
                    if (t < tb) {                                  // uniform
                        const uint4 h = smem[t * p.n_vec + hv];
                        a0[t] = dot_vec<DT>(w0[j], h, a0[t]);
                        a1[t] = dot_vec<DT>(w1[j], h, a1[t]);
                    }
            }
        }
        float y0 = 0.f, y1 = 0.f;                                  // lane t keeps token t's sums
#pragma unroll
        for (int t = 0; t < kPremixTok; ++t)
            if (t < tb) {
                const float s0 = wave_sum(a0[t]), s1 = wave_sum(a1[t]);
                if (lane == t) {
                    y0 = s0;
                    y1 = s1;
                }
            }
        if (lane < tb) {
            const size_t o = (size_t)(m0 + lane) * p.H;
            if (DT != kF32) {
                const unsigned short* hs = reinterpret_cast<const unsigned short*>(smem) + (size_t)lane * p.H;
                unsigned short* out = static_cast<unsigned short*>(p.out);
                out[o + r0] = narrow16<DT>(premix_act(y0, p.act) + widen16<DT>(hs[r0]));
                if (r1 != r0)
                    out[o + r1] = narrow16<DT>(premix_act(y1, p.act) + widen16<DT>(hs[r1]));
            } else {
                const float* hs = reinterpret_cast<const float*>(smem) + (size_t)lane * p.H;
                float* out = static_cast<float*>(p.out);
                out[o + r0] = premix_act(y0, p.act) + hs[r0];
                if (r1 != r0) out[o + r1] = premix_act(y1, p.act) + hs[r1];
            }
        }
    }
}

constexpr int kPremixTileTok = 16;               // tokens of a workgroup on the matrix cores
constexpr int kPremixLines = 16;                 // 128-byte lines of a row a wave holds at once
constexpr int kPremixTileStage = 32;             // 16-byte vectors a thread stages through registers

__host__ __device__ inline size_t premix_mfma_lds_bytes(int tok, int n_vec) {
    return ((size_t)tok * (n_vec + 1) + (size_t)kWavesPerBlock * kLinePairSlots) * sizeof(uint4) +
           (size_t)kWavesPerBlock * 256 * sizeof(float);
}

// bf16, H a multiple of 64 (whole 128-byte lines).  Tile of 16 output features x 16 tokens:
// A operand = rows of W1, B operand = hidden vectors from LDS (row stride padded by one
// vector: conflict-free); lane l of the result holds features 4*(l/16)..+4 of token l%16.
template <int DT>
__global__ __launch_bounds__(kBlock) void k_premix_mfma(PremixParams p) {
    extern __shared__ uint4 smem[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int r16 = lane & 15, q4 = lane >> 4;
    const int stride = p.n_vec + 1;
    uint4* hs = smem;                                              // [tok_per_wg][stride]
    uint4* my_slice = smem + (size_t)p.tok_per_wg * stride + (size_t)wave * kLinePairSlots;
    float* red = reinterpret_cast<float*>(smem + (size_t)p.tok_per_wg * stride +
                                          (size_t)kWavesPerBlock * kLinePairSlots);   // [4][256]
    const int m0 = blockIdx.y * p.tok_per_wg;
    const int tb = p.M - m0 < p.tok_per_wg ? p.M - m0 : p.tok_per_wg;
    const int r0 = blockIdx.x * 16;                                // H is a multiple of 16 here
    const int n_lines = p.n_vec / 8;
    // line L of the rows belongs to wave L % 4; a wave takes 16 of its lines per batch
    uint4 lo[kPremixLines], hi[kPremixLines];
    const uint4* wlo = p.W1 + (size_t)(r0 + line_load_row(lane)) * p.n_vec + line_load_chunk(lane);
    const uint4* whi = wlo + (size_t)8 * p.n_vec;
    auto load_batch = [&](int b) {
#pragma unroll
        for (int i = 0; i < kPremixLines; ++i) {
            const int L = (b * kPremixLines + i) * kWavesPerBlock + wave;
            lo[i] = make_uint4(0, 0, 0, 0);
            hi[i] = make_uint4(0, 0, 0, 0);
            if (L < n_lines) {                                     // wave-uniform
                lo[i] = load_stream(wlo + L * 8);
                hi[i] = load_stream(whi + L * 8);
            }
        }
    };
    // The tokens' vectors are requested before the weight lines and written to LDS after
    // those have been requested too: loads complete in order, so the tokens do not wait for
    // the 32 KB of weight lines per wave behind them, and the lines stream meanwhile.
    const int total = tb * p.n_vec;
    const uint4* hsrc = p.hidden + (size_t)m0 * p.n_vec;
    auto hs_slot = [&](int i) {
        const int t = i / p.n_vec;
        return hs + (size_t)t * stride + (i - t * p.n_vec);
    };
    uint4 st[kPremixTileStage];
#pragma unroll
    for (int j = 0; j < kPremixTileStage; ++j) {
        const int i = threadIdx.x + j * kBlock;
        if (i < total) st[j] = load_vec(hsrc + i);
    }
    for (int i = threadIdx.x + kPremixTileStage * kBlock; i < total; i += kBlock) *hs_slot(i) = hsrc[i];
    asm volatile("" ::: "memory");                                 // (keeps the order)
    load_batch(0);
    asm volatile("" ::: "memory");
#pragma unroll
    for (int j = 0; j < kPremixTileStage; ++j) {
        const int i = threadIdx.x + j * kBlock;
        if (i < total) store_vec(hs_slot(i), st[j]);
    }
    __syncthreads();
    f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const uint4* hb = hs + (size_t)(r16 < tb ? r16 : tb - 1) * stride + q4;   // columns past tb are not stored
    for (int b = 0; b * kPremixLines * kWavesPerBlock < n_lines; ++b) {       // block-uniform
        if (b) load_batch(b);
#pragma unroll
        for (int i = 0; i < kPremixLines; ++i) {
            const int L = (b * kPremixLines + i) * kWavesPerBlock + wave;
            if (L < n_lines) {                                     // wave-uniform
                uint4 s0, s1;
                mfma_operands_from_lines(lo[i], hi[i], lane, my_slice, s0, s1);
                const uint4 b0 = hb[L * 8], b1 = hb[L * 8 + 4];
                acc = mfma_tile<DT>(s0, b0, acc);
                acc = mfma_tile<DT>(s1, b1, acc);
            }
        }
    }
    *reinterpret_cast<f32x4_t*>(red + wave * 256 + lane * 4) = acc;
    __syncthreads();
    {
        const int e = threadIdx.x, l = e >> 2, i = e & 3;
        const int row = r0 + (l >> 4) * 4 + i, tok = l & 15;
        float y = 0.f;
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) y += red[w * 256 + e];    // wave order
        if (tok < tb) {
            const unsigned short* hrow = reinterpret_cast<const unsigned short*>(hs + (size_t)tok * stride);
            static_cast<unsigned short*>(p.out)[(size_t)(m0 + tok) * p.H + row] =
                narrow16<DT>(premix_act(y, p.act) + widen16<DT>(hrow[row]));
        }
    }
}

// More than 16 tokens: the token vectors no longer fit LDS whole, so they are staged in
// 512-column chunks for all token tiles at once (two buffers), and a workgroup of eight waves
// owns 16 output features: wave w takes the 64 columns w*64.. of every chunk, i.e. one
// 128-byte line of each of the 16 rows per chunk, and requests all its lines up front (the
// whole of W1 is in flight in one round).  A line pair's operands serve every token tile.
// A later chunk's token vectors are requested at the top of a chunk and written to a free
// buffer at its end.  From four tokens on; bf16 / fp16, H a multiple of 512, at most 8 chunks.
constexpr int kPremixWideWaves = 8;
constexpr int kPremixWideBlock = kPremixWideWaves * kWave;
constexpr int kPremixChunkVecs = 64;             // 16-byte vectors per 512-column chunk
constexpr int kPremixMaxChunks = 8;
constexpr int kPremixHbStride = kPremixChunkVecs + 1;            // padded rows: conflict-free B reads
constexpr int kPremixHbVecs = 64 * kPremixHbStride;              // one staging buffer: 64 token slots

__host__ __device__ inline size_t premix_wide_lds_bytes() {
    return ((size_t)2 * kPremixHbVecs + (size_t)kPremixWideWaves * kLinePairSlots) * sizeof(uint4);
}

template <int DT, int NCT, bool RING = false>
__global__ __launch_bounds__(kPremixWideBlock) void k_premix_wide(PremixParams p) {
    // NB staging buffers of 16 NCT token slots.  Loads return in order, so a token chunk
    // requested behind the weight lines would arrive only after the last of them: with one
    // or two token tiles every chunk's tokens are therefore requested first of all (they fit
    // the registers: 16 or 32 vectors per lane), staged as buffers come free, and the chunk
    // loop waits for nothing but its own weight lines.  With more token tiles the next
    // chunk's tokens are requested at the top of a chunk and staged at its end, behind the
    // weight lines (there the tokens' share of the work dominates anyway).
    // RING (three or four token tiles, H = 4096: every loop bound a constant, so that the
    // compiler's wait counts are exact): the tokens do not fit the registers whole, so both
    // streams are issued a few chunks ahead instead, interleaved in the order in which they
    // are wanted: tokens of chunk c + 2, then weight lines of chunk c + 4, at the top of
    // chunk c.  A wait for a chunk's tokens then leaves only younger requests outstanding.
    static_assert(!RING || NCT >= 3, "the ring is for token batches that do not fit the registers");
    constexpr int NB = NCT == 1 ? 8 : NCT == 2 ? 4 : 2;
    constexpr bool kUpFront = NCT <= 2;
    constexpr int D = NB - 1;
    constexpr int kBufVecs = 16 * NCT * kPremixHbStride;
    static_assert(NB * kBufVecs <= 2 * kPremixHbVecs, "the buffers fit the staging space");
    extern __shared__ uint4 smem[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int r16 = lane & 15, q4 = lane >> 4;
    uint4* hbuf = smem;
    uint4* my_slice = smem + 2 * kPremixHbVecs + (size_t)wave * kLinePairSlots;
    const int r0 = blockIdx.x * 16;
    const int n_chunks = p.n_vec / kPremixChunkVecs;

    // The residual term of the result this thread will write at the very end (feature and
    // token as in the last loop below): requested now, so that no trip to memory is left
    // behind the last weight line.
    constexpr int kOutPerThread = (NCT * 256 + kPremixWideBlock - 1) / kPremixWideBlock;
    unsigned short h_res[kOutPerThread];
#pragma unroll
    for (int j = 0; j < kOutPerThread; ++j) {
        const int e = threadIdx.x + j * kPremixWideBlock;
        const int ct = e >> 8, l = (e & 255) >> 2, i = e & 3;
        const int row = r0 + (l >> 4) * 4 + i, tok = ct * 16 + (l & 15);
        h_res[j] = 0;
        if (e < NCT * 256 && tok < p.M)
            h_res[j] = reinterpret_cast<const unsigned short*>(p.hidden)[(size_t)tok * p.H + row];
    }
    // token of slot wave + 8 i; slots past the last token hold zeros (never stored to u)
    auto fetch = [&](int c, uint4 (&st)[2 * NCT]) {
        const uint4* src = p.hidden + c * kPremixChunkVecs + lane;
#pragma unroll
        for (int i = 0; i < 2 * NCT; ++i) {
            const int s = wave + i * kPremixWideWaves;
            st[i] = make_uint4(0, 0, 0, 0);
            if (s < p.M) st[i] = load_vec(src + (size_t)s * p.n_vec);      // wave-uniform
        }
    };
    auto stage = [&](int c, const uint4 (&st)[2 * NCT]) {
        uint4* dst = hbuf + (size_t)(c % NB) * kBufVecs + (size_t)wave * kPremixHbStride + lane;
#pragma unroll
        for (int i = 0; i < 2 * NCT; ++i) store_vec(dst + (size_t)i * kPremixWideWaves * kPremixHbStride, st[i]);
    };
    if (RING) {
        constexpr int kN = kPremixMaxChunks;
        uint4 tka[2 * NCT], tkb[2 * NCT];              // token chunks: even ones in tka, odd ones in tkb
        uint4 lo[kN], hi[kN];
        const uint4* wlo = p.W1 + (size_t)(r0 + line_load_row(lane)) * p.n_vec + wave * 8 + line_load_chunk(lane);
        const uint4* whi = wlo + (size_t)8 * p.n_vec;
        auto lines = [&](int c) {
            lo[c] = load_stream(wlo + c * kPremixChunkVecs);
            hi[c] = load_stream(whi + c * kPremixChunkVecs);
        };
        fetch(0, tka);
        asm volatile("" ::: "memory");
        lines(0);
        asm volatile("" ::: "memory");
        fetch(1, tkb);
        asm volatile("" ::: "memory");
        lines(1);
        lines(2);
        lines(3);
        asm volatile("" ::: "memory");
        stage(0, tka);
        __syncthreads();
        f32x4_t acc[NCT];
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) acc[ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < kN; ++c) {
            if (c + 2 < kN) {                          // (chunk c's tokens left these registers before the last barrier)
                if (c % 2 == 0) fetch(c + 2, tka); else fetch(c + 2, tkb);
            }
            asm volatile("" ::: "memory");
            if (c + 4 < kN) lines(c + 4);
            asm volatile("" ::: "memory");
            uint4 s0, s1;
            mfma_operands_from_lines(lo[c], hi[c], lane, my_slice, s0, s1);
            const uint4* hb = hbuf + (size_t)(c % NB) * kBufVecs + wave * 8 + q4;
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const uint4 b0 = hb[(ct * 16 + r16) * kPremixHbStride];
                const uint4 b1 = hb[(ct * 16 + r16) * kPremixHbStride + 4];
                acc[ct] = mfma_tile<DT>(s0, b0, acc[ct]);
                acc[ct] = mfma_tile<DT>(s1, b1, acc[ct]);
            }
            // buffer (c + 1) % 2 was last read in chunk c - 1, before its barrier
            if (c + 1 < kN) {
                if ((c + 1) % 2 == 0) stage(c + 1, tka); else stage(c + 1, tkb);
                __syncthreads();
            }
        }
        __syncthreads();                               // every wave is done with the staging buffers
        float* red = reinterpret_cast<float*>(hbuf);   // [wave][token tile][256]
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct)
            *reinterpret_cast<f32x4_t*>(red + ((size_t)wave * NCT + ct) * 256 + lane * 4) = acc[ct];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kOutPerThread; ++j) {
            const int e = threadIdx.x + j * kPremixWideBlock;
            if (e >= NCT * 256) break;
            const int ct = e >> 8, l = (e & 255) >> 2, i = e & 3;
            const int row = r0 + (l >> 4) * 4 + i, tok = ct * 16 + (l & 15);
            float y = 0.f;
#pragma unroll
            for (int w = 0; w < kPremixWideWaves; ++w) y += red[((size_t)w * NCT + ct) * 256 + (e & 255)];
            if (tok < p.M)
                static_cast<unsigned short*>(p.out)[(size_t)tok * p.H + row] =
                    narrow16<DT>(premix_act(y, p.act) + widen16<DT>(h_res[j]));
        }
        return;
    }
    constexpr int kHeld = kUpFront ? kPremixMaxChunks : D;
    uint4 tk[kHeld][2 * NCT];
#pragma unroll
    for (int c = 0; c < kHeld; ++c)
        if (c < n_chunks) fetch(c, tk[c]);             // block-uniform
    asm volatile("" ::: "memory");                     // (keeps the order: tokens first, they return first)
    uint4 lo[kPremixMaxChunks], hi[kPremixMaxChunks];
    const uint4* wlo = p.W1 + (size_t)(r0 + line_load_row(lane)) * p.n_vec + wave * 8 + line_load_chunk(lane);
    const uint4* whi = wlo + (size_t)8 * p.n_vec;
#pragma unroll
    for (int c = 0; c < kPremixMaxChunks; ++c) {
        lo[c] = make_uint4(0, 0, 0, 0);
        hi[c] = make_uint4(0, 0, 0, 0);
        if (c < n_chunks) {                            // block-uniform
            lo[c] = load_stream(wlo + c * kPremixChunkVecs);
            hi[c] = load_stream(whi + c * kPremixChunkVecs);
        }
    }
    asm volatile("" ::: "memory");
#pragma unroll
    for (int c = 0; c < (kUpFront ? NB : D); ++c)
        if (c < n_chunks) stage(c, tk[c]);
    // The memory serves requests in the order it got them, and the other workgroups' weight
    // lines are ahead of a late workgroup's tokens: the last tokens arrive when most of W1
    // has (5 of 6.5 us at 8 tokens).  While the workgroup waits for them at the barrier, every
    // wave moves the weight lines it has got to the operand layout (its own lines, its own
    // LDS slice), so that only operand reads and matrix instructions are left behind it.
    if (kUpFront) {
#pragma unroll
        for (int c = 0; c < kPremixMaxChunks; ++c)
            if (c < n_chunks) {                        // block-uniform
                uint4 s0, s1;
                mfma_operands_from_lines(lo[c], hi[c], lane, my_slice, s0, s1);
                lo[c] = s0;
                hi[c] = s1;
            }
    }
    __syncthreads();
    f32x4_t acc[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) acc[ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < kPremixMaxChunks; ++c) {
        if (c < n_chunks) {                            // block-uniform
            const bool more = kUpFront ? c + NB < n_chunks : c + D < n_chunks;
            uint4 st[2 * NCT];
            if (!kUpFront && more) fetch(c + D, st);
            asm volatile("" ::: "memory");
            uint4 s0 = lo[c], s1 = hi[c];
            if (!kUpFront) mfma_operands_from_lines(lo[c], hi[c], lane, my_slice, s0, s1);
            const uint4* hb = hbuf + (size_t)(c % NB) * kBufVecs + wave * 8 + q4;
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const uint4 b0 = hb[(ct * 16 + r16) * kPremixHbStride];
                const uint4 b1 = hb[(ct * 16 + r16) * kPremixHbStride + 4];
                acc[ct] = mfma_tile<DT>(s0, b0, acc[ct]);
                acc[ct] = mfma_tile<DT>(s1, b1, acc[ct]);
            }
            if (kUpFront) {
                // buffer c % NB is free once every wave has read chunk c: its next tenant,
                // chunk c + NB, has been waiting in registers
                if (more) {
                    __syncthreads();
                    if (c + NB < kPremixMaxChunks) stage(c + NB, tk[c + NB < kHeld ? c + NB : 0]);
                    // (the next chunk's barrier, if it has one, also stands between this
                    // write and the reads of chunk c + NB)
                    if (!(c + 1 + NB < n_chunks)) __syncthreads();
                }
            } else {
                // buffer (c + D) % NB = (c - 1) % NB was last read in chunk c - 1, before its barrier
                if (more) stage(c + D, st);
                if (c + 1 < n_chunks) __syncthreads();
            }
        }
    }
    __syncthreads();                                   // every wave is done with the staging buffers
    // the waves' partial tiles, summed in wave order; lane l of a tile holds features
    // 4*(l/16)..+4 of token l%16
    float* red = reinterpret_cast<float*>(hbuf);       // [wave][token tile][256]
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct)
        *reinterpret_cast<f32x4_t*>(red + ((size_t)wave * NCT + ct) * 256 + lane * 4) = acc[ct];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kOutPerThread; ++j) {
        const int e = threadIdx.x + j * kPremixWideBlock;
        if (e >= NCT * 256) break;
        const int ct = e >> 8, l = (e & 255) >> 2, i = e & 3;
        const int row = r0 + (l >> 4) * 4 + i, tok = ct * 16 + (l & 15);
        float y = 0.f;
#pragma unroll
        for (int w = 0; w < kPremixWideWaves; ++w) y += red[((size_t)w * NCT + ct) * 256 + (e & 255)];
        if (tok < p.M)
            static_cast<unsigned short*>(p.out)[(size_t)tok * p.H + row] =
                narrow16<DT>(premix_act(y, p.act) + widen16<DT>(h_res[j]));
    }
}

}  // namespace
