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

}  // namespace
