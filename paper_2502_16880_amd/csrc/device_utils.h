// Device helpers shared by the kernels of the grouped LM head (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>

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
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

// Storage type of hidden vectors and weights (the template parameter DT of the kernels):
// fp32, bf16, or IEEE fp16; sums are fp32 in all three.  Values match coral_dtype.
enum StorageType { kF32 = 0, kBF16 = 1, kF16 = 2 };

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

// 16-byte accesses as native vectors (a struct copy is a memcpy to the compiler, which it
// cannot always turn back into registers).
__device__ __forceinline__ uint4 load_vec(const uint4* p) {
    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_vec(uint4* p, uint4 v) {
    u32x4_t o;
    o.x = v.x;
    o.y = v.y;
    o.z = v.z;
    o.w = v.w;
    *reinterpret_cast<u32x4_t*>(p) = o;
}

template <int DT>
__device__ __forceinline__ float dot_vec(uint4 w, uint4 h, float acc) {
    if (DT == kF16) {
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, w.x), __builtin_bit_cast(f16x2_t, h.x), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, w.y), __builtin_bit_cast(f16x2_t, h.y), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, w.z), __builtin_bit_cast(f16x2_t, h.z), acc, false);
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, w.w), __builtin_bit_cast(f16x2_t, h.w), acc, false);
    } else if (DT == kBF16) {
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

// One 16x16 tile step of 32 columns on the matrix cores: lane l feeds row l%16, columns
// 8*(l/16)..+8 of both operands (eight 16-bit values each) and holds rows 4*(l/16)..+4,
// column l%16 of the result.
template <int DT>
__device__ __forceinline__ f32x4_t mfma_tile(uint4 a, uint4 b, f32x4_t acc) {
    if (DT == kF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), acc, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), acc, 0, 0, 0);
}

// A 16-bit storage value as fp32, and fp32 rounded to the storage type (nearest even).
template <int DT>
__device__ __forceinline__ float widen16(unsigned short bits) {
    if (DT == kF16) return (float)__builtin_bit_cast(_Float16, bits);
    return __uint_as_float((unsigned)bits << 16);
}
template <int DT>
__device__ __forceinline__ unsigned short narrow16(float x) {
    if (DT == kF16) return __builtin_bit_cast(unsigned short, (_Float16)x);
    const unsigned u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;    // NaN stays NaN
    return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
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

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_add_i32(int x) {
    return x + __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, 0xf, false);
}

// Inclusive prefix sum over the 64 lanes (lane 63 holds the total).
__device__ __forceinline__ int wave_scan_inclusive(int x) {
    x = dpp_add_i32<0x111, 0xf>(x);   // row_shr:1
    x = dpp_add_i32<0x112, 0xf>(x);   // row_shr:2
    x = dpp_add_i32<0x114, 0xf>(x);   // row_shr:4
    x = dpp_add_i32<0x118, 0xf>(x);   // row_shr:8  -> scan inside each row of 16
    x = dpp_add_i32<0x142, 0xa>(x);   // row_bcast:15: rows 1 and 3 add the row before
    x = dpp_add_i32<0x143, 0xc>(x);   // row_bcast:31: rows 2 and 3 add the first half
    return x;
}

// MFMA operand loads.  v_mfma_f32_16x16x32_bf16 wants lane l to hold row l%16, 16-byte
// chunk l/16 of a 64-byte step; loading it that way makes neighbouring lanes touch
// different rows, which the texture addresser handles at a quarter of its rate.  So tiles
// are loaded with neighbouring lanes on contiguous bytes and moved to the layout the
// instruction wants afterwards: in registers (mfma_operands_from_quad_rows below), or
// through LDS:
// a wave load covers 8 rows x 128 bytes (lane p: row p/8, chunk p%8 of the line,
// i.e. both 32-column steps of a step pair), and the two registers that hold rows 0-7 and
// 8-15 of a tile go through a slice of kLinePairSlots slots together, which yields the
// operands of both steps (a slot of padding after every 8 keeps writes and reads
// conflict-free; LDS operations of a wave execute in order, so no barrier is needed).
__device__ __forceinline__ int line_load_row(int lane) { return lane >> 3; }
__device__ __forceinline__ int line_load_chunk(int lane) { return lane & 7; }
constexpr int kLinePairSlots = 144;
__device__ __forceinline__ void mfma_operands_from_lines(uint4 rows_lo, uint4 rows_hi, int lane,
                                                         uint4* slice, uint4& step0, uint4& step1) {
    const int w = lane + (lane >> 3);
    slice[w] = rows_lo;
    slice[72 + w] = rows_hi;
    const int r = lane & 15, q = lane >> 4;
    const int src = (r >> 3) * 72 + (r & 7) * 9 + q;
    step0 = slice[src];
    step1 = slice[src + 4];
}

// Transposition without LDS, for tiles loaded four rows x 256 contiguous bytes per wave
// load: load t of four (t = 0..3) has lane 16 q + 4 a + c on row 4 a + t, 16-byte chunk
// 4 q + c of the 256 bytes, so that every quad of lanes covers 64 contiguous bytes and every
// row two whole lines.  Exchanging t and c inside every quad of lanes (a 4 x 4 transposition
// of the four registers, two butterfly stages of DPP quad permutations) leaves in register c
// lane 16 q + i with row i, chunk 4 q + c: the operand of the 32-column step that takes the
// chunks {c, 4 + c, 8 + c, 12 + c} of the 256 bytes, as long as the other operand is read
// with the same choice of columns.
template <int CTRL>
__device__ __forceinline__ unsigned dpp_quad(unsigned x) {
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, true);   // (every source lane exists)
}
__device__ __forceinline__ void quad_transpose(unsigned& r0, unsigned& r1, unsigned& r2, unsigned& r3,
                                               bool odd, bool up) {
    // (the moves come first, with all lanes active: a DPP move under a divergent condition
    // would not see the other lanes)
    const unsigned x0 = dpp_quad<0xB1>(r0), x1 = dpp_quad<0xB1>(r1);   // quad_perm [1,0,3,2]
    const unsigned x2 = dpp_quad<0xB1>(r2), x3 = dpp_quad<0xB1>(r3);
    const unsigned a0 = odd ? x1 : r0, b0 = odd ? r1 : x0;
    const unsigned a1 = odd ? x3 : r2, b1 = odd ? r3 : x2;
    const unsigned ya0 = dpp_quad<0x4E>(a0), ya1 = dpp_quad<0x4E>(a1);  // quad_perm [2,3,0,1]
    const unsigned yb0 = dpp_quad<0x4E>(b0), yb1 = dpp_quad<0x4E>(b1);
    r0 = up ? ya1 : a0;
    r2 = up ? a1 : ya0;
    r1 = up ? yb1 : b0;
    r3 = up ? b1 : yb0;
    // (the results are wanted here, not where they are used: left to itself the compiler
    // keeps both stages' values alive across the whole gate and runs out of registers)
    asm volatile("" : "+v"(r0), "+v"(r1), "+v"(r2), "+v"(r3));
}
__device__ __forceinline__ void mfma_operands_from_quad_rows(uint4& r0, uint4& r1, uint4& r2, uint4& r3, int lane) {
    const bool odd = lane & 1, up = lane & 2;
    quad_transpose(r0.x, r1.x, r2.x, r3.x, odd, up);
    quad_transpose(r0.y, r1.y, r2.y, r3.y, odd, up);
    quad_transpose(r0.z, r1.z, r2.z, r3.z, odd, up);
    quad_transpose(r0.w, r1.w, r2.w, r3.w, odd, up);
}

// Value of the lane below (lane 0 keeps its own): one DPP move, no LDS round trip.
__device__ __forceinline__ int lane_below(int x) {
    return __builtin_amdgcn_update_dpp(x, x, 0x138 /* wave_shr:1 */, 0xf, 0xf, false);
}
__device__ __forceinline__ float lane_below(float x) {
    return __int_as_float(lane_below(__float_as_int(x)));
}

// Sorted list of the best candidates seen so far, lane i holding rank i.
// (v, id) is wave-uniform.  Lanes past the wanted k simply hold further ranks.
__device__ __forceinline__ void list_insert(float& lv, int& li, float v, int id, int lane, int k) {
    const float tv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(lv), k - 1));
    const int ti = __builtin_amdgcn_readlane(li, k - 1);
    if (!better(v, id, tv, ti)) return;                // does not reach the k best: wave-uniform
    const unsigned long long b = __ballot(better(v, id, lv, li));
    const int pos = __ffsll(b) - 1;                    // >= 0: the k-th entry is beaten
    const float sv = lane_below(lv);
    const int si = lane_below(li);
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


// Order-preserving 64-bit key: key(a) > key(b) exactly when a beats b (larger value
// first, then lower id).  -0.0 counts as +0.0, as it does for the float comparison.
__device__ __forceinline__ unsigned long long cand_key(float v, int id) {
    unsigned u = __float_as_uint(v + 0.0f);
    u ^= (u >> 31) ? 0xffffffffu : 0x80000000u;
    return ((unsigned long long)u << 32) | (unsigned)(~id);
}

// The candidate a key stands for (the value's -0.0 comes back as +0.0).
__device__ __forceinline__ float key_value(unsigned long long key) {
    const unsigned u = (unsigned)(key >> 32);
    return __uint_as_float((u >> 31) ? (u ^ 0x80000000u) : ~u);
}
__device__ __forceinline__ int key_id(unsigned long long key) { return (int)~(unsigned)key; }

}  // namespace
