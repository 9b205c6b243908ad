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
// A group selected by several tokens is read once for all of them (the union of the
// tokens' groups that the appendix's tree-decoding paragraph activates).
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <limits.h>
#include <stdint.h>
#include <stdlib.h>

#include <mutex>

#include "coral_lmhead.h"
#include "control_words.h"
#include "device_utils.h"
#include "fused_path.h"
#include "router_premix.h"
#include "staged_path.h"
#include "tile_path.h"
#include "tree_expand.h"

// Scratch memory of coral_lmhead_grouped_noalloc: what the other entry points take as their
// caller-provided workspace.  One copy per GPU the library runs on, held until the process
// ends; in host code the name is only a handle for hipGetSymbolAddress, never an address.
constexpr size_t kStaticScratchBytes = (size_t)CORAL_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// ---------------------------------------------------------------- host side
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline bool dtype_ok(coral_dtype dt) { return dt == CORAL_F32 || dt == CORAL_BF16 || dt == CORAL_F16; }
inline bool is_16bit(coral_dtype dt) { return dt != CORAL_F32; }
// One of three instantiations by storage type (kernels without an fp32 form pass nullptr).
#define CORAL_PICK_DT(dt, f32, bf16, f16) ((dt) == CORAL_F32 ? (f32) : (dt) == CORAL_BF16 ? (bf16) : (f16))

constexpr int kMaxWorkgroups = 256;    // upper bound of the single-launch path's grid
constexpr size_t kCtrlBytes = coral_ctrl::kWords * sizeof(unsigned int);   // control words at the start of the workspace
static_assert(coral_ctrl::kLpGroupArrivalWords >= kWave, "one arrival counter per activated group");
static_assert(coral_ctrl::kGateSelectArrivalWords * 16 >= kMaxM, "one arrival counter per token tile");

struct Layout {
    size_t ctrl, fused_part, fused_lse, fused_glist, fused_pairs, s, sel, mask, union_list, n_union, chunk_base, slot_count, part, lse_part, logp_sel, tile_mask, tile_first_block, tile_z, tile_stat, total;
    int part_stride;
};

bool sizes_ok(int M, int H, int V, int G, int g, int k) {
    if (M < 1 || H < 1 || V < 1 || k < 1) return false;
    if (G < 0 || g < 0 || (G == 0) != (g == 0) || g > G) return false;
    return true;
}

// pair_pieces: the shape can take the single-launch kernel's log-probability mode (the table
// of its per-pair pieces is the largest item and is left out otherwise).  tiles: the shape
// can take the matrix-core path (its logits buffer and span lists are left out otherwise).
// tiles_only: a layout for a call that is known to take the matrix-core path (the other
// paths' lists are left out).
Layout make_layout(int M, int V, int G, int g, int k, bool pair_pieces, bool tiles, bool tiles_only = false) {
    Layout L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    L.ctrl = take(kCtrlBytes);
    const size_t others = tiles_only ? 0 : 1;
    L.fused_part = take(others * kMaxWorkgroups * M * k * sizeof(Cand));
    L.fused_lse = take(others * kMaxWorkgroups * M * sizeof(unsigned long long));   // log-probability mode
    L.fused_glist = take(others * M * (g ? g : 1) * k * sizeof(Cand));
    // one (max, sum) piece per (row pair of a selected group, token that selected it): a
    // token's g groups are distinct, so their pairs number V / 2 + g at most
    L.fused_pairs = take(pair_pieces ? (size_t)M * ((size_t)V / 2 + g) * sizeof(unsigned long long) : 0);
    L.s = take((size_t)kGateParts * M * (G ? G : 1) * sizeof(float));
    L.sel = take((size_t)M * (g ? g : 1) * sizeof(int32_t));
    L.mask = take((size_t)(G ? G : 1) * sizeof(unsigned long long));
    L.union_list = take((size_t)(G ? G : 1) * sizeof(int32_t));
    L.n_union = take(sizeof(int32_t));
    L.chunk_base = take((size_t)M * (g ? g : 1) * sizeof(int32_t));
    L.slot_count = take((size_t)M * (g ? g : 1) * sizeof(int32_t));
    L.part_stride = (V + kChunkRows - 1) / kChunkRows + g;
    L.part = take(others * M * L.part_stride * k * sizeof(Cand));
    L.lse_part = take(others * M * L.part_stride * 2 * sizeof(float));     // log-probability mode
    L.logp_sel = take((size_t)M * (g ? g : 1) * sizeof(float));
    L.tile_mask = take((size_t)((kMaxM + 15) / 16) * (G ? G : 1) * sizeof(unsigned long long));
    L.tile_first_block = take((size_t)(G ? G : 1) * sizeof(int32_t));
    // a group's blocks round up: V / 128 + G blocks at most (+ 1: V itself rounds up)
    const size_t tile_blocks = (size_t)V / kTileRows + G + 1;
    L.tile_z = take(tiles ? tile_blocks * M * kTileRows * sizeof(float) : 0);
    L.tile_stat = take(tiles ? tile_blocks * M * sizeof(float2) : 0);
    L.total = off;
    return L;
}

coral_status check_common(const void* hidden, const void* lm_W, int M, int H, int V, int k,
                          coral_dtype dt, const int32_t* topk_ids, const float* topk_logits) {
    if (!hidden || !lm_W || !topk_ids || !topk_logits) return CORAL_ERR_NULL;
    if (!dtype_ok(dt)) return CORAL_ERR_SHAPE;
    if (M < 1 || H < 1 || V < 1 || k < 1) return CORAL_ERR_SHAPE;
    if (M > kMaxM || k > kMaxK) return CORAL_ERR_UNSUPPORTED;
    if (H % (is_16bit(dt) ? 8 : 4) != 0) return CORAL_ERR_UNSUPPORTED;
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

// Launch of the kernel that streams the weight rows.  The measurement entry points pass two
// events: they are bound to this launch and take the kernel's own start and stop times (what
// a kernel trace reports as its duration), not the times at which event records before and
// after it would be reached, which include the dispatch latency.
template <class F, class... Args>
coral_status launch_timed(F fn, dim3 grid, dim3 block, size_t lds, hipStream_t stream, void* ev_before,
                          void* ev_after, Args... args) {
    if (ev_before && ev_after)
        hipExtLaunchKernelGGL(fn, grid, block, (uint32_t)lds, stream, static_cast<hipEvent_t>(ev_before),
                              static_cast<hipEvent_t>(ev_after), 0, args...);
    else
        hipLaunchKernelGGL(fn, grid, block, lds, stream, args...);
    return launch_status();
}

// The only state the library keeps between calls: per device, the number of compute units
// (the single-launch path runs one workgroup on each) and the largest dynamic LDS size each
// kernel has been allowed so far.  Both are properties of the device and of the loaded code
// object, looked up once instead of on every call; a mutex guards them.
constexpr int kMaxDevices = 64;
constexpr int kMaxKernels = 96;
struct DeviceCache {
    int compute_units;
    void* scratch_ptr;          // this device's copy of `scratch`, looked up on first use
    int n_kernels;
    const void* kernel[kMaxKernels];
    int lds_bytes[kMaxKernels];
};
DeviceCache g_cache[kMaxDevices];
std::mutex g_cache_mutex;

int compute_units() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    if (g_cache[dev].compute_units == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return 0;
        g_cache[dev].compute_units = n;
    }
    return g_cache[dev].compute_units;
}

// Device address of this device's copy of the static scratch array.
coral_status static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CORAL_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    if (!g_cache[dev].scratch_ptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return CORAL_ERR_HIP;
        g_cache[dev].scratch_ptr = ptr;
    }
    *out = g_cache[dev].scratch_ptr;
    return CORAL_OK;
}

// Lets kernel `fn` use `bytes` of dynamic LDS on the current device (needed above 64 KB).
bool allow_lds(const void* fn, int bytes) {
    if (bytes <= 64 * 1024) return true;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    DeviceCache* c = dev >= 0 && dev < kMaxDevices ? &g_cache[dev] : nullptr;
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    int slot = -1;
    if (c) {
        for (int i = 0; i < c->n_kernels; ++i)
            if (c->kernel[i] == fn) slot = i;
        if (slot >= 0 && c->lds_bytes[slot] >= bytes) return true;
    }
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
        return false;
    if (c) {
        if (slot < 0 && c->n_kernels < kMaxKernels) {
            slot = c->n_kernels++;
            c->kernel[slot] = fn;
        }
        if (slot >= 0) c->lds_bytes[slot] = bytes;
    }
    return true;
}

// Gate of the single-launch path: from four tokens on it goes through the matrix cores (16-bit
// storage only; measured at the Llama3 shape: two tokens 52.1 against 50.8 us on the vector
// units, three equal, four 81.0 against 81.5).
int fused_gate_mode(bool dense, int M, int G, int g, int k, int jp, coral_dtype dt, bool logprob = false) {
    (void)G; (void)g; (void)k; (void)jp; (void)logprob;
    return dense || !is_16bit(dt) || M <= 3 ? kGateVector : kGateMfma;
}

// Activated groups at most.
inline long long max_union(int M, int G, int g) { return (long long)M * g < G ? (long long)M * g : G; }

// The single-launch kernel's log-probability mode gives every activated group workgroups of
// its own and ranks the groups in one wave: at most 64 activated groups, fewer than half the
// workgroups; a token's g lists share the LDS of one wave's lists.
bool fused_logprob_fits(int M, int G, int g, int k, int jp, coral_dtype dt, int workgroups) {
    if (jp > kFusedSegs || g > kFusedWaves) return false;
    const long long um = max_union(M, G, g);
    if (um > kWave || 2 * um > workgroups) return false;
    return fused_lds_layout(M, G, g, k, jp, false, fused_gate_mode(false, M, G, g, k, jp, dt, true), true)
               .total <= kLdsLimit;
}

// What a draft-level call adds to the log-probability head: the expansion of the tree level
// whose nodes are the call's tokens.
struct LevelExpand {
    const float* parent_score;
    int n_next;
    int32_t* next_parent;
    int32_t* next_token;
    float* next_score;
};

bool layout_has_pair_pieces(int M, int H, int G, int g, int k, coral_dtype dt) {
    if (G < 1 || !dtype_ok(dt)) return false;
    const int n_vec = H / (is_16bit(dt) ? 8 : 4);
    return fused_logprob_fits(M, G, g, k, (n_vec + kWave - 1) / kWave, dt, kMaxWorkgroups);
}

// Enqueues the single-launch path (the caller has checked with plan_path that it fits).
coral_status launch_fused(bool dense, const void* hidden, const void* gate_hidden, const void* gate_W,
               const float* gate_bias,
               const void* lm_W, const coral_group_index* gi, int M, int H, int V, int G, int g,
               int k, coral_dtype dt, int32_t* topk_ids, float* topk_logits, int32_t* sel_groups,
               char* ws, const Layout& L, hipStream_t stream, void* ev_before, void* ev_after,
               bool logprob = false, const LevelExpand* level = nullptr, int max_group_rows = 0) {
    const int n_vec = H / (is_16bit(dt) ? 8 : 4);
    const int jp = (n_vec + kWave - 1) / kWave;
    const int gate = fused_gate_mode(dense, M, G, g, k, jp, dt, logprob);
    int P = compute_units();
    if (P < 1) return CORAL_ERR_HIP;
    if (P > kMaxWorkgroups) P = kMaxWorkgroups;
    // Collected candidates instead of per-wave lists, where a workgroup is sure to meet at
    // most kCollectCap rows per token: it takes 16 consecutive row pairs out of every 16 P of
    // the concatenated activated groups, so of any group (a run of at most `pairs` pairs) it
    // meets no more than 16 * (pairs / 16P) + min(16, pairs % 16P), and a token has g groups.
    bool collect = false;
    if (!dense && !logprob && max_group_rows > 0) {
        const long long period = (long long)kFusedWaves * P;
        const long long pairs = ((long long)max_group_rows + kFusedRows - 1) / kFusedRows;
        const long long rest = pairs % period;
        const long long per_group = kFusedWaves * (pairs / period) + (rest < kFusedWaves ? rest : kFusedWaves);
        collect = kFusedRows * per_group * g <= kCollectCap &&
                  fused_lds_layout(M, G, g, k, jp, false, gate, false, true).total <= kLdsLimit;
    }
    const FusedLds F = fused_lds_layout(M, G, g, k, jp, dense, gate, logprob, collect);
    if (jp > kFusedSegs || F.total > kLdsLimit) return CORAL_ERR_UNSUPPORTED;   // not reached
    FusedParams p = {};
    p.collect = collect ? 1 : 0;
    // Measured with rows of 8 KB (Llama shapes): dense head, one or two tokens: 6 waves 158 us
    // against 165 us with all 16 (Llama2: 46.5 against 48.5 us); four tokens: 10 waves 162 us
    // against 168 us.  Rows of 7 KB (Qwen shape) and the grouped head's gathered rows are
    // fastest with all 16 (Qwen dense: 163 us against 170 us with 6).
    const bool rows_of_8k = ((size_t)n_vec * 16) % 8192 == 0;
    p.stream_waves = !dense || !rows_of_8k ? kFusedWaves : M <= 2 ? 6 : M <= 4 ? 10 : kFusedWaves;
    p.hidden = static_cast<const uint4*>(hidden);
    p.gate_hidden = static_cast<const uint4*>(gate_hidden);
    p.gate_W = static_cast<const uint4*>(gate_W);
    p.bias = gate_bias;
    p.lm_W = static_cast<const uint4*>(lm_W);
    p.offsets = gi ? gi->group_offsets : nullptr;
    p.rows = gi ? gi->group_rows : nullptr;
    p.sel_out = sel_groups;
    p.part = reinterpret_cast<Cand*>(ws + L.fused_part);
    p.lse_part = reinterpret_cast<unsigned long long*>(ws + L.fused_lse);
    p.glist = reinterpret_cast<Cand*>(ws + L.fused_glist);
    p.pair_lse = reinterpret_cast<unsigned long long*>(ws + L.fused_pairs);
    if (level) {
        p.parent_score = level->parent_score;
        p.n_next = level->n_next;
        p.next_parent = level->next_parent;
        p.next_token = level->next_token;
        p.next_score = level->next_score;
    }
    p.counter = reinterpret_cast<unsigned int*>(ws + L.ctrl) + coral_ctrl::kFusedArrival;
    p.topk_ids = topk_ids;
    p.topk_logits = topk_logits;
    p.M = M; p.V = V; p.G = G; p.g = g; p.k = k;
    p.n_vec = n_vec; p.jp = jp;
    typedef void (*fused_fn)(FusedParams);
    const bool routed = !dense && gate_hidden != hidden;
    fused_fn fn;
#define CORAL_FUSED_GATES(DT, R, LP)                                                             \
    (gate == kGateMfma ? k_fused<DT, false, kGateMfma, R, LP> : k_fused<DT, false, kGateVector, R, LP>)
    if (logprob && (dense || 2 * max_union(M, G, g) > P)) return CORAL_ERR_UNSUPPORTED;   // not reached
    if (logprob && routed)
        fn = CORAL_PICK_DT(dt, (k_fused<kF32, false, kGateVector, true, true>),
                           CORAL_FUSED_GATES(kBF16, true, true), CORAL_FUSED_GATES(kF16, true, true));
    else if (logprob)
        fn = CORAL_PICK_DT(dt, (k_fused<kF32, false, kGateVector, false, true>),
                           CORAL_FUSED_GATES(kBF16, false, true), CORAL_FUSED_GATES(kF16, false, true));
    else if (dense)
        fn = CORAL_PICK_DT(dt, (k_fused<kF32, true, kGateVector>), (k_fused<kBF16, true, kGateVector>),
                           (k_fused<kF16, true, kGateVector>));
    else if (routed)
        fn = CORAL_PICK_DT(dt, (k_fused<kF32, false, kGateVector, true>), CORAL_FUSED_GATES(kBF16, true, false),
                           CORAL_FUSED_GATES(kF16, true, false));
    else
        fn = CORAL_PICK_DT(dt, (k_fused<kF32, false, kGateVector, false>), CORAL_FUSED_GATES(kBF16, false, false),
                           CORAL_FUSED_GATES(kF16, false, false));
#undef CORAL_FUSED_GATES
    if (!allow_lds(reinterpret_cast<const void*>(fn), F.total)) return CORAL_ERR_HIP;
    return launch_timed(fn, dim3(P), dim3(kFusedBlock), F.total, stream, ev_before, ev_after, p);
}

// The dense head goes to the matrix-core path from 8 tokens on, if the vocabulary gives every
// workgroup at least two 128-row blocks (below that its per-block set-up and epilogue
// dominate and the vector path is faster).
bool dense_prefers_tiles(int M, int V) { return M >= 8 && V >= 2 * kMaxWorkgroups * kTileRows; }

// Matrix-core path: 16-bit storage, whole 512-column chunks, weights below 4 GiB, LDS plan within the limit.
bool tiles_fit(int M, int H, int V, int G, int g, int k, coral_dtype dt, int* u_max_out, int* lds_out) {
    if (!is_16bit(dt) || k > kMaxK || M > 64 || H % (kChunkVecs * 8) != 0) return false;
    if ((unsigned long long)V * H * 2ull >= (1ull << 32)) return false;   // 32-bit weight offsets
    long long um = (long long)M * g < G ? (long long)M * g : G;
    if (um < 1) um = 1;
    const TileLds T = tile_lds_layout((int)um);
    if (T.total > kLdsLimit) return false;
    // the ranking kernel keeps a few words per block of a token's groups in LDS
    if ((long long)V / kTileRows + g + 1 > (1 << 16)) return false;
    if (tile_select_lds_layout(g > 0 ? g : 1, V / kTileRows + g + 1).total > kLdsLimit) return false;
    *u_max_out = (int)um;
    *lds_out = T.total;
    return true;
}

// Which path a call takes, decided in one place for the entry points and the path query.
struct PathPlan {
    int path;            // 0 staged, 1 single launch, 2 tiles, -1 none (the staged path's
                         // token batch and lists do not fit LDS: rows beyond about 10 K values)
    int tile_umax, tile_lds;
};

bool staged_fits(int M, int jp, int k) {
    return logits_lds_bytes(M < kTokBatch ? M : kTokBatch, jp, k) <= (size_t)kLdsLimit;
}

PathPlan plan_path(bool dense, int M, int H, int V, int G, int g, int k, coral_dtype dt,
                   bool logprob = false) {
    PathPlan pl = {};
    const int n_vec = H / (is_16bit(dt) ? 8 : 4);
    const int jp = (n_vec + kWave - 1) / kWave;
    if (logprob) {     // the single-launch kernel where it fits, else the tile path, else the staged path
        pl.path = staged_fits(M, jp, k) ? 0 : -1;
        if (dense) return pl;
        if (fused_logprob_fits(M, G, g, k, jp, dt, kMaxWorkgroups)) {
            pl.path = 1;
        } else if (tiles_fit(M, H, V, G, g, k, dt, &pl.tile_umax, &pl.tile_lds) && G <= kWave) {
            pl.path = 2;                    // (k_gate_select leaves log p_router for up to 64 groups)
        }
        return pl;
    }
    const bool fused_ok =
        jp <= kFusedSegs &&
        fused_lds_layout(M, dense ? 0 : G, dense ? 0 : g, k, jp, dense,
                         fused_gate_mode(dense, M, dense ? 0 : G, dense ? 0 : g, k, jp, dt)).total <= kLdsLimit;
    const bool tiles_ok =
        tiles_fit(M, H, V, dense ? 0 : G, dense ? 0 : g, k, dt, &pl.tile_umax, &pl.tile_lds);
    if (dense && dense_prefers_tiles(M, V) && tiles_ok)
        pl.path = 2;
    else if (fused_ok)
        pl.path = 1;
    else if (tiles_ok)
        pl.path = 2;
    else
        pl.path = staged_fits(M, jp, k) ? 0 : -1;
    return pl;
}

// Whether a call with these sizes (grouped in either output mode, or dense when G = 0) can
// take the matrix-core path: the workspace then holds its logits buffer and span lists.
bool layout_has_tiles(int M, int H, int V, int G, int g, int k, coral_dtype dt) {
    if (!dtype_ok(dt) || H % (is_16bit(dt) ? 8 : 4) != 0) return false;
    if (plan_path(true, M, H, V, 0, 0, k, dt).path == 2) return true;
    if (G < 1) return false;
    return plan_path(false, M, H, V, G, g, k, dt).path == 2 ||
           plan_path(false, M, H, V, G, g, k, dt, true).path == 2;
}

// Enqueues k_tiles and the ranking of the logits it leaves.  For the grouped head the gate
// and selection kernel must already be enqueued (selection, the token tiles' masks; in the
// log-probability mode log p_router of the selection too).
coral_status launch_tiles(bool dense, const void* hidden, const void* lm_W,
                          const coral_group_index* gi, int M, int H, int V,
                          int G, int k, coral_dtype dt, int u_max, int lds, int32_t* topk_ids,
                          float* topk_out, char* ws, const Layout& L, hipStream_t stream,
                          void* ev_before, void* ev_after, const int32_t* sel = nullptr, int g = 0,
                          bool logprob = false) {
    int P = compute_units();
    if (P < 1) return CORAL_ERR_HIP;
    if (P > kMaxWorkgroups) P = kMaxWorkgroups;
    TileParams p = {};
    p.hidden = static_cast<const uint4*>(hidden);
    p.lm_W = static_cast<const uint4*>(lm_W);
    p.rows = gi ? gi->group_rows : nullptr;
    p.offsets = gi ? gi->group_offsets : nullptr;
    p.tile_mask = reinterpret_cast<const unsigned long long*>(ws + L.tile_mask);
    p.group_mask = reinterpret_cast<unsigned long long*>(ws + L.mask);
    p.group_first_block = reinterpret_cast<int32_t*>(ws + L.tile_first_block);
    p.z = reinterpret_cast<float*>(ws + L.tile_z);
    p.stat = reinterpret_cast<float2*>(ws + L.tile_stat);
    p.want_lse = logprob ? 1 : 0;
    p.next_block = reinterpret_cast<unsigned int*>(ws + L.ctrl) + coral_ctrl::kTileQueue;
    p.M = M; p.V = V; p.G = G;
    p.n_vec = H / 8;
    p.n_chunks = (p.n_vec + kChunkVecs - 1) / kChunkVecs;
    p.u_max = u_max;
    typedef void (*tiles_fn)(TileParams, int);
    const tiles_fn fn = dt == CORAL_F16 ? k_tiles<kF16> : k_tiles<kBF16>;
    if (!allow_lds(reinterpret_cast<const void*>(fn), lds)) return CORAL_ERR_HIP;
    coral_status st;
    if ((st = launch_timed(fn, dim3(P), dim3(kTileBlock), lds, stream, ev_before, ev_after, p, dense ? 1 : 0)) !=
        CORAL_OK)
        return st;

    TileSelectParams q = {};
    q.z = p.z;
    q.stat = p.stat;
    q.sel = sel;
    q.offsets = p.offsets;
    q.rows = p.rows;
    q.group_first_block = p.group_first_block;
    q.group_mask = p.group_mask;
    q.logp_sel = reinterpret_cast<const float*>(ws + L.logp_sel);
    q.next_block = p.next_block;
    q.topk_ids = topk_ids;
    q.topk_out = topk_out;
    q.M = M; q.V = V; q.g = g; q.k = k;
    q.max_blocks = V / kTileRows + g + 1;
    const int select_lds = tile_select_lds_layout(dense ? 1 : g, q.max_blocks).total;
    typedef void (*select_fn)(TileSelectParams);
    const select_fn sf = dense ? k_tile_select<true, false>
                               : logprob ? k_tile_select<false, true> : k_tile_select<false, false>;
    if (!allow_lds(reinterpret_cast<const void*>(sf), select_lds)) return CORAL_ERR_HIP;
    hipLaunchKernelGGL(sf, dim3(M), dim3(kSelectThreads), select_lds, stream, q);
    return launch_status();
}

}  // namespace

// Yardstick for the bench line: a kernel that only reads, in the single-launch path's shape.
// One workgroup per compute unit, `waves` waves each; a wave takes consecutive 16 KB pieces
// dealt round robin over waves and workgroups, 16 non-temporal 1 KB loads in flight per piece.
namespace {
__global__ __launch_bounds__(kFusedBlock) void k_probe_read(const uint4* __restrict__ src, unsigned long long pieces) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const unsigned long long stride = (unsigned long long)gridDim.x * (blockDim.x / kWave);
    unsigned x = 0u;
    for (unsigned long long q = (unsigned long long)blockIdx.x * (blockDim.x / kWave) + wave; q < pieces; q += stride) {
        const uint4* p = src + q * 1024 + lane;
        uint4 v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = load_stream(p + i * kWave);
#pragma unroll
        for (int i = 0; i < 16; ++i) x ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
    }
    asm volatile("" ::"v"(x));                          // (keeps the loads: nothing is written)
}
}  // namespace

extern "C" coral_status coral_probe_read(const void* src, size_t bytes, int waves, void* hip_stream,
                                         void* ev_before, void* ev_after) {
    if (!src || !ev_before || !ev_after) return CORAL_ERR_NULL;
    if (bytes < 16384 || bytes % 16384 != 0 || waves < 1 || waves > kFusedWaves) return CORAL_ERR_SHAPE;
    if ((uintptr_t)src & 15u) return CORAL_ERR_UNSUPPORTED;
    int P = compute_units();
    if (P < 1) return CORAL_ERR_HIP;
    if (P > kMaxWorkgroups) P = kMaxWorkgroups;
    return launch_timed(k_probe_read, dim3(P), dim3(waves * kWave), 0, static_cast<hipStream_t>(hip_stream),
                        ev_before, ev_after, static_cast<const uint4*>(src), (unsigned long long)(bytes / 16384));
}

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
    if (!sizes_ok(M, H, V, G, g, k)) return 0;
    return make_layout(M, V, G, g, k, layout_has_pair_pieces(M, H, G, g, k, dt),
                       layout_has_tiles(M, H, V, G, g, k, dt)).total;
}

extern "C" int coral_lmhead_path(int dense, int M, int H, int V, int G, int g, int k,
                                 coral_dtype dt) {
    if (!dtype_ok(dt)) return -1;
    if (M < 1 || H < 1 || V < 1 || k < 1 || M > kMaxM || k > kMaxK) return -1;
    if (H % (is_16bit(dt) ? 8 : 4) != 0) return -1;
    if (!dense && (G < 1 || g < 1 || g > G || G > kMaxG)) return -1;
    return plan_path(dense != 0, M, H, V, G, g, k, dt).path;
}

extern "C" int coral_lmhead_logprob_path(int M, int H, int V, int G, int g, int k, coral_dtype dt) {
    if (coral_lmhead_path(0, M, H, V, G, g, k, dt) < 0) return -1;
    return plan_path(false, M, H, V, G, g, k, dt, true).path;
}

extern "C" coral_status coral_lmhead_workspace_init(void* workspace, size_t workspace_bytes,
                                                    void* hip_stream) {
    coral_status st = check_workspace(workspace, workspace_bytes, kCtrlBytes);
    if (st != CORAL_OK) return st;
    hipLaunchKernelGGL(k_zero_words, dim3((kCtrlBytes / 4 + 255) / 256), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<unsigned int*>(workspace),
                       (int)(kCtrlBytes / 4));
    return launch_status();
}

namespace {

coral_status grouped_impl(const void* hidden, const void* gate_hidden, const void* gate_W,
                          const float* gate_bias, const void* lm_W, const coral_group_index* gi, int M, int H, int V,
                          int g, int k, coral_dtype dt, int32_t* topk_ids, float* topk_logits,
                          int32_t* sel_groups, void* workspace, size_t workspace_bytes,
                          void* hip_stream, void* ev_before, void* ev_after, bool logprob,
                          const LevelExpand* level = nullptr, bool static_workspace = false) {
    if (!gate_W || !gi) return CORAL_ERR_NULL;
    coral_status st = check_common(hidden, lm_W, M, H, V, k, dt, topk_ids, topk_logits);
    if (st != CORAL_OK) return st;
    if (!gi->group_offsets_host || !gi->group_offsets || !gi->group_rows) return CORAL_ERR_NULL;
    const int G = gi->G;
    if (G < 1 || g < 1 || g > G) return CORAL_ERR_SHAPE;
    if (G > kMaxG) return CORAL_ERR_UNSUPPORTED;
    if (!gate_hidden) gate_hidden = hidden;      // the router sees what the LM head sees
    if (((uintptr_t)gate_W | (uintptr_t)gate_hidden) & 15u) return CORAL_ERR_UNSUPPORTED;
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
    // (the static scratch serves the logit ranking only: no table of per-pair pieces, and the
    // matrix-core path's buffers only if this very call takes that path)
    const bool static_tiles = static_workspace && plan_path(false, M, H, V, G, g, k, dt).path == 2;
    const Layout L = make_layout(M, V, G, g, k, !static_workspace && layout_has_pair_pieces(M, H, G, g, k, dt),
                                 static_workspace ? static_tiles : layout_has_tiles(M, H, V, G, g, k, dt),
                                 static_tiles);
    if (static_workspace) {
        if (logprob || L.total > kStaticScratchBytes) return CORAL_ERR_WORKSPACE;
    } else {
        st = check_workspace(workspace, workspace_bytes, L.total);
        if (st != CORAL_OK) return st;
    }

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    PathPlan plan = plan_path(false, M, H, V, G, g, k, dt, logprob);
    if (logprob && plan.path == 1) {   // a device with few compute units: see fused_logprob_fits
        const int cu = compute_units();
        if (2 * max_union(M, G, g) > (cu < kMaxWorkgroups ? cu : kMaxWorkgroups))
            plan.path = staged_fits(M, ((H / (is_16bit(dt) ? 8 : 4)) + kWave - 1) / kWave, k) ? 0 : -1;
    }
    if (plan.path < 0) return CORAL_ERR_UNSUPPORTED;       // before anything is enqueued
    if (static_workspace) {
        // this device's copy of the array; its control words are cleared by a fill kernel on
        // the call's stream (the array keeps whatever the last call on this GPU left there)
        if ((st = static_scratch(&workspace)) != CORAL_OK) return st;
        hipLaunchKernelGGL(k_zero_words, dim3((kCtrlBytes / 4 + 255) / 256), dim3(256), 0, stream,
                           static_cast<unsigned int*>(workspace), (int)(kCtrlBytes / 4));
        if ((st = launch_status()) != CORAL_OK) return st;
    }
    char* ws = static_cast<char*>(workspace);
    if (plan.path == 1)
        return launch_fused(false, hidden, gate_hidden, gate_W, gate_bias, lm_W, gi, M, H, V, G, g, k, dt, topk_ids,
                            topk_logits, sel_groups, ws, L, stream, ev_before, ev_after, logprob, level, max_rows);
    float* s = reinterpret_cast<float*>(ws + L.s);
    int32_t* sel = sel_groups ? sel_groups : reinterpret_cast<int32_t*>(ws + L.sel);
    unsigned long long* mask = reinterpret_cast<unsigned long long*>(ws + L.mask);
    int32_t* union_list = reinterpret_cast<int32_t*>(ws + L.union_list);
    int32_t* n_union = reinterpret_cast<int32_t*>(ws + L.n_union);
    int32_t* chunk_base = reinterpret_cast<int32_t*>(ws + L.chunk_base);
    Cand* part = reinterpret_cast<Cand*>(ws + L.part);

    const int n_vec = H / (is_16bit(dt) ? 8 : 4);
    const uint4* hid = static_cast<const uint4*>(hidden);
    const uint4* ghid = static_cast<const uint4*>(gate_hidden);
    const uint4* gw = static_cast<const uint4*>(gate_W);
    if (plan.path == 2) {
        GateSelParams q = {};
        q.hidden = ghid; q.gate_W = gw; q.bias = gate_bias; q.s = s; q.sel = sel;
        q.tile_mask = reinterpret_cast<unsigned long long*>(ws + L.tile_mask);
        q.counters = reinterpret_cast<unsigned int*>(ws + L.ctrl) + coral_ctrl::kGateSelectArrival;
        q.M = M; q.G = G; q.g = g; q.n_vec = n_vec;
        if (logprob) q.logp_sel = reinterpret_cast<float*>(ws + L.logp_sel);
        const int tiles = ((G + 15) / 16) * ((M + 15) / 16);
        typedef void (*gate_select_fn)(GateSelParams);
        const gate_select_fn gs = dt == CORAL_F16 ? k_gate_select<kF16> : k_gate_select<kBF16>;
        hipLaunchKernelGGL(gs, dim3(tiles, kGateParts), dim3(kFusedBlock), 0, stream, q);
        if ((st = launch_status()) != CORAL_OK) return st;
        st = launch_tiles(false, hidden, lm_W, gi, M, H, V, G, k, dt,
                          plan.tile_umax, plan.tile_lds, topk_ids, topk_logits, ws, L, stream, ev_before,
                          ev_after, sel, g, logprob);
        if (st != CORAL_OK || !level) return st;
        hipLaunchKernelGGL(k_tree_expand, dim3(M), dim3(kWave), (size_t)M * k * sizeof(unsigned long long),
                           stream, level->parent_score, topk_ids, topk_logits, M, k, level->n_next,
                           level->next_parent, level->next_token, level->next_score);
        return launch_status();
    }
    typedef void (*gate_fn)(const uint4*, const uint4*, const float*, int, int, int, float*);
    const gate_fn gate_kernel = CORAL_PICK_DT(dt, k_gate<kF32>, k_gate<kBF16>, k_gate<kF16>);
    hipLaunchKernelGGL(gate_kernel, dim3(G), dim3(kBlock), 0, stream, ghid, gw, gate_bias, M, G, n_vec, s);
    if ((st = launch_status()) != CORAL_OK) return st;
    float* logp_sel = logprob ? reinterpret_cast<float*>(ws + L.logp_sel) : nullptr;
    hipLaunchKernelGGL(k_select, dim3(1), dim3(kBlock), 0, stream, s, gi->group_offsets, M, G, g, sel,
                       mask, union_list, n_union, chunk_base, logp_sel,
                       logprob ? reinterpret_cast<int32_t*>(ws + L.slot_count) : nullptr);
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
    p.lse_part = logprob ? reinterpret_cast<float*>(ws + L.lse_part) : nullptr;
    p.M = M; p.V = V; p.G = G; p.g = g; p.k = k;
    p.n_vec = n_vec;
    p.jp = (n_vec + kWave - 1) / kWave;
    p.tb_max = M < kTokBatch ? M : kTokBatch;
    p.part_stride = L.part_stride;
    const size_t lds = logits_lds_bytes(p.tb_max, p.jp, k);       // fits: plan_path checked it
    const int chunks = (max_rows + kChunkRows - 1) / kChunkRows;
    const long long union_max = max_union(M, G, g);
    if (chunks < 1) return CORAL_ERR_SHAPE;
    dim3 grid(chunks, (unsigned)union_max);
    typedef void (*logits_fn)(LogitsParams);
    const logits_fn fn =
        logprob ? CORAL_PICK_DT(dt, (k_logits<kF32, false, true>), (k_logits<kBF16, false, true>),
                                (k_logits<kF16, false, true>))
                : CORAL_PICK_DT(dt, (k_logits<kF32, false, false>), (k_logits<kBF16, false, false>),
                                (k_logits<kF16, false, false>));
    if (!allow_lds(reinterpret_cast<const void*>(fn), (int)lds)) return CORAL_ERR_HIP;
    if ((st = launch_timed(fn, grid, dim3(kBlock), lds, stream, ev_before, ev_after, p)) != CORAL_OK) return st;
    if (logprob)
        hipLaunchKernelGGL(k_merge_logprob<4>, dim3(M), dim3(kBlock), 0, stream, part, p.lse_part,
                           L.part_stride, reinterpret_cast<const int32_t*>(ws + L.slot_count), chunk_base,
                           logp_sel, g, k, topk_ids, topk_logits);
    else
        hipLaunchKernelGGL(k_merge, dim3(M), dim3(kBlock), 0, stream, part, L.part_stride, sel,
                           gi->group_offsets, g, 0, k, topk_ids, topk_logits);
    if ((st = launch_status()) != CORAL_OK || !level) return st;
    // draft-level call on the multi-kernel path: the expansion is one more launch
    hipLaunchKernelGGL(k_tree_expand, dim3(M), dim3(kWave), (size_t)M * k * sizeof(unsigned long long),
                       stream, level->parent_score, topk_ids, topk_logits, M, k, level->n_next,
                       level->next_parent, level->next_token, level->next_score);
    return launch_status();
}

coral_status dense_impl(const void* hidden, const void* lm_W, int M, int H, int V, int k,
                        coral_dtype dt, int32_t* topk_ids, float* topk_logits, void* workspace,
                        size_t workspace_bytes, void* hip_stream, void* ev_before,
                        void* ev_after) {
    coral_status st = check_common(hidden, lm_W, M, H, V, k, dt, topk_ids, topk_logits);
    if (st != CORAL_OK) return st;
    if (k > V) return CORAL_ERR_SHAPE;
    const Layout L = make_layout(M, V, 0, 0, k, false, layout_has_tiles(M, H, V, 0, 0, k, dt));
    st = check_workspace(workspace, workspace_bytes, L.total);
    if (st != CORAL_OK) return st;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    const PathPlan plan = plan_path(true, M, H, V, 0, 0, k, dt);
    if (plan.path < 0) return CORAL_ERR_UNSUPPORTED;
    // many tokens per row: the contraction is no longer cheap on the vector units
    if (plan.path == 2)
        return launch_tiles(true, hidden, lm_W, nullptr, M, H, V, 0, k, dt,
                            plan.tile_umax, plan.tile_lds, topk_ids, topk_logits, ws, L, stream,
                            ev_before, ev_after);
    if (plan.path == 1)
        return launch_fused(true, hidden, nullptr, nullptr, nullptr, lm_W, nullptr, M, H, V, 0, 0, k, dt, topk_ids,
                            topk_logits, nullptr, ws, L, stream, ev_before, ev_after);
    LogitsParams p = {};
    p.hidden = static_cast<const uint4*>(hidden);
    p.lm_W = static_cast<const uint4*>(lm_W);
    p.part = reinterpret_cast<Cand*>(ws + L.part);
    p.M = M; p.V = V; p.G = 0; p.g = 0; p.k = k;
    p.n_vec = H / (is_16bit(dt) ? 8 : 4);
    p.jp = (p.n_vec + kWave - 1) / kWave;
    p.tb_max = M < kTokBatch ? M : kTokBatch;
    p.part_stride = L.part_stride;
    const size_t lds = logits_lds_bytes(p.tb_max, p.jp, k);
    const int chunks = (V + kChunkRows - 1) / kChunkRows;
    typedef void (*logits_fn)(LogitsParams);
    const logits_fn fn = CORAL_PICK_DT(dt, (k_logits<kF32, true>), (k_logits<kBF16, true>), (k_logits<kF16, true>));
    if (!allow_lds(reinterpret_cast<const void*>(fn), (int)lds)) return CORAL_ERR_HIP;
    if ((st = launch_timed(fn, dim3(chunks), dim3(kBlock), lds, stream, ev_before, ev_after, p)) != CORAL_OK) return st;
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
    return grouped_impl(hidden, nullptr, gate_W, gate_bias, lm_W, gi, M, H, V, g, k, dt, topk_ids,
                        topk_logits, sel_groups, workspace, workspace_bytes, hip_stream, nullptr,
                        nullptr, false);
}

extern "C" coral_status coral_lmhead_grouped_noalloc(const void* hidden, const void* gate_W,
                                                     const float* gate_bias, const void* lm_W,
                                                     const coral_group_index* gi, int M, int H, int V,
                                                     int g, int k, coral_dtype dt, int32_t* topk_ids,
                                                     float* topk_logits, int32_t* sel_groups,
                                                     void* hip_stream) {
    return grouped_impl(hidden, nullptr, gate_W, gate_bias, lm_W, gi, M, H, V, g, k, dt, topk_ids,
                        topk_logits, sel_groups, nullptr, 0, hip_stream, nullptr, nullptr, false,
                        nullptr, true);
}

extern "C" coral_status coral_lmhead_grouped_routed(
    const void* hidden, const void* gate_hidden, const void* gate_W, const float* gate_bias,
    const void* lm_W, const coral_group_index* gi, int M, int H, int V, int g, int k,
    coral_dtype dt, int logprob, int32_t* topk_ids, float* topk_out, int32_t* sel_groups,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
    return grouped_impl(hidden, gate_hidden, gate_W, gate_bias, lm_W, gi, M, H, V, g, k, dt, topk_ids,
                        topk_out, sel_groups, workspace, workspace_bytes, hip_stream, nullptr,
                        nullptr, logprob != 0);
}

extern "C" coral_status coral_lmhead_draft_level(
    const void* hidden, const void* gate_hidden, const void* gate_W, const float* gate_bias,
    const void* lm_W, const coral_group_index* gi, int M, int H, int V, int g, int k,
    coral_dtype dt, const float* parent_score, int n_next, int32_t* topk_ids, float* topk_logprob,
    int32_t* sel_groups, int32_t* next_parent, int32_t* next_token, float* next_score,
    void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!next_parent || !next_token || !next_score) return CORAL_ERR_NULL;
    if (M < 1 || k < 1 || n_next < 1) return CORAL_ERR_SHAPE;
    if (M > kMaxM || k > kMaxK) return CORAL_ERR_UNSUPPORTED;
    if (n_next > M * k) return CORAL_ERR_SHAPE;
    const LevelExpand level = {parent_score, n_next, next_parent, next_token, next_score};
    return grouped_impl(hidden, gate_hidden, gate_W, gate_bias, lm_W, gi, M, H, V, g, k, dt, topk_ids,
                        topk_logprob, sel_groups, workspace, workspace_bytes, hip_stream, nullptr,
                        nullptr, true, &level);
}

extern "C" coral_status coral_tree_expand(const float* parent_score, const int32_t* cand_ids,
                                          const float* cand_logp, int M, int k, int n_next,
                                          int32_t* next_parent, int32_t* next_token,
                                          float* next_score, void* hip_stream) {
    if (!cand_ids || !cand_logp || !next_parent || !next_token || !next_score) return CORAL_ERR_NULL;
    if (M < 1 || k < 1 || n_next < 1) return CORAL_ERR_SHAPE;
    if (M > kMaxM || k > kMaxK) return CORAL_ERR_UNSUPPORTED;
    if (n_next > M * k) return CORAL_ERR_SHAPE;
    hipLaunchKernelGGL(k_tree_expand, dim3(M), dim3(kWave), (size_t)M * k * sizeof(unsigned long long),
                       static_cast<hipStream_t>(hip_stream),
                       parent_score, cand_ids, cand_logp, M, k, n_next, next_parent, next_token,
                       next_score);
    return launch_status();
}

extern "C" coral_status coral_router_premix(const void* hidden, const void* W1, int M, int H,
                                            coral_dtype dt, coral_activation act, void* u_out,
                                            void* hip_stream) {
    if (!hidden || !W1 || !u_out) return CORAL_ERR_NULL;
    if (!dtype_ok(dt)) return CORAL_ERR_SHAPE;
    if (act != CORAL_ACT_SILU && act != CORAL_ACT_RELU && act != CORAL_ACT_IDENTITY) return CORAL_ERR_SHAPE;
    if (M < 1 || H < 1) return CORAL_ERR_SHAPE;
    const bool w16 = is_16bit(dt);
    if (H % (w16 ? 8 : 4) != 0) return CORAL_ERR_UNSUPPORTED;
    if (((uintptr_t)hidden | (uintptr_t)W1 | (uintptr_t)u_out) & 15u) return CORAL_ERR_UNSUPPORTED;
    const size_t row_bytes = (size_t)H * (w16 ? 2 : 4);
    if (row_bytes > (size_t)kLdsLimit) return CORAL_ERR_UNSUPPORTED;
    {   // u_out must not overlap hidden: workgroups read hidden rows that others write
        const uintptr_t a = (uintptr_t)hidden, b = (uintptr_t)u_out;
        const size_t bytes = (size_t)M * row_bytes;
        if (a < b + bytes && b < a + bytes) return CORAL_ERR_UNSUPPORTED;
    }
    PremixParams p = {};
    p.hidden = static_cast<const uint4*>(hidden);
    p.W1 = static_cast<const uint4*>(W1);
    p.out = u_out;
    p.M = M; p.H = H; p.act = (int)act;
    p.n_vec = H / (w16 ? 8 : 4);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    typedef void (*premix_fn)(PremixParams);
    if (w16 && M >= 4 && M <= 64 && H % (kPremixChunkVecs * 8) == 0 &&
        H / (kPremixChunkVecs * 8) <= kPremixMaxChunks) {     // matrix cores, tokens staged in chunks
        typedef void (*wide_fn)(PremixParams);
        const int n_ct = (M + 15) / 16;
        const bool f16 = dt == CORAL_F16;
        // (three or four token tiles at the full width of 8 chunks: both streams issued a few
        // chunks ahead, see k_premix_wide)
        const bool ring = n_ct >= 3 && p.n_vec / kPremixChunkVecs == kPremixMaxChunks;
        const wide_fn wf =
            n_ct == 1   ? (f16 ? k_premix_wide<kF16, 1> : k_premix_wide<kBF16, 1>)
            : n_ct == 2 ? (f16 ? k_premix_wide<kF16, 2> : k_premix_wide<kBF16, 2>)
            : n_ct == 3 ? (ring ? (f16 ? k_premix_wide<kF16, 3, true> : k_premix_wide<kBF16, 3, true>)
                                : (f16 ? k_premix_wide<kF16, 3> : k_premix_wide<kBF16, 3>))
                        : (ring ? (f16 ? k_premix_wide<kF16, 4, true> : k_premix_wide<kBF16, 4, true>)
                                : (f16 ? k_premix_wide<kF16, 4> : k_premix_wide<kBF16, 4>));
        const int lds = (int)premix_wide_lds_bytes();
        if (!allow_lds(reinterpret_cast<const void*>(wf), lds)) return CORAL_ERR_HIP;
        hipLaunchKernelGGL(wf, dim3(H / 16), dim3(kPremixWideBlock), lds, stream, p);
        return launch_status();
    }
    if (w16 && H % 64 == 0 && M >= 4) {                       // matrix cores
        int tok = M < kPremixTileTok ? M : kPremixTileTok;
        while (tok > 4 && premix_mfma_lds_bytes(tok, p.n_vec) > (size_t)kLdsLimit) --tok;
        const size_t lds = premix_mfma_lds_bytes(tok, p.n_vec);
        if (lds <= (size_t)kLdsLimit) {
            p.tok_per_wg = tok;
            const premix_fn mf = dt == CORAL_F16 ? k_premix_mfma<kF16> : k_premix_mfma<kBF16>;
            if (!allow_lds(reinterpret_cast<const void*>(mf), (int)lds)) return CORAL_ERR_HIP;
            hipLaunchKernelGGL(mf, dim3(H / 16, (M + tok - 1) / tok), dim3(kBlock), lds, stream, p);
            return launch_status();
        }
    }
    int tok = (int)((size_t)kLdsLimit / 2 / row_bytes);       // two workgroups per compute unit
    if (tok < 1) tok = 1;
    if (tok > kPremixTok) tok = kPremixTok;
    if (tok > M) tok = M;
    p.tok_per_wg = tok;
    const int lds = (int)((size_t)tok * row_bytes);
    const int pairs = (H + 1) / 2;
    int gx = (pairs + kWavesPerBlock - 1) / kWavesPerBlock;
    if (gx > 2 * kMaxWorkgroups) gx = 2 * kMaxWorkgroups;
    const dim3 grid(gx, (M + tok - 1) / tok);
    const premix_fn fn = CORAL_PICK_DT(dt, k_premix<kF32>, k_premix<kBF16>, k_premix<kF16>);
    if (!allow_lds(reinterpret_cast<const void*>(fn), lds)) return CORAL_ERR_HIP;
    hipLaunchKernelGGL(fn, grid, dim3(kBlock), lds, stream, p);
    return launch_status();
}

extern "C" coral_status coral_lmhead_grouped_logprob(
    const void* hidden, const void* gate_W, const float* gate_bias, const void* lm_W,
    const coral_group_index* gi, int M, int H, int V, int g, int k, coral_dtype dt,
    int32_t* topk_ids, float* topk_logprob, int32_t* sel_groups, void* workspace,
    size_t workspace_bytes, void* hip_stream) {
    return grouped_impl(hidden, nullptr, gate_W, gate_bias, lm_W, gi, M, H, V, g, k, dt, topk_ids,
                        topk_logprob, sel_groups, workspace, workspace_bytes, hip_stream, nullptr,
                        nullptr, true);
}

extern "C" coral_status coral_lmhead_grouped_logprob_profiled(
    const void* hidden, const void* gate_W, const float* gate_bias, const void* lm_W,
    const coral_group_index* gi, int M, int H, int V, int g, int k, coral_dtype dt,
    int32_t* topk_ids, float* topk_logprob, int32_t* sel_groups, void* workspace,
    size_t workspace_bytes, void* hip_stream, void* ev_before, void* ev_after) {
    if (!ev_before || !ev_after) return CORAL_ERR_NULL;
    return grouped_impl(hidden, nullptr, gate_W, gate_bias, lm_W, gi, M, H, V, g, k, dt, topk_ids,
                        topk_logprob, sel_groups, workspace, workspace_bytes, hip_stream, ev_before,
                        ev_after, true);
}

extern "C" coral_status coral_lmhead_grouped_profiled(
    const void* hidden, const void* gate_W, const float* gate_bias, const void* lm_W,
    const coral_group_index* gi, int M, int H, int V, int g, int k, coral_dtype dt,
    int32_t* topk_ids, float* topk_logits, int32_t* sel_groups, void* workspace,
    size_t workspace_bytes, void* hip_stream, void* ev_before, void* ev_after) {
    if (!ev_before || !ev_after) return CORAL_ERR_NULL;
    return grouped_impl(hidden, nullptr, gate_W, gate_bias, lm_W, gi, M, H, V, g, k, dt, topk_ids,
                        topk_logits, sel_groups, workspace, workspace_bytes, hip_stream, ev_before,
                        ev_after, false);
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
