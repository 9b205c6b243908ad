// Map of the control words at the start of the workspace (32-bit words, all zero between
// calls; coral_lmhead_workspace_init zeroes them once, every kernel that uses one leaves it
// zero again).  Plain constants so that a host compiler can include this file too: a test
// builds the table below and checks that no two entries overlap and all lie inside the
// control area.
#pragma once

namespace coral_ctrl {

struct Entry {
    const char* name;
    int first_word;
    int n_words;
};

constexpr int kWords = 128;                 // size of the control area in words (512 bytes)
constexpr int kFusedArrival = 0;            // single-launch path: workgroups that have published
constexpr int kGateSelectArrival = 8;       // tile path: per token tile, k_gate_select workgroups that
constexpr int kGateSelectArrivalWords = 4;  //   have stored their scores (at most 4 token tiles)
constexpr int kTileQueue = 4;               // tile path: next block of k_tiles
constexpr int kLpGroupArrival = 64;         // log-probability mode: one counter per activated
constexpr int kLpGroupArrivalWords = 64;    //   group (at most 64 in the single-launch kernel)

constexpr Entry kMap[] = {
    {"fused_arrival", kFusedArrival, 1},
    {"gate_select_arrival", kGateSelectArrival, kGateSelectArrivalWords},
    {"tile_queue", kTileQueue, 1},
    {"logprob_group_arrival", kLpGroupArrival, kLpGroupArrivalWords},
};
constexpr int kMapEntries = sizeof(kMap) / sizeof(kMap[0]);

}  // namespace coral_ctrl
