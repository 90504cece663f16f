// Internal layout of dqn_envs (the synchronized samplers' shared arrays and device-resident frame stacks), shared by
// its implementation and the Algorithm 1 orchestrator.
#pragma once
#include "common.h"

struct dqn_envs {
    dqn_ctx* ctx = nullptr;
    replay* rb = nullptr;        // may be null: experiences are not stored
    int W = 0, A = 0;
    hipStream_t act_stream = nullptr;
    // pinned host arrays the sampler threads address ...
    uint8_t* h_obs = nullptr;    // [W][84*84]
    int32_t* h_actions = nullptr;
    float* h_rewards = nullptr;
    uint8_t* h_terminals = nullptr;
    float* h_q = nullptr;        // [W][A]
    // ... and the same memory as the kernels address it
    uint8_t* hd_obs = nullptr;
    int32_t* hd_actions = nullptr;
    float* hd_rewards = nullptr;
    uint8_t* hd_terminals = nullptr;
    float* hd_q = nullptr;
    uint8_t* d_states = nullptr; // [W][4][84][84], device
    bool started = false;        // dqn_envs_reset has run
};
