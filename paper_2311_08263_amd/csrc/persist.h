// One-launch-per-step persistent kernel for bf16 models with up to 16 rows per step (see persist.hip).
#pragma once
#include "fast.h"

struct PMat { size_t off; int32_t K, NT, ncg, NU; };   // fused matrix: inputs, n-tiles, column groups, units of 256 inputs

struct PersistArgs {
    const char* weights;
    size_t layers_off, layer_stride, g1_off, g2_off, gf_off;
    PMat mat[5];                  // QKV, O, gate/up, down (offsets inside a layer), LM head (absolute)
    int32_t L, M, Bact, lmhead, do_accept, G;
    int32_t H, Hkv, B, S, W, kvp, V, d, F;
    float eps;
    float *x, *q, *att, *h;       // activations fp32
    float* part; float* sspart; int32_t* cnt; int32_t cmax[5];   // split-K hand-off
    float* apart; int32_t* acnt;  // attention split hand-off
    int32_t* sync;                // [0] grid-barrier arrivals, [1] abort flag
    const float* cosT; const float* sinT;
    bf16_t* kc; bf16_t* vc;
    float* amax_val; int32_t* amax_idx; float* logits; float* topv;
    int32_t* state; StateMap sm;
    const void* emb;
    uint64_t* trace;              // FC_TRACE builds: phase timestamps of two workgroups
    int32_t dbg_stop;             // debug: run only this many stages (QKV, attention, O, gate/up, down per layer); < 0 = all
};

bool fc_persist_supported(const KernelDims& kd, int rows);
size_t fc_persist_part_bytes(const KernelDims& kd);
// enqueues the step: begin kernel (barrier reset + embedding) and the persistent kernel
hipError_t fc_persist_step(const FastArgs& a, int do_accept, void* prof, hipError_t (*prof_mark)(void*, int));
