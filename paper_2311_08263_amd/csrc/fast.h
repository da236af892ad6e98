// MFMA (matrix-core) forward path for bf16 models: launch plan and entry points.
#pragma once
#include "common.h"

#define FC_MAX_COUNTERS 8192
#define FC_MAX_ATTN_SPLITS 16 // largest split of the key range across workgroups

struct FastPlan {
    int32_t attn_splits;
    int32_t attn_bpw;  // key blocks of 32 per attention workgroup (decides at run time how many of the splits work)
    int32_t attn_many; // many-row attention kernel (attnp.hip): 0 never, 1 where it gives half of the CUs a workgroup, 2 for every pass of more than 32 rows per sequence
    int32_t co_single; // column-owner GEMM: 1 = one weight batch in flight per wave, 0 = two, 2 = chosen per GEMM
    int32_t co_sb[2][5];   // the per-GEMM choice (1 = one batch, 0 = two, 2 = whole slice) for up to 16 rows [0] and 17..32 rows [1]: defaults
                           // from the 7B shape, replaced by fc_fast_tune's measurement on the actual shape
    int32_t co_rot[2][5];  // per-GEMM: walk the K batches in a per-wave rotated order (same defaults / measurement)
    int32_t ks[5];     // column-owner GEMM: K slices per owner (residual GEMMs only; 1 elsewhere)
    int32_t nw2[5], ks2[5];   // the same for passes of 17..32 rows (two row tiles per workgroup)
    int32_t nw[5];     // column-owner GEMM: workgroups for QKV, O, gate/up, down, LM head
};
struct FastArgs {
    KernelDims kd;     // kd.M = rows of this pass
    int Bact, lmhead;
    const ModelMap* mm;
    const WorkspaceMap* wm;
    const char* weights;
    char* ws;
    float* dbg_logits;
    const FastPlan* plan;
    hipStream_t st;
    void* prof;
    hipError_t (*prof_mark)(void*, int);
    RowMap rm = RowMap{nullptr, nullptr, nullptr};   // packed rows of a step with per-sequence windows (kd.M = their sum, kd.W = the largest)
    int dbg_stop;      // debug: number of stages to run (5 per layer), < 0 = all
    int tune_gi = -1;  // >= 0: launch only GEMM tune_gi (0 QKV, 1 O, 2 gate/up, 3 down, 4 LM head) of layer 0 ...
    int tune_sb = 0;   // ... with this many-batches choice, this batch order and this many K slices per owner
    int tune_rot = 0, tune_ks = 1;   // (timing runs of fc_fast_tune; results are scratch)
};

// true when the MFMA path covers this shape (else the caller uses the plain kernels)
bool fc_fast_supported(const KernelDims& kd, int rows);
void fc_fast_scratch_sizes(const KernelDims& kd, size_t* gemm_part_bytes, size_t* attn_part_bytes);
void fc_fast_plan(const KernelDims& kd, FastPlan* plan);
hipError_t fc_fast_forward(const FastArgs& a);
// Times every column-owner GEMM of the pass shape a.kd (at most 32 rows) with one and with two weight batches in
// flight per wave or the wave's whole K slice at once and records the fastest in the plan.  Only that choice is
// measured: it moves loads, not additions, so the results are the same bits whichever wins.  Overwrites activations and layer 0's first cache rows:
// call it before a prefill.  Synchronises the stream.
hipError_t fc_fast_tune(FastArgs a, FastPlan* plan);

// isolation launchers (same kernels as the step)
size_t fc_attn_iso_scratch_bytes(int W, int H, int Dh);
hipError_t fc_attn_iso(const float* q, const void* kc, const void* vc, int n, int W, int H, int Hkv, int Dh, int S,
                       int dt, float* out, void* scratch, hipStream_t st);
size_t fc_lmhead_iso_scratch_bytes(int M, int d, int V);
hipError_t fc_lmhead_iso(const float* act, const void* packed, int M, int d, int V, int32_t* ids, float* top, float* top2,
                         float* logits, void* scratch, hipStream_t st);
