// Argument block and launcher of the weight-streaming bf16 GEMM (see gemm16.hip).
#pragma once
#include "fast.h"

enum { EPI_RESID = 0, EPI_SWIGLU = 1, EPI_QKV = 2, EPI_LMHEAD = 3 };

struct Gemm16Args {
    const bf16_t* W;       // fused matrix in fragment order
    int32_t K, NT;         // inputs, n-tiles (columns / 16)
    int32_t sk;            // K slices per column group
    const float* X;        // activations fp32 [M][ldx]
    int32_t ldx, M;        // M rows in this launch (<= 32); X and out already point at the first of them
    int32_t m0;            // index of that first row in the step (row m0 + m belongs to sequence (m0 + m) / W)
    const float* gain;     // RMSNorm gain [K]; NULL = no norm in front of this GEMM
    float eps;
    float* part;           // split-K partial tiles
    float* sspart;         // split-K partial row sums of squares
    int32_t* cnt;          // one arrival counter per column group, zero between launches
    float* out;            // RESID: residual stream (+=); SWIGLU: hidden [M][F]; QKV: q [M][H*Dh]; LMHEAD: logits or NULL
    int32_t ldo;
    // QKV epilogue
    const int32_t* n_state; const float* cosT; const float* sinT;
    bf16_t* kc; bf16_t* vc;
    int32_t layer, H, Hkv, B, S, Wn, kvp;
    // LM-head epilogue: per column group winners [ncg][16*MT]
    float* amax_val; int32_t* amax_idx;
};

size_t fc_gemm16_lds_bytes(int K, int sk, int MT, int nsplit);
hipError_t fc_gemm16(int epi, const Gemm16Args& a, int ncg, hipStream_t st);
hipError_t fc_argmax_final(const float* val, const int32_t* idx, int ncg, int stride, int M, int32_t* ids, float* top,
                           hipStream_t st);
