// Argument block and launchers of the many-row bf16 GEMM (see gemm256.hip).
#pragma once
#include "gemmco.h"

struct Gemm256Args {
    const bf16_t* W;       // fused matrix in fragment order
    int32_t K, NT;         // inputs (multiple of 256), n-tiles
    const bf16_t* AF;      // activations as bf16 hi + lo B-fragments [row tile][k-tile][hi|lo][64 lanes][8] (fc_split)
    int32_t M;             // rows
    float* out;            // RESID: residual stream (+=); SWIGLU: hidden [M][F]; QKV: q [M][H*128]; LMHEAD: logits or NULL
    int32_t ldo;
    const int32_t* n_state; const float* cosT; const float* sinT;
    bf16_t* kc; bf16_t* vc;
    int32_t layer, H, Hkv, B, S, Wn, kvp, kvq;
    RowMap rm;             // QKV: which sequence and slot a row is (dense when rm.rowb is NULL)
    float* amax_val; int32_t* amax_idx;   // LM head: winners per column block of 256 [column blocks][amax_stride]
    int32_t amax_stride;
    int32_t sk;            // K slices (RESID only when > 1: partial tiles to `part`, then added in slice order)
    float* part;           // [sk][M][NT*16] fp32
    int32_t cw;            // n-tiles per wave: 0 = chosen from the shape, 1, 2 or 4 = forced
    // Activations that arrive without their RMSNorm row scale (fragments written by fc_gemm256's own reduction,
    // see rf_AF): ssq [nssq][row tiles * 16] partial row sums of squares; the epilogue multiplies row m by
    // 1 / sqrt(sum_c ssq[c][m] / K + eps) before anything else.  NULL = the fragments are final.
    const float* ssq; int32_t nssq; float eps;
    // SWIGLU: also (or, with out == NULL, only) write the hidden activations as hi + lo fragments for the
    // down projection, [row tile][F / 32][hi|lo][64][8]
    bf16_t* hfrag;
    // RESID with sk > 1: the reduction also writes the new residual rows times rf_gain (the next norm's gain)
    // as hi + lo fragments to rf_AF and their partial sums of squares to rf_ssq [N / 256][row tiles * 16]
    bf16_t* rf_AF; const float* rf_gain; float* rf_ssq;
};
#define FC_GEMM256_MAX_SK 8
int fc_gemm256_cw(int epi, int M, int NT);          // n-tiles per wave the launcher picks: 4, 2 or 1 (64 x 256, 64 x 128, 64 x 64 tiles)
int fc_gemm256_mode(int epi, int M, int K, int NT, int sk, int cw);   // 1, 2 or 3: see gemm256.hip; 3 doubles the columns per workgroup
int fc_gemm256_sk(int M, int K, int NT);   // slices that fill the chip for a matrix with few columns

// X [M][ldx] fp32 -> AF; gain != NULL applies RMSNorm (fp32 statistics over the K inputs) first
hipError_t fc_split(const float* X, int ldx, int M, int K, const float* gain, float eps, bf16_t* AF, hipStream_t st);
static inline size_t fc_split_bytes(int M, int K) { return (size_t)((M + 15) / 16) * 16 * K * 4; }
hipError_t fc_gemm256(int epi, const Gemm256Args& a, hipStream_t st);
