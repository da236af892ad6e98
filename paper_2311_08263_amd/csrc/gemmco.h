// Argument block and launcher of the column-owner weight-streaming GEMM (see gemmco.hip).
#pragma once
#include "fast.h"

enum { EPI_RESID = 0, EPI_SWIGLU = 1, EPI_QKV = 2, EPI_LMHEAD = 3 };

struct GemmCoArgs {
    const bf16_t* W;       // fused matrix in fragment order
    int32_t K, NT;         // inputs (multiple of 256), n-tiles
    const float* X;        // activations fp32 [M][ldx]
    int32_t ldx, M;        // M <= 32 rows
    const float* gain;     // RMSNorm gain [K]; NULL = no norm in front of this GEMM
    float eps;
    float* out;            // RESID: residual stream (+=); SWIGLU: hidden [M][F]; QKV: q [M][H*128]; LMHEAD: logits or NULL
    int32_t ldo;
    const int32_t* n_state; const float* cosT; const float* sinT;
    bf16_t* kc; bf16_t* vc;
    int32_t layer, H, Hkv, B, S, Wn, kvp, kvq;
    RowMap rm;             // QKV: which sequence and slot a row is (dense when rm.rowb is NULL: m / Wn, m % Wn)
    float* amax_val; int32_t* amax_idx;   // LM head: winners per workgroup [workgroups][16 or 32 rows]
    int32_t ks;            // workgroups per column owner, each taking 1/ks of K (1..8; 1 for the LM head)
    float* xpart;          // ks > 1: partial tiles [workgroup][8 or 16 (more than 8 output tiles)][64 lanes][4], then each
                           // workgroup's share of the row sums of squares [workgroup][16 or 32]
    int32_t* xcnt;         // ks > 1: one arrival counter per owner, zero between launches
    int32_t hi_only;       // precision study: the activations enter as plain bf16 (their lo halves dropped)
    int32_t rotate;        // walk the K batches in a per-wave rotated order (spreads the streams over the memory channels)
    int32_t single_buffer; // weights in flight per wave: 1 = one batch, 0 = two batches, 2 = the wave's whole K slice requested up front
                           // (QKV and residual GEMMs, up to 16 rows, slices of at most 16 k-tiles per wave; else rejected)
};

// G workgroups = G / ks owners x ks K slices; owner i owns n-tiles [i*NT/owners, (i+1)*NT/owners), at most
// 8; fc_gemmco_grid picks one workgroup per CU (all resident, one round) unless the matrix is wider than
// 8 n-tiles per CU
int fc_gemmco_grid(int NT, int most = 8);
// most n-tiles a workgroup may own so that its partial tiles (8 sets x n-tiles x row tiles x 1 KB up to eight output tiles, 4 sets beyond) and, with a
// norm in front, the gain vector (K floats) fit the LDS of a CU
int fc_gemmco_most(int M, int K, bool gain);
int fc_num_cus();      // compute units of the current device
hipError_t fc_gemmco(int epi, const GemmCoArgs& a, int G, hipStream_t st);
// reduction of the LM head's per-workgroup winners [nparts][stride] to one id and value per row (lowest id on ties)
// (with a row map the result of row m goes to entry rowb[m] * W + rowj[m] of ids and top)
hipError_t fc_argmax_final(const float* val, const int32_t* idx, int nparts, int stride, int M, int32_t* ids, float* top,
                           hipStream_t st, RowMap rm = RowMap{nullptr, nullptr, nullptr}, int W = 0);
