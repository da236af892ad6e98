// Host-side launchers of all kernels (each enqueues on `st` and returns the hipGetLastError code).
#pragma once
#include "common.h"

// text of the last failure of a context-less call (what fastcot_last_error(NULL) returns)
void fc_set_error(const char* msg);

// ---- plain kernels (one thread per output; used for fp32 models and as the on-device cross-check)
// x[m] = embedding of win[m] (dense), or of win[rowb[m] * W + rowj[m]] with a row map
hipError_t fc_embed(const void* emb, int dt, const int32_t* win, float* x, int M, int d, int V, hipStream_t st,
                    RowMap rm = RowMap{nullptr, nullptr, nullptr}, int W = 0);
hipError_t fc_rmsnorm_plain(const float* x, const float* g, float* out, int M, int d, float eps, hipStream_t st);
hipError_t fc_gemm_plain(const void* W, int dt, int K, int NP, int N, const float* X, int ldx, float* Y, int ldy,
                         int M, int accumulate, hipStream_t st);
hipError_t fc_rope_cache_plain(const float* qkv, float* qrot, const KernelDims& kd, int layer, const int32_t* n_state,
                               const float* cosT, const float* sinT, void* kc, void* vc, int dt, hipStream_t st);
hipError_t fc_attn_plain(const float* q, int ldq, const void* kc, const void* vc, int dt, const KernelDims& kd,
                         int layer, const int32_t* n_state, float* out, hipStream_t st);
hipError_t fc_swiglu_plain(const float* gu, float* h, int M, int F, int ldgu, hipStream_t st);
hipError_t fc_argmax_plain(const float* logits, int M, int V, int32_t* ids, float* top, hipStream_t st);

// ---- decoding-state kernels
hipError_t fc_prefill_window(int32_t* state, const StateMap& sm, int B, int R, int S, int p0, hipStream_t st);
hipError_t fc_prefill_advance(int32_t* state, const StateMap& sm, int B, int W, int S, int p1, int last,
                              hipStream_t st);
hipError_t fc_rewindow(int32_t* state, const StateMap& sm, int B, int W, int S, hipStream_t st);
hipError_t fc_accept_commit(int32_t* state, const StateMap& sm, int B, int W, int S, hipStream_t st);
// sequences b1 and b2 trade slots: state entries and K/V cache (seq_bytes per sequence and layer, layers layer_stride_bytes apart)
hipError_t fc_swap_sequences(int32_t* state, const StateMap& sm, int b1, int b2, int W, int S, void* kc, void* vc,
                             size_t seq_bytes, int layers, size_t layer_stride_bytes, hipStream_t st);

// ---- weight packing
hipError_t fc_pack(const void* src, int dt, int rows, int cols, void* dst_base, const FusedMat& fm, int col_off,
                   int mode /*0 natural, 1 gate, 2 up, 3 + Dh: q/k heads of Dh*/, hipStream_t st);
hipError_t fc_fill_f32(float* dst, size_t n, float v, hipStream_t st);
hipError_t fc_copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t st);
hipError_t fc_kv_scatter(const void* k, const void* v, int S_in, int Hkv, int Dh, int S, int dt, void* kc, void* vc,
                         hipStream_t st);
