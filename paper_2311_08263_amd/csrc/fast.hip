#include <string.h>
#include "fast.h"
void fc_fast_scratch_sizes(const KernelDims& kd, size_t* g, size_t* a) { *g = 256; *a = 256; }
void fc_fast_plan(const KernelDims& kd, FastPlan* plan) { memset(plan, 0, sizeof(*plan)); }
hipError_t fc_fast_forward(const FastArgs& a) { return hipErrorNotSupported; }
#include "kernels.h"
__global__ void k_set_i32_(int32_t* p, int32_t v) { if (threadIdx.x == 0) *p = v; }
size_t fc_attn_iso_scratch_bytes(int W, int H, int Dh) { return 256; }
hipError_t fc_attn_iso(const float* q, const void* kc, const void* vc, int n, int W, int H, int Hkv, int Dh, int S,
                       int dt, float* out, void* scratch, hipStream_t st) {
    KernelDims kd{}; kd.L = 1; kd.H = H; kd.Hkv = Hkv; kd.Dh = Dh; kd.B = 1; kd.S = S; kd.W = W; kd.M = W;
    k_set_i32_<<<1, 64, 0, st>>>((int32_t*)scratch, n);
    return fc_attn_plain(q, H * Dh, kc, vc, dt, kd, 0, (const int32_t*)scratch, out, st);
}
size_t fc_lmhead_iso_scratch_bytes(int M, int d, int V) { return (size_t)M * V * 4 + 256; }
hipError_t fc_lmhead_iso(const float* act, const void* packed, int M, int d, int V, int32_t* ids, float* top,
                         float* logits, void* scratch, hipStream_t st) {
    float* lg = logits ? logits : (float*)scratch;
    hipError_t e = fc_gemm_plain(packed, FASTCOT_BF16, d, V, V, act, d, lg, V, M, 0, st);
    if (e != hipSuccess) return e;
    return fc_argmax_plain(lg, M, V, ids, top, st);
}
