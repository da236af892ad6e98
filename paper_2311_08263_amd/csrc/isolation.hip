// Kernel-isolation entry points: the step's attention and LM-head kernels on raw device pointers.
#include <stdio.h>
#include "kernels.h"
#include "fast.h"
#include "gemmco.h"


// Plain streaming read, shaped like the weight stream of the step's GEMMs: one workgroup of 8 waves per compute
// unit (256 workgroups), every wave reads a contiguous run of 1 KB pieces (16 bytes per lane) with 16 loads in
// flight, non-temporal.  Its rate over a buffer far larger than the caches is the read bandwidth this device
// delivers to the simplest possible kernel; a chain of such launches with the byte counts of the step's kernels
// is what the step would cost if every kernel did nothing but read its weights.
__global__ __launch_bounds__(512) void k_stream_read(const uint4* __restrict__ p, size_t n16, uint4* sink) {
    typedef __attribute__((__vector_size__(16))) uint32_t u32x4;
    const int lane = threadIdx.x & 63;
    const size_t gw = (size_t)blockIdx.x * 8 + (threadIdx.x >> 6), nw = (size_t)gridDim.x * 8;
    const size_t tiles = n16 >> 6, per = (tiles + nw - 1) / nw;
    const size_t t0 = gw * per < tiles ? gw * per : tiles, t1 = t0 + per < tiles ? t0 + per : tiles;
    const u32x4* q = (const u32x4*)p + lane;
    u32x4 acc = {0, 0, 0, 0};
    u32x4 ring[16];
    const size_t n = t1 - t0;
    if (n > 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) ring[r] = __builtin_nontemporal_load(q + (t0 + ((size_t)r < n ? r : 0)) * 64);
        for (size_t i = 0; i < n; i += 16) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc ^= ring[r];
                const size_t j = i + 16 + r;
                ring[r] = __builtin_nontemporal_load(q + (t0 + (j < n ? j : 0)) * 64);
            }
        }
    }
    // the pieces past the last whole kilobyte
    for (size_t i = (tiles << 6) + gw * 64 + lane; i < n16; i += nw * 64) { const uint4 v = p[i]; acc[0] ^= v.x ^ v.y ^ v.z ^ v.w; }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u && acc[1] == 0x12345678u) sink[0] = make_uint4(acc[0], acc[1], acc[2], acc[3]);   // keeps the loads alive
}
extern "C" int fastcot_stream_read(const void* d_src, size_t bytes, void* d_sink16, void* hip_stream) {
    if (!d_src || !d_sink16 || bytes < 16 || ((uintptr_t)d_src & 15)) return FASTCOT_EINVAL;
    k_stream_read<<<fc_num_cus(), 512, 0, (hipStream_t)hip_stream>>>((const uint4*)d_src, bytes / 16, (uint4*)d_sink16);
    return hipGetLastError() == hipSuccess ? 0 : FASTCOT_EHIP;
}
extern "C" int fastcot_stream_read_chain(const void* d_src, size_t src_bytes, const uint64_t* launch_bytes, int32_t n_launches,
                                         void* d_sink16, void* hip_stream) {
    if (!d_src || !d_sink16 || !launch_bytes || n_launches < 1 || ((uintptr_t)d_src & 15)) return FASTCOT_EINVAL;
    size_t off = 0;
    for (int i = 0; i < n_launches; ++i) {
        const size_t b = (size_t)launch_bytes[i] & ~(size_t)1023;
        if (b < 1024 || b > src_bytes) return FASTCOT_EINVAL;
        if (off + b > src_bytes) off = 0;             // wrap: the buffer is far larger than the caches
        k_stream_read<<<fc_num_cus(), 512, 0, (hipStream_t)hip_stream>>>((const uint4*)((const char*)d_src + off), b / 16, (uint4*)d_sink16);
        off += b;
    }
    return hipGetLastError() == hipSuccess ? 0 : FASTCOT_EHIP;
}

extern "C" size_t fastcot_attn_scratch_bytes(int32_t W, int32_t H, int32_t Dh) {
    if (W <= 0 || H <= 0 || Dh <= 0) return 0;
    return fc_attn_iso_scratch_bytes(W, H, Dh);
}

extern "C" int fastcot_kv_scatter(const void* d_k, const void* d_v, int32_t S, int32_t Hkv, int32_t Dh, int32_t max_seq,
                                  int32_t dtype, void* d_k_cache, void* d_vt_cache, void* hip_stream) {
    if (!d_k || !d_v || !d_k_cache || !d_vt_cache || S <= 0 || S > max_seq || max_seq % 32 || Hkv <= 0 || Dh <= 0 || Dh % 32 ||
        (dtype != FASTCOT_F32 && dtype != FASTCOT_BF16)) return FASTCOT_EINVAL;
    hipError_t e = fc_kv_scatter(d_k, d_v, S, Hkv, Dh, max_seq, dtype, d_k_cache, d_vt_cache, (hipStream_t)hip_stream);
    return e == hipSuccess ? 0 : FASTCOT_EHIP;
}

extern "C" int fastcot_attn_window(const float* d_q, const void* d_k_cache, const void* d_vt_cache, int32_t n, int32_t W,
                                   int32_t H, int32_t Hkv, int32_t Dh, int32_t max_seq, int32_t dtype, float* d_out,
                                   void* d_scratch, void* hip_stream) {
    if (!d_q || !d_k_cache || !d_vt_cache || !d_out || !d_scratch) return FASTCOT_EINVAL;
    if (n < 0 || W <= 0 || H <= 0 || Hkv <= 0 || H % Hkv || Dh <= 0 || Dh % 32 || max_seq > 16000 || max_seq % 32) return FASTCOT_EINVAL;
    if (dtype != FASTCOT_F32 && dtype != FASTCOT_BF16) return FASTCOT_EINVAL;
    if (n + W > max_seq) return FASTCOT_ECAPACITY;
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e = fc_attn_iso(d_q, d_k_cache, d_vt_cache, n, W, H, Hkv, Dh, max_seq, dtype, d_out, d_scratch, st);
    return e == hipSuccess ? 0 : FASTCOT_EHIP;
}

// ------------------------------------------------------------------ attention without any allocation
// For callers that cannot allocate device memory (code under graph capture, tight serving loops): the split-key
// partial results and arrival counters of the attention kernel live in a file-scope device array instead of a
// caller buffer.  Every GPU holds its own copy of the array; its address is looked up once per device.
#define FC_NOALLOC_MAX_H 64
#define FC_NOALLOC_MAX_W 16
#define FC_NOALLOC_BYTES (512 + (size_t)FC_NOALLOC_MAX_H * FC_MAX_ATTN_SPLITS * (8 * 64 * 4 + 128) * 4)
static __device__ __align__(256) unsigned char scratch[FC_NOALLOC_BYTES];
#define FC_NOALLOC_MAX_DEVICES 64
static void* g_scratch_ptr[FC_NOALLOC_MAX_DEVICES];

__global__ void k_zero_i32(int32_t* p, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

extern "C" int fastcot_attn_window_noalloc(const float* d_q, const void* d_k_cache, const void* d_vt_cache, int32_t n, int32_t W,
                                           int32_t H, int32_t Hkv, int32_t Dh, int32_t max_seq, int32_t dtype, float* d_out,
                                           void* hip_stream) {
    if (!d_q || !d_k_cache || !d_vt_cache || !d_out) { fc_set_error("fastcot_attn_window_noalloc: NULL device pointer"); return FASTCOT_EINVAL; }
    if (n < 0 || W <= 0 || H <= 0 || Hkv <= 0 || H % Hkv || Dh <= 0 || Dh % 32 || max_seq > 16000 || max_seq % 32 ||
        (dtype != FASTCOT_F32 && dtype != FASTCOT_BF16)) { fc_set_error("fastcot_attn_window_noalloc: bad shape argument"); return FASTCOT_EINVAL; }
    if (n + W > max_seq) { fc_set_error("fastcot_attn_window_noalloc: n + W exceeds max_seq"); return FASTCOT_ECAPACITY; }
    if (H > FC_NOALLOC_MAX_H || W > FC_NOALLOC_MAX_W) {
        fc_set_error("fastcot_attn_window_noalloc: at most 64 heads and 16 window rows fit the built-in scratch array");
        return FASTCOT_ECAPACITY;
    }
    if (fc_attn_iso_scratch_bytes(W, H, Dh) > FC_NOALLOC_BYTES) { fc_set_error("fastcot_attn_window_noalloc: scratch need exceeds the built-in array"); return FASTCOT_ECAPACITY; }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= FC_NOALLOC_MAX_DEVICES) { fc_set_error("fastcot_attn_window_noalloc: no current device"); return FASTCOT_EHIP; }
    if (!g_scratch_ptr[dev]) {        // once per device, with that device current
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { fc_set_error("fastcot_attn_window_noalloc: hipGetSymbolAddress failed"); return FASTCOT_EHIP; }
        g_scratch_ptr[dev] = p;
    }
    char* sc = (char*)g_scratch_ptr[dev];
    hipStream_t st = (hipStream_t)hip_stream;
    // the array keeps the last call's contents: the arrival counters must start at zero (a fill kernel, not a
    // memset node, so that the call may be captured into a graph)
    k_zero_i32<<<1, 64, 0, st>>>((int32_t*)(sc + 256), H);
    if (hipGetLastError() != hipSuccess) { fc_set_error("fastcot_attn_window_noalloc: launch failed"); return FASTCOT_EHIP; }
    hipError_t e = fc_attn_iso(d_q, d_k_cache, d_vt_cache, n, W, H, Hkv, Dh, max_seq, dtype, d_out, sc, st);
    if (e != hipSuccess) { fc_set_error("fastcot_attn_window_noalloc: attention launch failed"); return FASTCOT_EHIP; }
    return 0;
}

extern "C" size_t fastcot_lmhead_packed_bytes(int32_t d, int32_t V) {
    if (d <= 0 || V <= 0 || d % 32 || V % 16) return 0;
    return (size_t)d * V * 2;
}
extern "C" size_t fastcot_lmhead_scratch_bytes(int32_t M, int32_t d, int32_t V) {
    if (M <= 0 || d <= 0 || V <= 0) return 0;
    return fc_lmhead_iso_scratch_bytes(M, d, V);
}
extern "C" int fastcot_lmhead_pack(const void* src, int32_t d, int32_t V, void* d_packed, void* hip_stream) {
    if (!src || !d_packed || d <= 0 || V <= 0 || d % 32 || V % 16) return FASTCOT_EINVAL;
    FusedMat fm; fm.off = 0; fm.K = d; fm.N = V; fm.NP = V;
    hipError_t e = fc_pack(src, FASTCOT_BF16, d, V, d_packed, fm, 0, 0, (hipStream_t)hip_stream);
    return e == hipSuccess ? 0 : FASTCOT_EHIP;
}
extern "C" int fastcot_lmhead_argmax(const float* d_act, const void* d_packed, int32_t M, int32_t d, int32_t V,
                                     int32_t* d_ids, float* d_top, float* d_top2, float* d_logits, void* d_scratch, void* hip_stream) {
    if (!d_act || !d_packed || !d_ids || !d_top || !d_scratch) return FASTCOT_EINVAL;
    if (M <= 0 || d <= 0 || V <= 0 || d % 32 || V % 16) return FASTCOT_EINVAL;
    hipError_t e = fc_lmhead_iso(d_act, d_packed, M, d, V, d_ids, d_top, d_top2, d_logits, d_scratch, (hipStream_t)hip_stream);
    return e == hipSuccess ? 0 : FASTCOT_EHIP;
}
