// Plain kernels: one thread per output element, fp32 arithmetic, no matrix cores.
// They run fp32 models (the small parity configuration) and serve as the on-device
// cross-check of the MFMA kernels.  Each follows the model definition the benchmark
// configurations fix (RMSNorm, rotary embedding pairing i with i + Dh/2, grouped-query
// attention with the causal mask of Eq. (2), SwiGLU).
#include "kernels.h"

template <int DT> __device__ inline float wat(const void* W, size_t i) {
    if (DT == FASTCOT_F32) return ((const float*)W)[i];
    return bf16_to_f32(((const bf16_t*)W)[i]);
}
// cached value: fp32 models one fp32 plane; bf16 models a bf16 hi plane plus (kvp == 2) a bf16 lo plane or
// (kvp == 3) a plane of 8-bit residuals; i is the element index of plane 0's entry, `plane` the elements per plane
template <int DT> __device__ inline void kvstore(void* C, size_t i, size_t plane, int kvp, float v) {
    if (DT == FASTCOT_F32) { ((float*)C)[i] = v; return; }
    if (kvp == 3) {
        // (the block's base is part of i: the byte plane of a block starts one plane after its hi plane)
        uint32_t h, l; kv24_split(v, h, l);
        ((bf16_t*)C)[i] = (bf16_t)h;
        const size_t blk = i / plane * plane;
        ((uint8_t*)((bf16_t*)C + blk + plane))[i - blk] = (uint8_t)l;
        return;
    }
    bf16_t hi = f32_to_bf16(v);
    ((bf16_t*)C)[i] = hi;
    if (kvp == 2) ((bf16_t*)C)[i + plane] = f32_to_bf16(v - bf16_to_f32(hi));
}
template <int DT> __device__ inline float kvload(const void* C, size_t i, size_t plane, int kvp) {
    if (DT == FASTCOT_F32) return ((const float*)C)[i];
    if (kvp == 3) {
        const size_t blk = i / plane * plane;
        return kv24_join(((const bf16_t*)C)[i], ((const uint8_t*)((const bf16_t*)C + blk + plane))[i - blk]);
    }
    float v = bf16_to_f32(((const bf16_t*)C)[i]);
    if (kvp == 2) v += bf16_to_f32(((const bf16_t*)C)[i + plane]);
    return v;
}

// ------------------------------------------------------------------ embedding gather
template <int DT>
__global__ void k_embed(const void* emb, const int32_t* win, float* x, int d, int V, RowMap rm, int W) {
    int m = blockIdx.x;
    int t = win[rm.rowb ? rm.rowb[m] * W + rm.rowj[m] : m];
    if (t < 0 || t >= V) t = 0;
    if (DT == FASTCOT_BF16 && d % 8 == 0) {          // eight elements (16 bytes) per thread and pass
        const uint4* src = (const uint4*)((const bf16_t*)emb + (size_t)t * d);
        float4* dst = (float4*)(x + (size_t)m * d);
        for (int i = threadIdx.x; i < d / 8; i += blockDim.x) {
            const uint4 v = src[i];
            dst[2 * i] = make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u), __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xFFFF0000u));
            dst[2 * i + 1] = make_float4(__uint_as_float(v.z << 16), __uint_as_float(v.z & 0xFFFF0000u), __uint_as_float(v.w << 16), __uint_as_float(v.w & 0xFFFF0000u));
        }
        return;
    }
    for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)m * d + i] = wat<DT>(emb, (size_t)t * d + i);
}
hipError_t fc_embed(const void* emb, int dt, const int32_t* win, float* x, int M, int d, int V, hipStream_t st, RowMap rm, int W) {
    if (dt == FASTCOT_F32) k_embed<FASTCOT_F32><<<M, 256, 0, st>>>(emb, win, x, d, V, rm, W);
    else k_embed<FASTCOT_BF16><<<M, 256, 0, st>>>(emb, win, x, d, V, rm, W);
    return hipGetLastError();
}

// ------------------------------------------------------------------ RMSNorm
__device__ inline float block_sum(float v, float* red) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float s = 0;
    for (int i = 0; i < nw; ++i) s += red[i];
    return s;
}
__global__ void k_rmsnorm(const float* x, const float* g, float* out, int d, float eps) {
    __shared__ float red[16];
    const float* xr = x + (size_t)blockIdx.x * d;
    float ss = 0;
    for (int i = threadIdx.x; i < d; i += blockDim.x) ss += xr[i] * xr[i];
    ss = block_sum(ss, red);
    float r = 1.0f / sqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += blockDim.x) out[(size_t)blockIdx.x * d + i] = xr[i] * r * g[i];
}
hipError_t fc_rmsnorm_plain(const float* x, const float* g, float* out, int M, int d, float eps, hipStream_t st) {
    k_rmsnorm<<<M, 256, 0, st>>>(x, g, out, d, eps);
    return hipGetLastError();
}

// ------------------------------------------------------------------ GEMM  Y[m][n] (+)= sum_k X[m][k] W[k][n]
template <int DT>
__global__ void k_gemm_plain(const void* W, int K, int NP, int N, const float* X, int ldx, float* Y, int ldy,
                             int M, int accumulate) {
    constexpr int RB = 8;
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    int m0 = blockIdx.y * RB;
    if (n >= N) return;
    float acc[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) acc[r] = 0.f;
    for (int k = 0; k < K; ++k) {
        float w = (DT == FASTCOT_F32) ? ((const float*)W)[(size_t)k * NP + n]
                                      : bf16_to_f32(((const bf16_t*)W)[frag_index(K, k, n)]);
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            int m = m0 + r < M ? m0 + r : M - 1;
            acc[r] += X[(size_t)m * ldx + k] * w;
        }
    }
#pragma unroll
    for (int r = 0; r < RB; ++r)
        if (m0 + r < M) {
            float* y = Y + (size_t)(m0 + r) * ldy + n;
            *y = accumulate ? *y + acc[r] : acc[r];
        }
}
hipError_t fc_gemm_plain(const void* W, int dt, int K, int NP, int N, const float* X, int ldx, float* Y, int ldy,
                         int M, int accumulate, hipStream_t st) {
    dim3 grid((N + 255) / 256, (M + 7) / 8);
    if (dt == FASTCOT_F32) k_gemm_plain<FASTCOT_F32><<<grid, 256, 0, st>>>(W, K, NP, N, X, ldx, Y, ldy, M, accumulate);
    else k_gemm_plain<FASTCOT_BF16><<<grid, 256, 0, st>>>(W, K, NP, N, X, ldx, Y, ldy, M, accumulate);
    return hipGetLastError();
}

// ------------------------------------------------------------------ rotary embedding + KV-cache write
// Row m = b*W + j sits at absolute position n[b] + j.  The GEMM output row is in packed column
// order (head_col); rotated q goes to qrot in natural order, k heads are rotated and stored to the
// K cache, v heads stored to the transposed V cache.
template <int DT>
__global__ void k_rope_cache(const float* qkv, float* qrot, KernelDims kd, int layer, const int32_t* n_state,
                             const float* cosT, const float* sinT, void* kc, void* vc) {
    int m = blockIdx.x, b = m / kd.W, j = m % kd.W;
    int pos = n_state[b] + j;
    if (pos >= kd.S) return;  // capacity guard: never write outside the cache
    int half = kd.Dh / 2;
    const size_t plane = (size_t)kd.S * kd.Dh;
    const float* row = qkv + (size_t)m * kd.qkvN;
    int nrot = (kd.H + kd.Hkv) * half;
    for (int i = threadIdx.x; i < nrot; i += blockDim.x) {
        int hh = i / half, e = i % half;
        float c = cosT[(size_t)pos * half + e], s = sinT[(size_t)pos * half + e];
        const float* v = row + (size_t)hh * kd.Dh;
        float a = v[head_col(e, kd.Dh)], bb = v[head_col(e + half, kd.Dh)];
        float ra = a * c - bb * s, rb = bb * c + a * s;
        if (hh < kd.H) {
            float* q = qrot + (size_t)m * kd.H * kd.Dh + (size_t)hh * kd.Dh;
            q[e] = ra; q[e + half] = rb;
        } else {
            int kh = hh - kd.H;
            size_t base = kv_block(kd, layer, b, kh);
            kvstore<DT>(kc, base + k_index(pos, e, kd.Dh), plane, kd.kvp, ra);
            kvstore<DT>(kc, base + k_index(pos, e + half, kd.Dh), plane, kd.kvp, rb);
        }
    }
    const float* vrow = row + (size_t)(kd.H + kd.Hkv) * kd.Dh;
    for (int i = threadIdx.x; i < kd.Hkv * kd.Dh; i += blockDim.x) {
        int kh = i / kd.Dh, e = i % kd.Dh;
        size_t base = kv_block(kd, layer, b, kh) + v_index(e, pos, kd.Dh);
        kvstore<DT>(vc, base, plane, kd.kvp, vrow[i]);
    }
}
hipError_t fc_rope_cache_plain(const float* qkv, float* qrot, const KernelDims& kd, int layer, const int32_t* n_state,
                               const float* cosT, const float* sinT, void* kc, void* vc, int dt, hipStream_t st) {
    if (dt == FASTCOT_F32) k_rope_cache<FASTCOT_F32><<<kd.M, 256, 0, st>>>(qkv, qrot, kd, layer, n_state, cosT, sinT, kc, vc);
    else k_rope_cache<FASTCOT_BF16><<<kd.M, 256, 0, st>>>(qkv, qrot, kd, layer, n_state, cosT, sinT, kc, vc);
    return hipGetLastError();
}

// ------------------------------------------------------------------ window-causal attention
// One block per (row m, query head h): scores over cache positions 0 .. n[b]+j, softmax, weighted V.
template <int DT>
__global__ void k_attn_plain(const float* q, int ldq, const void* kc, const void* vc, KernelDims kd, int layer,
                             const int32_t* n_state, float* out) {
    extern __shared__ float sc[];   // [S] scores, then [16] reduction scratch
    float* red = sc + kd.S;
    int m = blockIdx.x, h = blockIdx.y, b = m / kd.W, j = m % kd.W;
    int last = n_state[b] + j;
    if (last >= kd.S) last = kd.S - 1;
    int kh = h / (kd.H / kd.Hkv);
    const float* qv = q + (size_t)m * ldq + (size_t)h * kd.Dh;
    const size_t kbase = kv_block(kd, layer, b, kh), plane = (size_t)kd.S * kd.Dh;
    float scale = 1.0f / sqrtf((float)kd.Dh);
    float mx = -3.0e38f;
    for (int t = threadIdx.x; t <= last; t += blockDim.x) {
        float s = 0;
        for (int i = 0; i < kd.Dh; ++i) s += qv[i] * kvload<DT>(kc, kbase + k_index(t, i, kd.Dh), plane, kd.kvp);
        s *= scale;
        sc[t] = s;
        mx = fmaxf(mx, s);
    }
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_down(mx, o, 64));
    int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = mx;
    __syncthreads();
    mx = red[0];
    for (int i = 1; i < nw; ++i) mx = fmaxf(mx, red[i]);
    float den = 0;
    for (int t = threadIdx.x; t <= last; t += blockDim.x) { float e = expf(sc[t] - mx); sc[t] = e; den += e; }
    den = block_sum(den, red);
    __syncthreads();
    for (int i = threadIdx.x; i < kd.Dh; i += blockDim.x) {
        float acc = 0;                          // transposed V in blocks of 32 positions
        for (int t = 0; t <= last; ++t) acc += sc[t] * kvload<DT>(vc, kbase + v_index(i, t, kd.Dh), plane, kd.kvp);
        out[(size_t)m * kd.H * kd.Dh + (size_t)h * kd.Dh + i] = acc / den;
    }
}
hipError_t fc_attn_plain(const float* q, int ldq, const void* kc, const void* vc, int dt, const KernelDims& kd,
                         int layer, const int32_t* n_state, float* out, hipStream_t st) {
    dim3 grid(kd.M, kd.H);
    size_t sh = ((size_t)kd.S + 16) * sizeof(float);
    if (dt == FASTCOT_F32) k_attn_plain<FASTCOT_F32><<<grid, 128, sh, st>>>(q, ldq, kc, vc, kd, layer, n_state, out);
    else k_attn_plain<FASTCOT_BF16><<<grid, 128, sh, st>>>(q, ldq, kc, vc, kd, layer, n_state, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------ SwiGLU on the fused gate/up output
__global__ void k_swiglu(const float* gu, float* h, int M, int F, int ldgu) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)M * F) return;
    int m = (int)(i / F), f = (int)(i % F);
    float g = gu[(size_t)m * ldgu + gu_col(f, 0)], u = gu[(size_t)m * ldgu + gu_col(f, 1)];
    h[i] = g / (1.0f + expf(-g)) * u;
}
hipError_t fc_swiglu_plain(const float* gu, float* h, int M, int F, int ldgu, hipStream_t st) {
    size_t n = (size_t)M * F;
    k_swiglu<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(gu, h, M, F, ldgu);
    return hipGetLastError();
}

// ------------------------------------------------------------------ per-row argmax, lowest index on ties
__global__ void k_argmax(const float* logits, int V, int32_t* ids, float* top) {
    __shared__ float bv[4];
    __shared__ int bi[4];
    const float* r = logits + (size_t)blockIdx.x * V;
    float best = -3.0e38f; int idx = 0x7fffffff;
    for (int i = threadIdx.x; i < V; i += blockDim.x) {
        float v = r[i];
        if (v > best || (v == best && i < idx)) { best = v; idx = i; }
    }
    for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_down(best, o, 64); int oi = __shfl_down(idx, o, 64);
        if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
    }
    if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = idx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w)
            if (bv[w] > best || (bv[w] == best && bi[w] < idx)) { best = bv[w]; idx = bi[w]; }
        ids[blockIdx.x] = idx; top[blockIdx.x] = best;
    }
}
hipError_t fc_argmax_plain(const float* logits, int M, int V, int32_t* ids, float* top, hipStream_t st) {
    k_argmax<<<M, 256, 0, st>>>(logits, V, ids, top);
    return hipGetLastError();
}

// ------------------------------------------------------------------ packing
// canonical [rows][cols] -> fused matrix columns; mode selects the column map: 0 natural at col_off,
// 1 / 2 gate / up interleave, 3 + Dh rotary-pair order inside heads of Dh columns (q and k heads).
template <int DT>
__global__ void k_pack(const void* src, int rows, int cols, void* dst, FusedMat fm, int col_off, int mode) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)rows * cols) return;
    int k = (int)(i / cols), c = (int)(i % cols);
    int n = mode == 0 ? col_off + c : (mode <= 2 ? gu_col(c, mode - 1) : qkv_col(col_off + c, mode - 3, 0x7fffffff));
    char* base = (char*)dst + fm.off;
    if (DT == FASTCOT_F32) ((float*)base)[(size_t)k * fm.NP + n] = ((const float*)src)[i];
    else ((bf16_t*)base)[frag_index(fm.K, k, n)] = ((const bf16_t*)src)[i];
}
hipError_t fc_pack(const void* src, int dt, int rows, int cols, void* dst_base, const FusedMat& fm, int col_off,
                   int mode, hipStream_t st) {
    size_t n = (size_t)rows * cols;
    unsigned blocks = (unsigned)((n + 255) / 256);
    if (dt == FASTCOT_F32) k_pack<FASTCOT_F32><<<blocks, 256, 0, st>>>(src, rows, cols, dst_base, fm, col_off, mode);
    else k_pack<FASTCOT_BF16><<<blocks, 256, 0, st>>>(src, rows, cols, dst_base, fm, col_off, mode);
    return hipGetLastError();
}

__global__ void k_fill_f32(float* dst, size_t n, float v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = v;
}
hipError_t fc_fill_f32(float* dst, size_t n, float v, hipStream_t st) {
    if (n == 0) return hipSuccess;
    k_fill_f32<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(dst, n, v);
    return hipGetLastError();
}
__global__ void k_copy_u32(uint32_t* dst, const uint32_t* src, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}
hipError_t fc_copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t st) {  // bytes % 4 == 0
    size_t n = bytes / 4;
    if (n == 0) return hipSuccess;
    k_copy_u32<<<(unsigned)((n + 255) / 256), 256, 0, st>>>((uint32_t*)dst, (const uint32_t*)src, n);
    return hipGetLastError();
}

// canonical K, V [S_in][Hkv][Dh] -> cache layout of one sequence: per head [S/32 blocks][32 * Dh] in fragment order (k_index, v_index)
template <int DT>
__global__ void k_kv_scatter(const void* k, const void* v, int S_in, int Hkv, int Dh, int S, void* kc, void* vc) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)S_in * Hkv * Dh) return;
    int e = (int)(i % Dh), h = (int)((i / Dh) % Hkv), t = (int)(i / ((size_t)Dh * Hkv));
    if (DT == FASTCOT_F32) {
        ((float*)kc)[(size_t)h * S * Dh + k_index(t, e, Dh)] = ((const float*)k)[i];
        ((float*)vc)[(size_t)h * Dh * S + v_index(e, t, Dh)] = ((const float*)v)[i];
    } else {
        ((bf16_t*)kc)[(size_t)h * S * Dh + k_index(t, e, Dh)] = ((const bf16_t*)k)[i];
        ((bf16_t*)vc)[(size_t)h * Dh * S + v_index(e, t, Dh)] = ((const bf16_t*)v)[i];
    }
}
hipError_t fc_kv_scatter(const void* k, const void* v, int S_in, int Hkv, int Dh, int S, int dt, void* kc, void* vc,
                         hipStream_t st) {
    size_t n = (size_t)S_in * Hkv * Dh;
    unsigned blocks = (unsigned)((n + 255) / 256);
    if (dt == FASTCOT_F32) k_kv_scatter<FASTCOT_F32><<<blocks, 256, 0, st>>>(k, v, S_in, Hkv, Dh, S, kc, vc);
    else k_kv_scatter<FASTCOT_BF16><<<blocks, 256, 0, st>>>(k, v, S_in, Hkv, Dh, S, kc, vc);
    return hipGetLastError();
}
