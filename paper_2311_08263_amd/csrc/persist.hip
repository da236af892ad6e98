// Persistent step kernel: the whole Jacobi step in one launch, one workgroup per compute unit.
//
// Why.  At 16 rows per step the forward is a chain of ~160 dependent weight-streaming GEMMs of
// 4-25 us each.  Launched one by one, each pays a fixed few microseconds (ramp-up, split-K
// hand-off, tail) during which HBM idles.  Here all workgroups stay resident for the whole step,
// stages are separated by grid barriers, and -- the point -- weight tiles do not depend on
// activations, so every wave keeps the tiles of its *next* units of work in flight (two register
// banks of 8 tiles) across barriers and stage changes: HBM keeps streaming while a barrier,
// a split-K hand-off or the attention stage is in progress.
//
// Work split.  A GEMM stage's work is the flat list of (column group of 128 outputs, unit of 256
// inputs) pairs; workgroup i takes the contiguous range [i*U/G, (i+1)*U/G), so every workgroup
// streams the same number of bytes (+-1 unit) whatever the matrix shape.  A range covers parts of
// one or more column groups; for each the workgroup produces a partial 16 x 128 tile, and the
// last contributor of a column group to arrive (atomic counter, no spinning) adds the partials
// in contributor order -- deterministic -- and runs the fused epilogue (RMSNorm scale, RoPE + KV
// cache write, residual add, SwiGLU, LM-head argmax).
//
// Coherence.  Each XCD has its own L2, so data produced and consumed inside this one launch by
// different workgroups (activations, partial tiles, this step's K/V rows) moves with agent-scope
// stores and loads; weights and the committed part of the KV cache use ordinary loads.
// Grid barrier: monotone arrival counter; a bounded spin that raises an abort flag on timeout, so
// every wave exits even if the grid were not co-resident.
#include <string.h>
#include "persist.h"
#include "kernels.h"
#include "xwg.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
union Frag { u32x4_t u; bf16x8_t v; };

#define NEG_BIG (-1.0e30f)
#define PART_FLOATS (8 * 64 * 4 + 128)
#define CHUNK_UNITS 4                       // activation units staged in LDS at a time (64 KB)
#define LDS_ACT_BYTES (CHUNK_UNITS * 8 * 2 * 1024)
#define LDS_EX_BYTES (16 * 132 * 4)
#define LDS_USED (LDS_ACT_BYTES + LDS_EX_BYTES + 9 * 16 * 4 + 2 * 8 * 16 * 4 + 64)
#define LDS_TOTAL (96 * 1024)               // more than half of a CU's 160 KB: exactly one workgroup per CU
#define BARRIER_SPIN_MAX (1 << 21)
#ifdef FC_TRACE
#define TRACE(code) do { if (tid == 0 && (wg == 0 || wg == 100) && a.trace && ntrace < 4000) { a.trace[(wg ? 8192 : 0) + 2 * ntrace] = wall_clock64(); a.trace[(wg ? 8192 : 0) + 2 * ntrace + 1] = (code); ++ntrace; } } while (0)
#else
#define TRACE(code) do { } while (0)
#endif

__device__ inline uint32_t rne16(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ inline float up16(uint32_t b) { return __uint_as_float(b << 16); }
__device__ inline void split8(const float* v, Frag& hi, Frag& lo) {
    uint32_t h[8], l[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { h[e] = rne16(v[e]); l[e] = rne16(v[e] - up16(h[e])); }
    hi.u = (u32x4_t){h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    lo.u = (u32x4_t){l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16)};
}
__device__ inline void st_agent_u16(bf16_t* p, uint32_t v) {
    __hip_atomic_store(p, (bf16_t)v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 16 bytes of bf16 from the KV cache: ordinary load, or agent-scope when the data is this step's
__device__ inline u32x4_t ld_kv16(const bf16_t* p, bool coherent) {
    if (!coherent) return *(const u32x4_t*)p;
    const uint64_t a = __hip_atomic_load((const uint64_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint64_t b = __hip_atomic_load((const uint64_t*)p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return (u32x4_t){(uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32)};
}

// ------------------------------------------------------------------ prefetch cursor over the step's GEMM units
struct Cur { int layer, st, f, f1; };      // st 0..3 inside a layer, 4 = LM head; layer < 0: exhausted

__device__ inline void cur_range(const PersistArgs& a, Cur& c, int wg) {
    const int U = a.mat[c.st].ncg * a.mat[c.st].NU;
    c.f = (int)(((unsigned)wg * (unsigned)U) / (unsigned)a.G);
    c.f1 = (int)(((unsigned)(wg + 1) * (unsigned)U) / (unsigned)a.G);
}
__device__ inline void cur_next_stage(const PersistArgs& a, Cur& c, int wg) {
    for (;;) {
        if (c.st == 4) { c.layer = -1; return; }
        if (c.st == 3) {
            if (c.layer + 1 < a.L) { c.layer++; c.st = 0; }
            else if (a.lmhead) c.st = 4;
            else { c.layer = -1; return; }
        } else c.st++;
        cur_range(a, c, wg);
        if (c.f < c.f1) return;
    }
}
__device__ inline void cur_begin(const PersistArgs& a, Cur& c, int wg) {
    c.layer = 0; c.st = 0;
    if (a.L == 0) { if (!a.lmhead) { c.layer = -1; return; } c.st = 4; }
    cur_range(a, c, wg);
    if (c.f >= c.f1) cur_next_stage(a, c, wg);
}
__device__ inline void cur_advance(const PersistArgs& a, Cur& c, int wg) {
    if (c.layer < 0) return;
    if (++c.f >= c.f1) cur_next_stage(a, c, wg);
}
// this wave's 8 tiles of the unit under the cursor; a valid dummy address (always the same 8 KB, so
// the loads hit in cache) when there is nothing to prefetch: bank loads are issued unconditionally,
// because a conditionally assigned register bank forces the compiler to copy it, and a copy waits
// for every load in flight
__device__ inline const u32x4_t* cur_ptr(const PersistArgs& a, const Cur& c, int w, int lane, bool want) {
    if (c.layer < 0 || !want) return (const u32x4_t*)a.weights + lane;
    const PMat& m = a.mat[c.st];
    const char* base = a.weights + (c.st == 4 ? m.off : a.layers_off + (size_t)c.layer * a.layer_stride + m.off);
    const int cg = c.f / m.NU, u = c.f - cg * m.NU, nt = cg * 8 + w;
    if (nt >= m.NT) return (const u32x4_t*)a.weights + lane;
    return (const u32x4_t*)base + ((size_t)nt * (m.K >> 5) + (size_t)u * 8) * 64 + lane;
}
#define LOAD_BANK(BANK, CURSOR, WANT)                                                \
    do {                                                                             \
        const u32x4_t* p_ = cur_ptr(a, CURSOR, w, lane, WANT);                       \
        _Pragma("unroll") for (int j_ = 0; j_ < 8; ++j_) BANK[j_] = __builtin_nontemporal_load(p_ + (size_t)j_ * 64); \
    } while (0)

// ------------------------------------------------------------------ grid barrier
// Precondition: every wave of the workgroup has waited for its agent-scope stores (wait_vmem_done).
__device__ inline bool grid_barrier(int32_t* sync, int target, int* lds_flag) {
    __syncthreads();
    if (threadIdx.x == 0) {
        arrive_agent(sync);
        int ok = 0;
        for (int it = 0; it < BARRIER_SPIN_MAX; ++it) {
            if (__hip_atomic_load(sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) { ok = 1; break; }
            if (__hip_atomic_load(sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
            __builtin_amdgcn_s_sleep(4);
        }
        if (!ok) st_agent_i32(sync + 1, 1);     // timeout or abort seen: tell everyone, leave
        *lds_flag = ok;
    }
    __syncthreads();
    return *lds_flag != 0;
}

// ------------------------------------------------------------------ the kernel
__global__ __launch_bounds__(512) void k_step(PersistArgs a) {
    extern __shared__ u32x4_t smem[];
    float* lds_ex = (float*)((char*)smem + LDS_ACT_BYTES);             // [16][132] epilogue exchange
    float* lds_ss = (float*)((char*)lds_ex + LDS_EX_BYTES);            // [8][16] per-wave row sums of squares
    float* lds_rs = lds_ss + 8 * 16;                                   // [16]
    float* lds_amv = lds_rs + 16;                                      // [8][16]
    int* lds_ami = (int*)(lds_amv + 8 * 16);                           // [8][16]
    int* lds_flag = lds_ami + 8 * 16;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int lm = lane & 15, g4 = lane >> 4;
    const int wg = blockIdx.x, G = a.G;
    int nbar = 0;
    int ntrace = 0; (void)ntrace;

    Cur pre;
    cur_begin(a, pre, wg);
    u32x4_t A[8], B[8];
    LOAD_BANK(A, pre, true); cur_advance(a, pre, wg);
    LOAD_BANK(B, pre, true); cur_advance(a, pre, wg);

    // ---------------------------------------------------------------- one GEMM stage
    auto gemm_stage = [&](int st, int layer) {
        const PMat& mt = a.mat[st];
        const int NU = mt.NU, U = mt.ncg * NU, K = mt.K;
        const float* X; const float* gain = nullptr;
        const char* lb = a.weights + a.layers_off + (size_t)layer * a.layer_stride;
        if (st == 0) { X = a.x; gain = (const float*)(lb + a.g1_off); }
        else if (st == 1) X = a.att;
        else if (st == 2) { X = a.x; gain = (const float*)(lb + a.g2_off); }
        else if (st == 3) X = a.h;
        else { X = a.x; gain = (const float*)(a.weights + a.gf_off); }
        const int f0 = (int)(((unsigned)wg * (unsigned)U) / (unsigned)G);
        const int f1 = (int)(((unsigned)(wg + 1) * (unsigned)U) / (unsigned)G);
        int f = f0;
        int par = 0;                      // 0: next unit sits in bank A, 1: in bank B
        const int row = lm < a.M ? lm : a.M - 1;

        while (f < f1) {
            // ---- sub-task: units [u_lo, u_hi) of column group cg
            const int cg = f / NU, u_lo = f - cg * NU;
            const int u_hi = (NU - u_lo < f1 - f) ? NU : u_lo + (f1 - f);
            const int nt = cg * 8 + w;
            const bool active = nt < mt.NT;
            f32x4_t acc = (f32x4_t){0.f, 0.f, 0.f, 0.f};
            float ss = 0.f;

            for (int uc = u_lo; uc < u_hi; uc += CHUNK_UNITS) {
                const int nc = (u_hi - uc < CHUNK_UNITS) ? u_hi - uc : CHUNK_UNITS;
                TRACE(1);
                __syncthreads();                                   // LDS free: previous reads are done
                // stage units [uc, uc+nc): wave w converts k-tiles w, w+8, .. (nc tiles)
                {
                    const float* xr = X + (size_t)row * K + (size_t)uc * 256 + 8 * g4;
                    float xv[CHUNK_UNITS][8];
#pragma unroll
                    for (int i = 0; i < CHUNK_UNITS; ++i)
                        if (i < nc) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) xv[i][e] = ld_agent_f32(xr + (w + 8 * i) * 32 + e);
                        }
#pragma unroll
                    for (int i = 0; i < CHUNK_UNITS; ++i)
                        if (i < nc) {
                            float v[8];
#pragma unroll
                            for (int e = 0; e < 8; ++e) { v[e] = xv[i][e]; ss += v[e] * v[e]; }
                            if (gain) {
                                const float* gp = gain + (size_t)uc * 256 + 8 * g4 + (w + 8 * i) * 32;
                                const float4 g0 = *(const float4*)gp, g1 = *(const float4*)(gp + 4);
                                v[0] *= g0.x; v[1] *= g0.y; v[2] *= g0.z; v[3] *= g0.w;
                                v[4] *= g1.x; v[5] *= g1.y; v[6] *= g1.z; v[7] *= g1.w;
                            }
                            Frag hi, lo;
                            split8(v, hi, lo);
                            smem[((size_t)(w + 8 * i) * 2) * 64 + lane] = hi.u;
                            smem[((size_t)(w + 8 * i) * 2 + 1) * 64 + lane] = lo.u;
                        }
                }
                TRACE(2);
                __syncthreads();
                TRACE(3);
                // consume nc units, alternating banks; refill each bank right after its use
                for (int k = 0; k < nc; ++k) {
                    // the QKV stage prefetches only inside itself: the banks are reloaded behind attention
                    const bool want = st != 0 || (pre.layer == layer && pre.st == 0);
                    if (par == 0) {
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            Frag wf; wf.u = A[j];
#pragma unroll
                            for (int p = 0; p < 2; ++p) {
                                Frag af; af.u = smem[((size_t)(k * 8 + j) * 2 + p) * 64 + lane];
                                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf.v, af.v, acc, 0, 0, 0);
                            }
                        }
                        LOAD_BANK(A, pre, want);
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            Frag wf; wf.u = B[j];
#pragma unroll
                            for (int p = 0; p < 2; ++p) {
                                Frag af; af.u = smem[((size_t)(k * 8 + j) * 2 + p) * 64 + lane];
                                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf.v, af.v, acc, 0, 0, 0);
                            }
                        }
                        LOAD_BANK(B, pre, want);
                    }
                    if (want) cur_advance(a, pre, wg);
                    par ^= 1;
                }
            }
            f += u_hi - u_lo;
            TRACE(4);

            // ---- row sums of squares of this workgroup's units
            ss += __shfl_xor(ss, 16, 64);
            ss += __shfl_xor(ss, 32, 64);
            if (g4 == 0) lds_ss[w * 16 + lm] = ss;
            __syncthreads();
            if (tid < 16) {
                float s = 0.f;
#pragma unroll
                for (int q = 0; q < 8; ++q) s += lds_ss[q * 16 + tid];
                lds_rs[tid] = s;
            }
            __syncthreads();

            // ---- hand-off between the contributors of this column group
            const int g_first = cg * NU, g_last = cg * NU + NU - 1;
            const int c_first = (int)((((unsigned)g_first + 1u) * (unsigned)G + (unsigned)U - 1u) / (unsigned)U) - 1;
            const int c_last = (int)((((unsigned)g_last + 1u) * (unsigned)G + (unsigned)U - 1u) / (unsigned)U) - 1;
            // with fewer units than workgroups every unit has its own workgroup (the ones between own nothing)
            const int count = U >= G ? c_last - c_first + 1 : NU;
            const int idx = U >= G ? wg - c_first : u_lo;
            if (count > 1) {
                const int cmax = a.cmax[st];
                float* mypart = a.part + (((size_t)(cg * cmax + idx) * 8 + w) * 64 + lane) * 4;
#pragma unroll
                for (int r = 0; r < 4; ++r) st_agent_f32(mypart + r, acc[r]);
                if (tid < 16) st_agent_f32(a.sspart + (size_t)(cg * cmax + idx) * 16 + tid, lds_rs[tid]);
                TRACE(5);
                wait_vmem_done();
                TRACE(6);
                __syncthreads();
                if (tid == 0) *lds_flag = (arrive_agent(a.cnt + cg) == count - 1);
                __syncthreads();
                TRACE(7);
                if (!*lds_flag) continue;                           // someone else finishes this column group
                acc = (f32x4_t){0.f, 0.f, 0.f, 0.f};
                for (int s0 = 0; s0 < count; s0 += 8) {
                    float pv[8][4];
#pragma unroll
                    for (int s = 0; s < 8; ++s)
                        if (s0 + s < count) {
                            const float* p = a.part + (((size_t)(cg * cmax + s0 + s) * 8 + w) * 64 + lane) * 4;
#pragma unroll
                            for (int r = 0; r < 4; ++r) pv[s][r] = ld_agent_f32(p + r);
                        }
#pragma unroll
                    for (int s = 0; s < 8; ++s)
                        if (s0 + s < count) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) acc[r] += pv[s][r];
                        }
                }
                if (tid < 16) {
                    float s = 0.f;
                    for (int q = 0; q < count; ++q) s += ld_agent_f32(a.sspart + (size_t)(cg * cmax + q) * 16 + tid);
                    lds_rs[tid] = s;
                }
                if (tid == 0) st_agent_i32(a.cnt + cg, 0);
                __syncthreads();
            }

            TRACE(8);
            // ---- epilogue: lane holds row lm, columns nt*16 + 4*g4 + r
            const float rs = gain ? 1.0f / sqrtf(lds_rs[lm] / (float)K + a.eps) : 1.0f;
            if (st == 1 || st == 3) {                       // residual add into x
                if (active && lm < a.M) {
                    float* o = a.x + (size_t)lm * a.d + nt * 16 + 4 * g4;
                    float v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = ld_agent_f32(o + r);
#pragma unroll
                    for (int r = 0; r < 4; ++r) st_agent_f32(o + r, v[r] + acc[r]);
                }
            } else if (st == 2) {                           // SwiGLU: gate in lanes g4 < 2, up in lane ^ 32
                float hv[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float mine = acc[r] * rs;
                    const float other = __shfl_xor(mine, 32, 64);
                    hv[r] = mine / (1.0f + expf(-mine)) * other;
                }
                if (active && g4 < 2 && lm < a.M) {
                    float* o = a.h + (size_t)lm * a.F + nt * 8 + 4 * g4;
#pragma unroll
                    for (int r = 0; r < 4; ++r) st_agent_f32(o + r, hv[r]);
                }
            } else if (st == 0) {                           // rotary embedding, q store, KV-cache write
                if (active) *(f32x4_t*)(lds_ex + (size_t)lm * 132 + (cg < a.H + a.Hkv ? (g4 < 2 ? 8 * w + 4 * g4 : 64 + 8 * w + 4 * (g4 - 2)) : w * 16 + 4 * g4)) = acc * rs;
                __syncthreads();
                const int hh = cg;
                const size_t plane = (size_t)a.S * 128;
                if (hh < a.H + a.Hkv) {
                    for (int id = tid; id < 16 * 64; id += 512) {
                        const int m = id >> 6, i = id & 63;
                        if (m >= a.M) continue;
                        const int b = m / a.W, j = m % a.W;
                        const int pos = a.state[a.sm.n + b] + j;
                        if (pos >= a.S) continue;
                        const float c = a.cosT[(size_t)pos * 64 + i], s = a.sinT[(size_t)pos * 64 + i];
                        const float x0 = lds_ex[(size_t)m * 132 + i], x1 = lds_ex[(size_t)m * 132 + i + 64];
                        const float r0 = x0 * c - x1 * s, r1 = x1 * c + x0 * s;
                        if (hh < a.H) {
                            float* q = a.q + (size_t)m * (a.H * 128) + hh * 128;
                            st_agent_f32(q + i, r0); st_agent_f32(q + i + 64, r1);
                        } else {
                            bf16_t* kr = a.kc + ((((size_t)layer * a.B + b) * a.Hkv + (hh - a.H)) * a.kvp) * plane;
                            const size_t i0 = k_index(pos, i, 128), i1 = k_index(pos, i + 64, 128);
                            const uint32_t h0 = rne16(r0), h1 = rne16(r1);
                            st_agent_u16(kr + i0, h0); st_agent_u16(kr + i1, h1);
                            if (a.kvp == 2) {
                                st_agent_u16(kr + plane + i0, rne16(r0 - up16(h0)));
                                st_agent_u16(kr + plane + i1, rne16(r1 - up16(h1)));
                            }
                        }
                    }
                } else {
                    const int kh = hh - a.H - a.Hkv;
                    for (int id = tid; id < 16 * 128; id += 512) {
                        const int m = id & 15, e = id >> 4;
                        if (m >= a.M) continue;
                        const int b = m / a.W, j = m % a.W;
                        const int pos = a.state[a.sm.n + b] + j;
                        if (pos >= a.S) continue;
                        bf16_t* vr = a.vc + ((((size_t)layer * a.B + b) * a.Hkv + kh) * a.kvp) * plane + v_index(e, pos, 128);
                        const float vv = lds_ex[(size_t)m * 132 + e];
                        const uint32_t h0 = rne16(vv);
                        st_agent_u16(vr, h0);
                        if (a.kvp == 2) st_agent_u16(vr + plane, rne16(vv - up16(h0)));
                    }
                }
            } else {                                        // LM head: per-row winner of this column group
                float best = NEG_BIG * 1.0e8f; int bi = 0x7fffffff;
                if (active) {
                    const int n0 = nt * 16 + 4 * g4;
                    float v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = acc[r] * rs;
                    if (a.logits && lm < a.M) *(float4*)(a.logits + (size_t)lm * a.V + n0) = make_float4(v[0], v[1], v[2], v[3]);
#pragma unroll
                    for (int r = 0; r < 4; ++r) if (v[r] > best) { best = v[r]; bi = n0 + r; }
                }
#pragma unroll
                for (int o = 16; o <= 32; o <<= 1) {
                    const float ov = __shfl_xor(best, o, 64); const int oi = __shfl_xor(bi, o, 64);
                    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
                }
                if (g4 == 0) { lds_amv[w * 16 + lm] = best; lds_ami[w * 16 + lm] = bi; }
                __syncthreads();
                if (tid < 16) {
                    float bv = lds_amv[tid]; int bx = lds_ami[tid];
                    for (int q = 1; q < 8; ++q) {
                        const float ov = lds_amv[q * 16 + tid]; const int oi = lds_ami[q * 16 + tid];
                        if (ov > bv || (ov == bv && oi < bx)) { bv = ov; bx = oi; }
                    }
                    st_agent_f32(a.amax_val + (size_t)cg * 16 + tid, bv);
                    st_agent_i32(a.amax_idx + (size_t)cg * 16 + tid, bx);
                }
            }
        }
        TRACE(9);
        // the next unit must sit in bank A when the following stage starts (after the QKV stage the
        // banks are reloaded behind the attention stage instead)
        if (par && st != 0) {
#pragma unroll
            for (int j = 0; j < 8; ++j) { const u32x4_t t = A[j]; A[j] = B[j]; B[j] = t; }
        }
        wait_vmem_done();
        TRACE(10);
    };

    // ---------------------------------------------------------------- attention stage
    auto attention = [&](int layer) {
        const int pairs = a.Bact * a.H;
        int nsp = 1;
        if (pairs <= G) { nsp = G / pairs; if (nsp > FC_MAX_ATTN_SPLITS) nsp = FC_MAX_ATTN_SPLITS; }
        float* lds = (float*)smem;
        TRACE(20);
        for (int item = wg; item < pairs * nsp; item += G) {
            const int bh = item / nsp, sp = item - bh * nsp;
            const int b = bh / a.H, h = bh - b * a.H, kvh = h / (a.H / a.Hkv);
            const int n = a.state[a.sm.n + b];
            int T = n + a.W;
            if (T > a.S) T = a.S;
            const int NB = (T + 31) >> 5;
            const int blk0 = (int)(((unsigned)sp * (unsigned)NB) / (unsigned)nsp);
            const int blk1 = (int)(((unsigned)(sp + 1) * (unsigned)NB) / (unsigned)nsp);
            const size_t plane = (size_t)a.S * 128;
            const bf16_t* kbase = a.kc + ((((size_t)layer * a.B + b) * a.Hkv + kvh) * a.kvp) * plane;
            const bf16_t* vbase = a.vc + ((((size_t)layer * a.B + b) * a.Hkv + kvh) * a.kvp) * plane;
            const bool two = a.kvp == 2;

            Frag qh[4], ql[4];
            {
                int j = lm;
                if (j >= a.W) j = a.W - 1;
                const float* qr = a.q + (size_t)(b * a.W + j) * (a.H * 128) + h * 128 + 32 * g4;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    float v[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = ld_agent_f32(qr + 8 * s + e);
                    split8(v, qh[s], ql[s]);
                }
            }
            f32x4_t acc[8];
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) acc[dt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
            float mrun = NEG_BIG, lrun = 0.f;
            const float scale = 0.08838834764831845f;

            for (int blk = blk0 + w; blk < blk1; blk += 8) {
                const int kb = blk << 5;
                const bool coh = kb + 32 > n;                 // block holds rows written in this launch
                f32x4_t sc[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const bf16_t* kp = kbase + (size_t)blk * 4096 + (size_t)(t * 4 * 64 + lane) * 8;   // fragment (t, s) at + s * 512
                    sc[t] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        Frag kf; kf.u = ld_kv16(kp + 512 * s, coh);
                        sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, qh[s].v, sc[t], 0, 0, 0);
                        sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf.v, ql[s].v, sc[t], 0, 0, 0);
                        if (two) {
                            Frag kl; kl.u = ld_kv16(kp + plane + 512 * s, coh);
                            sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kl.v, qh[s].v, sc[t], 0, 0, 0);
                        }
                    }
                }
                const int lastvis = n + (lm < a.W ? lm : a.W - 1);
                float p[8];
                float bm = NEG_BIG;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int key = kb + 8 * g4 + e;
                    const bool vis = key <= lastvis && key < T;
                    p[e] = vis ? sc[e >> 2][e & 3] * scale : NEG_BIG;
                    bm = fmaxf(bm, p[e]);
                }
                bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
                bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
                const float mnew = fmaxf(mrun, bm);
                const float alpha = expf(mrun - mnew);
                float ps = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int key = kb + 8 * g4 + e;
                    const bool vis = key <= lastvis && key < T;
                    p[e] = vis ? expf(p[e] - mnew) : 0.f;
                    ps += p[e];
                }
                mrun = mnew;
                lrun = lrun * alpha + ps;
                Frag ph, pl;
                split8(p, ph, pl);
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) {
                    const bf16_t* vp = vbase + (size_t)(kb >> 5) * 4096 + (size_t)(dt * 64 + lane) * 8;
                    Frag vf; vf.u = ld_kv16(vp, coh);
                    acc[dt] *= alpha;
                    acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, ph.v, acc[dt], 0, 0, 0);
                    acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, pl.v, acc[dt], 0, 0, 0);
                    if (two) {
                        Frag vl; vl.u = ld_kv16(vp + plane, coh);
                        acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vl.v, ph.v, acc[dt], 0, 0, 0);
                    }
                }
            }
            lrun += __shfl_xor(lrun, 16, 64);
            lrun += __shfl_xor(lrun, 32, 64);
            TRACE(21);

            // merge the 8 waves through LDS (wave 0 folds waves 1..7 in order)
            __syncthreads();
            if (w > 0) {
                float* dst = lds + (size_t)(w - 1) * PART_FLOATS;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) *(f32x4_t*)(dst + (dt * 64 + lane) * 4) = acc[dt];
                dst[2048 + lane] = mrun;
                dst[2112 + lane] = lrun;
            }
            __syncthreads();
            if (w == 0) {
                for (int w2 = 1; w2 < 8; ++w2) {
                    const float* s = lds + (size_t)(w2 - 1) * PART_FLOATS;
                    const float mo = s[2048 + lane], lo = s[2112 + lane];
                    const float mnew = fmaxf(mrun, mo);
                    const float wa = expf(mrun - mnew), wb = expf(mo - mnew);
                    lrun = lrun * wa + lo * wb;
                    mrun = mnew;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) acc[dt] = acc[dt] * wa + *(const f32x4_t*)(s + (dt * 64 + lane) * 4) * wb;
                }
                bool finish = true;
                if (nsp > 1) {
                    float* mine = a.apart + ((size_t)bh * nsp + sp) * PART_FLOATS;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) st_agent_f32(mine + (dt * 64 + lane) * 4 + r, acc[dt][r]);
                    st_agent_f32(mine + 2048 + lane, mrun);
                    st_agent_f32(mine + 2112 + lane, lrun);
                    wait_vmem_done();
                    int old = 0;
                    if (lane == 0) old = arrive_agent(a.acnt + bh);
                    old = __shfl(old, 0, 64);
                    finish = (old == nsp - 1);
                    if (finish) {
                        mrun = NEG_BIG; lrun = 0.f;
#pragma unroll
                        for (int dt = 0; dt < 8; ++dt) acc[dt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
                        for (int s2 = 0; s2 < nsp; ++s2) {
                            const float* s = a.apart + ((size_t)bh * nsp + s2) * PART_FLOATS;
                            const float mo = ld_agent_f32(s + 2048 + lane), lo = ld_agent_f32(s + 2112 + lane);
                            const float mnew = fmaxf(mrun, mo);
                            const float wa = expf(mrun - mnew), wb = expf(mo - mnew);
                            lrun = lrun * wa + lo * wb;
                            mrun = mnew;
#pragma unroll
                            for (int dt = 0; dt < 8; ++dt) {
                                f32x4_t o;
#pragma unroll
                                for (int r = 0; r < 4; ++r) o[r] = ld_agent_f32(s + (dt * 64 + lane) * 4 + r);
                                acc[dt] = acc[dt] * wa + o * wb;
                            }
                        }
                        if (lane == 0) st_agent_i32(a.acnt + bh, 0);
                    }
                }
                if (finish && lm < a.W) {
                    const float inv = 1.0f / lrun;
                    float* o = a.att + (size_t)(b * a.W + lm) * (a.H * 128) + h * 128 + 4 * g4;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) st_agent_f32(o + 16 * dt + r, acc[dt][r] * inv);
                }
            }
        }
        TRACE(22);
        wait_vmem_done();
        TRACE(23);
    };

#define BARRIER()                                                   \
    do {                                                            \
        ++nbar;                                                     \
        if (!grid_barrier(a.sync, nbar * G, lds_flag)) return;      \
        TRACE(11);                                                  \
    } while (0)

    // stage sequence: per layer QKV, attention, O, gate/up, down; then the LM head
    const int n_gemm = 4 * a.L + (a.lmhead ? 1 : 0);
#pragma nounroll
    for (int idx = 0; idx < n_gemm; ++idx) {
        const int l = idx >> 2;
        const int st = (idx == 4 * a.L) ? 4 : (idx & 3);
        if (a.dbg_stop >= 0 && 5 * l + (st == 0 ? 0 : st + 1) >= a.dbg_stop) return;
        gemm_stage(st, l);
        BARRIER();
        if (st == 0) {
            if (a.dbg_stop >= 0 && 5 * l + 1 >= a.dbg_stop) return;
            attention(l);
            // weight tiles are not kept in registers across attention: restart the prefetch behind it
            pre.layer = l; pre.st = 0; pre.f = pre.f1 = 0;
            cur_next_stage(a, pre, wg);
            LOAD_BANK(A, pre, true); cur_advance(a, pre, wg);
            LOAD_BANK(B, pre, true); cur_advance(a, pre, wg);
            BARRIER();
        }
    }
    if (!a.lmhead) return;
    if (wg != 0) return;

    // ---------------------------------------------------------------- final argmax + accept/commit (workgroup 0)
    int32_t* st = a.state;
    const StateMap& sm = a.sm;
    if (tid < a.M) {
        float best = NEG_BIG * 1.0e8f; int bi = 0x7fffffff;
        const int ncg = a.mat[4].ncg;
        for (int c = 0; c < ncg; ++c) {
            const float v = ld_agent_f32(a.amax_val + (size_t)c * 16 + tid);
            const int i = __hip_atomic_load(a.amax_idx + (size_t)c * 16 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v > best || (v == best && i < bi)) { best = v; bi = i; }
        }
        st[sm.o + tid] = bi;
        a.topv[tid] = best;
    }
    __syncthreads();
    if (!a.do_accept) return;
    // verification (Eq. 5), acceptance, buffer update, window shift, stop conditions: one thread per sequence
    int* not_done = lds_flag + 1;
    if (tid == 0) *not_done = 0;
    __syncthreads();
    const int W = a.W, S = a.S;
    const int max_new = st[sm.params + PARAM_MAX_NEW], eos = st[sm.params + PARAM_EOS];
    const int max_steps = st[sm.params + PARAM_MAX_STEPS], buf_len = st[sm.params + PARAM_BUF_LEN];
    for (int b = tid; b < a.Bact; b += 512) {
        if (st[sm.done + b]) { st[sm.lastK + b] = -1; continue; }
        const int32_t* wv = st + sm.win + b * W;
        const int32_t* o = st + sm.o + b * W;
        int32_t* buf = st + sm.buf + (size_t)b * S;
        int32_t* out = st + sm.out + (size_t)b * S;
        int n = st[sm.n + b], g = st[sm.g + b], steps = st[sm.steps + b];
        const int ws = st[sm.wseq + b], Wb = ws > 0 && ws < W ? ws : W;     // the sequence's own window, if it has one
        int K = 0;
        while (K < Wb - 1 && o[K] == wv[K + 1]) ++K;
        for (int j = 0; j < Wb; ++j) if (g + j < buf_len) buf[g + j] = o[j];
        int stop = 0, emitted = 0;
        for (int j = 0; j <= K && !stop; ++j) {
            if (g + j < max_new && g + j < S) { out[g + j] = o[j]; emitted = g + j + 1; }
            if (eos >= 0 && o[j] == eos) stop = 1;
        }
        if (emitted > st[sm.olen + b]) st[sm.olen + b] = emitted;
        const int newest = o[K];
        n += K + 1; g += K + 1; ++steps;
        if (g >= max_new || (max_steps > 0 && steps >= max_steps)) stop = 1;
        if (n + W > S || g + 2 * W - 1 > buf_len) {
            if (!stop) st[sm.flags + FLAG_ERROR] = 1;
            stop = 1;
        }
        st[sm.n + b] = n; st[sm.g + b] = g; st[sm.steps + b] = steps; st[sm.lastK + b] = K;
        st[sm.newest + b] = newest; st[sm.done + b] = stop;
        int32_t* wn = st + sm.win + b * W;
        wn[0] = newest;
        for (int j = 1; j < W; ++j) { const int p = g + j - 1; wn[j] = p < buf_len ? buf[p] : 0; }
        if (!stop) atomicAdd(not_done, 1);
    }
    __syncthreads();
    if (tid == 0) st[sm.flags + FLAG_ALL_DONE] = (*not_done == 0);
}

// barrier reset + embedding gather (rows of the window)
__global__ void k_step_begin(int32_t* sync, const bf16_t* emb, const int32_t* win, float* x, int d, int V) {
    if (blockIdx.x == 0 && threadIdx.x == 0) { sync[0] = 0; sync[1] = 0; }
    int t = win[blockIdx.x];
    if (t < 0 || t >= V) t = 0;
    for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)blockIdx.x * d + i] = bf16_to_f32(emb[(size_t)t * d + i]);
}

// ------------------------------------------------------------------ host side
static int g_num_cu = 0;
static bool g_attr_set = false;

bool fc_persist_supported(const KernelDims& kd, int rows) {
    return kd.esz == 2 && kd.Dh == 128 && rows >= 1 && rows <= 16 && kd.W <= 16 && kd.d % 256 == 0 && kd.F % 256 == 0 &&
           (kd.H * kd.Dh) % 256 == 0 && kd.S % 32 == 0 && kd.V % 128 == 0 && ((kd.H + 2 * kd.Hkv) * kd.Dh) % 128 == 0 &&
           (2 * kd.F) % 128 == 0 && kd.d % 128 == 0;
}

hipError_t fc_persist_step(const FastArgs& fa, int do_accept, void* prof, hipError_t (*prof_mark)(void*, int)) {
    hipError_t e;
    if (!g_num_cu) {
        int dev = 0;
        if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
        hipDeviceProp_t p;
        if ((e = hipGetDeviceProperties(&p, dev)) != hipSuccess) return e;
        g_num_cu = p.multiProcessorCount;
    }
    if (!g_attr_set) {
        if ((e = hipFuncSetAttribute((const void*)k_step, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_TOTAL)) != hipSuccess) return e;
        int per_cu = 0;
        if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_step, 512, LDS_TOTAL)) != hipSuccess) return e;
        if (per_cu < 1) return hipErrorLaunchOutOfResources;
        g_attr_set = true;
    }
    const KernelDims& kd = fa.kd; const ModelMap& mm = *fa.mm; const WorkspaceMap& wm = *fa.wm;
    PersistArgs a; memset(&a, 0, sizeof(a));
    a.weights = fa.weights; a.layers_off = mm.layers_off; a.layer_stride = mm.layer_stride;
    a.g1_off = mm.g1_off; a.g2_off = mm.g2_off; a.gf_off = mm.gf_off;
    const FusedMat* fm[5] = {&mm.qkv, &mm.o, &mm.gu, &mm.down, &mm.lm};
    a.G = g_num_cu;
    for (int i = 0; i < 5; ++i) {
        a.mat[i].off = fm[i]->off; a.mat[i].K = fm[i]->K; a.mat[i].NT = fm[i]->N / 16;
        a.mat[i].ncg = (a.mat[i].NT + 7) / 8; a.mat[i].NU = fm[i]->K / 256;
        a.cmax[i] = a.G / a.mat[i].ncg + 2;
    }
    a.L = kd.L; a.M = kd.M; a.Bact = fa.Bact; a.lmhead = fa.lmhead; a.do_accept = do_accept;
    a.H = kd.H; a.Hkv = kd.Hkv; a.B = kd.B; a.S = kd.S; a.W = kd.W; a.kvp = kd.kvp; a.V = kd.V; a.d = kd.d; a.F = kd.F;
    a.eps = kd.eps;
    char* ws = fa.ws;
    a.x = (float*)(ws + wm.x); a.q = (float*)(ws + wm.qkv); a.att = (float*)(ws + wm.att); a.h = (float*)(ws + wm.h);
    a.part = (float*)(ws + wm.gemm_part);
    a.sspart = a.part + (size_t)(a.G + 2 * 512) * 8 * 256;      // behind (G + 2 ncg) partial tiles, ncg <= 512
    a.cnt = (int32_t*)(ws + wm.gemm_cnt);
    a.apart = (float*)(ws + wm.attn_part); a.acnt = (int32_t*)(ws + wm.attn_cnt);
    a.sync = (int32_t*)(ws + wm.gemm_cnt) + FC_MAX_COUNTERS - 8;
    a.cosT = (const float*)(ws + wm.rope_cos); a.sinT = (const float*)(ws + wm.rope_sin);
    a.kc = (bf16_t*)(ws + wm.kc); a.vc = (bf16_t*)(ws + wm.vc);
    a.amax_val = (float*)(ws + wm.amax_part); a.amax_idx = (int32_t*)(a.amax_val + (size_t)a.mat[4].ncg * 16);
    a.logits = fa.dbg_logits; a.topv = (float*)(ws + wm.topv);
    a.state = (int32_t*)(ws + wm.state); a.sm = wm.st; a.dbg_stop = fa.dbg_stop;
    a.trace = (uint64_t*)(ws + wm.logits);      // debug builds only: timestamps land in the (otherwise unused) plain-path logits buffer
    for (int i = 0; i < 5; ++i) if (a.mat[i].ncg > 512) return hipErrorInvalidValue;
    if (prof && (e = prof_mark(prof, 13)) != hipSuccess) return e;
    k_step_begin<<<kd.M, 256, 0, fa.st>>>(a.sync, (const bf16_t*)(fa.weights + mm.emb_off), a.state + a.sm.win, a.x, kd.d, kd.V);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    k_step<<<a.G, 512, LDS_TOTAL, fa.st>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (prof && (e = prof_mark(prof, -1)) != hipSuccess) return e;
    return hipSuccess;
}

size_t fc_persist_part_bytes(const KernelDims& kd) {
    return (size_t)(512 + 2 * 512) * 8 * 1024 + (size_t)(512 + 2 * 512) * 64 + 4096;
}
