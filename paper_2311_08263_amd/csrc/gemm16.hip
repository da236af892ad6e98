// Weight-streaming bf16 GEMM for a few activation rows (M <= 16*MT), the dominant kernel of a
// Jacobi step: out[m][n] = sum_k act[m][k] * W[k][n] with every weight read from HBM exactly once.
//
// Mapping.  The fused weight matrix is stored in MFMA fragment order (see frag_index): the tile of
// 16 output columns x 32 inputs is 1 KB, one 16-byte load per lane.  A workgroup of 8 waves owns a
// column group of 8 n-tiles (128 columns) and one K slice; wave w streams n-tile w over the slice
// with DEPTH tile loads in flight and feeds v_mfma_f32_16x16x32_bf16 with the weights as the
// A operand (16 columns x 32 k) and the activations as the B operand (32 k x 16 rows), so that a
// lane ends up with 4 consecutive output columns of one activation row.  The activations of the
// K slice are staged once per workgroup into LDS, converted from fp32 to a bf16 hi + bf16 lo pair
// (two MFMAs per weight tile: the weights are exact in bf16, hi+lo carries 16 mantissa bits of the
// activation, accumulation is fp32), in B-fragment order so LDS reads are conflict-free.
// With sk > 1 the K slices of a column group are different workgroups: each writes its partial
// tile, the last to arrive (atomic counter) sums the partials in slice order -- deterministic --
// and runs the epilogue.  Epilogues fuse what follows the contraction: RMSNorm scale (the norm
// commutes with the GEMM as a per-row factor; the gain is applied while staging), rotary
// embedding + KV-cache write, residual add, SwiGLU, or the LM head's per-row argmax.
#include "gemm16.h"
#include "xwg.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
union Frag { u32x4_t u; bf16x8_t v; };

__device__ inline uint32_t bf16_rne_bits(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ inline float bf16_bits_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Slices are cut at units of 8 k-tiles (K % 256 == 0); a wave keeps two banks of 8 tiles in flight.
template <int EPI, int MT, int NSPLIT>
__global__ __launch_bounds__(512) void k_gemm16(Gemm16Args a) {
    extern __shared__ u32x4_t smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int sk = a.sk, cg = (int)(blockIdx.x / (unsigned)sk), ks = (int)(blockIdx.x - (unsigned)cg * (unsigned)sk);
    const int KT = a.K >> 5, NU = KT >> 3;
    const int nt = cg * 8 + w;
    const bool active = nt < a.NT;
    const int u0 = (int)(((unsigned)ks * (unsigned)NU) / (unsigned)sk), u1 = (int)(((unsigned)(ks + 1) * (unsigned)NU) / (unsigned)sk);
    const int nu = u1 - u0, nk = nu * 8, kt0 = u0 * 8;
    const int numax = (NU + sk - 1) / sk;                  // LDS is sized for the largest slice
    float* lds_ss = (float*)(smem + (size_t)numax * 8 * MT * NSPLIT * 64);   // [8 waves][MT*16], then [MT*16]
    float* lds_rs = lds_ss + 8 * MT * 16;
    int* lds_flag = (int*)(lds_rs + MT * 16);

    // 1. activation loads of the first two staged k-tiles (they return first), then two banks of weights
    const int lm = lane & 15, g4 = lane >> 4;
    const int row0 = lm < a.M ? lm : a.M - 1;               // rows past M repeat a valid row; never written out
    const float* xr0 = a.X + (size_t)row0 * a.ldx + kt0 * 32 + 8 * g4;
    float4 xa[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
        if (w + 8 * i < nk) {
            xa[i][0] = *(const float4*)(xr0 + (w + 8 * i) * 32);
            xa[i][1] = *(const float4*)(xr0 + (w + 8 * i) * 32 + 4);
        }
    const u32x4_t* wp = (const u32x4_t*)a.W + ((size_t)(active ? nt : 0) * KT + kt0) * 64 + lane;
    u32x4_t wa[8], wb[8];
    if (active) {
#pragma unroll
        for (int j = 0; j < 8; ++j) wa[j] = __builtin_nontemporal_load(wp + (size_t)j * 64);
        if (nu > 1) {
#pragma unroll
            for (int j = 0; j < 8; ++j) wb[j] = __builtin_nontemporal_load(wp + (size_t)(8 + j) * 64);
        }
    }

    // 2. stage the activation slice: fp32 -> (gain) -> bf16 hi/lo in B-fragment order (wave w takes
    //    k-tiles w, w+8, ..; lane = fragment lane, 8 consecutive k of row lane%16); row sum of squares
    const float* gp = a.gain ? a.gain + kt0 * 32 + 8 * g4 : nullptr;
    auto stage = [&](int t, int mt, float4 x0, float4 x1) -> float {
        float v[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += v[e] * v[e];
        if (gp) {
            const float4 g0 = *(const float4*)(gp + t * 32), g1 = *(const float4*)(gp + t * 32 + 4);
            v[0] *= g0.x; v[1] *= g0.y; v[2] *= g0.z; v[3] *= g0.w; v[4] *= g1.x; v[5] *= g1.y; v[6] *= g1.z; v[7] *= g1.w;
        }
        uint32_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = bf16_rne_bits(v[e]);
        u32x4_t* dst = smem + ((size_t)(t * MT + mt) * NSPLIT) * 64 + lane;
        dst[0] = (u32x4_t){h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
        if (NSPLIT == 2) {
            uint32_t l[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) l[e] = bf16_rne_bits(v[e] - bf16_bits_f32(h[e]));
            dst[64] = (u32x4_t){l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16)};
        }
        return ss;
    };
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int r = mt * 16 + lm;
        const float* xr = a.X + (size_t)(r < a.M ? r : a.M - 1) * a.ldx + kt0 * 32 + 8 * g4;
        float ss = 0.f;
        if (mt == 0) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
                if (w + 8 * i < nk) ss += stage(w + 8 * i, 0, xa[i][0], xa[i][1]);
        }
#pragma unroll 1
        for (int t = (mt == 0 ? w + 16 : w); t < nk; t += 8)
            ss += stage(t, mt, *(const float4*)(xr + t * 32), *(const float4*)(xr + t * 32 + 4));
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        if (g4 == 0) lds_ss[w * MT * 16 + mt * 16 + lm] = ss;
    }
    __syncthreads();
    if (tid < MT * 16) {
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) s += lds_ss[q * MT * 16 + tid];
        lds_rs[tid] = s;
    }

    // 3. stream the slice: consume a bank of 8 tiles, refill it two units ahead
    f32x4_t acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    if (active) {
        for (int u = 0; u < nu; u += 2) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                Frag wf; wf.u = wa[j];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int p = 0; p < NSPLIT; ++p) {
                        Frag af; af.u = smem[((size_t)((u * 8 + j) * MT + mt) * NSPLIT + p) * 64 + lane];
                        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf.v, af.v, acc[mt], 0, 0, 0);
                    }
            }
            if (u + 2 < nu) {
#pragma unroll
                for (int j = 0; j < 8; ++j) wa[j] = __builtin_nontemporal_load(wp + (size_t)((u + 2) * 8 + j) * 64);
            }
            if (u + 1 < nu) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    Frag wf; wf.u = wb[j];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int p = 0; p < NSPLIT; ++p) {
                            Frag af; af.u = smem[((size_t)(((u + 1) * 8 + j) * MT + mt) * NSPLIT + p) * 64 + lane];
                            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf.v, af.v, acc[mt], 0, 0, 0);
                        }
                }
                if (u + 3 < nu) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) wb[j] = __builtin_nontemporal_load(wp + (size_t)((u + 3) * 8 + j) * 64);
                }
            }
        }
    }

    // 4. cross-workgroup split-K: ordered fix-up by the last workgroup of the column group
    if (sk > 1) {
        float* mypart = a.part + ((((size_t)(cg * sk + ks) * 8 + w) * MT) * 64 + lane) * 4;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) st_agent_f32(mypart + mt * 256 + r, acc[mt][r]);
        float* sspart = a.sspart + (size_t)(cg * sk + ks) * (MT * 16);
        if (tid < MT * 16) st_agent_f32(sspart + tid, lds_rs[tid]);
        wait_vmem_done();
        __syncthreads();
        if (tid == 0) *lds_flag = (arrive_agent(a.cnt + cg) == sk - 1);
        __syncthreads();
        if (!*lds_flag) return;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
        // all loads of a batch of slices are issued before the first add: one memory round trip per
        // batch instead of one per slice; the adds stay in slice order
        for (int s0 = 0; s0 < sk; s0 += 8) {
            float pv[8][MT][4];
#pragma unroll
            for (int s = 0; s < 8; ++s)
                if (s0 + s < sk) {
                    const float* p = a.part + ((((size_t)(cg * sk + s0 + s) * 8 + w) * MT) * 64 + lane) * 4;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) pv[s][mt][r] = ld_agent_f32(p + mt * 256 + r);
                }
#pragma unroll
            for (int s = 0; s < 8; ++s)
                if (s0 + s < sk) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[mt][r] += pv[s][mt][r];
                }
        }
        if (tid < MT * 16) {
            float s = 0.f;
            for (int q0 = 0; q0 < sk; q0 += 16) {
                float sv[16];
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    if (q0 + q < sk) sv[q] = ld_agent_f32(a.sspart + (size_t)(cg * sk + q0 + q) * (MT * 16) + tid);
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    if (q0 + q < sk) s += sv[q];
            }
            lds_rs[tid] = s;
        }
        if (tid == 0) st_agent_i32(a.cnt + cg, 0);    // ready for the next launch
        __syncthreads();
    } else {
        __syncthreads();                // every wave is past its LDS reads before the region is reused
    }

    // 5. epilogue.  Lane holds rows m = mt*16 + (lane & 15), columns nt*16 + 4*(lane >> 4) + r.
    float rs[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
        rs[mt] = a.gain ? 1.0f / sqrtf(lds_rs[mt * 16 + lm] / (float)a.K + a.eps) : 1.0f;

    if (EPI == EPI_RESID) {
        if (!active) return;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = mt * 16 + lm;
            if (m < a.M) {
                float4* o = (float4*)(a.out + (size_t)m * a.ldo + nt * 16 + 4 * g4);
                float4 v = *o;
                v.x += acc[mt][0]; v.y += acc[mt][1]; v.z += acc[mt][2]; v.w += acc[mt][3];
                *o = v;
            }
        }
    } else if (EPI == EPI_SWIGLU) {
        // a tile holds gate features f0..f0+7 in columns 0..7 and their up values in columns 8..15:
        // the partner of lane l is lane l ^ 32
        if (!active) return;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = mt * 16 + lm;
            float4 h;
            float* hp = &h.x;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float mine = acc[mt][r] * rs[mt];
                const float other = __shfl_xor(mine, 32, 64);
                hp[r] = mine / (1.0f + expf(-mine)) * other;       // meaningful in the gate lanes (g4 < 2)
            }
            if (g4 < 2 && m < a.M) *(float4*)(a.out + (size_t)m * a.ldo + nt * 8 + 4 * g4) = h;
        }
    } else if (EPI == EPI_QKV) {
        // column group = one head of 128 (q heads, then k heads, then v heads)
        float* ex = (float*)smem;       // [MT*16][132]
        if (active) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                // q/k heads: tile w holds elements 8w..8w+7 and their rotary partners 64+8w..; v heads: natural
                *(float4*)(ex + (size_t)(mt * 16 + lm) * 132 + (cg < a.H + a.Hkv ? (g4 < 2 ? 8 * w + 4 * g4 : 64 + 8 * w + 4 * (g4 - 2)) : w * 16 + 4 * g4)) =
                    make_float4(acc[mt][0] * rs[mt], acc[mt][1] * rs[mt], acc[mt][2] * rs[mt], acc[mt][3] * rs[mt]);
        }
        __syncthreads();
        const int hh = cg;
        const size_t plane = (size_t)a.S * 128;
        if (hh < a.H + a.Hkv) {
            for (int idx = tid; idx < MT * 16 * 64; idx += 512) {
                const int m = idx >> 6, i = idx & 63;
                if (m >= a.M) continue;
                const int b = (a.m0 + m) / a.Wn, j = (a.m0 + m) % a.Wn;
                const int pos = a.n_state[b] + j;
                if (pos >= a.S) continue;                       // capacity guard
                const float c = a.cosT[(size_t)pos * 64 + i], s = a.sinT[(size_t)pos * 64 + i];
                const float x0 = ex[(size_t)m * 132 + i], x1 = ex[(size_t)m * 132 + i + 64];
                const float r0 = x0 * c - x1 * s, r1 = x1 * c + x0 * s;
                if (hh < a.H) {
                    float* q = a.out + (size_t)m * a.ldo + hh * 128;
                    q[i] = r0; q[i + 64] = r1;
                } else {
                    bf16_t* kr = a.kc + ((((size_t)a.layer * a.B + b) * a.Hkv + (hh - a.H)) * a.kvp) * plane;
                    const size_t i0 = k_index(pos, i, 128), i1 = k_index(pos, i + 64, 128);
                    const uint32_t h0 = bf16_rne_bits(r0), h1 = bf16_rne_bits(r1);
                    kr[i0] = (bf16_t)h0; kr[i1] = (bf16_t)h1;
                    if (a.kvp == 2) {
                        kr[plane + i0] = (bf16_t)bf16_rne_bits(r0 - bf16_bits_f32(h0));
                        kr[plane + i1] = (bf16_t)bf16_rne_bits(r1 - bf16_bits_f32(h1));
                    }
                }
            }
        } else {
            const int kh = hh - a.H - a.Hkv;
            for (int idx = tid; idx < MT * 16 * 128; idx += 512) {
                const int m = (idx & 15) + 16 * (idx >> 11), e = (idx >> 4) & 127;
                if (m >= a.M) continue;
                const int b = (a.m0 + m) / a.Wn, j = (a.m0 + m) % a.Wn;
                const int pos = a.n_state[b] + j;
                if (pos >= a.S) continue;
                bf16_t* vr = a.vc + ((((size_t)a.layer * a.B + b) * a.Hkv + kh) * a.kvp) * plane + v_index(e, pos, 128);
                const float vv = ex[(size_t)m * 132 + e];
                const uint32_t h0 = bf16_rne_bits(vv);
                vr[0] = (bf16_t)h0;
                if (a.kvp == 2) vr[plane] = (bf16_t)bf16_rne_bits(vv - bf16_bits_f32(h0));
            }
        }
    } else if (EPI == EPI_LMHEAD) {
        float* amv = (float*)smem;              // [8][MT*16]
        int* ami = (int*)(amv + 8 * MT * 16);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = mt * 16 + lm;
            float best = -3.0e38f; int bi = 0x7fffffff;
            if (active) {
                float v[4] = {acc[mt][0] * rs[mt], acc[mt][1] * rs[mt], acc[mt][2] * rs[mt], acc[mt][3] * rs[mt]};
                const int n0 = nt * 16 + 4 * g4;
                if (a.out && m < a.M) *(float4*)(a.out + (size_t)m * a.ldo + n0) = make_float4(v[0], v[1], v[2], v[3]);
#pragma unroll
                for (int r = 0; r < 4; ++r) if (v[r] > best) { best = v[r]; bi = n0 + r; }
            }
#pragma unroll
            for (int o = 16; o <= 32; o <<= 1) {
                float ov = __shfl_xor(best, o, 64); int oi = __shfl_xor(bi, o, 64);
                if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
            }
            if (g4 == 0) { amv[w * MT * 16 + m] = best; ami[w * MT * 16 + m] = bi; }
        }
        __syncthreads();
        if (tid < MT * 16) {
            float best = amv[tid]; int bi = ami[tid];
            for (int q = 1; q < 8; ++q) {
                float ov = amv[q * MT * 16 + tid]; int oi = ami[q * MT * 16 + tid];
                if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
            }
            a.amax_val[(size_t)cg * (MT * 16) + tid] = best;
            a.amax_idx[(size_t)cg * (MT * 16) + tid] = bi;
        }
    }
}

size_t fc_gemm16_lds_bytes(int K, int sk, int MT, int nsplit) {
    const int NU = K >> 8, numax = (NU + sk - 1) / sk;
    size_t act = (size_t)numax * 8 * MT * nsplit * 1024;
    return act + (size_t)9 * MT * 16 * 4 + 64;
}

template <int EPI, int MT>
static hipError_t launch_epi(const Gemm16Args& a, int ncg, hipStream_t st) {
    const size_t lds = fc_gemm16_lds_bytes(a.K, a.sk, MT, 2);
    if (lds > 140 * 1024) return hipErrorInvalidValue;
    static bool raised = false;          // per instantiation: allow dynamic LDS beyond the 64 KB default
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void*)k_gemm16<EPI, MT, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, 140 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    k_gemm16<EPI, MT, 2><<<ncg * a.sk, 512, lds, st>>>(a);
    return hipGetLastError();
}

hipError_t fc_gemm16(int epi, const Gemm16Args& a, int ncg, hipStream_t st) {
    if (a.M < 1 || a.M > 32 || a.sk < 1 || a.sk > FC_MAX_SK || ncg * 8 < a.NT || ncg > FC_MAX_COUNTERS) return hipErrorInvalidValue;
    if (a.K % 256 || a.sk > (a.K >> 8) || ((a.K >> 8) + a.sk - 1) / a.sk > 4) return hipErrorInvalidValue;   // slices of 1..4 units
    const bool two = a.M > 16;
    switch (epi) {
        case EPI_RESID: return two ? launch_epi<EPI_RESID, 2>(a, ncg, st) : launch_epi<EPI_RESID, 1>(a, ncg, st);
        case EPI_SWIGLU: return two ? launch_epi<EPI_SWIGLU, 2>(a, ncg, st) : launch_epi<EPI_SWIGLU, 1>(a, ncg, st);
        case EPI_QKV: return two ? launch_epi<EPI_QKV, 2>(a, ncg, st) : launch_epi<EPI_QKV, 1>(a, ncg, st);
        case EPI_LMHEAD: return two ? launch_epi<EPI_LMHEAD, 2>(a, ncg, st) : launch_epi<EPI_LMHEAD, 1>(a, ncg, st);
    }
    return hipErrorInvalidValue;
}

// reduction of the LM head's per-column-group winners: lowest id on ties
__global__ void k_argmax_final(const float* val, const int32_t* idx, int ncg, int stride, int32_t* ids, float* top) {
    __shared__ float bv[4];
    __shared__ int bi[4];
    const int m = blockIdx.x;
    float best = -3.0e38f; int b = 0x7fffffff;
    for (int c = threadIdx.x; c < ncg; c += blockDim.x) {
        float v = val[(size_t)c * stride + m]; int i = idx[(size_t)c * stride + m];
        if (v > best || (v == best && i < b)) { best = v; b = i; }
    }
    for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(best, o, 64); int oi = __shfl_xor(b, o, 64);
        if (ov > best || (ov == best && oi < b)) { best = ov; b = oi; }
    }
    if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = b; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int q = 1; q < (int)(blockDim.x >> 6); ++q)
            if (bv[q] > best || (bv[q] == best && bi[q] < b)) { best = bv[q]; b = bi[q]; }
        ids[m] = b; top[m] = best;
    }
}
hipError_t fc_argmax_final(const float* val, const int32_t* idx, int ncg, int stride, int M, int32_t* ids, float* top,
                           hipStream_t st) {
    k_argmax_final<<<M, 256, 0, st>>>(val, idx, ncg, stride, ids, top);
    return hipGetLastError();
}
