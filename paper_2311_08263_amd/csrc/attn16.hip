// Window-causal attention on matrix cores (bf16 KV cache, head_dim 128).
//
// The queries of a step are the W window rows of a sequence; the keys are the committed cache
// positions 0..n-1 plus the window positions n..n+W-1, row j seeing positions <= n+j -- the causal
// mask that lets one forward do lossless and Jacobi decoding together (Sec. 4.3, Eq. 2/4).
//
// One workgroup (4 waves) per (sequence, query head, key split); waves take 32-key blocks round
// robin.  Per block the wave computes S^T = K . Q^T with v_mfma_f32_16x16x32_bf16 (K rows as the
// A operand, straight from the cache with 16-byte loads; Q as the B operand, bf16 hi + lo), a
// running-max softmax in fp32, and O^T += V^T . P^T with V^T rows as the A operand (the V cache is
// stored transposed, [Dh][positions], so these are 16-byte loads too) and P^T, which is exactly the
// register layout the score tiles already have, as the B operand.  The two 16-key score tiles of a
// block interleave keys (tile t row r <-> key 8*(r/4) + 4*t + r%4) so that a lane ends with 8
// consecutive keys.  Waves are merged through LDS (each wave finishes a quarter of the head), key
// splits through a scratch buffer by the last workgroup to arrive, always in index order, so results
// do not depend on timing.  How many of the launched splits work on a sequence is decided at run
// time from its length.
#include "attn16.h"
#include "xwg.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2_t;
union Frag { u32x4_t u; bf16x8_t v; };

__device__ inline void split8(const float* v, Frag& hi, Frag& lo) {
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) pk_bf16_hilo(v[2 * e], v[2 * e + 1], h[e], l[e]);
    hi.u = (u32x4_t){h[0], h[1], h[2], h[3]};
    lo.u = (u32x4_t){l[0], l[1], l[2], l[3]};
}

#define NEG_BIG (-1.0e30f)
#define PART_FLOATS (8 * 64 * 4 + 128)   // per (bh, split, qt): O^T tiles, then m[64], l[64] per lane

// the bf16 lo operand of eight cached values kept as bf16 hi (h, four words) + 8-bit residual (two words of bytes):
// value - hi = byte * 2^-15 * 2^(exponent of hi), exact in bf16
__device__ inline void expand_lo8(const u32x4_t& h, uint32_t b0, uint32_t b1, Frag& lo) {
    uint32_t o[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t w = h[p], bw = p < 2 ? b0 : b1;
        // scale of the residual's unit: sign and exponent of hi, times 2^-15 (a hi of zero or below the normal
        // range has exponent field 0: its residual is dropped, an error below 2^-126)
        const float s0 = __uint_as_float((w << 16) & 0xFF800000u) * 3.0517578125e-05f;
        const float s1 = __uint_as_float(w & 0xFF800000u) * 3.0517578125e-05f;
        const float d0 = (float)((bw >> (16 * (p & 1))) & 0xFFu) * s0;
        const float d1 = (float)((bw >> (16 * (p & 1) + 8)) & 0xFFu) * s1;
        o[p] = pk_bf16(d0, d1);
    }
    lo.u = (u32x4_t){o[0], o[1], o[2], o[3]};
}

// KVP: 1 = one bf16 plane, 2 = bf16 hi + bf16 lo planes, 3 = bf16 hi plane + a plane of 8-bit residuals
template <int QT, int KVP>
__global__ __launch_bounds__(256, QT) void k_attn16(AttnArgs a) {
    extern __shared__ float lds[];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int lm = lane & 15, g = lane >> 4;
    // a window of more rows than a workgroup takes (16 per query tile) is cut into sub-windows: sub-window `sub` of a sequence is a
    // unit of its own whose rows see the committed positions plus the window rows up to their own (the
    // K/V of all window rows are already in the cache when this kernel starts)
    constexpr int SUBR = 16 * QT;                            // rows of a unit
    const int nsub = (a.W + SUBR - 1) / SUBR;
    // workgroups go to the eight XCDs (each with an L2 of its own) round robin by index, so with grouped
    // K/V heads consecutive indices take different K/V heads: the query heads that share one then follow
    // each other at a stride of Hkv, land on the same XCD when Hkv is a multiple of eight, and fetch the
    // shared planes from memory once instead of once per query head
    const int bh = blockIdx.x, hr = bh % a.H, G = a.H / a.Hkv, kvh = hr % a.Hkv, h = kvh * G + hr / a.Hkv;
    const int sub = (bh / a.H) % nsub, b = bh / (a.H * nsub);
    const int sp = blockIdx.y, nsp_max = gridDim.y;
    const int Wb = a.rstart ? a.rstart[b + 1] - a.rstart[b] : a.W, rbase = a.rstart ? a.rstart[b] : b * a.W;
    const int row0 = SUBR * sub, Wr = Wb - row0 < SUBR ? Wb - row0 : SUBR;        // rows of this unit
    if (Wr <= 0) return;                                     // a sequence with a smaller window of its own
    const int n = a.n_state[b] + row0;                       // positions every row of the unit sees
    int T = n + Wr;
    if (T > a.S) T = a.S;                                    // capacity guard (the host checks first)
    const int NB = (T + 31) >> 5;
    // splits actually used: about a.bpw key blocks per workgroup (the launch provides nsp_max for the
    // longest context; every workgroup of this (sequence, head) derives the same number from n)
    int nsp = (NB + a.bpw - 1) / a.bpw;
    if (nsp > nsp_max) nsp = nsp_max;
    if (sp >= nsp) return;
    const int blk0 = (int)(((unsigned)sp * (unsigned)NB) / (unsigned)nsp);
    const int blk1 = (int)(((unsigned)(sp + 1) * (unsigned)NB) / (unsigned)nsp);
    const size_t plane = (size_t)a.S * 128;
    constexpr int NPL = KVP == 1 ? 1 : 2;                   // planes of S * 128 elements a block occupies; register sets
    const bf16_t* kbase = a.kc + ((((size_t)a.layer * a.B + b) * a.Hkv + kvh) * NPL) * plane;
    const bf16_t* vbase = a.vc + ((((size_t)a.layer * a.B + b) * a.Hkv + kvh) * NPL) * plane;

    // Q as B operand: lane (row lm, dh 32*g + 8*s + e), hi and lo
    Frag qh[QT][4], ql[QT][4];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        int j = qt * 16 + lm;
        if (j >= Wr) j = Wr - 1;
        const float* qr = a.q + (size_t)(rbase + row0 + j) * a.ldq + h * 128 + 32 * g;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            float4 x0 = *(const float4*)(qr + 8 * s), x1 = *(const float4*)(qr + 8 * s + 4);
            float v[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
            split8(v, qh[qt][s], ql[qt][s]);
        }
    }

    f32x4_t acc[QT][8];
    float mrun[QT], lrun[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        mrun[qt] = NEG_BIG; lrun[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) acc[qt][dt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    }
    const float scale = 0.08838834764831845f;   // 1/sqrt(128)

    // one 32-key block: K tiles and V^T tiles of block `blk` into registers
    struct KV { Frag kf[NPL][2][4], vf[NPL][8]; };
    auto load = [&](KV& r, int blk_want) {
        const int blk = blk_want < NB ? blk_want : NB - 1;       // past the end: a valid block, never used
        Frag (&kf)[NPL][2][4] = r.kf; Frag (&vf)[NPL][8] = r.vf;
        // K tiles (A operand): tile t row r=lm <-> key 32*blk + 8*(lm/4) + 4*t + lm%4 ; dh 32*g + 8*s..
        // (the cache stores each block as these eight fragments, one contiguous kilobyte each; the loads are
        // non-temporal: K and V are read once per step, and letting them allocate in L2 cost 40% at batch 8)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const u32x4_t* kp = (const u32x4_t*)(kbase + (size_t)blk * 4096) + lane;
#pragma unroll
            for (int s = 0; s < 4; ++s) kf[0][t][s].u = __builtin_nontemporal_load(kp + (t * 4 + s) * 64);
            if (KVP == 2) {
                const u32x4_t* kl = (const u32x4_t*)(kbase + plane + (size_t)blk * 4096) + lane;
#pragma unroll
                for (int s = 0; s < 4; ++s) kf[NPL - 1][t][s].u = __builtin_nontemporal_load(kl + (t * 4 + s) * 64);
            } else if (KVP == 3) {      // eight residual bytes per lane and fragment; expanded in compute()
                const u32x2_t* kl = (const u32x2_t*)((const uint8_t*)(kbase + plane) + (size_t)blk * 4096) + lane;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const u32x2_t bw = __builtin_nontemporal_load(kl + (t * 4 + s) * 64);
                    kf[NPL - 1][t][s].u = (u32x4_t){bw[0], bw[1], 0u, 0u};
                }
            }
        }
        // V^T tiles (A operand): row 16*dt + lm, keys kb + 8*g .. +7
        // (stored as eight fragments per block as well)
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            vf[0][dt].u = __builtin_nontemporal_load((const u32x4_t*)(vbase + (size_t)blk * 4096) + dt * 64 + lane);
            if (KVP == 2) vf[NPL - 1][dt].u = __builtin_nontemporal_load((const u32x4_t*)(vbase + plane + (size_t)blk * 4096) + dt * 64 + lane);
            else if (KVP == 3) {
                const u32x2_t bw = __builtin_nontemporal_load((const u32x2_t*)((const uint8_t*)(vbase + plane) + (size_t)blk * 4096) + dt * 64 + lane);
                vf[NPL - 1][dt].u = (u32x4_t){bw[0], bw[1], 0u, 0u};
            }
        }
    };
    auto compute = [&](KV& r, int blk) {
        const int kb = blk << 5;
        if (KVP == 3) {          // the residual bytes become bf16 lo operands
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int s = 0; s < 4; ++s) { const u32x4_t bw = r.kf[NPL - 1][t][s].u; expand_lo8(r.kf[0][t][s].u, bw[0], bw[1], r.kf[NPL - 1][t][s]); }
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) { const u32x4_t bw = r.vf[NPL - 1][dt].u; expand_lo8(r.vf[0][dt].u, bw[0], bw[1], r.vf[NPL - 1][dt]); }
        }
        const Frag (&kf)[NPL][2][4] = r.kf; const Frag (&vf)[NPL][8] = r.vf;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            f32x4_t sc[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                sc[t] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][t][s].v, qh[qt][s].v, sc[t], 0, 0, 0);
                    sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][t][s].v, ql[qt][s].v, sc[t], 0, 0, 0);
                    if (KVP >= 2)   // lo x lo is below fp32 resolution and is dropped
                        sc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[NPL - 1][t][s].v, qh[qt][s].v, sc[t], 0, 0, 0);
                }
            }
            // lane: row j = qt*16 + lm, keys kb + 8*g + e  (e = 4*t + r)
            const int j = qt * 16 + lm;
            const int lastvis = n + (j < Wr ? j : Wr - 1);
            float p[8];
            float bm = NEG_BIG;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int key = kb + 8 * g + e;
                const bool vis = key <= lastvis && key < T;
                p[e] = vis ? sc[e >> 2][e & 3] * scale : NEG_BIG;
                bm = fmaxf(bm, p[e]);
            }
            bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
            bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
            const float mnew = fmaxf(mrun[qt], bm);
            const float alpha = expf(mrun[qt] - mnew);
            float ps = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int key = kb + 8 * g + e;
                const bool vis = key <= lastvis && key < T;
                p[e] = vis ? expf(p[e] - mnew) : 0.f;
                ps += p[e];
            }
            mrun[qt] = mnew;
            lrun[qt] = lrun[qt] * alpha + ps;
            Frag ph, pl;
            split8(p, ph, pl);
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                acc[qt][dt] *= alpha;
                acc[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[0][dt].v, ph.v, acc[qt][dt], 0, 0, 0);
                acc[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[0][dt].v, pl.v, acc[qt][dt], 0, 0, 0);
                if (KVP >= 2)
                    acc[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[NPL - 1][dt].v, ph.v, acc[qt][dt], 0, 0, 0);
            }
        }
    };
    // two register sets: the next block of this wave travels while the current one is used.  With one
    // query tile there are registers to spare and the scheduler is told to keep all loads of the next
    // block ahead of the current block's arithmetic; with two tiles the compiler is left to reuse each
    // register as soon as it is free (two workgroups share a CU instead).
    {
        KV ra, rb;
        int blk = blk0 + wv;
        if (blk < blk1) {
            load(ra, blk);
            for (;;) {
                load(rb, blk + 4);
                if (QT == 1) __builtin_amdgcn_sched_barrier(0);
                compute(ra, blk);
                blk += 4;
                if (blk >= blk1) break;
                load(ra, blk + 4);
                if (QT == 1) __builtin_amdgcn_sched_barrier(0);
                compute(rb, blk);
                blk += 4;
                if (blk >= blk1) break;
            }
        }
    }
    // row sums over the 4 lanes of a row
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        lrun[qt] += __shfl_xor(lrun[qt], 16, 64);
        lrun[qt] += __shfl_xor(lrun[qt], 32, 64);
    }

    // ---- merge the 4 waves: everyone publishes to LDS, then wave w finishes output tiles 2w and 2w+1
    // (16 head elements each) over the four partials, in wave order
    {
        float* dst = lds + (size_t)wv * QT * PART_FLOATS;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) *(f32x4_t*)(dst + qt * PART_FLOATS + (dt * 64 + lane) * 4) = acc[qt][dt];
            dst[qt * PART_FLOATS + 2048 + lane] = mrun[qt];
            dst[qt * PART_FLOATS + 2112 + lane] = lrun[qt];
        }
    }
    __syncthreads();
    f32x4_t o2[QT][2];
    float mw[QT], lw[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        float mv[4], m = NEG_BIG;
#pragma unroll
        for (int v = 0; v < 4; ++v) { mv[v] = lds[(size_t)(v * QT + qt) * PART_FLOATS + 2048 + lane]; m = fmaxf(m, mv[v]); }
        float l = 0.f;
        o2[qt][0] = o2[qt][1] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float* src = lds + (size_t)(v * QT + qt) * PART_FLOATS;
            const float wgt = expf(mv[v] - m);
            l += src[2112 + lane] * wgt;
#pragma unroll
            for (int t = 0; t < 2; ++t) o2[qt][t] += *(const f32x4_t*)(src + ((2 * wv + t) * 64 + lane) * 4) * wgt;
        }
        mw[qt] = m; lw[qt] = l;
    }

    if (nsp > 1) {
        // ---- key splits: partial tiles go to memory with agent-scope stores; the last workgroup to
        // arrive reads all of them back -- every load of the merge is in flight at once (each wave its
        // two tiles of every split), splits folded in index order
        float* mine = a.part + ((size_t)bh * nsp_max + sp) * QT * PART_FLOATS;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                float* dst = mine + qt * PART_FLOATS + ((2 * wv + t) * 64 + lane) * 4;
                st_agent_f32x2(dst, o2[qt][t][0], o2[qt][t][1]);
                st_agent_f32x2(dst + 2, o2[qt][t][2], o2[qt][t][3]);
            }
            if (wv == 0) {
                st_agent_f32(mine + qt * PART_FLOATS + 2048 + lane, mw[qt]);
                st_agent_f32(mine + qt * PART_FLOATS + 2112 + lane, lw[qt]);
            }
        }
        wait_vmem_done();
        __syncthreads();                                   // all four waves' stores have completed
        int* flag = (int*)(lds + 4 * QT * PART_FLOATS);
        if (tid == 0) *flag = arrive_agent(a.cnt + bh);
        __syncthreads();
        if (*flag != nsp - 1) return;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            float m = NEG_BIG, l = 0.f;
            o2[qt][0] = o2[qt][1] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
            for (int s0 = 0; s0 < nsp; s0 += 8) {          // eight splits' loads in flight at a time
                float ms[8], ls[8];
                f32x4_t os[8][2];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int s2 = s0 + u < nsp ? s0 + u : nsp - 1;
                    const float* src = a.part + ((size_t)bh * nsp_max + s2) * QT * PART_FLOATS + qt * PART_FLOATS;
                    ms[u] = ld_agent_f32(src + 2048 + lane);
                    ls[u] = ld_agent_f32(src + 2112 + lane);
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const float* p4 = src + ((2 * wv + t) * 64 + lane) * 4;
                        float v0, v1, v2, v3;
                        ld_agent_f32x2(p4, v0, v1);
                        ld_agent_f32x2(p4 + 2, v2, v3);
                        os[u][t] = (f32x4_t){v0, v1, v2, v3};
                    }
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const bool valid = s0 + u < nsp;
                    const float mu = valid ? ms[u] : NEG_BIG;
                    const float mnew = fmaxf(m, mu);
                    const float wa = expf(m - mnew), wb = valid ? expf(mu - mnew) : 0.f;
                    l = l * wa + ls[u] * wb;
                    o2[qt][0] = o2[qt][0] * wa + os[u][0] * wb;
                    o2[qt][1] = o2[qt][1] * wa + os[u][1] * wb;
                    m = mnew;
                }
            }
            lw[qt] = l;
        }
        if (tid == 0) st_agent_i32(a.cnt + bh, 0);
    }
    // out[row][h*128 + 16*dt + 4*g + r] = O / l, this wave's tiles dt = 2*wv, 2*wv + 1
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int j = qt * 16 + lm;
        if (j < Wr) {
            const float inv = 1.0f / lw[qt];
            const int row = rbase + row0 + j;
            if (a.out) {
                float* o = a.out + (size_t)row * a.ldo + h * 128 + 4 * g;
#pragma unroll
                for (int t = 0; t < 2; ++t) *(f32x4_t*)(o + 16 * (2 * wv + t)) = o2[qt][t] * inv;
            }
            if (a.ofrag) {
                // head elements 32 * wv + 16 * t + 4 * g + r: k-tile 4 * h + wv, octet 2 * t + g / 2, elements 4 * (g % 2) + r
                const size_t KTo = (size_t)a.H * 4;
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const f32x4_t v = o2[qt][t] * inv;
                    uint32_t h0, l0, h1, l1;
                    pk_bf16_hilo(v[0], v[1], h0, l0);
                    pk_bf16_hilo(v[2], v[3], h1, l1);
                    char* dst = (char*)a.ofrag + ((((size_t)(row >> 4) * KTo + 4 * h + wv) * 2) * 64 + (row & 15) + 16 * (2 * t + (g >> 1))) * 16 + 8 * (g & 1);
                    *(uint2*)dst = make_uint2(h0, h1);
                    *(uint2*)(dst + 1024) = make_uint2(l0, l1);
                }
            }
        }
    }
}

size_t fc_attn16_part_bytes(int BH, int nsplit, int W) {      // covers both unit sizes
    const int tiles = W > 16 ? 2 * ((W + 31) / 32) : 1;
    return (size_t)BH * tiles * nsplit * PART_FLOATS * 4;
}

hipError_t fc_attn16(const AttnArgs& a, int Bact, int nsplit, hipStream_t st) {
    const int QT = a.W > 16 && a.subrows != 16 ? 2 : 1, nsub = (a.W + 16 * QT - 1) / (16 * QT);
    if (a.W < 1 || nsplit < 1 || nsplit > FC_MAX_ATTN_SPLITS || Bact * nsub * a.H > FC_MAX_COUNTERS || a.S < 32 || a.S % 32 || a.bpw < 1)
        return hipErrorInvalidValue;
    dim3 grid(Bact * nsub * a.H, nsplit);
    const size_t l1 = (size_t)4 * PART_FLOATS * 4 + 16, l2 = (size_t)8 * PART_FLOATS * 4 + 16;
    static bool lds_ok = false;                          // two query tiles need more than the default 64 KB
    if (!lds_ok) {
        hipError_t e = hipFuncSetAttribute((const void*)k_attn16<2, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)l2);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_attn16<2, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)l2);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_attn16<2, 3>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)l2);
        if (e != hipSuccess) return e;
        lds_ok = true;
    }
    if (a.kvp == 2) {
        if (QT == 2) k_attn16<2, 2><<<grid, 256, l2, st>>>(a);
        else k_attn16<1, 2><<<grid, 256, l1, st>>>(a);
    } else if (a.kvp == 1) {
        if (QT == 2) k_attn16<2, 1><<<grid, 256, l2, st>>>(a);
        else k_attn16<1, 1><<<grid, 256, l1, st>>>(a);
    } else if (a.kvp == 3) {
        if (QT == 2) k_attn16<2, 3><<<grid, 256, l2, st>>>(a);
        else k_attn16<1, 3><<<grid, 256, l1, st>>>(a);
    } else return hipErrorInvalidValue;
    return hipGetLastError();
}
