// bf16 GEMM for steps with many rows (batch x window up to a few hundred): out = act . W with the
// weights in MFMA fragment order and the activations pre-split into bf16 hi + lo fragments.
//
// At 256 rows the step is no longer a pure weight stream: 2 x 256 x params x 2 (hi, lo) flops per
// step put it on the matrix-core side of the ridge.  Tiling: a workgroup of 4 waves computes 64
// rows x 256 columns; wave w owns 4 n-tiles (64 columns) for all 4 row tiles (16 accumulator
// tiles), so every activation fragment read from LDS feeds 4 MFMAs and every weight fragment (read
// straight from global memory, 4 k-tiles ahead) feeds 8.  Activation fragments of 4 k-tiles at a
// time are copied global -> LDS by the whole workgroup, double buffered (2 x 32 KB), one barrier per
// stage.  The four workgroups of a column block re-read the same weights: HBM sees them once, the
// repeats come from L2.  What bounds the kernel at 256 rows (measured with per-workgroup time stamps at the
// 13B gate/up shape): MFMA issue at 21-23 cycles per MFMA instead of 16 plus the L2 -> CU load path (96 KB per
// workgroup and stage; with most loads removed the loop is a quarter faster).  A workgroup alone on a CU runs
// its 40 stages in 70 us, two on a CU finish after 86 and 118 us (the arbiter favours the older waves).  Not the
// bound: LDS read latency (software-pipelined reads changed nothing), MFMA busy is 38 %, no bank conflicts.
// Variants that were slower: 128-row tiles with both operands staged through LDS (gate/up 170 us against
// 156 us) and 8 x 2 tiles per wave (182 us).  Workgroup ids are mapped so that the row blocks of one column block run on
// the same XCD (ids that are equal mod 8 share an XCD and its L2), back to back.  Matrices with few
// columns (O and down projections) are also split along K so that the launch fills the chip; the
// slices store partial tiles and k_resid_reduce adds them to the residual stream in slice order.
//
// k_split prepares the activations: optional RMSNorm (row statistics in fp32, gain applied), then
// bf16 hi + lo, stored in B-fragment order [row tile][k-tile][hi|lo][lane][8].
#include "gemm256.h"
#include "gemmco.h"      // fc_num_cus

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
union Frag { u32x4_t u; bf16x8_t v; };

__device__ inline uint32_t rne16(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ inline float up16(uint32_t b) { return __uint_as_float(b << 16); }

// ------------------------------------------------------------------ activation split (+ RMSNorm)
// grid (row tiles of 16 rows, K chunks); X [M][K] fp32 -> AF [MT][KT][2][64][8] bf16.  With a gain every
// workgroup computes the statistics of its 16 rows over the whole row (the rows sit in L2) and then
// converts its own K chunk.
__global__ __launch_bounds__(512) void k_split(const float* X, int ldx, int M, int K, const float* gain, float eps,
                                               bf16_t* AF) {
    __shared__ float red[8][16];
    __shared__ float rs[16];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int lm = lane & 15, g4 = lane >> 4;
    const int mt = blockIdx.x, KT = K >> 5;
    const int kt_lo = (int)((unsigned)KT * blockIdx.y / gridDim.y), kt_hi = (int)((unsigned)KT * (blockIdx.y + 1) / gridDim.y);
    const int row = mt * 16 + lm < M ? mt * 16 + lm : M - 1;
    const float* xr = X + (size_t)row * ldx + 8 * g4;
    float scale = 1.0f;
    if (gain) {
        float ss = 0.f;
        for (int kt = w; kt < KT; kt += 8) {
            const float4 a = *(const float4*)(xr + kt * 32), b = *(const float4*)(xr + kt * 32 + 4);
            ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w + b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
        }
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        if (g4 == 0) red[w][lm] = ss;
        __syncthreads();
        if (tid < 16) {
            float s = 0.f;
            for (int q = 0; q < 8; ++q) s += red[q][tid];
            rs[tid] = 1.0f / sqrtf(s / (float)K + eps);
        }
        __syncthreads();
        scale = rs[lm];
    }
    u32x4_t* dst = (u32x4_t*)AF + (size_t)mt * KT * 2 * 64 + lane;
    for (int kt = kt_lo + w; kt < kt_hi; kt += 8) {
        const float4 a = *(const float4*)(xr + kt * 32), b = *(const float4*)(xr + kt * 32 + 4);
        float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        if (gain) {
            const float4 g0 = *(const float4*)(gain + kt * 32 + 8 * g4), g1 = *(const float4*)(gain + kt * 32 + 8 * g4 + 4);
            const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = v[e] * scale * g[e];
        }
        uint32_t h[4], l[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) pk_bf16_hilo(v[2 * e], v[2 * e + 1], h[e], l[e]);
        dst[(size_t)kt * 128] = (u32x4_t){h[0], h[1], h[2], h[3]};
        dst[(size_t)kt * 128 + 64] = (u32x4_t){l[0], l[1], l[2], l[3]};
    }
}

hipError_t fc_split(const float* X, int ldx, int M, int K, const float* gain, float eps, bf16_t* AF, hipStream_t st) {
    if (M < 1 || K % 256) return hipErrorInvalidValue;
    const int MT = (M + 15) / 16;
    int kc = (512 + MT - 1) / MT;                       // about 512 workgroups, at least 8 k-tiles each
    if (kc > K / 256) kc = K / 256;
    k_split<<<dim3(MT, kc), 512, 0, st>>>(X, ldx, M, K, gain, eps, AF);
    return hipGetLastError();
}

// ------------------------------------------------------------------ the GEMM
// CW = n-tiles per wave: 4 (tiles of 64 rows x 256 columns) where that gives the chip enough workgroups,
// 2 or 1 (64 x 128, 64 x 64) for few rows x few columns, where the GEMM is still a weight stream and needs
// the workgroups more than the reuse.
// KG = 2: eight waves per workgroup, two groups of four that take the even and the odd k-tiles of every stage
// (each wave still its 4 x CW tiles) and add their accumulators through LDS at the end.  One such workgroup per
// CU does what two four-wave workgroups of different tiles would, with one activation stage for both groups;
// used where the launch has no more workgroups than CUs anyway.
// KG = 3: eight waves per workgroup, two groups of four that take neighbouring column blocks (a tile of 64 rows x
// 128 * CW columns) and share the activation stage; used where that brings the launch down to one workgroup per
// CU (with four waves two workgroups would share a CU, each staging the same activations).
template <int EPI, int CW, int KG>
__global__ __launch_bounds__(KG == 1 ? 256 : 512, KG == 1 ? 2 : 1) void k_gemm256(Gemm256Args a) {
    __shared__ u32x4_t stage[2][4][4][2][64];           // [buffer][k-tile][row tile][hi|lo][lane]: 2 x 32 KB
    constexpr bool KSPLIT = KG == 2, CSPLIT = KG == 3;
    constexpr int NWV = KG == 1 ? 4 : 8;                 // waves
    __shared__ float rowpart[NWV][64];
    constexpr int NTH = 64 * NWV, SL = 32 / NWV;         // threads, 16-byte stage loads per thread
    const int tid = threadIdx.x, lane = tid & 63, w = (tid >> 6) & 3, kg = tid >> 8, w8 = tid >> 6;
    const int lm = lane & 15, g4 = lane >> 4;
    const int KT = a.K >> 5, NS = KT >> 2, MT = (a.M + 15) >> 4;
    // id -> (XCD x, sequence number q on that XCD) -> row block q % nrb of unit 8 * (q / nrb) + x
    constexpr int WCOLS = CSPLIT ? 8 * CW : 4 * CW;      // n-tiles per workgroup
    const int nrb = (MT + 3) >> 2, ncb = (a.NT + WCOLS - 1) / WCOLS;
    const int xq = blockIdx.x >> 3, unit = (xq / nrb) * 8 + (blockIdx.x & 7), rb = xq % nrb;
    if (unit >= ncb * a.sk) return;                      // grid padding (whole workgroup leaves together)
    const int cb = unit / a.sk, ks = unit % a.sk;
    const int s_lo = (int)((unsigned)NS * (unsigned)ks / (unsigned)a.sk), s_hi = (int)((unsigned)NS * (unsigned)(ks + 1) / (unsigned)a.sk);
    const int nt0 = cb * WCOLS + CW * (CSPLIT ? w8 : w);      // this wave's CW n-tiles
    const int mt0 = rb * 4;
    // QKV: the cache positions of this wave's rows (a dependent load of the sequence length) are fetched here,
    // a whole K loop ahead of the epilogue that needs them
    int qpos[4], qb[4];
    if (EPI == EPI_QKV) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int row = (mt0 + m) * 16 + lm;
            const bool rok = (!KSPLIT || kg == (m >> 1)) && mt0 + m < MT && row < a.M;
            qb[m] = rok ? (a.rm.rowb ? a.rm.rowb[row] : row / a.Wn) : 0;
            qpos[m] = rok ? a.n_state[qb[m]] + (a.rm.rowb ? a.rm.rowj[row] : row % a.Wn) : a.S;
        }
    }

    // stage copy: 32 fragments of 1 KB per stage, 8 x 16 bytes per thread.  Addresses are a uniform 64-bit base
    // (scalar registers, advanced per stage) plus a per-thread 32-bit byte offset fixed for the whole kernel:
    // no 64-bit vector arithmetic in the loop.
    const char* AFb = (const char*)a.AF;
    uint32_t aoff[SL];
#pragma unroll
    for (int i = 0; i < SL; ++i) {
        const int idx = tid + NTH * i, f = idx >> 6, ln = idx & 63;
        const int ktl = f >> 3, mtl = (f >> 1) & 3, part = f & 1;
        const int mt = mt0 + mtl < MT ? mt0 + mtl : MT - 1;
        aoff[i] = ((((uint32_t)mt * KT + ktl) * 2 + part) * 64 + ln) * 16;
    }
    auto stage_load = [&](u32x4_t (&r)[SL], int s) {
        const char* base = AFb + (size_t)s * 8192;            // 4 k-tiles x (hi, lo) x 1 KB
#pragma unroll
        for (int i = 0; i < SL; ++i) r[i] = *(const u32x4_t*)(base + aoff[i]);
    };
    auto stage_store = [&](const u32x4_t (&r)[SL], int buf) {
#pragma unroll
        for (int i = 0; i < SL; ++i) {
            const int idx = tid + NTH * i, f = idx >> 6, ln = idx & 63;
            stage[buf][f >> 3][(f >> 1) & 3][f & 1][ln] = r[i];
        }
    };
    const char* Wb = (const char*)a.W;
    uint32_t woff[CW];
#pragma unroll
    for (int j = 0; j < CW; ++j) {
        const int nt = nt0 + j < a.NT ? nt0 + j : a.NT - 1;
        woff[j] = ((uint32_t)nt * KT * 64 + lane) * 16;
    }
    auto wload = [&](u32x4_t (&wt)[CW], int kt) {
        const int kc = kt < KT ? kt : KT - 1;                 // past the end: re-read the last k-tile (never used)
        const char* base = Wb + (size_t)kc * 1024;
#pragma unroll
        for (int j = 0; j < CW; ++j) wt[j] = *(const u32x4_t*)(base + woff[j]);   // plain loads: the row blocks of a column block share these lines in L2
    };

    f32x4_t acc[CW][4];
#pragma unroll
    for (int j = 0; j < CW; ++j)
#pragma unroll
        for (int m = 0; m < 4; ++m) acc[j][m] = (f32x4_t){0.f, 0.f, 0.f, 0.f};

    u32x4_t sr[SL];
    u32x4_t W0[CW], W1[CW], W2[CW], W3[CW];              // KG = 2: W0, W1 hold k-tiles kg and kg + 2 of a stage
    stage_load(sr, s_lo);
    if (!KSPLIT) { wload(W0, 4 * s_lo); wload(W1, 4 * s_lo + 1); wload(W2, 4 * s_lo + 2); wload(W3, 4 * s_lo + 3); }
    else { wload(W0, 4 * s_lo + kg); wload(W1, 4 * s_lo + kg + 2); }
    stage_store(sr, 0);
    if (a.ssq) {
        // row statistics of the 64 rows (activations that come without their norm scale): wave w adds every
        // fourth partial sum, all its loads in flight together; the epilogue adds the four
        const int MP = MT * 16;
        const int row = mt0 * 16 + lane < MP ? mt0 * 16 + lane : MP - 1;
        float ssum = 0.f;
#pragma unroll 8
        for (int c = w8; c < a.nssq; c += NWV) ssum += a.ssq[(size_t)c * MP + row];
        rowpart[w8][lane] = ssum;
    }
    __syncthreads();

#define STEP(WSET, U)                                                                               \
    do {                                                                                            \
        Frag ah[4], al[4];                                                                          \
        _Pragma("unroll") for (int m = 0; m < 4; ++m) { ah[m].u = stage[buf][U][m][0][lane]; al[m].u = stage[buf][U][m][1][lane]; } \
        _Pragma("unroll") for (int j = 0; j < CW; ++j) {                                            \
            Frag wf; wf.u = WSET[j];                                                                \
            _Pragma("unroll") for (int m = 0; m < 4; ++m) {                                         \
                acc[j][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf.v, ah[m].v, acc[j][m], 0, 0, 0); \
                acc[j][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf.v, al[m].v, acc[j][m], 0, 0, 0); \
            }                                                                                       \
        }                                                                                           \
        wload(WSET, 4 * s + U + 4);                                                                 \
        __builtin_amdgcn_sched_barrier(0);   /* keep these loads here: four k-tiles ahead of their use */ \
    } while (0)

    int buf = 0;
    for (int s = s_lo; s < s_hi; ++s) {
        stage_load(sr, s + 1 < s_hi ? s + 1 : s);        // next stage's activations travel while this one is used
        __builtin_amdgcn_sched_barrier(0);               // (left alone the scheduler sinks all loads to the end of the stage)
        if (!KSPLIT) {
            STEP(W0, 0);
            STEP(W1, 1);
            STEP(W2, 2);
            STEP(W3, 3);
        } else {
            STEP(W0, kg);
            STEP(W1, kg + 2);
        }
        stage_store(sr, buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
#undef STEP

    if (KSPLIT) {
        // the two k-groups meet: each publishes the half of its accumulators that the other group will finish
        // (group 0 keeps row tiles 0 and 1, group 1 row tiles 2 and 3: 8 KB per wave, the stage buffers are free
        // after the loop's last barrier), adds what it receives and runs the epilogue for its own half
        f32x4_t* red = (f32x4_t*)&stage[0][0][0][0][0];
#pragma unroll
        for (int j = 0; j < CW; ++j)
#pragma unroll
            for (int mm = 0; mm < 2; ++mm) red[((w8 * 4 + j) * 2 + mm) * 64 + lane] = kg == 1 ? acc[j][mm] : acc[j][2 + mm];
        __syncthreads();
        const int pw = kg == 0 ? w + 4 : w;             // the wave of the other group with the same n-tiles
#pragma unroll
        for (int j = 0; j < CW; ++j)
#pragma unroll
            for (int mm = 0; mm < 2; ++mm) {
                const f32x4_t o = red[((pw * 4 + j) * 2 + mm) * 64 + lane];
                if (kg == 0) acc[j][mm] += o; else acc[j][2 + mm] += o;
            }
        __syncthreads();
    }
    // ---- epilogue: acc[j][m]: rows (mt0 + m) * 16 + lm, columns (nt0 + j) * 16 + 4 * g4 + r
    float best[4]; int bidx[4];
    float rscale[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        best[m] = -3.0e38f; bidx[m] = 0x7fffffff;
        rscale[m] = 1.0f;
        if (EPI != EPI_RESID && a.ssq) {
            const int r = m * 16 + lm;
            float ssum = 0.f;
#pragma unroll
            for (int q = 0; q < NWV; ++q) ssum += rowpart[q][r];
            rscale[m] = 1.0f / sqrtf(ssum / (float)a.K + a.eps);
        }
    }
    // QKV: positions and rotary factors are requested a row tile ahead of their use, in front of the stores of
    // the tile before (a load behind a store that might alias it is not moved up by the compiler, and sixteen
    // tiles each waiting for their own factors cost sixteen round trips)
    f32x4_t qc[2][CW], qs[2][CW];
    auto qfactors = [&](int m, f32x4_t (&c)[CW], f32x4_t (&sn)[CW]) {
#pragma unroll
        for (int j = 0; j < CW; ++j) {
            const int nt = nt0 + j, hh = nt >> 3, t = nt & 7;
            c[j] = (f32x4_t){1.0f, 1.0f, 1.0f, 1.0f};
            sn[j] = (f32x4_t){0.0f, 0.0f, 0.0f, 0.0f};
            if (qpos[m] < a.S && nt < a.NT && hh < a.H + a.Hkv) {
                c[j] = *(const f32x4_t*)(a.cosT + (size_t)qpos[m] * 64 + 8 * t + 4 * (g4 & 1));
                sn[j] = *(const f32x4_t*)(a.sinT + (size_t)qpos[m] * 64 + 8 * t + 4 * (g4 & 1));
            }
        }
    };
    if (EPI == EPI_QKV) qfactors(0, qc[0], qs[0]);
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int row = (mt0 + m) * 16 + lm;
        const bool rok = (!KSPLIT || kg == (m >> 1)) && mt0 + m < MT && row < a.M;
        if (EPI == EPI_QKV && m + 1 < 4) qfactors(m + 1, qc[(m + 1) & 1], qs[(m + 1) & 1]);
#pragma unroll
        for (int j = 0; j < CW; ++j) {
            const int nt = nt0 + j;
            const bool ok = rok && nt < a.NT;
            f32x4_t v = acc[j][m];
            if (EPI != EPI_RESID && a.ssq) v *= rscale[m];
            if (EPI == EPI_RESID) {
                if (ok) {
                    if (a.sk > 1) *(f32x4_t*)(a.part + ((size_t)ks * a.M + row) * (a.NT * 16) + nt * 16 + 4 * g4) = v;
                    else {
                        f32x4_t* o = (f32x4_t*)(a.out + (size_t)row * a.ldo + nt * 16 + 4 * g4);
                        *o = *o + v;
                    }
                }
            } else if (EPI == EPI_SWIGLU) {
                f32x4_t h;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float other = __shfl_xor(v[r], 32, 64);
                    h[r] = v[r] / (1.0f + expf(-v[r])) * other;
                }
                if (ok && g4 < 2) {
                    if (a.out) *(f32x4_t*)(a.out + (size_t)row * a.ldo + nt * 8 + 4 * g4) = h;
                    if (a.hfrag) {
                        // features 8 * nt + 4 * g4 + r of row `row`: k-tile nt / 4, octet nt % 4, elements 4 * g4 + r
                        uint32_t h0, l0, h1, l1;
                        pk_bf16_hilo(h[0], h[1], h0, l0);
                        pk_bf16_hilo(h[2], h[3], h1, l1);
                        const size_t KTh = (size_t)(a.ldo >> 5);
                        char* dst = (char*)a.hfrag + ((((size_t)(mt0 + m) * KTh + (nt >> 2)) * 2) * 64 + lm + 16 * (nt & 3)) * 16 + 8 * g4;
                        *(uint2*)dst = make_uint2(h0, h1);
                        *(uint2*)(dst + 1024) = make_uint2(l0, l1);
                    }
                }
            } else if (EPI == EPI_QKV) {
                const int hh = nt >> 3, t = nt & 7;
                const int b = qb[m], pos = qpos[m];
                const bool pk = ok && pos < a.S;                 // capacity guard
                const size_t plane = (size_t)a.S * 128;
                if (hh < a.H + a.Hkv) {
                    const int i0 = 8 * t + 4 * (g4 & 1);
                    f32x4_t rr;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float other = __shfl_xor(v[e], 32, 64);
                        const float c = qc[m & 1][j][e], s = qs[m & 1][j][e];
                        rr[e] = g4 < 2 ? v[e] * c - other * s : v[e] * c + other * s;
                        if (hh >= a.H) rr[e] = kv_round(rr[e], a.kvq & 15);
                    }
                    const int el = (g4 < 2 ? 0 : 64) + i0;
                    if (pk) {
                        if (hh < a.H) *(f32x4_t*)(a.out + (size_t)row * a.ldo + hh * 128 + el) = rr;
                        else {
                            bf16_t* kb = a.kc + ((((size_t)a.layer * a.B + b) * a.Hkv + (hh - a.H)) * kv_alloc_planes(a.kvp)) * plane;
                            const size_t ki = k_index(pos, el, 128);
                            bf16_t* kr = kb + ki;
                            uint32_t h[4];
                            if (a.kvp == 3) {
                                uint32_t l[4];
#pragma unroll
                                for (int e = 0; e < 4; ++e) kv24_split(rr[e], h[e], l[e]);
                                *(uint2*)kr = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                                *(uint32_t*)((uint8_t*)(kb + plane) + ki) = l[0] | (l[1] << 8) | (l[2] << 16) | (l[3] << 24);
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; ++e) h[e] = rne16(rr[e]);
                                *(uint2*)kr = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                                if (a.kvp == 2) {
                                    uint32_t l[4];
#pragma unroll
                                    for (int e = 0; e < 4; ++e) l[e] = rne16(rr[e] - up16(h[e]));
                                    *(uint2*)(kr + plane) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
                                }
                            }
                        }
                    }
                } else if (pk) {
                    const int kh = hh - a.H - a.Hkv;
                    bf16_t* vb = a.vc + ((((size_t)a.layer * a.B + b) * a.Hkv + kh) * kv_alloc_planes(a.kvp)) * plane;
                    const size_t vi = v_index(16 * t + 4 * g4, pos, 128);
                    bf16_t* vr = vb + vi;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float vq = kv_round(v[e], a.kvq >> 4);
                        if (a.kvp == 3) {
                            uint32_t h0, l0; kv24_split(vq, h0, l0);
                            vr[e * 8] = (bf16_t)h0;
                            ((uint8_t*)(vb + plane))[vi + e * 8] = (uint8_t)l0;
                        } else {
                            const uint32_t h0 = rne16(vq);
                            vr[e * 8] = (bf16_t)h0;
                            if (a.kvp == 2) vr[e * 8 + plane] = (bf16_t)rne16(vq - up16(h0));
                        }
                    }
                }
            } else if (EPI == EPI_LMHEAD) {
                const int n0 = nt * 16 + 4 * g4;
                if (ok && a.out) *(f32x4_t*)(a.out + (size_t)row * a.ldo + n0) = v;
                if (nt < a.NT) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) if (v[r] > best[m]) { best[m] = v[r]; bidx[m] = n0 + r; }
                }
            }
        }
    }
    if (EPI == EPI_LMHEAD) {
        // winner per row over this workgroup's 256 columns: lanes of a row, then the 4 waves (the
        // stage buffers are free after the last barrier of the main loop)
        float (*amv)[64] = (float (*)[64])&stage[0][0][0][0][0];
        int (*ami)[64] = (int (*)[64])&stage[1][0][0][0][0];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
#pragma unroll
            for (int o = 16; o <= 32; o <<= 1) {
                const float ov = __shfl_xor(best[m], o, 64); const int oi = __shfl_xor(bidx[m], o, 64);
                if (ov > best[m] || (ov == best[m] && oi < bidx[m])) { best[m] = ov; bidx[m] = oi; }
            }
            if (g4 == 0 && (!KSPLIT || kg == (m >> 1))) { amv[CSPLIT ? w8 : w][m * 16 + lm] = best[m]; ami[CSPLIT ? w8 : w][m * 16 + lm] = bidx[m]; }
        }
        __syncthreads();
        if (tid < 64) {
            float bv = amv[0][tid]; int bx = ami[0][tid];
            for (int q = 1; q < (CSPLIT ? 8 : 4); ++q)
                if (amv[q][tid] > bv || (amv[q][tid] == bv && ami[q][tid] < bx)) { bv = amv[q][tid]; bx = ami[q][tid]; }
            const int row = mt0 * 16 + tid;
            if (row < a.M) {
                a.amax_val[(size_t)cb * a.amax_stride + row] = bv;
                a.amax_idx[(size_t)cb * a.amax_stride + row] = bx;
            }
        }
    }
}

// out[m][n] += part[0][m][n] + part[1][m][n] + ... (slice order: the result does not depend on timing)
__global__ __launch_bounds__(256) void k_resid_reduce(const float* part, int sk, int M, int N, float* out, int ldo) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, n4 = N >> 2;
    if (i >= (size_t)M * n4) return;
    const int m = (int)(i / n4), c = (int)(i % n4) * 4;
    f32x4_t s = *(const f32x4_t*)(part + (size_t)m * N + c);
    for (int k = 1; k < sk; ++k) s = s + *(const f32x4_t*)(part + ((size_t)k * M + m) * N + c);
    f32x4_t* o = (f32x4_t*)(out + (size_t)m * ldo + c);
    *o = *o + s;
}

// The same sum, and in the same pass the input of the next GEMM: the new residual rows times the next norm's
// gain as bf16 hi + lo B-fragments, plus partial row sums of squares (the consumer applies the norm's row scale
// in its epilogue).  grid (row tiles, N / 256); wave w of a workgroup converts k-tile 8 * blockIdx.y + w; lane
// (row lm, octet g4) as in the fragment.  Rows past M of the last row tile are not written.
__global__ __launch_bounds__(512) void k_resid_reduce_split(const float* part, int sk, int M, int N, float* out, int ldo,
                                                            const float* gain, bf16_t* AF, float* ssq) {
    __shared__ float red[8][16];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int lm = lane & 15, g4 = lane >> 4;
    const int mt = blockIdx.x, KT = N >> 5, kt = blockIdx.y * 8 + w, MP = gridDim.x * 16;
    const int m = mt * 16 + lm, c = kt * 32 + 8 * g4;
    float ss = 0.f;
    if (m < M) {
        f32x4_t s0 = *(const f32x4_t*)(part + (size_t)m * N + c), s1 = *(const f32x4_t*)(part + (size_t)m * N + c + 4);
        for (int k = 1; k < sk; ++k) {
            s0 = s0 + *(const f32x4_t*)(part + ((size_t)k * M + m) * N + c);
            s1 = s1 + *(const f32x4_t*)(part + ((size_t)k * M + m) * N + c + 4);
        }
        f32x4_t* o = (f32x4_t*)(out + (size_t)m * ldo + c);
        const f32x4_t x0 = o[0] + s0, x1 = o[1] + s1;
        o[0] = x0; o[1] = x1;
        const f32x4_t g0 = *(const f32x4_t*)(gain + c), g1 = *(const f32x4_t*)(gain + c + 4);
        uint32_t h[4], l[4];
        pk_bf16_hilo(x0[0] * g0[0], x0[1] * g0[1], h[0], l[0]);
        pk_bf16_hilo(x0[2] * g0[2], x0[3] * g0[3], h[1], l[1]);
        pk_bf16_hilo(x1[0] * g1[0], x1[1] * g1[1], h[2], l[2]);
        pk_bf16_hilo(x1[2] * g1[2], x1[3] * g1[3], h[3], l[3]);
        u32x4_t* dst = (u32x4_t*)AF + (((size_t)mt * KT + kt) * 2) * 64 + lane;
        dst[0] = (u32x4_t){h[0], h[1], h[2], h[3]};
        dst[64] = (u32x4_t){l[0], l[1], l[2], l[3]};
#pragma unroll
        for (int e = 0; e < 4; ++e) ss += x0[e] * x0[e] + x1[e] * x1[e];
    }
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if (g4 == 0) red[w][lm] = ss;
    __syncthreads();
    if (tid < 16) {
        float t = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) t += red[q][tid];
        ssq[(size_t)blockIdx.y * MP + mt * 16 + tid] = t;
    }
}

// n-tiles per wave: the widest tile (4, 2 or 1, i.e. 256, 128 or 64 columns per workgroup) that still gives about
// two thirds of the CUs a workgroup; with fewer the GEMM, still a weight stream at these row counts, starves
// (measured at the 7B shape, gate/up with 64 rows: 86 workgroups 69.9 us, 172 51.9 us, 344 63.1 us; with 128
// rows: 172 workgroups 69.7 us, 344 77.6 us, 688 92.5 us).  The residual GEMMs fill the chip with K slices
// instead, which keeps the reuse of the wide tile.
int fc_gemm256_cw(int epi, int M, int NT) {
    if (epi == EPI_RESID) return 4;
    const int nrb = ((M + 15) / 16 + 3) / 4;
    for (int cw = 4; cw > 1; cw >>= 1)
        if (((NT + 4 * cw - 1) / (4 * cw)) * nrb >= 160) return cw;
    return 1;
}

// K slices for a matrix with few columns: as many as give every CU at most one workgroup (measured at 256 rows,
// 13B O / down: 240 workgroups 41 / 77 us, 480 workgroups 46 / 81 us, 320 workgroups 50 / 99 us; 7B prefill of
// 256 rows: 256 workgroups 9.4 ms, 384 10.0 ms, 512 9.9 ms: a second workgroup on a CU gains little and the
// partial tiles cost); where one per CU would leave a quarter of the CUs idle, about two per CU instead
// workgroup shape: 1 = four waves; 2 = eight waves in two k-groups, where the launch has at most one workgroup
// per CU anyway; 3 = eight waves over two neighbouring column blocks, where that brings it down to one per CU or
// where four-wave workgroups would come to more than two per CU
int fc_gemm256_mode(int epi, int M, int K, int NT, int sk, int cw) {
    (void)epi;
    const int nrb = ((M + 15) / 16 + 3) / 4, cus = fc_num_cus();
    if (K < 512) return 1;
    if (((NT + 4 * cw - 1) / (4 * cw)) * sk * nrb <= cus) return 2;
    if (((NT + 8 * cw - 1) / (8 * cw)) * sk * nrb <= cus) return 3;
    if (((NT + 4 * cw - 1) / (4 * cw)) * sk * nrb > 2 * cus) return 3;     // several rounds either way: the shared stage wins
    return 1;
}

int fc_gemm256_sk(int M, int K, int NT) {
    const int nwg = ((NT + 15) / 16) * (((M + 15) / 16 + 3) / 4), NS = K / 128;
    if (nwg >= 200) return 1;
    const int cus = fc_num_cus();
    int sk = cus / nwg;
    if (sk < 1 || nwg * sk < (3 * cus) / 4) sk = (2 * cus - 32 + nwg - 1) / nwg;
    if (sk > FC_GEMM256_MAX_SK) sk = FC_GEMM256_MAX_SK;
    if (sk > NS / 2) sk = NS / 2;
    return sk < 1 ? 1 : sk;
}

template <int CW, int KG>
static hipError_t launch256(int epi, const Gemm256Args& a, dim3 grid, hipStream_t st) {
    switch (epi) {
        case EPI_RESID: k_gemm256<EPI_RESID, CW, KG><<<grid, KG == 1 ? 256 : 512, 0, st>>>(a); break;
        case EPI_SWIGLU: k_gemm256<EPI_SWIGLU, CW, KG><<<grid, KG == 1 ? 256 : 512, 0, st>>>(a); break;
        case EPI_QKV: k_gemm256<EPI_QKV, CW, KG><<<grid, KG == 1 ? 256 : 512, 0, st>>>(a); break;
        case EPI_LMHEAD: k_gemm256<EPI_LMHEAD, CW, KG><<<grid, KG == 1 ? 256 : 512, 0, st>>>(a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t fc_gemm256(int epi, const Gemm256Args& a, hipStream_t st) {
    if (a.M < 1 || a.K % 256 || a.NT < 1 || a.sk < 1 || a.sk > FC_GEMM256_MAX_SK || a.sk > a.K / 128) return hipErrorInvalidValue;
    if (a.sk > 1 && (epi != EPI_RESID || !a.part)) return hipErrorInvalidValue;
    // the kernel addresses weights and fragments with 32-bit byte offsets from their bases
    if ((size_t)a.NT * 16 * a.K * 2 >= ((size_t)1 << 32) || (size_t)((a.M + 15) / 16) * 16 * a.K * 4 >= ((size_t)1 << 32)) return hipErrorInvalidValue;
    // narrow tiles when wide ones would leave most of the chip idle
    const int nrb = ((a.M + 15) / 16 + 3) / 4;
    const int cw = (a.cw == 1 || a.cw == 2 || a.cw == 4) ? a.cw : fc_gemm256_cw(epi, a.M, a.NT);
    const int mode = fc_gemm256_mode(epi, a.M, a.K, a.NT, a.sk, cw);
    const int wcols = mode == 3 ? 8 * cw : 4 * cw;
    const int units = ((a.NT + wcols - 1) / wcols) * a.sk;
    dim3 grid((unsigned)((units + 7) / 8) * 8 * nrb);
    hipError_t e;
    if (mode == 2) e = cw == 1 ? launch256<1, 2>(epi, a, grid, st) : (cw == 2 ? launch256<2, 2>(epi, a, grid, st) : launch256<4, 2>(epi, a, grid, st));
    else if (mode == 3) e = cw == 1 ? launch256<1, 3>(epi, a, grid, st) : (cw == 2 ? launch256<2, 3>(epi, a, grid, st) : launch256<4, 3>(epi, a, grid, st));
    else e = cw == 1 ? launch256<1, 1>(epi, a, grid, st) : (cw == 2 ? launch256<2, 1>(epi, a, grid, st) : launch256<4, 1>(epi, a, grid, st));
    if (e != hipSuccess) return e;
    if (a.sk > 1) {
        const size_t n = (size_t)a.M * (a.NT * 4);
        if (a.rf_AF) {
            if ((a.NT * 16) % 256 || !a.rf_gain || !a.rf_ssq) return hipErrorInvalidValue;
            k_resid_reduce_split<<<dim3((a.M + 15) / 16, a.NT * 16 / 256), 512, 0, st>>>(a.part, a.sk, a.M, a.NT * 16, a.out, a.ldo,
                                                                                       a.rf_gain, a.rf_AF, a.rf_ssq);
        } else
            k_resid_reduce<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(a.part, a.sk, a.M, a.NT * 16, a.out, a.ldo);
    }
    return hipGetLastError();
}
