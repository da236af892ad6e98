// Column-owner weight-streaming bf16 GEMM for up to 32 activation rows (MT = 1 or 2 row tiles of 16).
//
// A workgroup of 8 waves owns NW n-tiles (16 output columns each) over the whole of K; wave w
// takes the w-th eighth of K.  No workgroup ever needs another workgroup's result: the eight
// partial tiles meet in LDS, then waves 0..NW-1 each finish one tile and run the fused epilogue.
// For the residual GEMMs with long K and few columns (down, O) the workgroups of a launch can also be
// grouped ks to an owner, each taking 1/ks of K and so reading only 1/ks of the activations (at the 7B
// shape the down projection reads 704 KB of activations per workgroup against 352 KB of weights); the ks
// partial tiles (1 KB each) meet through memory and the last workgroup to arrive adds them in slice order.
// Compared with slicing K across workgroups everywhere this trades the global hand-off (partial tiles through
// memory, an atomic counter, a second pass by the last arriver) for more activation reads out of
// L2: every workgroup reads all 16 x K activations, straight into registers in MFMA B-fragment
// order (lane = row % 16 + 16 * k-octet: two 16-byte loads per k-tile), converts them to a bf16
// hi + lo pair and reuses each fragment for its NW weight tiles.  Weights stream HBM -> VGPR once,
// in MFMA fragment order, KB k-tiles x NW n-tiles per batch.
#include "gemmco.h"
#include "xwg.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
union Frag { u32x4_t u; bf16x8_t v; };

__device__ inline uint32_t rne16(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ inline float up16(uint32_t b) { return __uint_as_float(b << 16); }


// One batch = KB k-tiles: the wave's weight tiles for its n-tiles and its activation octets.
template <int NW, int KB, int MT> struct Batch {
    u32x4_t wt[KB][NW];
    float4 xa[KB][MT][2];
};

// NW * MT <= 16 output tiles per workgroup: after the K slices of the eight waves have met in LDS, wave
// w finishes tiles ti = w and w + 8, tile ti = j * MT + mt (n-tile j of the workgroup, row tile mt).
// KW > 0 selects the up-front variant for K slices of at most KW k-tiles per wave (see the main loop); KB and DB
// are ignored then.
template <int EPI, int NW, int KB, bool DB, int MT, int KW = 0>
__global__ __launch_bounds__(512) void k_gemmco(GemmCoArgs a) {
    extern __shared__ float lds[];
    constexpr int TW = NW * MT;                          // output tiles per workgroup
    // up to 8 output tiles: all eight waves publish at once (one barrier); more: in two rounds of four sets
    constexpr int SETS = TW <= 8 ? 8 : 4;
    f32x4_t* lds_part = (f32x4_t*)lds;                  // [SETS][TW][64 lanes]
    float* lds_ss = lds + SETS * TW * 256;              // [8][MT * 16]
    float* lds_amv = lds_ss + 8 * MT * 16;              // [8][16]
    int* lds_ami = (int*)(lds_amv + 8 * 16);            // [8][16]
    float* lds_gain = (float*)(lds_ami + 8 * 16);       // [K] (only with a norm in front)
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int lm = lane & 15, g4 = lane >> 4;
    // workgroup i owns n-tiles [i*NT/G, (i+1)*NT/G): at most NW of them
    const int ks = (EPI != EPI_LMHEAD && a.ks > 1) ? a.ks : 1;
    const int G = gridDim.x / ks, owner = blockIdx.x / ks, slice = blockIdx.x % ks;
    const int nt0 = (int)(((unsigned)owner * (unsigned)a.NT) / (unsigned)G);
    const int nt1 = (int)(((unsigned)(owner + 1) * (unsigned)a.NT) / (unsigned)G);
    // this workgroup's K slice in k-tiles, cut in eight for the waves (ragged cuts allowed)
    const int KT = a.K >> 5;
    const int s_lo = (int)((unsigned)KT * (unsigned)slice / (unsigned)ks), s_len = (int)((unsigned)KT * (unsigned)(slice + 1) / (unsigned)ks) - s_lo;
    const int kt_begin = s_lo + ((w * s_len) >> 3), kt_end = s_lo + (((w + 1) * s_len) >> 3);
    const int nb = (((s_len + 7) >> 3) + KB - 1) / KB;          // batches of the longest wave
    // With a.rotate every wave walks its batches in a rotated order that differs from wave to wave and
    // workgroup to workgroup: the slices of different workgroups start at addresses that differ by multiples
    // of K * 32 bytes, so in step they would all sit on the same memory channels (measured at the 7B shape:
    // down -5 %, LM head -7 %, gate/up -2 %, QKV +4 %: the caller decides per GEMM).  Batch ib of the loop is
    // batch (ib + rot) mod nbw of the wave's own nbw batches; the loop indices beyond nbw stay invalid.
    const int nbw = (kt_end - kt_begin + KB - 1) / KB;
    const int rot = (a.rotate && nbw > 0) ? (int)(((unsigned)blockIdx.x * 7u + (unsigned)w * 3u) % (unsigned)nbw) : 0;
    auto rot_batch = [&](int ib) { int r = ib + rot; return ib < nbw ? (r >= nbw ? r - nbw : r) : ib; };
    const float* xr[MT];                                // rows past M repeat a valid row; never written
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xr[mt] = a.X + (size_t)(mt * 16 + lm < a.M ? mt * 16 + lm : a.M - 1) * a.ldx + 8 * g4;
    const u32x4_t* wbase = (const u32x4_t*)a.W + lane;

    // All loads are unconditional (a conditionally loaded register batch would be copied, and a copy
    // waits for every load in flight): past the end of the slice, or for n-tiles this workgroup does
    // not own, the address falls back to the first tile of the matrix (cached), and the activations
    // of such k-tiles are zeroed at use.
    auto load = [&](Batch<NW, KB, MT>& b, int ib) {
#pragma unroll
        for (int t = 0; t < KB; ++t) {
            const int kt = kt_begin + rot_batch(ib) * KB + t;
            const bool kv = ib < nb && kt < kt_end;
#pragma unroll
            for (int j = 0; j < NW; ++j) {
                const bool v = kv && nt0 + j < nt1;
                b.wt[t][j] = __builtin_nontemporal_load(wbase + (v ? ((size_t)(nt0 + j) * KT + kt) * 64 : 0));
            }
        }
#pragma unroll
        for (int t = 0; t < KB; ++t) {
            const int kt = kt_begin + rot_batch(ib) * KB + t;
            const int kc = (ib < nb && kt < kt_end) ? kt : kt_begin;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                b.xa[t][mt][0] = *(const float4*)(xr[mt] + kc * 32);
                b.xa[t][mt][1] = *(const float4*)(xr[mt] + kc * 32 + 4);
            }
        }
    };

    f32x4_t acc[NW][MT];
    float ss[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        ss[mt] = 0.f;
#pragma unroll
        for (int j = 0; j < NW; ++j) acc[j][mt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    }

    // one k-tile: activations -> bf16 hi + lo fragments (row statistics on the way), then NW x MT x 2 MFMAs
    auto ktile = [&](const u32x4_t (&wk)[NW], const float4 (&x)[MT][2], int kt, bool valid) {
        const float keep = valid ? 1.0f : 0.0f;
        const int kc = valid ? kt : kt_begin;
        float4 g0, g1;
        if (a.gain) { g0 = *(const float4*)(lds_gain + kc * 32 + 8 * g4); g1 = *(const float4*)(lds_gain + kc * 32 + 8 * g4 + 4); }
        Frag hi[MT], lo[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float v[8] = {x[mt][0].x, x[mt][0].y, x[mt][0].z, x[mt][0].w, x[mt][1].x, x[mt][1].y, x[mt][1].z, x[mt][1].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) { v[e] *= keep; ss[mt] += v[e] * v[e]; }
            if (a.gain) { v[0] *= g0.x; v[1] *= g0.y; v[2] *= g0.z; v[3] *= g0.w; v[4] *= g1.x; v[5] *= g1.y; v[6] *= g1.z; v[7] *= g1.w; }
            uint32_t h[4], l[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) pk_bf16_hilo(v[2 * e], v[2 * e + 1], h[e], l[e]);
            hi[mt].u = (u32x4_t){h[0], h[1], h[2], h[3]};
            lo[mt].u = a.hi_only ? (u32x4_t){0u, 0u, 0u, 0u} : (u32x4_t){l[0], l[1], l[2], l[3]};
        }
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            Frag wf; wf.u = wk[j];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf.v, hi[mt].v, acc[j][mt], 0, 0, 0);
                acc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf.v, lo[mt].v, acc[j][mt], 0, 0, 0);
            }
        }
    };
    auto compute = [&](const Batch<NW, KB, MT>& b, int ib) {
#pragma unroll
        for (int t = 0; t < KB; ++t) {
            const int kt = kt_begin + rot_batch(ib) * KB + t;
            ktile(b.wt[t], b.xa[t], kt, ib < nb && kt < kt_end);
        }
    };

    // What the epilogue will need from memory is requested now, a whole K loop ahead of its use: the rotary
    // factors of this wave's output tiles (behind a dependent load of the sequence length) and the residual
    // tile that the result is added to.
    constexpr int NF = (TW + 7) / 8;
    float rcos[NF][4], rsin[NF][4];
    f32x4_t xold[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        const int ti = w + 8 * f, nt = nt0 + ti / MT, m = (w % MT) * 16 + lm;
        const bool mine = ti < TW && nt < nt1 && m < a.M;
        xold[f] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 4; ++e) { rcos[f][e] = 1.0f; rsin[f][e] = 0.0f; }
        if (EPI == EPI_RESID) {
            if (mine) xold[f] = *(const f32x4_t*)(a.out + (size_t)m * a.ldo + nt * 16 + 4 * g4);
        } else if (EPI == EPI_QKV) {
            const int hh = nt >> 3, t = nt & 7;
            if (mine && hh < a.H + a.Hkv) {
                const int pos = a.rm.rowb ? a.n_state[a.rm.rowb[m]] + a.rm.rowj[m] : a.n_state[m / a.Wn] + m % a.Wn;
                if (pos < a.S) {
                    const f32x4_t c4 = *(const f32x4_t*)(a.cosT + (size_t)pos * 64 + 8 * t + 4 * (g4 & 1));
                    const f32x4_t s4 = *(const f32x4_t*)(a.sinT + (size_t)pos * 64 + 8 * t + 4 * (g4 & 1));
#pragma unroll
                    for (int e = 0; e < 4; ++e) { rcos[f][e] = c4[e]; rsin[f][e] = s4[e]; }
                }
            }
        }
    }

    if constexpr (KW > 0) {
        // Up-front variant for short K slices (at most KW k-tiles per wave): the wave requests its weights at
        // once, as many k-tiles as 28-32 fragments of registers hold (KA), and refills the slot of a k-tile that
        // has been used with the k-tile KA further on; the slice then costs about one memory round trip instead
        // of one per batch.  Activations (L2 hits) travel one k-tile ahead.  (A ring of the same depth with a
        // run-time trip count, with or without the activations travelling in the ring, was no faster than the
        // batches: what pays is the burst at the start of the kernel.)
        constexpr int FR = EPI == EPI_QKV ? 28 : 32;       // (the QKV epilogue keeps its rotary factors in registers too)
        constexpr int KA = NW * KW <= FR ? KW : FR / NW;
        u32x4_t wt[KA][NW];
        auto wload = [&](u32x4_t (&wk)[NW], int t) {
            const int kt = kt_begin + t;
#pragma unroll
            for (int j = 0; j < NW; ++j) {
                const bool v = kt < kt_end && nt0 + j < nt1;
                wk[j] = __builtin_nontemporal_load(wbase + (v ? ((size_t)(nt0 + j) * KT + kt) * 64 : 0));
            }
        };
#pragma unroll
        for (int t = 0; t < KA; ++t) wload(wt[t], t);
        if (a.gain) {       // the norm gain goes through LDS once per workgroup
            for (int i = tid * 4; i < a.K; i += 512 * 4) *(float4*)(lds_gain + i) = *(const float4*)(a.gain + i);
            __syncthreads();
        }
        float4 xa[2][MT][2];
        auto xload = [&](float4 (&x)[MT][2], int t) {
            const int kt = kt_begin + t, kc = kt < kt_end ? kt : kt_begin;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                x[mt][0] = *(const float4*)(xr[mt] + kc * 32);
                x[mt][1] = *(const float4*)(xr[mt] + kc * 32 + 4);
            }
        };
        xload(xa[0], 0);
#pragma unroll
        for (int t = 0; t < KW; ++t) {
            if (t + 1 < KW) xload(xa[(t + 1) & 1], t + 1);
            __builtin_amdgcn_sched_barrier(0);
            ktile(wt[t % KA], xa[t & 1], kt_begin + t, kt_begin + t < kt_end);
            if (t + KA < KW) wload(wt[t % KA], t + KA);
        }
    } else {
    // two batches in flight per wave: the next one is requested before the current one is used
    // (DB = false keeps one batch per wave in flight and fewer registers, so that two workgroups
    // share a CU and overlap each other's phases instead)
    Batch<NW, KB, MT> A;
    load(A, 0);
    if (DB) {
        Batch<NW, KB, MT> B;
        load(B, 1);
        if (a.gain) {       // the norm gain goes through LDS once per workgroup
            for (int i = tid * 4; i < a.K; i += 512 * 4) *(float4*)(lds_gain + i) = *(const float4*)(a.gain + i);
            __syncthreads();
        }
        for (int ib = 0; ib < nb; ib += 2) {
            compute(A, ib);
            load(A, ib + 2);
            __builtin_amdgcn_sched_barrier(0);          // the loads stay here, ahead of the other batch's arithmetic
            compute(B, ib + 1);
            load(B, ib + 3);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        if (a.gain) {
            for (int i = tid * 4; i < a.K; i += 512 * 4) *(float4*)(lds_gain + i) = *(const float4*)(a.gain + i);
            __syncthreads();
        }
        for (int ib = 0; ib < nb; ++ib) {
            compute(A, ib);
            load(A, ib + 1);
        }
    }
    }

    // the eight K slices meet in LDS: with up to eight output tiles every wave publishes its partial tiles and one
    // barrier later each tile's finisher adds the eight in wave order; with more tiles in two rounds, so that
    // four partial sets (4 x TW KB) are enough: waves 4..7 publish, waves 0..3 add those to their own and
    // publish the sums
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        ss[mt] += __shfl_xor(ss[mt], 16, 64);
        ss[mt] += __shfl_xor(ss[mt], 32, 64);
        if (g4 == 0) lds_ss[(w * MT + mt) * 16 + lm] = ss[mt];
    }
    if constexpr (SETS == 8) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < NW; ++j) lds_part[(w * TW + j * MT + mt) * 64 + lane] = acc[j][mt];
        __syncthreads();
    } else {
    if (w >= 4) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < NW; ++j) lds_part[((w - 4) * TW + j * MT + mt) * 64 + lane] = acc[j][mt];
    }
    __syncthreads();
    if (w < 4) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < NW; ++j) acc[j][mt] += lds_part[(w * TW + j * MT + mt) * 64 + lane];
    }
    __syncthreads();
    if (w < 4) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int j = 0; j < NW; ++j) lds_part[(w * TW + j * MT + mt) * 64 + lane] = acc[j][mt];
    }
    __syncthreads();
    }

    // wave w finishes tiles w and (with more than 8 tiles) w + 8: lane holds row tm*16 + lm, columns
    // nt*16 + 4*g4 + r.  MT divides 8, so both tiles of a wave belong to the same row tile tm.
    const int tm = w % MT;
    const int m = tm * 16 + lm;
    int ntf[NF];
    bool fin[NF];
    f32x4_t v[NF];
    float rs = 1.0f, ssrow = 0.f;
    if (a.gain) {
#pragma unroll
        for (int q = 0; q < 8; ++q) ssrow += lds_ss[(q * MT + tm) * 16 + lm];
        rs = 1.0f / sqrtf(ssrow / (float)a.K + a.eps);
    }
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        const int ti = w + 8 * f;
        ntf[f] = nt0 + ti / MT;
        fin[f] = ti < TW && ntf[f] < nt1;
        v[f] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
        if (fin[f]) {
#pragma unroll
            for (int q = 0; q < SETS; ++q) v[f] += lds_part[(q * TW + ti) * 64 + lane];
            if (ks == 1) v[f] *= rs;
        }
    }
    if (EPI != EPI_LMHEAD && ks > 1) {
        // partial tiles of the ks slices (and, with a norm in front, each slice's share of the row sums of
        // squares) meet through memory; the last workgroup to arrive adds them in slice order
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            float* mine = a.xpart + ((size_t)blockIdx.x * (8 * NF) + w + 8 * f) * 256 + lane * 4;
            if (fin[f]) {
                st_agent_f32x2(mine, v[f][0], v[f][1]);
                st_agent_f32x2(mine + 2, v[f][2], v[f][3]);
            }
        }
        float* sspart = a.xpart + (size_t)gridDim.x * (8 * NF) * 256;       // [workgroup][MT * 16]
        if (a.gain && w < MT && g4 == 0) st_agent_f32(sspart + (size_t)blockIdx.x * (MT * 16) + tm * 16 + lm, ssrow);
        wait_vmem_done();
        __syncthreads();
        int* flag = (int*)lds_ss;
        if (tid == 0) *flag = arrive_agent(a.xcnt + owner);
        __syncthreads();
        if (*flag != ks - 1) return;
        if (a.gain) {
            float s = 0.f;
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2) {
                const float p = ld_agent_f32(sspart + (size_t)(owner * ks + (s2 < ks ? s2 : 0)) * (MT * 16) + tm * 16 + lm);
                if (s2 < ks) s += p;
            }
            rs = 1.0f / sqrtf(s / (float)a.K + a.eps);
        }
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            if (!fin[f]) continue;
            f32x4_t part[8];
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2) {
                const float* src = a.xpart + ((size_t)(owner * ks + (s2 < ks ? s2 : 0)) * (8 * NF) + w + 8 * f) * 256 + lane * 4;
                float p0, p1, p2, p3;
                ld_agent_f32x2(src, p0, p1);
                ld_agent_f32x2(src + 2, p2, p3);
                part[s2] = (f32x4_t){p0, p1, p2, p3};
            }
            v[f] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2) if (s2 < ks) v[f] += part[s2];
            v[f] *= rs;
        }
        if (tid == 0) st_agent_i32(a.xcnt + owner, 0);
    }
    float best = -3.0e38f; int bi = 0x7fffffff;          // LM head: the wave's winner per row over its tiles
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        const int nt = ntf[f];
        const f32x4_t vv = v[f];
        if (!fin[f]) continue;
        if (EPI == EPI_RESID) {
            if (m < a.M) *(f32x4_t*)(a.out + (size_t)m * a.ldo + nt * 16 + 4 * g4) = xold[f] + vv;
        } else if (EPI == EPI_SWIGLU) {
            // columns 0..7 of a tile: gate of features 8*nt..; columns 8..15: their up values (lane ^ 32)
            f32x4_t h;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float other = __shfl_xor(vv[r], 32, 64);
                h[r] = vv[r] / (1.0f + expf(-vv[r])) * other;
            }
            if (g4 < 2 && m < a.M) *(f32x4_t*)(a.out + (size_t)m * a.ldo + nt * 8 + 4 * g4) = h;
        } else if (EPI == EPI_QKV) {
            // q/k heads: tile t of a head holds elements 8t..8t+7 (columns 0..7) and their rotary partners
            // 64+8t.. (columns 8..15, lane ^ 32); v heads are in natural order
            const int hh = nt >> 3, t = nt & 7;
            const int mc = m < a.M ? m : 0;
            const int b = a.rm.rowb ? a.rm.rowb[mc] : m / a.Wn, j = a.rm.rowb ? a.rm.rowj[mc] : m % a.Wn;
            const int pos = m < a.M ? a.n_state[b] + j : a.S;
            const bool ok = m < a.M && pos < a.S;               // capacity guard
            const size_t plane = (size_t)a.S * 128;
            if (hh < a.H + a.Hkv) {
                const int i0 = 8 * t + 4 * (g4 & 1);            // element index within the half
                f32x4_t r;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float other = __shfl_xor(vv[e], 32, 64);
                    const float c = rcos[f][e], s = rsin[f][e];
                    r[e] = g4 < 2 ? vv[e] * c - other * s : vv[e] * c + other * s;
                    if (hh >= a.H) r[e] = kv_round(r[e], a.kvq & 15);
                }
                const int el = (g4 < 2 ? 0 : 64) + i0;          // element index within the head
                if (ok) {
                    if (hh < a.H) *(f32x4_t*)(a.out + (size_t)m * a.ldo + hh * 128 + el) = r;
                    else {
                        bf16_t* kb = a.kc + ((((size_t)a.layer * a.B + b) * a.Hkv + (hh - a.H)) * kv_alloc_planes(a.kvp)) * plane;
                        const size_t ki = k_index(pos, el, 128);
                        bf16_t* kr = kb + ki;
                        uint32_t h[4];
                        if (a.kvp == 3) {
                            uint32_t l[4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) kv24_split(r[e], h[e], l[e]);
                            *(uint2*)kr = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                            *(uint32_t*)((uint8_t*)(kb + plane) + ki) = l[0] | (l[1] << 8) | (l[2] << 16) | (l[3] << 24);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e) h[e] = rne16(r[e]);
                            *(uint2*)kr = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                            if (a.kvp == 2) {
                                uint32_t l[4];
#pragma unroll
                                for (int e = 0; e < 4; ++e) l[e] = rne16(r[e] - up16(h[e]));
                                *(uint2*)(kr + plane) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
                            }
                        }
                    }
                }
            } else if (ok) {
                const int kh = hh - a.H - a.Hkv;
                bf16_t* vb = a.vc + ((((size_t)a.layer * a.B + b) * a.Hkv + kh) * kv_alloc_planes(a.kvp)) * plane;
                const size_t vi = v_index(16 * t + 4 * g4, pos, 128);
                bf16_t* vr = vb + vi;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float vq = kv_round(vv[e], a.kvq >> 4);
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
            if (a.out && m < a.M) *(f32x4_t*)(a.out + (size_t)m * a.ldo + n0) = vv;
#pragma unroll
            for (int r = 0; r < 4; ++r) if (vv[r] > best || (vv[r] == best && n0 + r < bi)) { best = vv[r]; bi = n0 + r; }
        }
    }
    if (EPI == EPI_LMHEAD) {
#pragma unroll
        for (int o = 16; o <= 32; o <<= 1) {
            const float ov = __shfl_xor(best, o, 64); const int oi = __shfl_xor(bi, o, 64);
            if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
        }
        if (g4 == 0) { lds_amv[w * 16 + lm] = best; lds_ami[w * 16 + lm] = bi; }
        __syncthreads();
        if (tid < 16 * MT) {                 // row tid: the waves whose tiles are row tile tid / 16
            const int rt = tid >> 4, r16 = tid & 15;
            float bv = -3.0e38f; int bx = 0x7fffffff;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (q % MT != rt) continue;
                const float ov = lds_amv[q * 16 + r16]; const int oi = lds_ami[q * 16 + r16];
                if (ov > bv || (ov == bv && oi < bx)) { bv = ov; bx = oi; }
            }
            a.amax_val[(size_t)blockIdx.x * (16 * MT) + tid] = bv;
            a.amax_idx[(size_t)blockIdx.x * (16 * MT) + tid] = bx;
        }
    }
}

static int g_cus = 0;
static int num_cus() {
    if (!g_cus) {
        int dev = 0; hipDeviceProp_t p;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess) g_cus = p.multiProcessorCount;
        if (g_cus <= 0) g_cus = 256;
    }
    return g_cus;
}

int fc_num_cus() { return num_cus(); }

// grid: one workgroup per CU unless that would give a workgroup more than `most` n-tiles (at most 8: with two
// row tiles a workgroup then finishes 16 output tiles, whose partial sums take 64 KB of LDS)
int fc_gemmco_grid(int NT, int most) {
    int G = num_cus();
    if (G > NT) G = NT;
    while ((NT + G - 1) / G > most) G += num_cus();
    return G;
}

static size_t co_lds_bytes(int nw, int mt, int K, bool gain) {
    return (size_t)(nw * mt <= 8 ? 8 : 4) * nw * mt * 1024 + (size_t)(8 * mt * 16 + 2 * 8 * 16) * 4 + (gain ? (size_t)K * 4 : 0) + 64;
}

int fc_gemmco_most(int M, int K, bool gain) {
    // the kernel is instantiated for 1, 2, 3, 4, 6 and 8 n-tiles per workgroup (5 runs as 6, 7 as 8) and
    // sizes its LDS for the instantiated count
    const int inst[6] = {8, 6, 4, 3, 2, 1};
    for (int i = 0; i < 6; ++i)
        if (co_lds_bytes(inst[i], M > 16 ? 2 : 1, K, gain) <= 150 * 1024) return inst[i];
    return 1;
}

template <int EPI, int NW, int KB, bool DB, int MT, int KW = 0>
static hipError_t launch_k(const GemmCoArgs& a, int G, hipStream_t st) {
    const size_t lds = co_lds_bytes(NW, MT, a.K, a.gain != nullptr);
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void*)k_gemmco<EPI, NW, KB, DB, MT, KW>, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    if (lds > 150 * 1024) return hipErrorInvalidValue;
    k_gemmco<EPI, NW, KB, DB, MT, KW><<<G, 512, lds, st>>>(a);
    return hipGetLastError();
}
// up-front variant: QKV and the residual GEMMs, up to 16 rows, K slices of at most 16 k-tiles per wave
template <int EPI>
static hipError_t launch_deep(const GemmCoArgs& a, int G, int nw, hipStream_t st) {
    if constexpr (EPI == EPI_QKV || EPI == EPI_RESID) {
        const int ks = a.ks > 1 ? a.ks : 1, KT = a.K >> 5;
        const int kw = ((KT + ks - 1) / ks + 7) / 8;          // most k-tiles any wave owns
        if (a.M > 16 || nw < 1) return hipErrorInvalidValue;
        if (kw <= 8) switch (nw) {
            case 1: return launch_k<EPI, 1, 1, false, 1, 8>(a, G, st);
            case 2: return launch_k<EPI, 2, 1, false, 1, 8>(a, G, st);
            case 3: return launch_k<EPI, 3, 1, false, 1, 8>(a, G, st);
            case 4: return launch_k<EPI, 4, 1, false, 1, 8>(a, G, st);
            case 5: case 6: return launch_k<EPI, 6, 1, false, 1, 8>(a, G, st);
        } else if (kw <= 12) switch (nw) {
            case 1: return launch_k<EPI, 1, 1, false, 1, 12>(a, G, st);
            case 2: return launch_k<EPI, 2, 1, false, 1, 12>(a, G, st);
            case 3: return launch_k<EPI, 3, 1, false, 1, 12>(a, G, st);
            case 4: return launch_k<EPI, 4, 1, false, 1, 12>(a, G, st);
        } else if (kw <= 16) switch (nw) {
            case 1: return launch_k<EPI, 1, 1, false, 1, 16>(a, G, st);
            case 2: return launch_k<EPI, 2, 1, false, 1, 16>(a, G, st);
            case 3: return launch_k<EPI, 3, 1, false, 1, 16>(a, G, st);
        }
    }
    return hipErrorInvalidValue;
}
template <int EPI>
static hipError_t launch_epi(const GemmCoArgs& a, int G, hipStream_t st) {
    const int owners = G / (a.ks > 1 ? a.ks : 1);
    const int nw = (a.NT + owners - 1) / owners;  // most n-tiles any workgroup owns
    if (a.single_buffer == 2) return launch_deep<EPI>(a, G, nw, st);
    if (a.M > 16 && nw > 8) return hipErrorInvalidValue;
    if (a.M > 16 && !a.single_buffer) {           // two row tiles, two batches in flight
        switch (nw) {
            case 1: return launch_k<EPI, 1, 2, true, 2>(a, G, st);
            case 2: return launch_k<EPI, 2, 2, true, 2>(a, G, st);
            case 3: return launch_k<EPI, 3, 2, true, 2>(a, G, st);
            case 4: return launch_k<EPI, 4, 1, true, 2>(a, G, st);
            case 5: case 6: return launch_k<EPI, 6, 1, true, 2>(a, G, st);
            case 7: case 8: return launch_k<EPI, 8, 1, true, 2>(a, G, st);
        }
        return hipErrorInvalidValue;
    }
    if (a.M > 16) {                               // two row tiles
        switch (nw) {
            case 1: return launch_k<EPI, 1, 4, false, 2>(a, G, st);
            case 2: return launch_k<EPI, 2, 4, false, 2>(a, G, st);
            case 3: return launch_k<EPI, 3, 2, false, 2>(a, G, st);
            case 4: return launch_k<EPI, 4, 2, false, 2>(a, G, st);
            case 5: case 6: return launch_k<EPI, 6, 2, false, 2>(a, G, st);
            case 7: case 8: return launch_k<EPI, 8, 2, false, 2>(a, G, st);
        }
        return hipErrorInvalidValue;
    }
    if (nw > 8) {                                 // 9..12 n-tiles per workgroup (K slices per owner make them short)
        if (nw > 12) return hipErrorInvalidValue;
        return a.single_buffer ? launch_k<EPI, 12, 1, false, 1>(a, G, st) : launch_k<EPI, 12, 1, true, 1>(a, G, st);
    }
    if (a.single_buffer) {
        switch (nw) {
            case 1: return launch_k<EPI, 1, 8, false, 1>(a, G, st);
            case 2: return launch_k<EPI, 2, 4, false, 1>(a, G, st);
            case 3: return launch_k<EPI, 3, 4, false, 1>(a, G, st);
            case 4: return launch_k<EPI, 4, 4, false, 1>(a, G, st);
            case 5: case 6: return launch_k<EPI, 6, 2, false, 1>(a, G, st);
            case 7: case 8: return launch_k<EPI, 8, 2, false, 1>(a, G, st);
        }
        return hipErrorInvalidValue;
    }
    switch (nw) {
        case 1: return launch_k<EPI, 1, 4, true, 1>(a, G, st);
        case 2: return launch_k<EPI, 2, 4, true, 1>(a, G, st);
        case 3: return launch_k<EPI, 3, 3, true, 1>(a, G, st);
        case 4: return launch_k<EPI, 4, 2, true, 1>(a, G, st);
        case 5: case 6: return launch_k<EPI, 6, 2, true, 1>(a, G, st);
        case 7: case 8: return launch_k<EPI, 8, 1, true, 1>(a, G, st);
    }
    return hipErrorInvalidValue;
}

hipError_t fc_gemmco(int epi, const GemmCoArgs& a, int G, hipStream_t st) {
    const int ks = a.ks > 1 ? a.ks : 1, most = a.M <= 16 ? 12 : 8;
    if (a.M < 1 || a.M > 32 || a.K % 256 || a.NT < 1 || G < 1 || ks > 8 || G % ks || G / ks > a.NT ||
        (a.NT + G / ks - 1) / (G / ks) > most || a.K / 256 < ks)
        return hipErrorInvalidValue;
    if (ks > 1 && (epi == EPI_LMHEAD || !a.xpart || !a.xcnt || G / ks > FC_MAX_COUNTERS)) return hipErrorInvalidValue;
    switch (epi) {
        case EPI_RESID: return launch_epi<EPI_RESID>(a, G, st);
        case EPI_SWIGLU: return launch_epi<EPI_SWIGLU>(a, G, st);
        case EPI_QKV: return launch_epi<EPI_QKV>(a, G, st);
        case EPI_LMHEAD: return launch_epi<EPI_LMHEAD>(a, G, st);
    }
    return hipErrorInvalidValue;
}

// reduction of the LM head's per-workgroup winners: lowest id on ties
__global__ void k_argmax_final(const float* val, const int32_t* idx, int nparts, int stride, int32_t* ids, float* top, RowMap rm, int W) {
    __shared__ float bv[4];
    __shared__ int bi[4];
    const int m = blockIdx.x;
    float best = -3.0e38f; int b = 0x7fffffff;
    for (int c = threadIdx.x; c < nparts; c += blockDim.x) {
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
        const int dst = rm.rowb ? rm.rowb[m] * W + rm.rowj[m] : m;
        ids[dst] = b; top[dst] = best;
    }
}
hipError_t fc_argmax_final(const float* val, const int32_t* idx, int nparts, int stride, int M, int32_t* ids, float* top,
                           hipStream_t st, RowMap rm, int W) {
    k_argmax_final<<<M, 256, 0, st>>>(val, idx, nparts, stride, ids, top, rm, W);
    return hipGetLastError();
}
