// Causal attention for passes with many query rows per sequence (prompt chunks, very wide windows): the first
// forward of the method (Sec. 4.1) sees a whole prompt, and the window-causal mask of Eq. 2 / Eq. 4 is the same
// mask over more rows.
//
// The step kernel (attn16.hip) gives every 16 or 32 query rows a workgroup of their own, which then reads all of
// K and V: fine while K/V is read once or twice, wasteful when a chunk of a prompt brings hundreds of rows.  Here
// a workgroup of four waves takes 128 query rows of one (sequence, head) -- a wave 32 rows, as two 16-row tiles --
// and walks the key blocks once for all of them: a block of 32 keys (K and V^T fragments, hi and lo planes:
// 32 KB) is copied global -> LDS by the whole workgroup while the previous one is being used (two buffers, one
// barrier per block), and every wave reads its matrix operands from LDS.  Scores S^T = K . Q^T, fp32 running-max
// softmax and O^T += V^T . P^T are the step kernel's, operand layouts included; a wave owns its rows from start
// to finish, so nothing is merged between waves or workgroups.  A wave skips the blocks none of its rows can see.
#include "attn16.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
union Frag { u32x4_t u; bf16x8_t v; };

__device__ inline void split8p(const float* v, Frag& hi, Frag& lo) {
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) pk_bf16_hilo(v[2 * e], v[2 * e + 1], h[e], l[e]);
    hi.u = (u32x4_t){h[0], h[1], h[2], h[3]};
    lo.u = (u32x4_t){l[0], l[1], l[2], l[3]};
}

#define NEG_BIG (-1.0e30f)

// KVP: 1 = one bf16 plane, 2 = bf16 hi + bf16 lo planes
template <int KVP>
__global__ __launch_bounds__(256, 2) void k_attnp(AttnArgs a) {
    __shared__ u32x4_t kv[2][2 * KVP][512];              // [buffer][K hi, (K lo,) V hi (, V lo)][8 fragments x 64 lanes]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int lm = lane & 15, g = lane >> 4;
    const int nrb = (a.W + 127) >> 7;
    // query heads that share a K/V head follow each other at a stride of Hkv (same XCD, see attn16.hip); the row
    // blocks of a head run latest first: they see the most keys
    const int bh = blockIdx.x / nrb, rbk = nrb - 1 - (int)(blockIdx.x % nrb);
    const int hr = bh % a.H, G = a.H / a.Hkv, kvh = hr % a.Hkv, h = kvh * G + hr / a.Hkv, b = bh / a.H;
    const int n = a.n_state[b];
    const int Wb = a.rstart ? a.rstart[b + 1] - a.rstart[b] : a.W, rbase = a.rstart ? a.rstart[b] : b * a.W;
    const int row_base = 128 * rbk, rows_wg = Wb - row_base < 128 ? Wb - row_base : 128;
    if (rows_wg <= 0) return;                             // a sequence with a smaller window of its own
    int T = n + row_base + rows_wg;                       // keys the last row of the workgroup sees
    if (T > a.S) T = a.S;                                 // capacity guard (the host checks first)
    const int NB = (T + 31) >> 5;
    const int r0 = row_base + 32 * wv;                    // this wave's rows r0 .. r0 + 31
    const int rows_wave = Wb - r0 < 32 ? Wb - r0 : 32;    // <= 0: a wave without rows (it still copies blocks)
    const int last_key = n + r0 + rows_wave - 1;          // newest key any row of the wave sees
    const size_t plane = (size_t)a.S * 128;
    const bf16_t* kbase = a.kc + ((((size_t)a.layer * a.B + b) * a.Hkv + kvh) * KVP) * plane;
    const bf16_t* vbase = a.vc + ((((size_t)a.layer * a.B + b) * a.Hkv + kvh) * KVP) * plane;

    // Q as B operand: lane (row lm, dh 32*g + 8*s + e), hi and lo
    Frag qh[2][4], ql[2][4];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        int j = r0 + qt * 16 + lm;
        if (j >= Wb) j = Wb - 1;
        const float* qr = a.q + (size_t)(rbase + j) * a.ldq + h * 128 + 32 * g;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const float4 x0 = *(const float4*)(qr + 8 * s), x1 = *(const float4*)(qr + 8 * s + 4);
            const float v[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
            split8p(v, qh[qt][s], ql[qt][s]);
        }
    }
    f32x4_t acc[2][8];
    float mrun[2], lrun[2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        mrun[qt] = NEG_BIG; lrun[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) acc[qt][dt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    }
    const float scale = 0.08838834764831845f;   // 1/sqrt(128)

    // block copy: 4 (or 2) chunks of 8 KB, 512 sixteen-byte words each; thread t takes words t and t + 256 of every chunk
    constexpr int NCH = 2 * KVP;
    u32x4_t sr[NCH][2];
    auto stage_load = [&](int blk) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const bf16_t* src = (c < KVP ? kbase : vbase) + (size_t)(c % KVP) * plane + (size_t)blk * 4096;
            sr[c][0] = __builtin_nontemporal_load((const u32x4_t*)src + tid);
            sr[c][1] = __builtin_nontemporal_load((const u32x4_t*)src + 256 + tid);
        }
    };
    auto stage_store = [&](int buf) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) { kv[buf][c][tid] = sr[c][0]; kv[buf][c][256 + tid] = sr[c][1]; }
    };

    auto compute = [&](int buf, int blk) {
        const int kb = blk << 5;
        f32x4_t sc[2][2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) sc[qt][0] = sc[qt][1] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag kh, kl;
                kh.u = kv[buf][0][(t * 4 + s) * 64 + lane];
                if (KVP == 2) kl.u = kv[buf][1][(t * 4 + s) * 64 + lane];
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    sc[qt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kh.v, qh[qt][s].v, sc[qt][t], 0, 0, 0);
                    sc[qt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kh.v, ql[qt][s].v, sc[qt][t], 0, 0, 0);
                    if (KVP == 2)   // lo x lo is below fp32 resolution and is dropped
                        sc[qt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kl.v, qh[qt][s].v, sc[qt][t], 0, 0, 0);
                }
            }
        Frag ph[2], pl[2];
        float alpha[2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            // lane: row j = r0 + qt*16 + lm, keys kb + 8*g + e  (e = 4*t + r)
            int j = r0 + qt * 16 + lm;
            if (j >= Wb) j = Wb - 1;
            const int lastvis = n + j;
            float p[8];
            float bm = NEG_BIG;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int key = kb + 8 * g + e;
                const bool vis = key <= lastvis && key < T;
                p[e] = vis ? sc[qt][e >> 2][e & 3] * scale : NEG_BIG;
                bm = fmaxf(bm, p[e]);
            }
            bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
            bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
            const float mnew = fmaxf(mrun[qt], bm);
            alpha[qt] = expf(mrun[qt] - mnew);
            float ps = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int key = kb + 8 * g + e;
                const bool vis = key <= lastvis && key < T;
                p[e] = vis ? expf(p[e] - mnew) : 0.f;
                ps += p[e];
            }
            mrun[qt] = mnew;
            lrun[qt] = lrun[qt] * alpha[qt] + ps;
            split8p(p, ph[qt], pl[qt]);
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            Frag vh, vl;
            vh.u = kv[buf][KVP][dt * 64 + lane];
            if (KVP == 2) vl.u = kv[buf][KVP + 1][dt * 64 + lane];
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                acc[qt][dt] *= alpha[qt];
                acc[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh.v, ph[qt].v, acc[qt][dt], 0, 0, 0);
                acc[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vh.v, pl[qt].v, acc[qt][dt], 0, 0, 0);
                if (KVP == 2)
                    acc[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vl.v, ph[qt].v, acc[qt][dt], 0, 0, 0);
            }
        }
    };

    stage_load(0);
    stage_store(0);
    __syncthreads();
    int buf = 0;
    for (int blk = 0; blk < NB; ++blk) {
        const bool more = blk + 1 < NB;                   // the same for every wave of the workgroup
        if (more) stage_load(blk + 1);                    // travels while this block is used
        __builtin_amdgcn_sched_barrier(0);
        if (rows_wave > 0 && (blk << 5) <= last_key) compute(buf, blk);
        if (more) stage_store(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    // out[row][h*128 + 16*dt + 4*g + r] = O / l
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        float l = lrun[qt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        const int j = r0 + qt * 16 + lm;
        if (j < Wb) {
            const float inv = 1.0f / l;
            const int row = rbase + j;
            if (a.out) {
                float* o = a.out + (size_t)row * a.ldo + h * 128 + 4 * g;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) *(f32x4_t*)(o + 16 * dt) = acc[qt][dt] * inv;
            }
            if (a.ofrag) {
                // head elements 16 * dt + 4 * g + r: k-tile 4 * h + dt / 2, octet 2 * (dt % 2) + g / 2, elements 4 * (g % 2) + r
                const size_t KTo = (size_t)a.H * 4;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) {
                    const f32x4_t v = acc[qt][dt] * inv;
                    uint32_t h0, l0, h1, l1;
                    pk_bf16_hilo(v[0], v[1], h0, l0);
                    pk_bf16_hilo(v[2], v[3], h1, l1);
                    char* dst = (char*)a.ofrag + ((((size_t)(row >> 4) * KTo + 4 * h + (dt >> 1)) * 2) * 64 + (row & 15) + 16 * (2 * (dt & 1) + (g >> 1))) * 16 + 8 * (g & 1);
                    *(uint2*)dst = make_uint2(h0, h1);
                    *(uint2*)(dst + 1024) = make_uint2(l0, l1);
                }
            }
        }
    }
}

// workgroups the many-row kernel would launch (the caller compares with the CU count)
int fc_attnp_workgroups(int Bact, int H, int W) { return Bact * H * ((W + 127) / 128); }

hipError_t fc_attnp(const AttnArgs& a, int Bact, hipStream_t st) {
    if (a.W < 1 || a.S < 32 || a.S % 32 || a.H % a.Hkv || (a.kvp != 1 && a.kvp != 2)) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)fc_attnp_workgroups(Bact, a.H, a.W);
    if (a.kvp == 2) k_attnp<2><<<grid, 256, 0, st>>>(a);
    else k_attnp<1><<<grid, 256, 0, st>>>(a);
    return hipGetLastError();
}
