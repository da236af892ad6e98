// Shared declarations of the FastCoT gfx950 library: workspace map, packed-weight map,
// device-side state block and small device helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/fastcot.h"

typedef uint16_t bf16_t;  // raw bf16 bit pattern

__host__ __device__ inline float bf16_to_f32(bf16_t b) {
    union { uint32_t u; float f; } v; v.u = (uint32_t)b << 16; return v.f;
}
__host__ __device__ inline bf16_t f32_to_bf16(float f) {  // round to nearest even, finite inputs
    union { uint32_t u; float f; } v; v.f = f;
    v.u += 0x7FFFu + ((v.u >> 16) & 1u);
    return (bf16_t)(v.u >> 16);
}

#if defined(__HIPCC__)
// Two floats -> one word of two bf16 (a in the low half), round to nearest even: one v_cvt_pk_bf16_f32.
__device__ inline uint32_t pk_bf16(float a, float b) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// hi + lo split of a pair: hi = bf16(a), bf16(b); lo = bf16 of what the hi parts leave over
__device__ inline void pk_bf16_hilo(float a, float b, uint32_t& hi, uint32_t& lo) {
    hi = pk_bf16(a, b);
    lo = pk_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xFFFF0000u));
}

// The 3-byte cache format (kvp == 3): a value is rounded to the upper 24 bits of its fp32 pattern (to nearest
// even); the upper 16 bits go to the hi plane (a bf16, truncated, not rounded), the next 8 to a plane of bytes.
// hi and value - hi are both exact bf16 numbers, so the attention kernel feeds them to the matrix cores as it
// feeds the hi + lo pair.
__host__ __device__ inline void kv24_split(float v, uint32_t& hi16, uint32_t& lo8) {
    union { uint32_t u; float f; } x; x.f = v;
    const uint32_t u = x.u + 0x7Fu + ((x.u >> 8) & 1u);
    hi16 = u >> 16; lo8 = (u >> 8) & 0xFFu;
}
__host__ __device__ inline float kv24_join(uint32_t hi16, uint32_t lo8) {
    union { uint32_t u; float f; } x; x.u = (hi16 << 16) | (lo8 << 8); return x.f;
}

// Precision study of the K/V cache: what a cached value would be after a round trip through a narrower
// storage format (0 as computed, 1 bf16, 2 fp16, 3 the upper 24 bits of fp32), round to nearest even.  The
// value is then stored in the hi + lo planes as usual (which hold any of these exactly), so the effect of a
// format on the logits can be measured before a kernel for it exists.
__device__ inline float kv_round(float v, int mode) {
    if (mode == 1) return __uint_as_float((uint32_t)f32_to_bf16(v) << 16);
    if (mode == 2) return (float)(_Float16)v;
    if (mode == 3) { uint32_t u = __float_as_uint(v); u += 0x7Fu + ((u >> 8) & 1u); return __uint_as_float(u & 0xFFFFFF00u); }
    return v;
}
#endif

// ------------------------------------------------------------------ packed weights
// A fused matrix has K rows (inputs) and NP columns (outputs, padded to a multiple of 16).
// fp32 models keep it row-major [K][NP].  bf16 models keep it in MFMA fragment order: the
// 16-column x 32-row tile (nt, kt) is 64 lanes x 8 values, lane = (col % 16) + 16 * ((row % 32) / 8),
// value = row % 8, tiles ordered [nt][kt]; one wave reads a tile with one 16-byte load per lane.
struct FusedMat {
    size_t off;     // byte offset inside the packed weights
    int32_t K, N;   // logical rows, logical columns
    int32_t NP;     // padded columns
};
__host__ __device__ inline size_t frag_index(int32_t K, int32_t k, int32_t n) {
    int32_t KT = K >> 5;
    int32_t nt = n >> 4, kt = k >> 5;
    int32_t lane = (n & 15) + 16 * ((k & 31) >> 3);
    return ((size_t)(nt * (size_t)KT + kt) * 64 + lane) * 8 + (k & 7);
}

// Column order inside the fused matrices.  Outputs that an epilogue must combine sit in the same
// 16-column MFMA tile, 8 columns apart, so that the two values end up in lanes l and l^32 of one
// wave: gate and up of a feature (SwiGLU), and the rotary pair (i, i + Dh/2) of a head.
__host__ __device__ inline int32_t gu_col(int32_t feature, int32_t is_up) {
    return ((feature >> 3) << 4) + (is_up << 3) + (feature & 7);
}
// position of element i of a head inside the head's Dh packed columns
__host__ __device__ inline int32_t head_col(int32_t i, int32_t Dh) {
    const int32_t half = Dh >> 1, lo = i < half ? i : i - half;
    return ((lo >> 3) << 4) + ((i < half ? 0 : 1) << 3) + (lo & 7);
}
// canonical fused QKV column (head-major, natural order inside a head) -> packed column;
// v heads (columns from v_begin on) keep the natural order
__host__ __device__ inline int32_t qkv_col(int32_t c, int32_t Dh, int32_t v_begin) {
    if (c >= v_begin) return c;
    return (c / Dh) * Dh + head_col(c % Dh, Dh);
}

struct ModelMap {
    FusedMat qkv, o, gu, down;   // per layer, offsets relative to the layer base
    size_t g1_off, g2_off;       // per layer fp32 gains
    size_t layer_stride;         // bytes per layer
    size_t layers_off;           // byte offset of layer 0
    size_t emb_off;              // [V][d] row-major, model dtype
    FusedMat lm;                 // absolute offset
    size_t gf_off;
    size_t total;
};

// ------------------------------------------------------------------ device state block (int32 words)
struct StateMap {      // offsets in int32 words from the state base
    int32_t n, g, done, steps, newest, lastK, plen, olen, win, o, buf, out, prompt, flags, params;
    int32_t wseq;      // per-sequence window size [B]: 0 = the batch's window, else the smaller of the two
    int32_t rowb, rowj; // packed rows of a step with per-sequence windows: row m is slot rowj[m] of sequence rowb[m] [B * window]
    int32_t rstart;    // ... and sequence b's rows are rstart[b] .. rstart[b + 1] - 1 [B + 1]
    int32_t words;
};
enum { FLAG_ALL_DONE = 0, FLAG_ERROR = 1 };
enum { PARAM_MAX_NEW = 0, PARAM_EOS = 1, PARAM_MAX_STEPS = 2, PARAM_BUF_LEN = 3, PARAM_B = 4 };

// Row layout of a pass.  Dense (all three NULL): row m = slot m % W of sequence m / W.  Packed (a step whose
// sequences have windows of their own, Sec. 5.4 Time Composition): sequence b contributes only its own W_b rows;
// row m belongs to sequence rowb[m], slot rowj[m], and the rows of sequence b start at rstart[b].
struct RowMap { const int32_t* rowb; const int32_t* rowj; const int32_t* rstart; };

struct WorkspaceMap {
    size_t kc, vc;              // KV cache [L][B][Hkv][planes][S/32 blocks][32 * Dh] in fragment order (k_index, v_index)
    size_t rope_cos, rope_sin;  // fp32 [S][Dh/2]
    size_t x, nx, qkv, qrot, att, gu, h, logits, topv;
    size_t gemm_part, gemm_cnt, attn_part, attn_cnt, amax_part;
    size_t state;
    size_t total;
    size_t gemm_part_bytes, attn_part_bytes;
    StateMap st;
};

struct KernelDims {    // model + capacities as the kernels need them
    int32_t L, d, H, Hkv, Dh, F, V, B, S, W, M;   // W = rows per sequence of a pass (the window, or a prefill chunk), M = rows of a pass
    int32_t Wcap;      // most rows per sequence any pass may have (the workspace is sized for B * Wcap rows)
    int32_t qkvN;      // (H + 2 Hkv) * Dh
    float eps;
    int32_t esz;       // bytes per weight / cache element
    int32_t kvp;       // cached value: 1 = one plane (fp32 models: fp32; bf16 models: plain bf16), 2 = bf16 hi + bf16 lo planes,
                       // 3 = bf16 hi plane + a plane of 8-bit residuals (kv24_split), kept in the space of two planes
    int32_t actq;      // precision study: bit g set = GEMM g (QKV, O, gate/up, down, LM head) takes its activations as plain bf16
    int32_t kvq;       // precision study: kv_round mode of K (bits 0..3) and of V (bits 4..7) before a value is cached; 0 = off
};

// element offset of plane 0 of one (layer, sequence, kv head) block of the K or V cache; plane p
// follows at p * S * Dh.  Inside a plane both caches are cut into blocks of 32 positions (32 * Dh
// elements), and a block is stored in the order in which the attention kernel's MFMA A-operand
// fragments want it, so that every 16-byte-per-lane load of a wave reads one contiguous kilobyte
// (whole cache lines) instead of 64 pieces of 16 bytes:
//  K: eight fragments (t, s), t = score tile (rows r <-> position 8*(r/4) + 4*t + r%4 of the block),
//     s = which eight of each 32 head elements; lane = r + 16 * (dh / 32), element dh % 8.
//  V (transposed): Dh/16 fragments of 16 head elements; lane = dh % 16 + 16 * (position / 8), element
//     position % 8.
// S is a multiple of 32 and Dh a multiple of 32.
__host__ __device__ inline int kv_alloc_planes(int kvp) { return kvp == 3 ? 2 : kvp; }   // planes of S * Dh elements a block occupies
__host__ __device__ inline size_t kv_block(const KernelDims& kd, int layer, int b, int kh) {
    return ((((size_t)layer * kd.B + b) * kd.Hkv + kh) * (size_t)kv_alloc_planes(kd.kvp)) * (size_t)kd.S * kd.Dh;
}
__host__ __device__ inline size_t k_index(int pos, int dh, int Dh) {
    const int kk = pos & 31, t = (kk >> 2) & 1, r = 4 * (kk >> 3) + (kk & 3);
    const int G = Dh >> 5, s = (dh & 31) >> 3, lane = r + 16 * (dh >> 5);
    return (size_t)(pos >> 5) * 32 * Dh + (size_t)((t * 4 + s) * 16 * G + lane) * 8 + (dh & 7);
}
__host__ __device__ inline size_t v_index(int dh, int pos, int Dh) {
    const int kk = pos & 31;
    return (size_t)(pos >> 5) * 32 * Dh + (size_t)((dh >> 4) * 64 + (dh & 15) + 16 * (kk >> 3)) * 8 + (kk & 7);
}

int fc_build_maps(const fastcot_config* cfg, ModelMap* mm, WorkspaceMap* wm, KernelDims* kd);

#define FC_ALIGN(x) (((x) + 255) & ~(size_t)255)
