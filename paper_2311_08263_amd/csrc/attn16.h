// Argument block and launcher of the matrix-core window-causal attention (see attn16.hip).
#pragma once
#include "fast.h"

struct AttnArgs {
    const float* q;        // rotated queries fp32, row (b*W + j), head h at column h*128
    int32_t ldq;
    const bf16_t* kc;      // K cache [L][B][Hkv][planes][S][128]: bf16 hi plane, optional bf16 lo plane
    const bf16_t* vc;      // V cache, transposed [L][B][Hkv][planes][128][S]
    int32_t layer, B, H, Hkv, S, W, kvp;
    const int32_t* n_state;   // committed length per sequence
    const int32_t* rstart;    // packed rows (per-sequence windows): sequence b owns rows rstart[b] .. rstart[b + 1] - 1 and W is the
                              // largest window; NULL = dense, W rows per sequence at b * W
    float* out;            // [rows][ldo], head h at column h*128 (may be NULL when ofrag is given)
    int32_t ldo;
    int32_t subrows;       // rows per workgroup: 0 = 32 where the window has more than 16 rows (two query tiles per workgroup),
                           // 16 = always one query tile (windows of 17..32 rows as two units that read K/V separately)
    bf16_t* ofrag;         // not NULL: the output also as bf16 hi + lo B-fragments [row tile][H*128/32][hi|lo][64][8],
                           // the layout the many-row O projection reads
    float* part;           // split partials
    int32_t* cnt;          // one arrival counter per (sequence, head), zero between launches
    int32_t bpw;           // key blocks (of 32) per workgroup that decide how many of the launched splits are used
};

size_t fc_attn16_part_bytes(int BH, int nsplit, int W);
// many query rows per sequence (attnp.hip): workgroups of 128 rows x one head that walk the keys once; uses q, kc,
// vc, layer, B, H, Hkv, S, W, kvp (1 or 2), n_state, out, ldo, ofrag of the argument block
int fc_attnp_workgroups(int Bact, int H, int W);
hipError_t fc_attnp(const AttnArgs& a, int Bact, hipStream_t st);
hipError_t fc_attn16(const AttnArgs& a, int Bact, int nsplit, hipStream_t st);
