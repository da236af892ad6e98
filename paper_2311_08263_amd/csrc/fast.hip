// MFMA forward path for bf16 models: per layer five launches (QKV+RoPE+cache write, attention,
// O-proj+residual, gate/up+SwiGLU, down+residual), then the LM head with fused argmax.
#include <string.h>
#include "kernels.h"
#include "attn16.h"
#include "gemmco.h"
#include "gemm256.h"

enum { KK_EMBED = 0, KK_QKV = 2, KK_ATTN = 4, KK_O = 5, KK_GU = 6, KK_DOWN = 8, KK_LM = 9, KK_ARGMAX = 10 };

bool fc_fast_supported(const KernelDims& kd, int rows) {
    return kd.esz == 2 && kd.Dh == 128 && rows >= 1 && kd.d % 256 == 0 && kd.F % 256 == 0 &&
           (kd.H * kd.Dh) % 256 == 0 && kd.S % 32 == 0 && kd.V % 16 == 0;
}

// inputs (K) of GEMM i: QKV, O, gate/up, down, LM head
static int kin0(const KernelDims& kd, int i) { return i == 1 ? kd.H * kd.Dh : (i == 3 ? kd.F : kd.d); }

void fc_fast_plan(const KernelDims& kd, FastPlan* p) {
    memset(p, 0, sizeof(*p));
    // at most 8 key splits: the last workgroup to arrive folds up to 8 partial results in one round of loads
    // (measured at 2050 positions, 32 heads: 8 splits 24 us, 12 splits 32 us; at 350 positions 6 splits of 2
    // key blocks 12.7 us, 3 splits of 4 blocks 14.9 us)
    int nb = (kd.S + 31) / 32, sp = (nb + 1) / 2;
    if (sp > 8) sp = 8;
    // and no more workgroups than CUs: the kernel's register budget allows one workgroup per CU, a second
    // round costs more than the split saves (measured: 64 heads, 600 positions: 4 splits 20.6 us, 8 splits
    // 24.3 us; batch 8 x 40 heads: 1 split 75 us, 2 splits 102 us)
    while (sp > 1 && kd.B * kd.H * sp > fc_num_cus()) --sp;
    p->attn_splits = sp < 1 ? 1 : sp;
    p->attn_bpw = 2;
    p->attn_many = 1;
    // column-owner kernel: workgroups per GEMM (one per CU where the matrix allows)
    const int nts[5] = {kd.qkvN / 16, kd.d / 16, 2 * kd.F / 16, kd.d / 16, kd.V / 16};
    // measured on the 7B shape: one workgroup per CU
    for (int i = 0; i < 5; ++i) { p->nw[i] = fc_gemmco_grid(nts[i]); p->ks[i] = 1; }
    if (nts[1] < 512) {                  // O projection with fewer than two n-tiles per CU
        // measured at the 7B shape: two K slices per owner (16.6 us against 17.6 us for one)
        const int G = p->nw[1], K = kd.H * kd.Dh;
        if (G % 2 == 0 && G / 2 <= nts[1] && (nts[1] + G / 2 - 1) / (G / 2) <= 8 && K >= 2048) p->ks[1] = 2;
    }
    // down projection: K is long and the columns few, so every workgroup would read far more activation
    // bytes than weight bytes; K slices per owner cut that (measured at the 7B shape)
    if (kd.F >= 2 * kd.d && kd.F >= 4096 && p->nw[3] % 4 == 0 && p->nw[3] / 4 <= nts[3] && (nts[3] + p->nw[3] / 4 - 1) / (p->nw[3] / 4) <= 8) p->ks[3] = 4;
    p->co_single = 2;    // measured (7B and 70B shapes): down and LM head 2-4 % faster with two batches in flight, QKV and O slower
    for (int i = 0; i < 5; ++i) { p->co_sb[0][i] = !(i == 3 || i == 4); p->co_sb[1][i] = 0; p->co_rot[0][i] = i >= 2; p->co_rot[1][i] = 1; }
    // Measured per shape (steps of up to 16 rows, every combination of K slices per owner x batch order x batches
    // in flight timed on the shape's own matrices, the fastest recorded here): {K slices, rotated order, batches in
    // flight} for QKV, O, gate/up, down, LM head.  Everything that fixes the order of the fp32 additions comes from
    // this table or the rules above, never from a timing at run time, so that every process computes the same bits.
    // The second triple is the same for steps of 17..32 rows (measured at 32 rows; 0 K slices = derived from the
    // first triple as below): 7B QKV 33.5 -> 31.7 us, O 20.4 -> 16.9 us, down 31.0 -> 29.4 us; 70B gate/up 183.9 -> 171.9 us.
    struct Row { int d, F, H, Hkv; int ks[5], rot[5], sb[5]; int ks2[5], rot2[5], sb2[5]; };
    static const Row table[] = {
        {4096, 11008, 32, 32, {1, 2, 1, 8, 1}, {0, 0, 1, 1, 1}, {2, 2, 1, 0, 0}, {1, 4, 1, 4, 1}, {1, 1, 1, 1, 1}, {1, 0, 0, 0, 0}},      // Llama-2-7B shape
        {5120, 13824, 40, 40, {1, 4, 1, 4, 1}, {1, 0, 1, 1, 1}, {0, 1, 0, 1, 0}, {0, 0, 0, 0, 0}, {1, 1, 1, 1, 1}, {0, 0, 0, 0, 0}},      // 13B shape
        {8192, 28672, 64, 8, {2, 4, 1, 4, 1}, {1, 1, 0, 1, 1}, {1, 1, 0, 0, 0}, {0, 2, 0, 0, 0}, {1, 1, 0, 1, 1}, {0, 0, 0, 0, 0}},       // 70B shape
    };
    const Row* mine = nullptr;
    for (const Row& r : table) {
        if (r.d != kd.d || r.F != kd.F || r.H != kd.H || r.Hkv != kd.Hkv || kd.Dh != 128) continue;
        for (int i = 0; i < 5; ++i) {
            const int G = p->nw[i], ks = r.ks[i], own = G / ks;
            if (G % ks == 0 && own >= 1 && own <= nts[i] && (nts[i] + own - 1) / own <= 12 && kin0(kd, i) / 256 >= ks) p->ks[i] = ks;
            p->co_rot[0][i] = r.rot[i]; p->co_sb[0][i] = r.sb[i];
            p->co_rot[1][i] = r.rot2[i]; p->co_sb[1][i] = r.sb2[i];
        }
        mine = &r;
    }
    // 17..32 rows (two row tiles per workgroup, up to 16 output tiles): the same grids where the partial tiles
    // fit the LDS, K slices halved until they divide the grid
    const int kin[5] = {kd.d, kd.H * kd.Dh, kd.d, kd.F, kd.d};
    const bool gained[5] = {true, false, true, false, true};
    for (int i = 0; i < 5; ++i) {
        const int most = fc_gemmco_most(32, kin[i], gained[i]);
        int G2 = p->nw[i];
        const int own = G2 > 0 ? G2 / p->ks[i] : 0;
        if (own < 1 || (nts[i] + own - 1) / own > most) G2 = fc_gemmco_grid(nts[i], most);
        int k2 = p->ks[i];
        while (k2 > 1 && (G2 % k2 || G2 / k2 > nts[i] || (nts[i] + G2 / k2 - 1) / (G2 / k2) > most)) k2 >>= 1;
        const int kt = mine ? mine->ks2[i] : 0;          // the table's own value for this class, where it fits
        if (kt >= 1 && i < 4 && G2 % kt == 0 && G2 / kt >= 1 && G2 / kt <= nts[i] && (nts[i] + G2 / kt - 1) / (G2 / kt) <= most && kin[i] / 256 >= kt) k2 = kt;
        p->nw2[i] = G2; p->ks2[i] = k2;
    }
}

// Layout of the many-row (more than 32 rows) part of the GEMM scratch, offsets in bytes
struct ManyRowScratch { size_t af_x, af_att, af_h, ssq, part, end; };
static ManyRowScratch many_row_scratch(const KernelDims& kd) {
    auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
    ManyRowScratch m;
    const size_t MP = (size_t)((kd.M + 15) / 16) * 16;
    m.af_x = 0;
    m.af_att = m.af_x + up(fc_split_bytes(kd.M, kd.d));
    m.af_h = m.af_att + up(fc_split_bytes(kd.M, kd.H * kd.Dh));
    m.ssq = m.af_h + up(fc_split_bytes(kd.M, kd.F));
    m.part = m.ssq + up((size_t)(kd.d / 256 + 1) * MP * 4);
    m.end = m.part + (size_t)FC_GEMM256_MAX_SK * kd.M * kd.d * 4;
    return m;
}

void fc_fast_scratch_sizes(const KernelDims& kd, size_t* gemm_part_bytes, size_t* attn_part_bytes) {
    // column-owner kernel with K slices per owner: per workgroup up to 16 partial tiles of 1 KB and 32 partial row
    // sums; at most as many workgroups as the widest matrix has n-tiles
    int nmax = 2 * kd.F;
    if (kd.qkvN > nmax) nmax = kd.qkvN;
    if (kd.V > nmax) nmax = kd.V;
    *gemm_part_bytes = (size_t)(nmax / 16 + 1) * (16 * 1024 + 32 * 4) + 4096;
    // many-row path: activation fragments, row statistics and split-K partial tiles live in the same scratch
    const size_t big = many_row_scratch(kd).end + 4096;
    if (*gemm_part_bytes < big) *gemm_part_bytes = big;
    *attn_part_bytes = fc_attn16_part_bytes(kd.B * kd.H, FC_MAX_ATTN_SPLITS, kd.Wcap > kd.W ? kd.Wcap : kd.W) + 4096;
}

#define FLAUNCH(kind, call)                                                          \
    do {                                                                             \
        hipError_t e_;                                                               \
        if (a.prof && (e_ = a.prof_mark(a.prof, kind)) != hipSuccess) return e_;     \
        if ((e_ = (call)) != hipSuccess) return e_;                                  \
        if (a.prof && (e_ = a.prof_mark(a.prof, -1)) != hipSuccess) return e_;       \
    } while (0)

hipError_t fc_fast_forward(const FastArgs& a) {
    const KernelDims& kd = a.kd;
    const ModelMap& mm = *a.mm; const WorkspaceMap& wm = *a.wm;
    const int M = kd.M, d = kd.d, qd = kd.H * kd.Dh;
    char* ws = a.ws; const char* wt = a.weights;
    int32_t* stp = (int32_t*)(ws + wm.state);
    float* x = (float*)(ws + wm.x); float* q = (float*)(ws + wm.qkv); float* att = (float*)(ws + wm.att);
    float* h = (float*)(ws + wm.h);
    struct { const int32_t* n_state; const float* cosT; const float* sinT; bf16_t* kc; bf16_t* vc; float* amax_val; int layer; } g;
    g.n_state = stp + wm.st.n; g.cosT = (const float*)(ws + wm.rope_cos); g.sinT = (const float*)(ws + wm.rope_sin);
    g.kc = (bf16_t*)(ws + wm.kc); g.vc = (bf16_t*)(ws + wm.vc);
    g.amax_val = (float*)(ws + wm.amax_part); g.layer = 0;
    AttnArgs at; memset(&at, 0, sizeof(at));
    at.q = q; at.ldq = qd; at.kc = g.kc; at.vc = g.vc; at.B = kd.B; at.H = kd.H; at.Hkv = kd.Hkv; at.S = kd.S; at.W = kd.W; at.kvp = kd.kvp;
    at.rstart = a.rm.rstart;
    at.n_state = g.n_state; at.out = att; at.ldo = qd; at.part = (float*)(ws + wm.attn_part); at.cnt = (int32_t*)(ws + wm.attn_cnt); at.bpw = a.plan->attn_bpw;

    GemmCoArgs co; memset(&co, 0, sizeof(co));
    co.M = M; co.eps = kd.eps; co.n_state = g.n_state; co.cosT = g.cosT; co.sinT = g.sinT; co.kc = g.kc; co.vc = g.vc;
    co.H = kd.H; co.Hkv = kd.Hkv; co.B = kd.B; co.S = kd.S; co.Wn = kd.W; co.kvp = kd.kvp; co.kvq = kd.kvq;
    co.amax_val = g.amax_val; co.single_buffer = 1; co.rm = a.rm;
    Gemm256Args big; memset(&big, 0, sizeof(big));
    big.M = M; big.n_state = g.n_state; big.cosT = g.cosT; big.sinT = g.sinT; big.kc = g.kc; big.vc = g.vc;
    big.H = kd.H; big.Hkv = kd.Hkv; big.B = kd.B; big.S = kd.S; big.Wn = kd.W; big.kvp = kd.kvp; big.kvq = kd.kvq;
    big.amax_stride = (M + 15) / 16 * 16; big.rm = a.rm;
    // many-row scratch: the fragments of x, of the attention output and of the hidden activations, the partial
    // row sums of squares of x, then the split-K partial tiles
    const ManyRowScratch mrs = many_row_scratch(kd);
    bf16_t* af_x = (bf16_t*)(ws + wm.gemm_part + mrs.af_x); bf16_t* af_att = (bf16_t*)(ws + wm.gemm_part + mrs.af_att);
    bf16_t* af_h = (bf16_t*)(ws + wm.gemm_part + mrs.af_h); float* ssq = (float*)(ws + wm.gemm_part + mrs.ssq);
    big.part = (float*)(ws + wm.gemm_part + mrs.part);
    big.eps = kd.eps;
    // which fragment buffers hold what their fp32 twin would: x (with the gain of the norm that comes next, row
    // scale still to be applied by the consumer), attention output, hidden activations
    bool x_frag = false, att_frag = false, h_frag = false;
    const float* next_gain = nullptr;          // gain the next reduction folds into the fragments of x
    // LM head: one winner per row and column block (16, 8 or 4 n-tiles)
    const int lm_cw = fc_gemm256_cw(EPI_LMHEAD, M, kd.V / 16);
    const int lm_cols = (fc_gemm256_mode(EPI_LMHEAD, M, d, kd.V / 16, 1, lm_cw) == 3 ? 8 : 4) * lm_cw;
    const int lm_ncb = (kd.V / 16 + lm_cols - 1) / lm_cols;
    big.amax_val = g.amax_val; big.amax_idx = (int32_t*)(g.amax_val + (size_t)lm_ncb * big.amax_stride);
    int gi = 0;        // which GEMM of the plan
    auto gemm = [&](int epi, const void* W, int K, int N, const float* X, int ldx, const float* gain,
                    float* out, int ldo) {
        // workgroups of the column-owner kernel and its K slices per owner
        const int nw = M <= 16 ? a.plan->nw[gi] : (M <= 32 ? a.plan->nw2[gi] : 0);
        const int ksl = a.tune_gi >= 0 ? a.tune_ks : (M <= 16 ? a.plan->ks[gi] : a.plan->ks2[gi]);
        if (nw > 0) {
            co.W = (const bf16_t*)W; co.K = K; co.NT = N / 16; co.X = X; co.ldx = ldx; co.gain = gain; co.out = out; co.ldo = ldo;
            co.layer = g.layer; co.ks = epi != EPI_LMHEAD ? ksl : 1; co.hi_only = (kd.actq >> gi) & 1;
            // one or two weight batches in flight per wave: which is faster depends on the GEMM and on the shape
            // (7B: two for down and LM head; 13B: two for QKV and gate/up, one for down), so it is a plan entry
            co.single_buffer = a.tune_gi >= 0 ? a.tune_sb : (a.plan->co_single == 2 ? a.plan->co_sb[M > 16][gi] : a.plan->co_single);
            co.rotate = a.tune_gi >= 0 ? a.tune_rot : a.plan->co_rot[M > 16][gi];
            co.xpart = (float*)(ws + wm.gemm_part); co.xcnt = (int32_t*)(ws + wm.gemm_cnt);
            co.amax_idx = (int32_t*)(co.amax_val + (size_t)nw * (M > 16 ? 32 : 16));
            return fc_gemmco(epi, co, nw, a.st);
        }
        if (M > 32) {        // matrix-core bound: activations split once, tiles of 64 rows x 256 columns
            // the input: fragments a producer has already written (x after a fused reduction, attention output,
            // hidden activations), else split here (RMSNorm included)
            bf16_t* af = X == x ? af_x : (X == att ? af_att : af_h);
            const bool ready = X == x ? x_frag : (X == att ? att_frag : h_frag);
            big.ssq = nullptr; big.nssq = 0;
            if (!ready) {
                hipError_t e = fc_split(X, ldx, M, K, gain, kd.eps, af, a.st);
                if (e != hipSuccess) return e;
            } else if (X == x) { big.ssq = ssq; big.nssq = d / 256; }
            big.sk = epi == EPI_RESID ? fc_gemm256_sk(M, K, N / 16) : 1;
            big.W = (const bf16_t*)W; big.K = K; big.NT = N / 16; big.AF = af; big.out = out; big.ldo = ldo; big.layer = g.layer;
            big.hfrag = nullptr; big.rf_AF = nullptr; big.rf_gain = nullptr; big.rf_ssq = nullptr;
            if (epi == EPI_SWIGLU) {            // the hidden activations leave as fragments (fp32 copy only for debugging)
                big.hfrag = af_h; h_frag = true;
                if (a.dbg_stop < 0) big.out = nullptr;
            }
            if (epi == EPI_RESID) {
                x_frag = big.sk > 1 && d % 256 == 0 && next_gain != nullptr;
                if (x_frag) { big.rf_AF = af_x; big.rf_gain = next_gain; big.rf_ssq = ssq; }
            }
            return fc_gemm256(epi, big, a.st);
        }
        return hipErrorInvalidValue;       // every plan gives the column-owner kernel a grid
    };

    if (a.tune_gi >= 0) {            // timing run of one GEMM (layer 0 weights, whatever the buffers hold)
        const char* lb = wt + mm.layers_off;
        g.layer = 0; gi = a.tune_gi;
        switch (gi) {
            case 0: return gemm(EPI_QKV, lb + mm.qkv.off, d, kd.qkvN, x, d, (const float*)(lb + mm.g1_off), q, qd);
            case 1: return gemm(EPI_RESID, lb + mm.o.off, qd, d, att, qd, nullptr, x, d);
            case 2: return gemm(EPI_SWIGLU, lb + mm.gu.off, d, 2 * kd.F, x, d, (const float*)(lb + mm.g2_off), h, kd.F);
            case 3: return gemm(EPI_RESID, lb + mm.down.off, kd.F, d, h, kd.F, nullptr, x, d);
            case 4: return gemm(EPI_LMHEAD, wt + mm.lm.off, d, kd.V, x, d, (const float*)(wt + mm.gf_off), nullptr, kd.V);
        }
        return hipErrorInvalidValue;
    }
    FLAUNCH(KK_EMBED, fc_embed(wt + mm.emb_off, FASTCOT_BF16, stp + wm.st.win, x, M, d, kd.V, a.st, a.rm, kd.W));
    int nstage = 0;
#define DBG_STOP() do { if (a.dbg_stop >= 0 && nstage++ >= a.dbg_stop) return hipSuccess; } while (0)
    for (int l = 0; l < kd.L; ++l) {
        const char* lb = wt + mm.layers_off + (size_t)l * mm.layer_stride;
        g.layer = l; at.layer = l;
        DBG_STOP();
        gi = 0;
        FLAUNCH(KK_QKV, gemm(EPI_QKV, lb + mm.qkv.off, d, kd.qkvN, x, d, (const float*)(lb + mm.g1_off), q, qd));
        DBG_STOP();
        if (M > 32) {                  // the many-row O projection reads fragments: attention writes them itself
            at.ofrag = af_att; att_frag = true;
            at.out = a.dbg_stop >= 0 ? att : nullptr;
        }
        // windows of more than 16 rows at a small batch: workgroups of one query tile each instead of two
        // (they read K/V twice, which costs nothing while the launch is latency-bound: 7B, 32 rows, 17.4 -> 13.9 us)
        int attn_splits = a.plan->attn_splits;
        at.subrows = 0;
        const int units16 = (kd.W + 15) / 16;
        if (kd.W > 16 && a.Bact * kd.H * units16 <= fc_num_cus() && kd.S <= 8192) {   // (long caches: K/V traffic counts)
            at.subrows = 16;
            while (attn_splits > 1 && a.Bact * kd.H * units16 * attn_splits > fc_num_cus()) --attn_splits;
        }
        // passes with many rows per sequence (prompt chunks): one walk over the keys per 128 rows, where that
        // still gives at least half of the CUs a workgroup
        const bool many = a.plan->attn_many == 2 ? kd.W > 32
                                                  : (a.plan->attn_many == 1 && kd.W >= 64 && 2 * fc_attnp_workgroups(a.Bact, kd.H, kd.W) >= fc_num_cus());
        if (many && kd.kvp != 3)
            FLAUNCH(KK_ATTN, fc_attnp(at, a.Bact, a.st));
        else
        FLAUNCH(KK_ATTN, fc_attn16(at, a.Bact, attn_splits, a.st));
        DBG_STOP();
        gi = 1;
        next_gain = (const float*)(lb + mm.g2_off);
        FLAUNCH(KK_O, gemm(EPI_RESID, lb + mm.o.off, qd, d, att, qd, nullptr, x, d));
        DBG_STOP();
        gi = 2;
        FLAUNCH(KK_GU, gemm(EPI_SWIGLU, lb + mm.gu.off, d, 2 * kd.F, x, d, (const float*)(lb + mm.g2_off), h, kd.F));
        DBG_STOP();
        gi = 3;
        next_gain = l + 1 < kd.L ? (const float*)(wt + mm.layers_off + (size_t)(l + 1) * mm.layer_stride + mm.g1_off) : (const float*)(wt + mm.gf_off);
        FLAUNCH(KK_DOWN, gemm(EPI_RESID, lb + mm.down.off, kd.F, d, h, kd.F, nullptr, x, d));
    }
    if (a.dbg_stop >= 0 && nstage >= a.dbg_stop) return hipSuccess;
    if (a.lmhead) {
        const int stride = M > 16 ? 32 : 16;
        const int nwlm = M <= 16 ? a.plan->nw[4] : (M <= 32 ? a.plan->nw2[4] : 0);
        const int nwin = nwlm;                                // partial winners to reduce
        gi = 4;
        FLAUNCH(KK_LM, gemm(EPI_LMHEAD, wt + mm.lm.off, d, kd.V, x, d, (const float*)(wt + mm.gf_off), a.dbg_logits, kd.V));
        if (M <= 32)
            FLAUNCH(KK_ARGMAX, fc_argmax_final(g.amax_val, (const int32_t*)(g.amax_val + (size_t)nwin * stride), nwin, stride, M, stp + wm.st.o,
                                               (float*)(ws + wm.topv), a.st, a.rm, kd.W));
        else
            FLAUNCH(KK_ARGMAX, fc_argmax_final(big.amax_val, big.amax_idx, lm_ncb, big.amax_stride, M,
                                               stp + wm.st.o, (float*)(ws + wm.topv), a.st, a.rm, kd.W));
    }
    return hipSuccess;
}

hipError_t fc_fast_tune(FastArgs a, FastPlan* plan) {
    const int M = a.kd.M;
    if (M < 1 || M > 32) return hipSuccess;
    const int cls = M > 16;
    a.prof = nullptr; a.prof_mark = nullptr; a.dbg_stop = -1; a.plan = plan;
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    if ((e = hipEventCreate(&e1)) != hipSuccess) { (void)hipEventDestroy(e0); return e; }
    // mean of 5 launches after 2 untimed ones; hipErrorInvalidValue from the first launch = the launcher
    // rejected the combination (nothing ran)
    auto measure = [&](float* ms) -> hipError_t {
        hipError_t r = fc_fast_forward(a);
        if (r != hipSuccess) return r;
        r = fc_fast_forward(a);
        if (r == hipSuccess) r = hipEventRecord(e0, a.st);
        for (int i = 0; i < 5 && r == hipSuccess; ++i) r = fc_fast_forward(a);
        if (r == hipSuccess) r = hipEventRecord(e1, a.st);
        if (r == hipSuccess) r = hipEventSynchronize(e1);
        if (r == hipSuccess) r = hipEventElapsedTime(ms, e0, e1);
        return r;
    };
    // Only the number of weight batches in flight is measured, and only for the GEMMs that walk their batches in
    // plain order: there it changes when loads are issued, never the order in which a wave adds its k-tiles, so
    // every choice gives the same bits.  The K slices per owner and the batch order do change the order of the
    // fp32 additions, and so does the batch size of a GEMM that walks its batches in rotated order: all of those
    // stay as fc_fast_plan fixed them from the shape.  Two processes therefore compute identical logits whatever
    // their timings were.
    for (int gi = 0; gi < 5 && e == hipSuccess; ++gi) {
        const int nw = cls ? plan->nw2[gi] : plan->nw[gi];
        if (nw <= 0) continue;                      // not a column-owner launch
        float best = 1e30f;
        int best_sb = plan->co_sb[cls][gi];
        const int rot = plan->co_rot[cls][gi], ks = cls ? plan->ks2[gi] : plan->ks[gi];
        if (rot) continue;
        a.tune_gi = gi; a.tune_ks = ks; a.tune_rot = rot;
        for (int sb = 0; sb < 3 && e == hipSuccess; ++sb) {      // two batches, one batch, the whole slice at once
            a.tune_sb = sb;
            float t = 1e30f;
            for (int rep = 0; rep < 3 && e == hipSuccess; ++rep) {
                float ms = 0.f;
                const hipError_t r = measure(&ms);
                if (r == hipErrorInvalidValue) { t = 1e30f; break; }
                e = r;
                if (e == hipSuccess && ms < t) t = ms;
            }
            if (e == hipSuccess && t < best) { best = t; best_sb = sb; }
        }
        if (e == hipSuccess) plan->co_sb[cls][gi] = best_sb;
    }
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    return e;
}

// ------------------------------------------------------------------ isolation launchers
__global__ void k_set_i32(int32_t* p, int32_t v) { if (threadIdx.x == 0) *p = v; }

static int iso_attn_splits(int S) {
    int nb = (S + 31) / 32, sp = (nb + 1) / 2;
    return sp < 1 ? 1 : (sp > 8 ? 8 : sp);
}
// scratch: [0,256) the committed length; [256, 256+4*H) counters; then split partials
size_t fc_attn_iso_scratch_bytes(int W, int H, int Dh) {
    return 256 + (((size_t)H * 4 + 255) & ~(size_t)255) + fc_attn16_part_bytes(H, FC_MAX_ATTN_SPLITS, W);
}
hipError_t fc_attn_iso(const float* q, const void* kc, const void* vc, int n, int W, int H, int Hkv, int Dh, int S,
                       int dt, float* out, void* scratch, hipStream_t st) {
    char* sc = (char*)scratch;
    k_set_i32<<<1, 64, 0, st>>>((int32_t*)sc, n);
    if (dt != FASTCOT_BF16 || Dh != 128 || W > 32 || S % 32 || H > FC_MAX_COUNTERS) {
        KernelDims kd{}; kd.L = 1; kd.H = H; kd.Hkv = Hkv; kd.Dh = Dh; kd.B = 1; kd.S = S; kd.W = W; kd.M = W; kd.kvp = 1;
        return fc_attn_plain(q, H * Dh, kc, vc, dt, kd, 0, (const int32_t*)sc, out, st);
    }
    AttnArgs at; memset(&at, 0, sizeof(at));
    at.q = q; at.ldq = H * 128; at.kc = (const bf16_t*)kc; at.vc = (const bf16_t*)vc; at.layer = 0; at.B = 1; at.H = H;
    at.Hkv = Hkv; at.S = S; at.W = W; at.kvp = 1; at.n_state = (const int32_t*)sc; at.out = out; at.ldo = H * 128;
    at.cnt = (int32_t*)(sc + 256); at.bpw = 2;
    at.part = (float*)(sc + 256 + (((size_t)H * 4 + 255) & ~(size_t)255));
    return fc_attn16(at, 1, iso_attn_splits(n + W), st);
}

// scratch: winners per workgroup [workgroups][32] value + index, then room for logits (plain path only)
static int lm_iso_grid(int M, int d, int V) { return fc_gemmco_grid(V / 16, M > 16 ? fc_gemmco_most(32, d, false) : 8); }
size_t fc_lmhead_iso_scratch_bytes(int M, int d, int V) {
    const size_t G = (size_t)(V / 16 + 1);
    return G * 32 * 8 + 256 + (size_t)M * V * 4;
}
// largest logit of every row among the ids other than the row's winner
__global__ void k_top2(const float* logits, int V, const int32_t* ids, float* top2) {
    __shared__ float sv[4];
    const int m = blockIdx.x, win = ids[m];
    float best = -3.0e38f;
    for (int n = threadIdx.x; n < V; n += blockDim.x) { const float v = logits[(size_t)m * V + n]; if (n != win && v > best) best = v; }
    for (int o = 32; o > 0; o >>= 1) best = fmaxf(best, __shfl_xor(best, o, 64));
    if ((threadIdx.x & 63) == 0) sv[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) top2[m] = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
}
hipError_t fc_lmhead_iso(const float* act, const void* packed, int M, int d, int V, int32_t* ids, float* top, float* top2,
                         float* logits, void* scratch, hipStream_t st) {
    char* sc = (char*)scratch;
    float* lg_scratch = (float*)(sc + (size_t)(V / 16 + 1) * 32 * 8 + 256);
    if (top2 && !logits) logits = lg_scratch;              // the runner-up is read off the logits
    if (M > 32 || d % 256) {
        float* lg = logits ? logits : lg_scratch;
        hipError_t e = fc_gemm_plain(packed, FASTCOT_BF16, d, V, V, act, d, lg, V, M, 0, st);
        if (e != hipSuccess) return e;
        e = fc_argmax_plain(lg, M, V, ids, top, st);
        if (e != hipSuccess || !top2) return e;
        k_top2<<<M, 256, 0, st>>>(lg, V, ids, top2);
        return hipGetLastError();
    }
    GemmCoArgs co; memset(&co, 0, sizeof(co));
    const int nwg = lm_iso_grid(M, d, V), stride = M > 16 ? 32 : 16;
    co.W = (const bf16_t*)packed; co.K = d; co.NT = V / 16; co.X = act; co.ldx = d; co.M = M; co.out = logits; co.ldo = V;
    co.single_buffer = 1;
    co.amax_val = (float*)sc;
    co.amax_idx = (int32_t*)(co.amax_val + (size_t)nwg * stride);
    hipError_t e = fc_gemmco(EPI_LMHEAD, co, nwg, st);
    if (e != hipSuccess) return e;
    e = fc_argmax_final(co.amax_val, co.amax_idx, nwg, stride, M, ids, top, st);
    if (e != hipSuccess || !top2) return e;
    k_top2<<<M, 256, 0, st>>>(logits, V, ids, top2);
    return hipGetLastError();
}
