// C ABI of the FastCoT gfx950 library: context, weight packing, prefill, Jacobi step, generate.
// The host code here only sequences kernel launches; every step of the decoding path (forward,
// argmax, verification, acceptance, commit, window shift) runs in device kernels.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <vector>
#include "kernels.h"
#include "fast.h"

static thread_local char g_err[512] = "";

struct fastcot_ctx {
    fastcot_config cfg;
    ModelMap mm;
    WorkspaceMap wm;
    KernelDims kd;
    const char* weights;
    char* ws;
    hipStream_t st;
    int Bact;            // sequences of the current run
    int prefilled, generated;
    int opt_compact;     // fastcot_generate moves finished sequences out of the way so that later steps run fewer rows
    int opt_tune;        // measure the plan's per-GEMM choices at prefill
    int tuned_rows[2];   // rows per step the plan's per-GEMM choices were last measured for (up to 16 / 17..32 rows)
    int last_eos;        // eos_id of the last fastcot_generate (-1 = none)
    int buf_len;
    int opt_plain, opt_graph, dbg_stop;
    int opt_packed;      // steps of sequences with windows of their own compute only those rows (MFMA path)
    int rows_dirty;      // the row map has to be rebuilt before the next step (windows, slots or the batch changed)
    int rows_step;       // rows of a packed step; 0 = dense
    float* dbg_logits;
    hipGraphExec_t graph_exec;
    hipGraph_t graph;
    int graph_valid;
    FastPlan plan;
    // profiling of single launches
    int prof_on;
    std::vector<hipEvent_t> prof_ev;
    std::vector<int> prof_kind;
    size_t prof_used;
    // step timing
    std::vector<hipEvent_t> step_ev;
    std::vector<float> step_ms;
    int32_t* pinned;     // small pinned host block for polling
    char err[512];
};

static int fail(fastcot_ctx* c, int code, const char* fmt, const char* a = "", long x = 0, long y = 0) {
    char* dst = c ? c->err : g_err;
    snprintf(dst, 512, fmt, a, x, y);
    if (c) snprintf(g_err, 512, "%s", dst);
    return code;
}
void fc_set_error(const char* msg) { snprintf(g_err, 512, "%s", msg); }
#define HIPCHK(c, call)                                                                          \
    do {                                                                                         \
        hipError_t e_ = (call);                                                                  \
        if (e_ != hipSuccess) return fail(c, FASTCOT_EHIP, "HIP error '%s' at line %ld", hipGetErrorString(e_), __LINE__); \
    } while (0)

static const char* kKernelNames[FASTCOT_N_KERNEL_KINDS] = {
    "embed", "rmsnorm", "gemm_qkv", "rope_cache", "attention", "gemm_o", "gemm_gate_up", "swiglu",
    "gemm_down", "lm_head", "argmax", "accept_commit", "attn_combine", "reserved13", "empty_kernel", "reserved15"};
enum { KK_EMBED = 0, KK_RMSNORM, KK_QKV, KK_ROPE, KK_ATTN, KK_O, KK_GU, KK_SWIGLU, KK_DOWN, KK_LM, KK_ARGMAX, KK_ACCEPT, KK_EMPTY = 14 };
__global__ void k_empty() {}

extern "C" const char* fastcot_kernel_name(int32_t kind) {
    return (kind >= 0 && kind < FASTCOT_N_KERNEL_KINDS) ? kKernelNames[kind] : "";
}
extern "C" const char* fastcot_last_error(const fastcot_ctx* ctx) { return ctx ? ctx->err : g_err; }

// ------------------------------------------------------------------ layout maps
// NULL if the configuration is usable, else what is wrong with it
static const char* cfg_problem(const fastcot_config* c) {
    if (!c) return "configuration is NULL";
    if (c->n_layers < 0 || c->d_model <= 0 || c->n_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 ||
        c->d_ffn <= 0 || c->vocab <= 0 || c->max_batch <= 0 || c->max_seq <= 0 || c->window <= 0) return "a dimension or capacity is not positive";
    if (c->dtype != FASTCOT_F32 && c->dtype != FASTCOT_BF16) return "dtype is neither FASTCOT_F32 nor FASTCOT_BF16";
    if (c->n_heads % c->n_kv_heads) return "n_heads is not a multiple of n_kv_heads";
    if (c->head_dim % 32 || c->d_model % 16 || c->d_ffn % 16 || c->vocab % 16) return "head_dim must be a multiple of 32; d_model, d_ffn and vocab multiples of 16";
    if (c->dtype == FASTCOT_BF16 && (c->d_model % 32 || c->d_ffn % 32 || (c->n_heads * c->head_dim) % 32)) return "bf16 models need d_model, d_ffn and n_heads*head_dim to be multiples of 32";
    if (c->max_seq > 16000) return "max_seq above 16000 positions is not supported";
    if (c->max_seq < 2 * c->window) return "max_seq must be at least 2*window";
    if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return "rms_eps must be >= 0 and rope_base > 0";
    return nullptr;
}
static int valid_cfg(const fastcot_config* c) { return cfg_problem(c) == nullptr; }

int fc_build_maps(const fastcot_config* c, ModelMap* mm, WorkspaceMap* wm, KernelDims* kd) {
    if (!valid_cfg(c)) return FASTCOT_EINVAL;
    const size_t esz = c->dtype == FASTCOT_F32 ? 4 : 2;
    const int d = c->d_model, qd = c->n_heads * c->head_dim, kvd = c->n_kv_heads * c->head_dim, F = c->d_ffn;
    auto fused = [&](size_t& cur, int K, int N) {
        FusedMat f; f.off = cur; f.K = K; f.N = N; f.NP = (N + 15) & ~15;
        cur = FC_ALIGN(cur + (size_t)K * f.NP * esz);
        return f;
    };
    if (mm) {
        size_t cur = 0;
        mm->qkv = fused(cur, d, qd + 2 * kvd);
        mm->o = fused(cur, qd, d);
        mm->gu = fused(cur, d, 2 * F);
        mm->down = fused(cur, F, d);
        mm->g1_off = cur; cur = FC_ALIGN(cur + (size_t)d * 4);
        mm->g2_off = cur; cur = FC_ALIGN(cur + (size_t)d * 4);
        mm->layer_stride = cur;
        size_t top = 0;
        mm->emb_off = top; top = FC_ALIGN(top + (size_t)c->vocab * d * esz);
        mm->lm = fused(top, d, c->vocab);
        mm->gf_off = top; top = FC_ALIGN(top + (size_t)d * 4);
        mm->layers_off = top;
        mm->total = top + (size_t)c->n_layers * mm->layer_stride;
    }
    KernelDims k;
    k.L = c->n_layers; k.d = d; k.H = c->n_heads; k.Hkv = c->n_kv_heads; k.Dh = c->head_dim; k.F = F;
    k.V = c->vocab; k.B = c->max_batch; k.S = (c->max_seq + 31) & ~31; k.W = c->window;
    k.qkvN = qd + 2 * kvd; k.eps = c->rms_eps; k.esz = (int)esz; k.kvp = c->dtype == FASTCOT_BF16 ? 2 : 1; k.kvq = 0; k.actq = 0;
    // prefill runs the same kernels over chunks of the prompt; where the matrix-core path covers the
    // shape a chunk is up to 1024 rows per sequence (at most 1024 rows in all), else one window
    k.Wcap = k.W; k.M = k.B * k.W;
    if (fc_fast_supported(k, k.M)) {
        int ch = 1024;
        while (ch > 32 && k.B * ch > 1024) ch >>= 1;
        if (ch > k.S) ch = k.S;
        if (ch > k.Wcap) k.Wcap = ch;
    }
    k.M = k.B * k.Wcap;
    if (kd) *kd = k;
    if (wm) {
        size_t cur = 0;
        auto take = [&](size_t bytes) { size_t o = cur; cur = FC_ALIGN(cur + bytes); return o; };
        const size_t M = (size_t)k.M;
        size_t cache = (size_t)k.L * k.B * k.Hkv * kv_alloc_planes(k.kvp) * k.S * k.Dh * esz;
        wm->kc = take(cache); wm->vc = take(cache);
        wm->rope_cos = take((size_t)k.S * (k.Dh / 2) * 4); wm->rope_sin = take((size_t)k.S * (k.Dh / 2) * 4);
        wm->x = take(M * d * 4); wm->nx = take(M * d * 4); wm->qkv = take(M * k.qkvN * 4); wm->qrot = take(M * qd * 4);
        wm->att = take(M * qd * 4); wm->gu = take(M * 2 * F * 4); wm->h = take(M * F * 4);
        wm->logits = take(M * k.V * 4); wm->topv = take(M * 4);
        fc_fast_scratch_sizes(k, &wm->gemm_part_bytes, &wm->attn_part_bytes);
        wm->gemm_part = take(wm->gemm_part_bytes); wm->gemm_cnt = take(FC_MAX_COUNTERS * 4);
        wm->attn_part = take(wm->attn_part_bytes); wm->attn_cnt = take(FC_MAX_COUNTERS * 4);
        {
            // column-owner / split-K kernels: per workgroup 32 rows; many-row kernel: per column block of 64
            // (narrow tiles) or 256 columns, all rows
            size_t am = (size_t)(k.V / 16 + 8) * 32 * 8, am2 = (size_t)(k.V / 64 + 1) * ((M + 15) / 16 * 16) * 8;
            wm->amax_part = take(am > am2 ? am : am2);
        }     // winners per column group / per workgroup
        StateMap s; int w = 0;
        auto ti = [&](int words) { int o = w; w += (words + 3) & ~3; return o; };
        s.n = ti(k.B); s.g = ti(k.B); s.done = ti(k.B); s.steps = ti(k.B); s.newest = ti(k.B); s.lastK = ti(k.B);
        s.plen = ti(k.B); s.olen = ti(k.B); s.win = ti(k.B * k.Wcap); s.o = ti(k.B * k.Wcap);
        s.buf = ti(k.B * k.S); s.out = ti(k.B * k.S); s.prompt = ti(k.B * k.S); s.flags = ti(8); s.params = ti(8);
        s.wseq = ti(k.B);
        s.rowb = ti(k.B * k.Wcap); s.rowj = ti(k.B * k.Wcap); s.rstart = ti(k.B + 1);
        s.words = w;
        wm->st = s;
        wm->state = take((size_t)w * 4);
        wm->total = cur;
    }
    return 0;
}

extern "C" size_t fastcot_weight_bytes(const fastcot_config* cfg) {
    ModelMap mm;
    return fc_build_maps(cfg, &mm, nullptr, nullptr) == 0 ? mm.total : 0;
}
extern "C" size_t fastcot_workspace_bytes(const fastcot_config* cfg) {
    WorkspaceMap wm;
    return fc_build_maps(cfg, nullptr, &wm, nullptr) == 0 ? wm.total : 0;
}

// ------------------------------------------------------------------ weight packing
extern "C" int fastcot_pack_tensor(const fastcot_config* cfg, int32_t tensor, int32_t layer, const void* src,
                                   void* d_packed, void* hip_stream) {
    ModelMap mm; KernelDims kd;
    if (fc_build_maps(cfg, &mm, nullptr, &kd) != 0) return fail(nullptr, FASTCOT_EINVAL, "invalid configuration: %s", cfg_problem(cfg));
    if (!d_packed) return fail(nullptr, FASTCOT_EINVAL, "d_packed is NULL%s");
    hipStream_t st = (hipStream_t)hip_stream;
    const int dt = cfg->dtype, d = kd.d, qd = kd.H * kd.Dh, kvd = kd.Hkv * kd.Dh;
    char* base = (char*)d_packed;
    const bool per_layer = tensor >= FASTCOT_T_WQ;
    if (per_layer && (layer < 0 || layer >= kd.L)) return fail(nullptr, FASTCOT_EINVAL, "layer out of range%s");
    char* lbase = base + mm.layers_off + (size_t)(per_layer ? layer : 0) * mm.layer_stride;
    const bool gain = tensor == FASTCOT_T_GF || tensor == FASTCOT_T_G1 || tensor == FASTCOT_T_G2;
    if (!src && !gain) return fail(nullptr, FASTCOT_EINVAL, "d_canonical is NULL%s");
    hipError_t e = hipSuccess;
    switch (tensor) {
        case FASTCOT_T_EMB: e = fc_copy_bytes(base + mm.emb_off, src, (size_t)kd.V * d * kd.esz, st); break;
        case FASTCOT_T_WLM: e = fc_pack(src, dt, d, kd.V, base, mm.lm, 0, 0, st); break;
        case FASTCOT_T_GF: case FASTCOT_T_G1: case FASTCOT_T_G2: {
            float* dst = (float*)(tensor == FASTCOT_T_GF ? base + mm.gf_off
                                  : lbase + (tensor == FASTCOT_T_G1 ? mm.g1_off : mm.g2_off));
            e = src ? fc_copy_bytes(dst, src, (size_t)d * 4, st) : fc_fill_f32(dst, d, 1.0f, st);
            break;
        }
        case FASTCOT_T_WQ: e = fc_pack(src, dt, d, qd, lbase, mm.qkv, 0, 3 + kd.Dh, st); break;
        case FASTCOT_T_WK: e = fc_pack(src, dt, d, kvd, lbase, mm.qkv, qd, 3 + kd.Dh, st); break;
        case FASTCOT_T_WV: e = fc_pack(src, dt, d, kvd, lbase, mm.qkv, qd + kvd, 0, st); break;
        case FASTCOT_T_WO: e = fc_pack(src, dt, qd, d, lbase, mm.o, 0, 0, st); break;
        case FASTCOT_T_WG: e = fc_pack(src, dt, d, kd.F, lbase, mm.gu, 0, 1, st); break;
        case FASTCOT_T_WU: e = fc_pack(src, dt, d, kd.F, lbase, mm.gu, 0, 2, st); break;
        case FASTCOT_T_WD: e = fc_pack(src, dt, kd.F, d, lbase, mm.down, 0, 0, st); break;
        default: return fail(nullptr, FASTCOT_EINVAL, "unknown tensor id%s");
    }
    if (e != hipSuccess) return fail(nullptr, FASTCOT_EHIP, "pack launch failed: %s", hipGetErrorString(e));
    return 0;
}

// canonical layout of a whole model: element count and element size of a tensor
static size_t canon_elems(const KernelDims& kd, int t) {
    const size_t d = kd.d, qd = (size_t)kd.H * kd.Dh, kvd = (size_t)kd.Hkv * kd.Dh, F = kd.F, V = kd.V;
    switch (t) {
        case FASTCOT_T_EMB: case FASTCOT_T_WLM: return V * d;
        case FASTCOT_T_GF: case FASTCOT_T_G1: case FASTCOT_T_G2: return d;
        case FASTCOT_T_WQ: case FASTCOT_T_WO: return d * qd;
        case FASTCOT_T_WK: case FASTCOT_T_WV: return d * kvd;
        case FASTCOT_T_WG: case FASTCOT_T_WU: case FASTCOT_T_WD: return d * F;
    }
    return 0;
}
static size_t canon_bytes(const KernelDims& kd, int t) {
    const bool gain = t == FASTCOT_T_GF || t == FASTCOT_T_G1 || t == FASTCOT_T_G2;
    return FC_ALIGN(canon_elems(kd, t) * (gain ? 4 : (size_t)kd.esz));
}
extern "C" size_t fastcot_canonical_offset(const fastcot_config* cfg, int32_t tensor, int32_t layer) {
    KernelDims kd;
    if (fc_build_maps(cfg, nullptr, nullptr, &kd) != 0 || tensor < FASTCOT_T_EMB || tensor > FASTCOT_T_G2) return (size_t)-1;
    size_t global = 0, per_layer = 0, off_in_layer = 0;
    for (int t = FASTCOT_T_EMB; t <= FASTCOT_T_GF; ++t) { if (t == tensor) return global; global += canon_bytes(kd, t); }
    if (layer < 0 || layer >= kd.L) return (size_t)-1;
    for (int t = FASTCOT_T_WQ; t <= FASTCOT_T_G2; ++t) { if (t == tensor) off_in_layer = per_layer; per_layer += canon_bytes(kd, t); }
    return global + (size_t)layer * per_layer + off_in_layer;
}
extern "C" size_t fastcot_canonical_bytes(const fastcot_config* cfg) {
    KernelDims kd;
    if (fc_build_maps(cfg, nullptr, nullptr, &kd) != 0) return 0;
    size_t total = 0;
    for (int t = FASTCOT_T_EMB; t <= FASTCOT_T_GF; ++t) total += canon_bytes(kd, t);
    size_t per_layer = 0;
    for (int t = FASTCOT_T_WQ; t <= FASTCOT_T_G2; ++t) per_layer += canon_bytes(kd, t);
    return total + (size_t)kd.L * per_layer;
}
extern "C" int fastcot_pack_weights(const fastcot_config* cfg, const void* d_canonical, void* d_packed, void* hip_stream) {
    KernelDims kd;
    if (fc_build_maps(cfg, nullptr, nullptr, &kd) != 0) return fail(nullptr, FASTCOT_EINVAL, "invalid configuration: %s", cfg_problem(cfg));
    if (!d_canonical || !d_packed) return fail(nullptr, FASTCOT_EINVAL, "NULL device buffer%s");
    const char* src = (const char*)d_canonical;
    for (int t = FASTCOT_T_EMB; t <= FASTCOT_T_GF; ++t) {
        const int rc = fastcot_pack_tensor(cfg, t, 0, src + fastcot_canonical_offset(cfg, t, 0), d_packed, hip_stream);
        if (rc) return rc;
    }
    for (int l = 0; l < kd.L; ++l)
        for (int t = FASTCOT_T_WQ; t <= FASTCOT_T_G2; ++t) {
            const int rc = fastcot_pack_tensor(cfg, t, l, src + fastcot_canonical_offset(cfg, t, l), d_packed, hip_stream);
            if (rc) return rc;
        }
    return 0;
}

// ------------------------------------------------------------------ context
static int32_t* state_ptr(fastcot_ctx* c) { return (int32_t*)(c->ws + c->wm.state); }

extern "C" int fastcot_init(const fastcot_config* cfg, const void* d_packed, void* d_workspace, size_t workspace_bytes,
                            void* hip_stream, fastcot_ctx** out) {
    if (!out) return fail(nullptr, FASTCOT_EINVAL, "out is NULL%s");
    *out = nullptr;
    if (!d_packed || !d_workspace) return fail(nullptr, FASTCOT_EINVAL, "NULL device buffer%s");
    fastcot_ctx* c = new (std::nothrow) fastcot_ctx();
    if (!c) return fail(nullptr, FASTCOT_ENOMEM, "out of host memory%s");
    if (fc_build_maps(cfg, &c->mm, &c->wm, &c->kd) != 0) { delete c; return fail(nullptr, FASTCOT_EINVAL, "invalid configuration: %s", cfg_problem(cfg)); }
    if (workspace_bytes < c->wm.total) { delete c; return fail(nullptr, FASTCOT_ECAPACITY, "workspace too small%s"); }
    c->cfg = *cfg; c->weights = (const char*)d_packed; c->ws = (char*)d_workspace; c->st = (hipStream_t)hip_stream;
    c->Bact = 0; c->prefilled = 0; c->generated = 0; c->buf_len = 0; c->opt_tune = 1; c->opt_compact = 1;
    c->opt_packed = 1; c->rows_dirty = 1; c->rows_step = 0;
    c->opt_plain = (cfg->dtype == FASTCOT_F32); c->opt_graph = 1; c->dbg_stop = -1; c->dbg_logits = nullptr;
    c->graph_exec = nullptr; c->graph = nullptr; c->graph_valid = 0; c->prof_on = 0; c->prof_used = 0;
    c->pinned = nullptr; c->err[0] = 0;
    fc_fast_plan(c->kd, &c->plan);
    // rotary table: cos/sin of pos * base^(-2i/Dh), evaluated in double on the host
    const int half = c->kd.Dh / 2;
    std::vector<float> cs((size_t)c->kd.S * half), sn((size_t)c->kd.S * half);
    for (int p = 0; p < c->kd.S; ++p)
        for (int i = 0; i < half; ++i) {
            double ang = (double)p * pow((double)cfg->rope_base, -2.0 * i / (double)c->kd.Dh);
            cs[(size_t)p * half + i] = (float)cos(ang); sn[(size_t)p * half + i] = (float)sin(ang);
        }
#define INITCHK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { int rc_ = fail(nullptr, FASTCOT_EHIP, "HIP error '%s' in init line %ld", hipGetErrorString(e_), __LINE__); if (c->pinned) (void)hipHostFree(c->pinned); delete c; return rc_; } } while (0)
    INITCHK(hipHostMalloc((void**)&c->pinned, 4096 * 4, hipHostMallocDefault));
    INITCHK(hipMemcpyAsync(c->ws + c->wm.rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice, c->st));
    INITCHK(hipMemcpyAsync(c->ws + c->wm.rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice, c->st));
    INITCHK(hipMemsetAsync(c->ws + c->wm.state, 0, (size_t)c->wm.st.words * 4, c->st));
    INITCHK(hipMemsetAsync(c->ws + c->wm.gemm_cnt, 0, FC_MAX_COUNTERS * 4, c->st));
    INITCHK(hipMemsetAsync(c->ws + c->wm.attn_cnt, 0, FC_MAX_COUNTERS * 4, c->st));
    INITCHK(hipMemsetAsync(c->ws + c->wm.kc, 0, c->wm.rope_cos - c->wm.kc, c->st));   // whole KV cache
    INITCHK(hipStreamSynchronize(c->st));
#undef INITCHK
    // a bf16 model the matrix-core kernels do not cover runs through the plain kernels: say so (not an error)
    if (cfg->dtype == FASTCOT_BF16 && !fc_fast_supported(c->kd, c->kd.B * c->kd.W)) {
        c->opt_plain = 1;
        snprintf(c->err, sizeof(c->err), "note: this bf16 model runs on the plain one-thread-per-output kernels: the matrix-core kernels need "
                 "head_dim 128 and d_model, d_ffn, n_heads*head_dim multiples of 256");
    }
    *out = c;
    return 0;
}

static void drop_graph(fastcot_ctx* c) {
    if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
    if (c->graph) (void)hipGraphDestroy(c->graph);
    c->graph_exec = nullptr; c->graph = nullptr; c->graph_valid = 0;
    c->rows_dirty = 1;          // whatever invalidates the graph may have changed who sits where
}

extern "C" void fastcot_free(fastcot_ctx* c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->st);
    drop_graph(c);
    for (hipEvent_t e : c->prof_ev) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->step_ev) (void)hipEventDestroy(e);
    if (c->pinned) (void)hipHostFree(c->pinned);
    delete c;
}

extern "C" int fastcot_set_option(fastcot_ctx* c, int32_t option, int32_t value) {
    if (!c) return fail(nullptr, FASTCOT_EINVAL, "ctx is NULL%s");
    const int nts[5] = {c->kd.qkvN / 16, c->kd.d / 16, 2 * c->kd.F / 16, c->kd.d / 16, c->kd.V / 16};
    const int Ks[5] = {c->kd.d, c->kd.H * c->kd.Dh, c->kd.d, c->kd.F, c->kd.d};
    if (option == FASTCOT_OPT_PLAIN_KERNELS) {
        if (!value && c->cfg.dtype == FASTCOT_F32) return fail(c, FASTCOT_EINVAL, "fp32 models only have the plain kernels%s");
        c->opt_plain = value != 0;
    } else if (option == FASTCOT_OPT_GRAPH) c->opt_graph = value != 0;
    else if (option == FASTCOT_OPT_DEBUG_STAGES) c->dbg_stop = value;
    else if (option == FASTCOT_OPT_PACKED_ROWS) c->opt_packed = value != 0;
    else if (option == FASTCOT_OPT_KV_PLANES) {
        if (c->cfg.dtype != FASTCOT_BF16 || value < 1 || value > 3) return fail(c, FASTCOT_EINVAL, "KV planes: 1, 2 or 3, bf16 models only%s");
        c->kd.kvp = value; c->prefilled = 0;      // the cache layout changes: a new prefill is required
    } else if (option == FASTCOT_OPT_KV_EMULATE) {
        if (c->cfg.dtype != FASTCOT_BF16 || value < 0 || (value & 15) > 3 || (value >> 4) > 3) return fail(c, FASTCOT_EINVAL, "KV format emulation: K mode + 16 * V mode, modes 0..3, bf16 models only%s");
        c->kd.kvq = value; c->prefilled = 0;
    } else if (option == FASTCOT_OPT_ACT_EMULATE) {
        if (c->cfg.dtype != FASTCOT_BF16 || value < 0 || value > 31) return fail(c, FASTCOT_EINVAL, "activation format emulation: a mask of the five GEMMs, bf16 models only%s");
        c->kd.actq = value;
    } else if (option == FASTCOT_OPT_COMPACT) c->opt_compact = value != 0;
    else if (option == FASTCOT_OPT_AUTOTUNE) { c->opt_tune = value != 0; c->tuned_rows[0] = c->tuned_rows[1] = 0; }
    else if (option >= FASTCOT_PLAN_NW && option < FASTCOT_PLAN_NW + 5) {
        const int gi = option - FASTCOT_PLAN_NW, NT = nts[gi], ks = c->plan.ks[gi] > 1 ? c->plan.ks[gi] : 1;
        if (value < 1 || value > NT || (NT + value - 1) / value > 8)
            return fail(c, FASTCOT_EINVAL, "workgroups of the column-owner GEMM: NT/8 .. NT%s");
        if (value % ks || value / ks > NT || (NT + value / ks - 1) / (value / ks) > 12)
            return fail(c, FASTCOT_EINVAL, "workgroups of the column-owner GEMM do not fit its K slices per owner%s");
        c->plan.nw[gi] = value; c->opt_tune = 0;
    } else if (option >= FASTCOT_PLAN_KS && option < FASTCOT_PLAN_KS + 4) {
        const int gi = option - FASTCOT_PLAN_KS, NT = nts[gi], nw = c->plan.nw[gi], K = Ks[gi];
        if (value < 1 || value > 8 || K / 256 < value) return fail(c, FASTCOT_EINVAL, "K slices per owner out of range%s");
        if (nw % value || nw / value > NT || nw / value < 1 || (NT + nw / value - 1) / (nw / value) > 12)
            return fail(c, FASTCOT_EINVAL, "K slices per owner do not fit the workgroup count of that GEMM%s");
        c->plan.ks[gi] = value; c->opt_tune = 0;
        // steps of 17..32 rows (two row tiles per workgroup, at most 8 n-tiles): the same value where it fits
        const int nw2 = c->plan.nw2[gi];
        if (nw2 > 0 && nw2 % value == 0 && nw2 / value >= 1 && nw2 / value <= NT && (NT + nw2 / value - 1) / (nw2 / value) <= 8)
            c->plan.ks2[gi] = value;
    } else if (option >= FASTCOT_PLAN_SB && option < FASTCOT_PLAN_SB + 5) {
        if (value < 0 || value > 2) return fail(c, FASTCOT_EINVAL, "weight batches in flight: 0 (two), 1 (one) or 2 (whole slice up front)%s");
        c->plan.co_sb[0][option - FASTCOT_PLAN_SB] = c->plan.co_sb[1][option - FASTCOT_PLAN_SB] = value; c->opt_tune = 0;
    } else if (option >= FASTCOT_PLAN_ROT && option < FASTCOT_PLAN_ROT + 5) {
        c->plan.co_rot[0][option - FASTCOT_PLAN_ROT] = c->plan.co_rot[1][option - FASTCOT_PLAN_ROT] = value != 0; c->opt_tune = 0;
    } else if (option == FASTCOT_PLAN_CO_SINGLE) {
        if (value < 0 || value > 2) return fail(c, FASTCOT_EINVAL, "buffering of the column-owner GEMM: 0, 1 or 2%s");
        c->plan.co_single = value; c->opt_tune = 0;
    } else if (option == FASTCOT_PLAN_ATTN_SPLITS) {
        if (value < 1 || value > FC_MAX_ATTN_SPLITS) return fail(c, FASTCOT_EINVAL, "attention splits out of range%s");
        c->plan.attn_splits = value;
    } else if (option == FASTCOT_PLAN_ATTN_BLOCKS) {
        if (value < 1 || value > 4096) return fail(c, FASTCOT_EINVAL, "attention blocks per workgroup out of range%s");
        c->plan.attn_bpw = value;
    } else if (option == FASTCOT_PLAN_ATTN_MANY_ROWS) {
        if (value < 0 || value > 2) return fail(c, FASTCOT_EINVAL, "many-row attention: 0 never, 1 by workgroup count, 2 for every pass of more than 32 rows%s");
        c->plan.attn_many = value;
    }
    else return fail(c, FASTCOT_EINVAL, "unknown option%s");
    drop_graph(c);
    return 0;
}

extern "C" int fastcot_debug_logits(fastcot_ctx* c, float* d_logits) {
    if (!c) return fail(nullptr, FASTCOT_EINVAL, "ctx is NULL%s");
    c->dbg_logits = d_logits;
    drop_graph(c);
    return 0;
}

// ------------------------------------------------------------------ forward pass
static hipError_t prof_mark(fastcot_ctx* c, int kind) {
    if (c->prof_used >= c->prof_ev.size()) {
        hipEvent_t e; hipError_t r = hipEventCreate(&e);
        if (r != hipSuccess) return r;
        c->prof_ev.push_back(e); c->prof_kind.push_back(0);
    }
    c->prof_kind[c->prof_used] = kind;
    return hipEventRecord(c->prof_ev[c->prof_used++], c->st);
}
#define LAUNCH(c, kind, call)                                                      \
    do {                                                                           \
        if ((c)->prof_on) HIPCHK(c, prof_mark(c, kind));                           \
        HIPCHK(c, call);                                                           \
        if ((c)->prof_on) HIPCHK(c, prof_mark(c, -1));                             \
    } while (0)

static int forward_plain(fastcot_ctx* c, int lmhead, int R) {
    const KernelDims kd0 = c->kd;
    KernelDims kd = kd0; kd.W = R; kd.M = c->Bact * R;
    const int dt = c->cfg.dtype, M = kd.M, d = kd.d, qd = kd.H * kd.Dh;
    char* ws = c->ws; const char* wt = c->weights;
    int32_t* stp = state_ptr(c);
    const StateMap& sm = c->wm.st;
    float* x = (float*)(ws + c->wm.x); float* nx = (float*)(ws + c->wm.nx); float* qkv = (float*)(ws + c->wm.qkv);
    float* att = (float*)(ws + c->wm.att); float* gu = (float*)(ws + c->wm.gu); float* h = (float*)(ws + c->wm.h);
    LAUNCH(c, KK_EMBED, fc_embed(wt + c->mm.emb_off, dt, stp + sm.win, x, M, d, kd.V, c->st));
    for (int l = 0; l < kd.L; ++l) {
        const char* lb = wt + c->mm.layers_off + (size_t)l * c->mm.layer_stride;
        LAUNCH(c, KK_RMSNORM, fc_rmsnorm_plain(x, (const float*)(lb + c->mm.g1_off), nx, M, d, kd.eps, c->st));
        LAUNCH(c, KK_QKV, fc_gemm_plain(lb + c->mm.qkv.off, dt, d, c->mm.qkv.NP, kd.qkvN, nx, d, qkv, kd.qkvN, M, 0, c->st));
        LAUNCH(c, KK_ROPE, fc_rope_cache_plain(qkv, (float*)(ws + c->wm.qrot), kd, l, stp + sm.n, (const float*)(ws + c->wm.rope_cos),
                                               (const float*)(ws + c->wm.rope_sin), ws + c->wm.kc, ws + c->wm.vc, dt, c->st));
        LAUNCH(c, KK_ATTN, fc_attn_plain((const float*)(ws + c->wm.qrot), qd, ws + c->wm.kc, ws + c->wm.vc, dt, kd, l, stp + sm.n, att, c->st));
        LAUNCH(c, KK_O, fc_gemm_plain(lb + c->mm.o.off, dt, qd, c->mm.o.NP, d, att, qd, x, d, M, 1, c->st));
        LAUNCH(c, KK_RMSNORM, fc_rmsnorm_plain(x, (const float*)(lb + c->mm.g2_off), nx, M, d, kd.eps, c->st));
        LAUNCH(c, KK_GU, fc_gemm_plain(lb + c->mm.gu.off, dt, d, c->mm.gu.NP, 2 * kd.F, nx, d, gu, 2 * kd.F, M, 0, c->st));
        LAUNCH(c, KK_SWIGLU, fc_swiglu_plain(gu, h, M, kd.F, 2 * kd.F, c->st));
        LAUNCH(c, KK_DOWN, fc_gemm_plain(lb + c->mm.down.off, dt, kd.F, c->mm.down.NP, d, h, kd.F, x, d, M, 1, c->st));
    }
    if (lmhead) {
        float* logits = c->dbg_logits ? c->dbg_logits : (float*)(ws + c->wm.logits);
        LAUNCH(c, KK_RMSNORM, fc_rmsnorm_plain(x, (const float*)(wt + c->mm.gf_off), nx, M, d, kd.eps, c->st));
        LAUNCH(c, KK_LM, fc_gemm_plain(wt + c->mm.lm.off, dt, d, c->mm.lm.NP, kd.V, nx, d, logits, kd.V, M, 0, c->st));
        LAUNCH(c, KK_ARGMAX, fc_argmax_plain(logits, M, kd.V, stp + sm.o, (float*)(ws + c->wm.topv), c->st));
    }
    return 0;
}

// one forward pass over R rows per sequence (R = 0: the window); step: the pass of a Jacobi step, which computes
// only the sequences' own rows when they have windows of their own
static int forward(fastcot_ctx* c, int lmhead, int R = 0, bool step = false) {
    if (R <= 0) R = c->kd.W;
    if (R > c->kd.Wcap) return fail(c, FASTCOT_ECAPACITY, "pass of %s%ld rows per sequence exceeds the workspace (%ld)", "", (long)R, (long)c->kd.Wcap);
    if (c->opt_plain || !fc_fast_supported(c->kd, c->Bact * R)) return forward_plain(c, lmhead, R);
    FastArgs a;
    a.kd = c->kd; a.kd.W = R; a.kd.M = c->Bact * R; a.Bact = c->Bact;
    if (step && c->rows_step > 0) {          // sequences with windows of their own: only those rows
        const StateMap& sm = c->wm.st; const int32_t* stp = state_ptr(c);
        a.kd.M = c->rows_step;
        a.rm = RowMap{stp + sm.rowb, stp + sm.rowj, stp + sm.rstart};
    }
    a.mm = &c->mm; a.wm = &c->wm; a.weights = c->weights; a.ws = c->ws; a.dbg_logits = c->dbg_logits;
    a.plan = &c->plan; a.st = c->st; a.lmhead = lmhead;
    a.dbg_stop = c->dbg_stop;
    a.prof = c->prof_on ? c : nullptr;
    a.prof_mark = c->prof_on ? [](void* p, int kind) { return prof_mark((fastcot_ctx*)p, kind); } : nullptr;
    hipError_t e = fc_fast_forward(a);
    if (e != hipSuccess) return fail(c, FASTCOT_EHIP, "forward launch failed: %s", hipGetErrorString(e));
    return 0;
}

static int step_body(fastcot_ctx* c) {
    int rc = forward(c, 1, 0, true);
    if (rc) return rc;
    LAUNCH(c, KK_ACCEPT, fc_accept_commit(state_ptr(c), c->wm.st, c->Bact, c->kd.W, c->kd.S, c->st));
    return 0;
}

// Row map of the next steps: with per-sequence windows (and the option on, and the matrix-core path) sequence b
// contributes its own W_b rows, packed one sequence after the other; otherwise the layout is dense.  Reads the
// windows back from the device, where they travel with their sequences when slots are traded.
static int rebuild_rows(fastcot_ctx* c) {
    const StateMap& sm = c->wm.st; const int B = c->Bact, W = c->kd.W;
    int32_t* stp = state_ptr(c);
    c->rows_dirty = 0; c->rows_step = 0;
    if (!c->opt_packed || c->opt_plain || B < 1) return 0;
    HIPCHK(c, hipStreamSynchronize(c->st));
    std::vector<int32_t> ws(B);
    HIPCHK(c, hipMemcpy(ws.data(), stp + sm.wseq, (size_t)B * 4, hipMemcpyDeviceToHost));
    bool own = false;
    for (int b = 0; b < B; ++b) own = own || (ws[b] > 0 && ws[b] < W);
    if (!own) return 0;
    std::vector<int32_t> rowb, rowj, rstart(B + 1);
    for (int b = 0; b < B; ++b) {
        const int Wb = ws[b] > 0 && ws[b] < W ? ws[b] : W;
        rstart[b] = (int32_t)rowb.size();
        for (int j = 0; j < Wb; ++j) { rowb.push_back(b); rowj.push_back(j); }
    }
    rstart[B] = (int32_t)rowb.size();
    if (!fc_fast_supported(c->kd, (int)rowb.size())) return 0;
    HIPCHK(c, hipMemcpy(stp + sm.rowb, rowb.data(), rowb.size() * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(stp + sm.rowj, rowj.data(), rowj.size() * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(stp + sm.rstart, rstart.data(), rstart.size() * 4, hipMemcpyHostToDevice));
    c->rows_step = (int)rowb.size();
    return 0;
}

static int enqueue_step(fastcot_ctx* c) {
    if (c->rows_dirty) { int rc = rebuild_rows(c); if (rc) return rc; }
    // the legacy default stream cannot be captured: launch kernel by kernel there
    if (!c->opt_graph || c->prof_on || c->st == nullptr) return step_body(c);
    if (!c->graph_valid) {
        HIPCHK(c, hipStreamBeginCapture(c->st, hipStreamCaptureModeThreadLocal));
        int rc = step_body(c);
        hipGraph_t g = nullptr;
        hipError_t e = hipStreamEndCapture(c->st, &g);
        if (rc) { if (g) (void)hipGraphDestroy(g); return rc; }
        if (e != hipSuccess) return fail(c, FASTCOT_EHIP, "graph capture failed: %s", hipGetErrorString(e));
        c->graph = g;
        HIPCHK(c, hipGraphInstantiate(&c->graph_exec, c->graph, nullptr, nullptr, 0));
        c->graph_valid = 1;
    }
    HIPCHK(c, hipGraphLaunch(c->graph_exec, c->st));
    return 0;
}

// ------------------------------------------------------------------ prefill
// Passes of R rows per sequence over prompt tokens 0 .. maxlen-2 of the first B slots (the last prompt token
// becomes slot 0 of the first window); the plain path keeps R = window.  Enqueues only.
static int prefill_passes(fastcot_ctx* c, int B, int maxlen) {
    const KernelDims& kd = c->kd; const StateMap& sm = c->wm.st;
    int32_t* stp = state_ptr(c);
    const int rows_cap = (c->opt_plain || !fc_fast_supported(kd, B * kd.W)) ? kd.W : kd.Wcap;
    int p0 = 0;
    do {
        const int left = maxlen - 1 - p0;
        int R = left < rows_cap ? ((left + 15) & ~15) : rows_cap;
        if (R > rows_cap) R = rows_cap;
        if (R < 1) R = rows_cap < 16 ? rows_cap : 16;          // 1-token prompts: no forward, only the window set-up
        const bool last = p0 + R >= maxlen - 1;
        HIPCHK(c, fc_prefill_window(stp, sm, B, R, kd.S, p0, c->st));
        if (left > 0) { int rc = forward(c, 0, R); if (rc) return rc; }
        HIPCHK(c, fc_prefill_advance(stp, sm, B, kd.W, kd.S, p0 + R, last, c->st));
        p0 += R;
    } while (p0 < maxlen - 1);
    return 0;
}

// two sequences trade slots: state rows and K/V cache
static hipError_t trade_slots(fastcot_ctx* c, int b1, int b2) {
    const KernelDims& kd = c->kd;
    const size_t seq_bytes = (size_t)kd.Hkv * kv_alloc_planes(kd.kvp) * kd.S * kd.Dh * kd.esz;
    return fc_swap_sequences(state_ptr(c), c->wm.st, b1, b2, kd.W, kd.S, c->ws + c->wm.kc, c->ws + c->wm.vc, seq_bytes, kd.L,
                             (size_t)kd.B * seq_bytes, c->st);
}

extern "C" int fastcot_prefill(fastcot_ctx* c, int32_t B, const int32_t* prompts, int32_t max_P, const int32_t* lens,
                               const int32_t* buffer_init, int32_t buf_len) {
    if (!c) return fail(nullptr, FASTCOT_EINVAL, "ctx is NULL%s");
    if (!prompts || !lens || !buffer_init || max_P < 1) return fail(c, FASTCOT_EINVAL, "NULL or empty prompt arguments%s");
    if (B < 1) return fail(c, FASTCOT_EINVAL, "batch must be >= 1%s");
    const KernelDims& kd = c->kd;
    if (B > kd.B) return fail(c, FASTCOT_ECAPACITY, "batch %s%ld exceeds max_batch %ld", "", B, kd.B);
    if (buf_len > c->cfg.max_seq) return fail(c, FASTCOT_ECAPACITY, "buf_len %s%ld exceeds max_seq %ld", "", buf_len, c->cfg.max_seq);
    if (buf_len < 2 * kd.W) return fail(c, FASTCOT_EINVAL, "buf_len %s%ld must be at least 2*window = %ld", "", buf_len, 2 * kd.W);
    int maxlen = 0;
    for (int b = 0; b < B; ++b) {
        if (lens[b] < 1 || lens[b] > max_P) return fail(c, FASTCOT_EINVAL, "prompt length out of range%s");
        if (lens[b] - 1 + 2 * kd.W > c->cfg.max_seq) return fail(c, FASTCOT_ECAPACITY, "prompt of %s%ld tokens does not fit max_seq %ld", "", lens[b], c->cfg.max_seq);
        for (int i = 0; i < lens[b]; ++i)
            if (prompts[(size_t)b * max_P + i] < 0 || prompts[(size_t)b * max_P + i] >= kd.V) return fail(c, FASTCOT_EINVAL, "prompt token out of vocabulary%s");
        if (lens[b] > maxlen) maxlen = lens[b];
    }
    for (size_t i = 0; i < (size_t)B * buf_len; ++i)
        if (buffer_init[i] < 0 || buffer_init[i] >= kd.V) return fail(c, FASTCOT_EINVAL, "buffer token out of vocabulary%s");
    const StateMap& sm = c->wm.st;
    int32_t* stp = state_ptr(c);
    HIPCHK(c, hipStreamSynchronize(c->st));
    std::vector<int32_t> tmp((size_t)B * kd.S, 0);
    for (int b = 0; b < B; ++b) memcpy(&tmp[(size_t)b * kd.S], prompts + (size_t)b * max_P, (size_t)lens[b] * 4);
    HIPCHK(c, hipMemcpy(stp + sm.prompt, tmp.data(), tmp.size() * 4, hipMemcpyHostToDevice));
    std::fill(tmp.begin(), tmp.end(), 0);
    for (int b = 0; b < B; ++b) memcpy(&tmp[(size_t)b * kd.S], buffer_init + (size_t)b * buf_len, (size_t)buf_len * 4);
    HIPCHK(c, hipMemcpy(stp + sm.buf, tmp.data(), tmp.size() * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(stp + sm.plen, lens, (size_t)B * 4, hipMemcpyHostToDevice));
    int32_t params[8] = {0x3fffffff, -1, 0, buf_len, B, 0, 0, 0};
    HIPCHK(c, hipMemcpy(stp + sm.params, params, sizeof(params), hipMemcpyHostToDevice));
    int32_t zeros[8] = {0};
    HIPCHK(c, hipMemcpy(stp + sm.flags, zeros, sizeof(zeros), hipMemcpyHostToDevice));
    HIPCHK(c, hipMemsetAsync(stp + sm.n, 0, (size_t)kd.B * 4, c->st));
    HIPCHK(c, hipMemsetAsync(stp + sm.wseq, 0, (size_t)kd.B * 4, c->st));
    if (B != c->Bact) drop_graph(c);
    c->Bact = B; c->buf_len = buf_len; c->prefilled = 0; c->generated = 0;
    // the plan's per-GEMM choices are measured once per step shape, on this model's own matrices (the buffers
    // hold nothing yet that the passes below do not overwrite)
    {
        const int rows = B * kd.W, cls = rows > 16;
        if (c->opt_tune && !c->opt_plain && c->plan.co_single == 2 && rows <= 32 && c->tuned_rows[cls] != rows &&
            fc_fast_supported(kd, rows)) {
            FastArgs a;
            a.kd = kd; a.kd.M = rows; a.Bact = B; a.mm = &c->mm; a.wm = &c->wm; a.weights = c->weights; a.ws = c->ws;
            a.dbg_logits = nullptr; a.plan = &c->plan; a.st = c->st; a.lmhead = 1; a.dbg_stop = -1; a.prof = nullptr; a.prof_mark = nullptr;
            HIPCHK(c, fc_fast_tune(a, &c->plan));
            c->tuned_rows[cls] = rows;
            drop_graph(c);
        }
    }
    { int rc = prefill_passes(c, B, maxlen); if (rc) return rc; }
    HIPCHK(c, hipStreamSynchronize(c->st));
    c->prefilled = 1;
    return 0;
}

// ------------------------------------------------------------------ one step
extern "C" int fastcot_jacobi_step(fastcot_ctx* c, int32_t* n_accepted, int32_t* accepted, int32_t* window_next) {
    if (!c) return fail(nullptr, FASTCOT_EINVAL, "ctx is NULL%s");
    if (!c->prefilled) return fail(c, FASTCOT_ESTATE, "fastcot_jacobi_step before fastcot_prefill%s");
    int rc = enqueue_step(c);
    if (rc) return rc;
    if (!n_accepted && !accepted && !window_next) return 0;
    const StateMap& sm = c->wm.st; const int B = c->Bact, W = c->kd.W;
    int32_t* stp = state_ptr(c);
    HIPCHK(c, hipStreamSynchronize(c->st));
    std::vector<int32_t> K(B), o((size_t)B * W);
    HIPCHK(c, hipMemcpy(K.data(), stp + sm.lastK, (size_t)B * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(o.data(), stp + sm.o, (size_t)B * W * 4, hipMemcpyDeviceToHost));
    for (int b = 0; b < B; ++b) {
        if (n_accepted) n_accepted[b] = K[b] + 1;    // lastK is -1 for a finished sequence
        if (accepted) for (int j = 0; j < W; ++j) accepted[(size_t)b * W + j] = (j <= K[b]) ? o[(size_t)b * W + j] : -1;
    }
    if (window_next) HIPCHK(c, hipMemcpy(window_next, stp + sm.win, (size_t)B * W * 4, hipMemcpyDeviceToHost));
    int32_t flags[2];
    HIPCHK(c, hipMemcpy(flags, stp + sm.flags, 8, hipMemcpyDeviceToHost));
    if (flags[FLAG_ERROR]) return fail(c, FASTCOT_ECAPACITY, "a sequence ran out of cache or buffer capacity%s");
    return 0;
}

// ------------------------------------------------------------------ window size between steps
// The paper fixes the window per run and names an adaptive size as future work (Limitations); this is the
// hook such a controller needs: from the next fastcot_jacobi_step on, every sequence runs `window` rows.
extern "C" int fastcot_set_window(fastcot_ctx* c, int32_t window) {
    if (!c) return fail(nullptr, FASTCOT_EINVAL, "ctx is NULL%s");
    if (!c->prefilled) return fail(c, FASTCOT_ESTATE, "fastcot_set_window before fastcot_prefill%s");
    if (c->generated) return fail(c, FASTCOT_ESTATE, "fastcot_set_window after fastcot_generate%s");
    if (window < 1 || window > c->kd.Wcap) return fail(c, FASTCOT_ECAPACITY, "window %s%ld outside 1..%ld", "", (long)window, (long)c->kd.Wcap);
    if (window == c->kd.W) return 0;
    const StateMap& sm = c->wm.st; const int B = c->Bact;
    int32_t* stp = state_ptr(c);
    HIPCHK(c, hipStreamSynchronize(c->st));
    std::vector<int32_t> hn(B), hg(B);
    HIPCHK(c, hipMemcpy(hn.data(), stp + sm.n, (size_t)B * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(hg.data(), stp + sm.g, (size_t)B * 4, hipMemcpyDeviceToHost));
    for (int b = 0; b < B; ++b)
        if (hn[b] + window > c->kd.S || hg[b] + 2 * window - 1 > c->buf_len)
            return fail(c, FASTCOT_ECAPACITY, "window %s%ld does not fit the cache or the buffer of a sequence", "", (long)window);
    drop_graph(c);
    c->kd.W = window; c->cfg.window = window;
    HIPCHK(c, fc_rewindow(stp, sm, B, window, c->kd.S, c->st));
    return 0;
}

// Per-sequence window sizes (ragged batches, Sec. 5.4 Time Composition): sequence b verifies, accepts and writes back only the
// first windows[b] rows of its share of the step.  On the matrix-core path the step then computes only those rows
// (rebuild_rows packs them); the plain kernels keep the dense layout (rows at b * W + j) and ignore the rest.
extern "C" int fastcot_set_windows(fastcot_ctx* c, const int32_t* windows) {
    if (!c) return fail(nullptr, FASTCOT_EINVAL, "ctx is NULL%s");
    if (!c->prefilled) return fail(c, FASTCOT_ESTATE, "fastcot_set_windows before fastcot_prefill%s");
    if (c->generated) return fail(c, FASTCOT_ESTATE, "fastcot_set_windows after fastcot_generate%s");
    if (!windows) return fail(c, FASTCOT_EINVAL, "windows is NULL%s");
    const int B = c->Bact;
    for (int b = 0; b < B; ++b)
        if (windows[b] < 1 || windows[b] > c->kd.W) return fail(c, FASTCOT_EINVAL, "window %s%ld outside 1..%ld", "", (long)windows[b], (long)c->kd.W);
    HIPCHK(c, hipStreamSynchronize(c->st));
    HIPCHK(c, hipMemcpy(state_ptr(c) + c->wm.st.wseq, windows, (size_t)B * 4, hipMemcpyHostToDevice));
    drop_graph(c);          // the rows of a step may change
    return 0;
}

extern "C" int fastcot_step_rows(fastcot_ctx* c, int32_t* row_start) {
    if (!c) return fail(nullptr, FASTCOT_EINVAL, "ctx is NULL%s");
    if (!row_start) return fail(c, FASTCOT_EINVAL, "row_start is NULL%s");
    if (!c->prefilled) return fail(c, FASTCOT_ESTATE, "fastcot_step_rows before fastcot_prefill%s");
    if (c->rows_dirty) { int rc = rebuild_rows(c); if (rc) return rc; }
    const int B = c->Bact, W = c->kd.W;
    if (c->rows_step > 0) {
        HIPCHK(c, hipStreamSynchronize(c->st));
        HIPCHK(c, hipMemcpy(row_start, state_ptr(c) + c->wm.st.rstart, (size_t)(B + 1) * 4, hipMemcpyDeviceToHost));
    } else
        for (int b = 0; b <= B; ++b) row_start[b] = b * W;
    return 0;
}

// ------------------------------------------------------------------ a sequence joins the running batch
// Ragged batches (Sec. 5.4 Time Composition, Table 2: a batch otherwise runs, padded, until its longest member ends): between two
// fastcot_jacobi_step calls a new prompt takes over slot `slot`; the other sequences keep their state, and
// since no term of Eq. 2 couples sequences, their streams are what they would have been.  The kernels work
// on the first slots of the batch, so the newcomer is prefilled in slot 0 as a batch of one: the sequence
// that lives there trades places with it for that long.
extern "C" int fastcot_join(fastcot_ctx* c, int32_t slot, const int32_t* prompt, int32_t len, const int32_t* buffer_init) {
    if (!c) return fail(nullptr, FASTCOT_EINVAL, "ctx is NULL%s");
    if (!c->prefilled) return fail(c, FASTCOT_ESTATE, "fastcot_join before fastcot_prefill%s");
    if (c->generated) return fail(c, FASTCOT_ESTATE, "fastcot_join after fastcot_generate%s");
    if (!prompt || !buffer_init) return fail(c, FASTCOT_EINVAL, "NULL prompt or buffer%s");
    const KernelDims& kd = c->kd; const StateMap& sm = c->wm.st; const int B = c->Bact;
    if (slot < 0 || slot >= B) return fail(c, FASTCOT_EINVAL, "slot %s%ld outside the batch of %ld", "", (long)slot, (long)B);
    if (len < 1 || len > kd.S) return fail(c, FASTCOT_EINVAL, "prompt length out of range%s");
    if (len - 1 + 2 * kd.W > c->cfg.max_seq) return fail(c, FASTCOT_ECAPACITY, "prompt of %s%ld tokens does not fit max_seq %ld", "", (long)len, (long)c->cfg.max_seq);
    for (int i = 0; i < len; ++i)
        if (prompt[i] < 0 || prompt[i] >= kd.V) return fail(c, FASTCOT_EINVAL, "prompt token out of vocabulary%s");
    for (int i = 0; i < c->buf_len; ++i)
        if (buffer_init[i] < 0 || buffer_init[i] >= kd.V) return fail(c, FASTCOT_EINVAL, "buffer token out of vocabulary%s");
    int32_t* stp = state_ptr(c);
    if (slot != 0) HIPCHK(c, trade_slots(c, 0, slot));
    HIPCHK(c, hipStreamSynchronize(c->st));
    std::vector<int32_t> row((size_t)kd.S, 0);
    memcpy(row.data(), prompt, (size_t)len * 4);
    HIPCHK(c, hipMemcpy(stp + sm.prompt, row.data(), row.size() * 4, hipMemcpyHostToDevice));
    std::fill(row.begin(), row.end(), 0);
    memcpy(row.data(), buffer_init, (size_t)c->buf_len * 4);
    HIPCHK(c, hipMemcpy(stp + sm.buf, row.data(), row.size() * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(stp + sm.plen, &len, 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemsetAsync(stp + sm.n, 0, 4, c->st));
    HIPCHK(c, hipMemsetAsync(stp + sm.wseq, 0, 4, c->st));    // the newcomer runs the batch's window
    if (c->rows_step > 0) drop_graph(c);                      // (with packed rows the step's row map changes with it)
    // a pass of R rows uses the first R window entries, which at R > W are the other sequences' windows
    std::vector<int32_t> wins((size_t)B * kd.W);
    HIPCHK(c, hipMemcpy(wins.data(), stp + sm.win, wins.size() * 4, hipMemcpyDeviceToHost));
    c->Bact = 1;                                   // the step graph, captured for B sequences, is not touched
    int rc = prefill_passes(c, 1, len);
    c->Bact = B;
    if (rc) return rc;
    HIPCHK(c, hipStreamSynchronize(c->st));
    if (B > 1) HIPCHK(c, hipMemcpy(stp + sm.win + kd.W, wins.data() + kd.W, (size_t)(B - 1) * kd.W * 4, hipMemcpyHostToDevice));
    if (slot != 0) HIPCHK(c, trade_slots(c, 0, slot));
    // the flags speak for the whole batch: they stand only if a remaining sequence still has them raised
    HIPCHK(c, hipMemcpyAsync(c->pinned, stp + sm.done, (size_t)B * 4, hipMemcpyDeviceToHost, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    bool any_done = false;
    for (int b = 0; b < B; ++b) any_done = any_done || c->pinned[b] != 0;
    if (!any_done) { int32_t zeros[2] = {0, 0}; HIPCHK(c, hipMemcpy(stp + sm.flags, zeros, 8, hipMemcpyHostToDevice)); }
    return 0;
}

// ------------------------------------------------------------------ generate
extern "C" int fastcot_generate(fastcot_ctx* c, int32_t max_new, int32_t max_steps, int32_t eos_id, int32_t* out_ids,
                                int32_t* out_len, int32_t* out_steps, int32_t* approx_tail) {
    if (!c) return fail(nullptr, FASTCOT_EINVAL, "ctx is NULL%s");
    if (!c->prefilled) return fail(c, FASTCOT_ESTATE, "fastcot_generate before fastcot_prefill%s");
    if (c->generated) return fail(c, FASTCOT_ESTATE, "fastcot_generate may be called once per prefill%s");
    if (!out_ids || !out_len || !out_steps || max_new < 1) return fail(c, FASTCOT_EINVAL, "bad output arguments%s");
    const KernelDims& kd = c->kd; const StateMap& sm = c->wm.st; const int B = c->Bact, W = kd.W;
    if (c->buf_len < max_new + 2 * W) return fail(c, FASTCOT_ECAPACITY, "buf_len %s%ld is below max_new_tokens + 2*window = %ld", "", c->buf_len, max_new + 2 * W);
    int32_t* stp = state_ptr(c);
    std::vector<int32_t> hn(B), hg(B), hdone(B, 0);
    HIPCHK(c, hipStreamSynchronize(c->st));
    HIPCHK(c, hipMemcpy(hn.data(), stp + sm.n, (size_t)B * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(hg.data(), stp + sm.g, (size_t)B * 4, hipMemcpyDeviceToHost));
    for (int b = 0; b < B; ++b) {
        if (hg[b] != 0) return fail(c, FASTCOT_ESTATE, "fastcot_generate after fastcot_jacobi_step is not supported%s");
        if (hn[b] + max_new + 2 * W > c->cfg.max_seq) return fail(c, FASTCOT_ECAPACITY, "prompt + max_new_tokens + 2*window exceeds max_seq%s");
    }
    int32_t params[8] = {max_new, eos_id < 0 ? -1 : eos_id, max_steps > 0 ? max_steps : 0, c->buf_len, B, 0, 0, 0};
    HIPCHK(c, hipMemcpy(stp + sm.params, params, sizeof(params), hipMemcpyHostToDevice));
    c->generated = 1; c->last_eos = eos_id < 0 ? -1 : eos_id;
    c->step_ms.clear();
    size_t ev_used = 0;
    auto next_event = [&](hipEvent_t* ev) -> hipError_t {
        if (ev_used >= c->step_ev.size()) {
            if (c->step_ev.size() >= 8192) { *ev = nullptr; return hipSuccess; }
            hipEvent_t e; hipError_t r = hipEventCreate(&e);
            if (r != hipSuccess) return r;
            c->step_ev.push_back(e);
        }
        *ev = c->step_ev[ev_used++];
        return hipSuccess;
    };
    int total_steps = 0;
    bool all_done = false;
    hipEvent_t ev;
    HIPCHK(c, next_event(&ev));
    if (ev) HIPCHK(c, hipEventRecord(ev, c->st));
    // Ragged finish: sequences that are done trade slots with unfinished ones further back, so that the
    // unfinished ones sit in slots 0..Bcur-1 and the following steps run Bcur * W rows (every kernel works on
    // the first Bact slots).  The trades are undone before returning: callers see their own order.
    int Bcur = B;
    std::vector<std::pair<int, int>> trades;
    auto trade = [&](int b1, int b2) -> hipError_t { return trade_slots(c, b1, b2); };
    while (!all_done) {
        // every unfinished sequence needs at least ceil((max_new - g) / W) more steps: enqueue that many
        int need = 1;
        for (int b = 0; b < Bcur; ++b) {
            int r = (max_new - hg[b] + W - 1) / W;
            if (total_steps == 0 || !hdone[b]) need = r > need ? r : need;
        }
        if (max_steps > 0 && need > max_steps - total_steps) need = max_steps - total_steps;
        if (need < 1) need = 1;
        for (int s = 0; s < need; ++s) {
            int rc = enqueue_step(c);
            if (rc) return rc;
            HIPCHK(c, next_event(&ev));
            if (ev) HIPCHK(c, hipEventRecord(ev, c->st));
            ++total_steps;
        }
        HIPCHK(c, hipMemcpyAsync(c->pinned, stp + sm.g, (size_t)B * 4, hipMemcpyDeviceToHost, c->st));
        HIPCHK(c, hipMemcpyAsync(c->pinned + B, stp + sm.done, (size_t)B * 4, hipMemcpyDeviceToHost, c->st));
        HIPCHK(c, hipMemcpyAsync(c->pinned + 2 * B, stp + sm.flags, 8, hipMemcpyDeviceToHost, c->st));
        HIPCHK(c, hipStreamSynchronize(c->st));
        all_done = c->pinned[2 * B + FLAG_ALL_DONE] != 0;
        for (int b = 0; b < B; ++b) { hg[b] = c->pinned[b]; hdone[b] = c->pinned[B + b]; }
        if (c->pinned[2 * B + FLAG_ERROR]) {
            for (size_t i = trades.size(); i-- > 0;) (void)trade(trades[i].first, trades[i].second);
            c->Bact = B; drop_graph(c);
            return fail(c, FASTCOT_ECAPACITY, "a sequence ran out of cache or buffer capacity%s");
        }
        if (!all_done && c->opt_compact && !(max_steps > 0 && total_steps >= max_steps)) {
            int lo = 0, hi = Bcur - 1, moved = 0;
            for (;;) {
                while (lo < hi && !hdone[lo]) ++lo;          // first finished slot
                while (hi > lo && hdone[hi]) --hi;           // last unfinished slot
                if (lo >= hi) break;
                HIPCHK(c, trade(lo, hi));
                trades.push_back({lo, hi});
                std::swap(hg[lo], hg[hi]); std::swap(hdone[lo], hdone[hi]);
                ++moved;
            }
            int nact = 0;
            while (nact < Bcur && !hdone[nact]) ++nact;
            if (nact >= 1 && nact < Bcur) { Bcur = nact; c->Bact = nact; drop_graph(c); }
            (void)moved;
        }
    }
    if (!trades.empty() || c->Bact != B) {
        for (size_t i = trades.size(); i-- > 0;) HIPCHK(c, trade(trades[i].first, trades[i].second));
        c->Bact = B; drop_graph(c);
        HIPCHK(c, hipStreamSynchronize(c->st));
    }
    for (size_t i = 0; i + 1 < ev_used; ++i) {
        float ms = 0; HIPCHK(c, hipEventElapsedTime(&ms, c->step_ev[i], c->step_ev[i + 1]));
        c->step_ms.push_back(ms);
    }
    std::vector<int32_t> tmp((size_t)B * kd.S);
    HIPCHK(c, hipMemcpy(tmp.data(), stp + sm.out, tmp.size() * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(out_len, stp + sm.olen, (size_t)B * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(out_steps, stp + sm.steps, (size_t)B * 4, hipMemcpyDeviceToHost));
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < max_new; ++i) out_ids[(size_t)b * max_new + i] = i < out_len[b] ? tmp[(size_t)b * kd.S + i] : -1;
    if (approx_tail && W > 1) {
        std::vector<int32_t> win((size_t)B * W);
        HIPCHK(c, hipMemcpy(win.data(), stp + sm.win, win.size() * 4, hipMemcpyDeviceToHost));
        for (int b = 0; b < B; ++b) for (int j = 1; j < W; ++j) approx_tail[(size_t)b * (W - 1) + j - 1] = win[(size_t)b * W + j];
    }
    return 0;
}

// ------------------------------------------------------------------ answer phase
// Sec. 4.4 "Trigger Answer": when the iterations have stopped, the complete prompt, all generated tokens --
// the exact ones and the approximate ones still in the window, the glimpse -- and the answer trigger are
// put together and the model decodes the answer directly.  Here the cache already holds the K/V of the
// prompt and the exact tokens, so only the newest exact token, the glimpse and the trigger are run through
// the model (one pass, no LM head; their last token becomes the input of the first decoding step), then
// the answer is decoded greedily one token per step (Eq. 1).  A sequence that ended with EOS has no
// glimpse: its context ends at the EOS.
extern "C" int fastcot_answer(fastcot_ctx* c, const int32_t* trigger_ids, int32_t n_trigger, int32_t max_new,
                              int32_t eos_id, int32_t* out_ids, int32_t* out_len) {
    if (!c) return fail(nullptr, FASTCOT_EINVAL, "ctx is NULL%s");
    if (!c->prefilled || !c->generated) return fail(c, FASTCOT_ESTATE, "fastcot_answer needs a finished fastcot_generate%s");
    if (!out_ids || !out_len || max_new < 1 || n_trigger < 0 || (n_trigger > 0 && !trigger_ids))
        return fail(c, FASTCOT_EINVAL, "bad arguments%s");
    const KernelDims& kd = c->kd; const StateMap& sm = c->wm.st; const int B = c->Bact, W = kd.W, S = kd.S;
    for (int i = 0; i < n_trigger; ++i)
        if (trigger_ids[i] < 0 || trigger_ids[i] >= kd.V) return fail(c, FASTCOT_EINVAL, "trigger token out of vocabulary%s");
    int32_t* stp = state_ptr(c);
    HIPCHK(c, hipStreamSynchronize(c->st));
    std::vector<int32_t> hn(B), hg(B), holen(B), hnew(B), hplen(B), hwin((size_t)B * W), hout((size_t)B * S);
    HIPCHK(c, hipMemcpy(hn.data(), stp + sm.n, (size_t)B * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(hg.data(), stp + sm.g, (size_t)B * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(holen.data(), stp + sm.olen, (size_t)B * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(hnew.data(), stp + sm.newest, (size_t)B * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(hplen.data(), stp + sm.plen, (size_t)B * 4, hipMemcpyDeviceToHost));
    std::vector<int32_t> hws(B);
    HIPCHK(c, hipMemcpy(hws.data(), stp + sm.wseq, (size_t)B * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(hwin.data(), stp + sm.win, hwin.size() * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(hout.data(), stp + sm.out, hout.size() * 4, hipMemcpyDeviceToHost));
    // per sequence: the tokens that still have to enter the cache, and the committed length they start at
    std::vector<std::vector<int32_t>> ctxrows(B);
    int R = 0;
    for (int b = 0; b < B; ++b) {
        std::vector<int32_t>& t = ctxrows[b];
        const bool eos_end = c->last_eos >= 0 && holen[b] > 0 && hout[(size_t)b * S + holen[b] - 1] == c->last_eos;
        if (eos_end) {       // keep the exact tokens up to the EOS; K/V valid below its position
            hn[b] = hplen[b] - 1 + holen[b];
            t.push_back(c->last_eos);
        } else {             // newest exact token (not in the cache yet), then the glimpse
            if (hn[b] != hplen[b] - 1 + hg[b]) return fail(c, FASTCOT_ESTATE, "inconsistent sequence state%s");
            t.push_back(hg[b] > 0 ? hnew[b] : hwin[(size_t)b * W]);
            const int Wb = hws[b] > 0 && hws[b] < W ? hws[b] : W;
            for (int j = 1; j < Wb; ++j) t.push_back(hwin[(size_t)b * W + j]);
        }
        for (int i = 0; i < n_trigger; ++i) t.push_back(trigger_ids[i]);
        if ((int)t.size() - 1 > R) R = (int)t.size() - 1;
        if (hn[b] + (int)t.size() + max_new + 1 > S) return fail(c, FASTCOT_ECAPACITY, "answer phase does not fit max_seq%s");
    }
    HIPCHK(c, hipMemcpy(stp + sm.n, hn.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    // context passes of at most Wcap rows per sequence (all but the last context token): rows beyond a
    // sequence's own are pads whose K/V is never committed
    const int rows_cap = (c->opt_plain || !fc_fast_supported(kd, B * kd.W)) ? kd.W : kd.Wcap;
    for (int p0 = 0; p0 < R; p0 += rows_cap) {
        const int Rp = R - p0 < rows_cap ? R - p0 : rows_cap;
        std::vector<int32_t> rows((size_t)B * Rp, 0);
        for (int b = 0; b < B; ++b)
            for (int j = 0; j < Rp && p0 + j + 1 < (int)ctxrows[b].size(); ++j) rows[(size_t)b * Rp + j] = ctxrows[b][p0 + j];
        HIPCHK(c, hipMemcpy(stp + sm.win, rows.data(), rows.size() * 4, hipMemcpyHostToDevice));
        int rc = forward(c, 0, Rp);
        if (rc) return rc;
        HIPCHK(c, hipStreamSynchronize(c->st));
        for (int b = 0; b < B; ++b) {
            int adv = (int)ctxrows[b].size() - 1 - p0;
            hn[b] += adv < 0 ? 0 : (adv > Rp ? Rp : adv);
        }
        HIPCHK(c, hipMemcpy(stp + sm.n, hn.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    }
    // one-token window per sequence: slot 0 = the last context token
    std::vector<int32_t> slot0(B), zero(B, 0);
    for (int b = 0; b < B; ++b) slot0[b] = ctxrows[b].back();
    HIPCHK(c, hipMemcpy(stp + sm.win, slot0.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(stp + sm.newest, slot0.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(stp + sm.g, zero.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(stp + sm.done, zero.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(stp + sm.steps, zero.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(stp + sm.olen, zero.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    int32_t params[8] = {max_new, eos_id < 0 ? -1 : eos_id, 0, S, B, 0, 0, 0};
    HIPCHK(c, hipMemcpy(stp + sm.params, params, sizeof(params), hipMemcpyHostToDevice));
    int32_t zeros[8] = {0};
    HIPCHK(c, hipMemcpy(stp + sm.flags, zeros, sizeof(zeros), hipMemcpyHostToDevice));
    c->prefilled = 0;        // the windowed state is gone: the next run starts with fastcot_prefill
    // greedy decoding, one row per sequence and step; as many steps at a time as every unfinished sequence
    // still needs at least
    std::vector<int32_t> g2(B, 0), d2(B, 0);
    bool all_done = false;
    while (!all_done) {
        int need = 1;
        for (int b = 0; b < B; ++b) if (!d2[b] && max_new - g2[b] > need) need = max_new - g2[b];
        for (int s = 0; s < need; ++s) {
            int rc = forward(c, 1, 1);
            if (rc) return rc;
            HIPCHK(c, fc_accept_commit(stp, sm, B, 1, S, c->st));
        }
        HIPCHK(c, hipMemcpyAsync(c->pinned, stp + sm.g, (size_t)B * 4, hipMemcpyDeviceToHost, c->st));
        HIPCHK(c, hipMemcpyAsync(c->pinned + B, stp + sm.done, (size_t)B * 4, hipMemcpyDeviceToHost, c->st));
        HIPCHK(c, hipMemcpyAsync(c->pinned + 2 * B, stp + sm.flags, 8, hipMemcpyDeviceToHost, c->st));
        HIPCHK(c, hipStreamSynchronize(c->st));
        all_done = c->pinned[2 * B + FLAG_ALL_DONE] != 0;
        for (int b = 0; b < B; ++b) { g2[b] = c->pinned[b]; d2[b] = c->pinned[B + b]; }
        if (c->pinned[2 * B + FLAG_ERROR]) return fail(c, FASTCOT_ECAPACITY, "a sequence ran out of cache capacity%s");
    }
    HIPCHK(c, hipMemcpy(hout.data(), stp + sm.out, hout.size() * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(out_len, stp + sm.olen, (size_t)B * 4, hipMemcpyDeviceToHost));
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < max_new; ++i) out_ids[(size_t)b * max_new + i] = i < out_len[b] ? hout[(size_t)b * S + i] : -1;
    return 0;
}

extern "C" int fastcot_step_times(fastcot_ctx* c, float* ms, int32_t cap, int32_t* n_steps) {
    if (!c || !n_steps) return fail(c, FASTCOT_EINVAL, "NULL argument%s");
    *n_steps = (int32_t)c->step_ms.size();
    for (int i = 0; ms && i < cap && i < *n_steps; ++i) ms[i] = c->step_ms[i];
    return 0;
}

extern "C" int fastcot_get_state(fastcot_ctx* c, int32_t* n, int32_t* generated, int32_t* done, int32_t* window,
                                 int32_t* last_o, int32_t* last_K) {
    if (!c) return fail(nullptr, FASTCOT_EINVAL, "ctx is NULL%s");
    if (!c->prefilled) return fail(c, FASTCOT_ESTATE, "no sequences: call fastcot_prefill first%s");
    const StateMap& sm = c->wm.st; const int B = c->Bact, W = c->kd.W;
    int32_t* stp = state_ptr(c);
    HIPCHK(c, hipStreamSynchronize(c->st));
    if (n) HIPCHK(c, hipMemcpy(n, stp + sm.n, (size_t)B * 4, hipMemcpyDeviceToHost));
    if (generated) HIPCHK(c, hipMemcpy(generated, stp + sm.g, (size_t)B * 4, hipMemcpyDeviceToHost));
    if (done) HIPCHK(c, hipMemcpy(done, stp + sm.done, (size_t)B * 4, hipMemcpyDeviceToHost));
    if (window) HIPCHK(c, hipMemcpy(window, stp + sm.win, (size_t)B * W * 4, hipMemcpyDeviceToHost));
    if (last_o) HIPCHK(c, hipMemcpy(last_o, stp + sm.o, (size_t)B * W * 4, hipMemcpyDeviceToHost));
    if (last_K) HIPCHK(c, hipMemcpy(last_K, stp + sm.lastK, (size_t)B * 4, hipMemcpyDeviceToHost));
    return 0;
}

// ------------------------------------------------------------------ per-kernel timing of the forward
extern "C" int fastcot_profile_step(fastcot_ctx* c, int32_t iters, float* mean_ms, int32_t* launches_per_step) {
    if (!c || !mean_ms || !launches_per_step || iters < 1) return fail(c, FASTCOT_EINVAL, "bad arguments%s");
    if (!c->prefilled) return fail(c, FASTCOT_ESTATE, "fastcot_profile_step before fastcot_prefill%s");
    double sum[FASTCOT_N_KERNEL_KINDS] = {0}; long cnt[FASTCOT_N_KERNEL_KINDS] = {0};
    for (int it = 0; it < iters; ++it) {
        c->prof_on = 1; c->prof_used = 0;
        int rc = c->rows_dirty ? rebuild_rows(c) : 0;
        if (!rc) rc = forward(c, 1, 0, true);
        // what an event pair itself adds to a launch: the same pair around a kernel that does nothing
        if (!rc) {
            hipError_t e1 = prof_mark(c, KK_EMPTY);
            k_empty<<<1, 64, 0, c->st>>>();
            hipError_t e2 = prof_mark(c, -1);
            if (e1 != hipSuccess || e2 != hipSuccess) { c->prof_on = 0; return fail(c, FASTCOT_EHIP, "event record failed%s"); }
        }
        c->prof_on = 0;
        if (rc) return rc;
        HIPCHK(c, hipStreamSynchronize(c->st));
        for (size_t i = 0; i + 1 < c->prof_used; i += 2) {
            float ms = 0; HIPCHK(c, hipEventElapsedTime(&ms, c->prof_ev[i], c->prof_ev[i + 1]));
            int k = c->prof_kind[i];
            if (k >= 0 && k < FASTCOT_N_KERNEL_KINDS) { sum[k] += ms; cnt[k]++; }
        }
    }
    for (int k = 0; k < FASTCOT_N_KERNEL_KINDS; ++k) {
        mean_ms[k] = cnt[k] ? (float)(sum[k] / cnt[k]) : 0.f;
        launches_per_step[k] = (int32_t)(cnt[k] / iters);
    }
    return 0;
}

// ------------------------------------------------------------------ debug read-back of activations
extern "C" int fastcot_debug_read(fastcot_ctx* c, int32_t what, float* host, size_t count) {
    if (!c || !host) return fail(c, FASTCOT_EINVAL, "NULL argument%s");
    const size_t M = (size_t)c->kd.M;
    size_t off, cap;
    switch (what) {
        case 0: off = c->wm.x; cap = M * c->kd.d; break;
        case 1: off = c->wm.qkv; cap = M * c->kd.qkvN; break;
        case 2: off = c->wm.att; cap = M * c->kd.H * c->kd.Dh; break;
        case 3: off = c->wm.h; cap = M * c->kd.F; break;
        case 4: off = c->wm.logits; cap = M * c->kd.V; break;     // plain-path logits buffer
        default: return fail(c, FASTCOT_EINVAL, "unknown buffer%s");
    }
    if (count > cap) return fail(c, FASTCOT_ECAPACITY, "count exceeds the buffer%s");
    HIPCHK(c, hipStreamSynchronize(c->st));
    HIPCHK(c, hipMemcpy(host, c->ws + off, count * 4, hipMemcpyDeviceToHost));
    return 0;
}
