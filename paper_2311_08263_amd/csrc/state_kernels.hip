// Decoding-state kernels: all per-sequence state (committed length n, generated count g, the
// Approximate Tokens Buffer, the window, done flags) lives in device memory so that a captured
// step can be replayed without host arguments.
#include "kernels.h"

// Prefill pass of R rows per sequence starting at prompt position p0: row j of sequence b carries
// prompt token p0 + j if that token is one of the first len-1 prompt tokens, else a pad (its K/V is
// never committed).
__global__ void k_prefill_window(int32_t* st, StateMap sm, int B, int R, int S, int p0) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B * R) return;
    int b = i / R, j = i % R;
    int len = st[sm.plen + b];
    int p = p0 + j;
    st[sm.win + i] = (p < len - 1) ? st[sm.prompt + (size_t)b * S + p] : 0;
}
hipError_t fc_prefill_window(int32_t* state, const StateMap& sm, int B, int R, int S, int p0, hipStream_t st) {
    k_prefill_window<<<(B * R + 255) / 256, 256, 0, st>>>(state, sm, B, R, S, p0);
    return hipGetLastError();
}

// After the forward of a prefill pass that ended at prompt position p1: commit the K/V of the real
// prompt rows.  After the last pass, set up the first Jacobi window: slot 0 = last prompt token,
// slots 1.. = buffer[0..W-2].
__global__ void k_prefill_advance(int32_t* st, StateMap sm, int B, int W, int S, int p1, int last) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int len = st[sm.plen + b];
    int n = p1;
    if (n > len - 1) n = len - 1;
    st[sm.n + b] = n;
    if (last) {
        st[sm.g + b] = 0; st[sm.done + b] = 0; st[sm.steps + b] = 0; st[sm.lastK + b] = 0; st[sm.olen + b] = 0;
        int newest = st[sm.prompt + (size_t)b * S + len - 1];
        st[sm.newest + b] = newest;
        st[sm.win + b * W] = newest;
        for (int j = 1; j < W; ++j) st[sm.win + b * W + j] = st[sm.buf + (size_t)b * S + j - 1];
    }
}
hipError_t fc_prefill_advance(int32_t* state, const StateMap& sm, int B, int W, int S, int p1, int last,
                              hipStream_t st) {
    k_prefill_advance<<<(B + 63) / 64, 64, 0, st>>>(state, sm, B, W, S, p1, last);
    return hipGetLastError();
}

// Verification (Eq. 5), acceptance, cache update and window shift (Sec. 4.3), stop conditions
// (Sec. 4.4) for every sequence.  o[b][j] is the argmax of row j, i.e. the prediction for the
// token after window slot j.  Approximate slot i is verified when o[i-1] == win[i]; slots are
// checked in order and the first miss stops.  K verified slots => K+1 exact tokens o[0..K].
// Committing their K/V is the bump of n: rows 0..K of this step wrote their K/V at positions
// n..n+K already.  All W fresh outputs go back to the buffer; the window slides by K+1.
// One wave per sequence, lane j on window slot j (in rounds of 64 for wider windows): the scans of Eq. 5 and of
// the EOS rule are ballots, the copies one load and one store per lane.
__global__ void k_accept_commit(int32_t* st, StateMap sm, int B, int W, int S) {
    __shared__ int not_done;
    if (threadIdx.x == 0) not_done = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int max_new = st[sm.params + PARAM_MAX_NEW], eos = st[sm.params + PARAM_EOS];
    const int max_steps = st[sm.params + PARAM_MAX_STEPS], buf_len = st[sm.params + PARAM_BUF_LEN];
    for (int b = wave; b < B; b += nwaves) {
        if (st[sm.done + b]) { if (lane == 0) st[sm.lastK + b] = -1; continue; }
        const int32_t* w = st + sm.win + b * W;
        const int32_t* o = st + sm.o + b * W;
        int32_t* buf = st + sm.buf + (size_t)b * S;
        int32_t* out = st + sm.out + (size_t)b * S;
        int n = st[sm.n + b], g = st[sm.g + b], steps = st[sm.steps + b];
        const int g0 = g, olen0 = st[sm.olen + b];
        // a sequence with a window of its own uses the first Wb rows of its W: the others are ignored (or not computed)
        const int ws = st[sm.wseq + b], Wb = ws > 0 && ws < W ? ws : W;
        // K = verified slots: the first i in 1..Wb-1 with o[i-1] != w[i] ends the scan (Eq. 5); E = first accepted
        // row that is an EOS (rows after it are not emitted)
        int K = Wb - 1, E = Wb;
        for (int j0 = 0; j0 < Wb - 1; j0 += 64) {
            const int j = j0 + lane;
            const bool miss = j < Wb - 1 && o[j] != w[j + 1];
            const unsigned long long mask = __ballot(miss);
            if (mask) { K = j0 + __ffsll((long long)mask) - 1; break; }
        }
        if (eos >= 0)
            for (int j0 = 0; j0 <= K; j0 += 64) {
                const int j = j0 + lane;
                const unsigned long long mask = __ballot(j <= K && o[j] == eos);
                if (mask) { E = j0 + __ffsll((long long)mask) - 1; break; }
            }
        // all Wb fresh outputs go back to the buffer ("Cache Update", Sec. 4.3); the next window is read from the
        // values themselves where they were just written (slot p of the buffer, p - g0 < Wb), else from the buffer
        const int last = E < K ? E : K;                         // last emitted row
        for (int j = lane; j < Wb; j += 64) {
            const int oj = o[j];
            if (g0 + j < buf_len) buf[g0 + j] = oj;
            if (j <= last && g0 + j < max_new && g0 + j < S) out[g0 + j] = oj;
        }
        int jmax = last;
        if (jmax > max_new - 1 - g0) jmax = max_new - 1 - g0;
        if (jmax > S - 1 - g0) jmax = S - 1 - g0;
        const int emitted = jmax >= 0 ? g0 + jmax + 1 : 0;
        int stop = E <= K;
        const int newest = o[K];
        n += K + 1; g += K + 1; ++steps;
        if (g >= max_new || (max_steps > 0 && steps >= max_steps)) stop = 1;
        bool err = false;
        if (n + W > S || g + 2 * W - 1 > buf_len) {       // no room for another window: stop, flag it
            err = !stop;
            stop = 1;
        }
        // (the window is rewritten only after every lane has read its o and w above: a wave runs in lockstep, and
        // the reads below touch o and the part of the buffer this step did not write)
        int32_t* wn = st + sm.win + b * W;
        for (int j = lane; j < W; j += 64) {
            int v;
            if (j == 0) v = newest;
            else {
                const int p = g + j - 1;
                v = p >= buf_len ? 0 : (p - g0 < Wb ? o[p - g0] : buf[p]);
            }
            wn[j] = v;
        }
        if (lane == 0) {
            if (emitted > olen0) st[sm.olen + b] = emitted;
            if (err) st[sm.flags + FLAG_ERROR] = 1;
            st[sm.n + b] = n; st[sm.g + b] = g; st[sm.steps + b] = steps; st[sm.lastK + b] = K;
            st[sm.newest + b] = newest; st[sm.done + b] = stop;
            if (!stop) atomicAdd(&not_done, 1);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) st[sm.flags + FLAG_ALL_DONE] = (not_done == 0);
}
// A new window size between steps: the window is rebuilt from the newest exact token and the buffer
// (the buffer already holds every output of the previous steps, Sec. 4.3 "Cache Update").
__global__ void k_rewindow(int32_t* st, StateMap sm, int B, int W, int S) {
    const int buf_len = st[sm.params + PARAM_BUF_LEN];
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B * W) return;
    const int b = i / W, j = i % W;
    const int p = st[sm.g + b] + j - 1;
    st[sm.win + i] = j == 0 ? st[sm.newest + b] : (p < buf_len ? st[sm.buf + (size_t)b * S + p] : 0);
}
hipError_t fc_rewindow(int32_t* state, const StateMap& sm, int B, int W, int S, hipStream_t st) {
    k_rewindow<<<(B * W + 255) / 256, 256, 0, st>>>(state, sm, B, W, S);
    return hipGetLastError();
}

hipError_t fc_accept_commit(int32_t* state, const StateMap& sm, int B, int W, int S, hipStream_t st) {
    const int waves = B < 16 ? (B < 1 ? 1 : B) : 16;
    k_accept_commit<<<1, 64 * waves, 0, st>>>(state, sm, B, W, S);
    return hipGetLastError();
}

// ------------------------------------------------------------------ sequence slots
// Two sequences trade slots: every per-sequence entry of the state block (one workgroup) ...
__global__ void k_swap_seq(int32_t* st, StateMap sm, int b1, int b2, int W, int S) {
    const int t = threadIdx.x;
    if (t < 9) {
        const int32_t offs[9] = {sm.n, sm.g, sm.done, sm.steps, sm.newest, sm.lastK, sm.plen, sm.olen, sm.wseq};
        const int32_t v1 = st[offs[t] + b1], v2 = st[offs[t] + b2];
        st[offs[t] + b1] = v2; st[offs[t] + b2] = v1;
    }
    for (int j = t; j < W; j += blockDim.x) {
        const int32_t v1 = st[sm.win + b1 * W + j], v2 = st[sm.win + b2 * W + j];
        st[sm.win + b1 * W + j] = v2; st[sm.win + b2 * W + j] = v1;
    }
    const int32_t rows[3] = {sm.buf, sm.out, sm.prompt};
    for (int r = 0; r < 3; ++r)
        for (int j = t; j < S; j += blockDim.x) {
            const int32_t v1 = st[rows[r] + b1 * S + j], v2 = st[rows[r] + b2 * S + j];
            st[rows[r] + b1 * S + j] = v2; st[rows[r] + b2 * S + j] = v1;
        }
}
// ... and their K/V cache: `count` chunks of n16 sixteen-byte words, chunk i at a + i * stride16 and b + i * stride16
__global__ void k_swap_chunks(uint4* a, uint4* b, size_t n16, size_t stride16) {
    uint4* pa = a + (size_t)blockIdx.y * stride16; uint4* pb = b + (size_t)blockIdx.y * stride16;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) {
        const uint4 va = pa[i], vb = pb[i];
        pa[i] = vb; pb[i] = va;
    }
}
hipError_t fc_swap_sequences(int32_t* state, const StateMap& sm, int b1, int b2, int W, int S, void* kc, void* vc,
                             size_t seq_bytes, int layers, size_t layer_stride_bytes, hipStream_t st) {
    if (b1 == b2) return hipSuccess;
    if (seq_bytes % 16 || layer_stride_bytes % 16) return hipErrorInvalidValue;
    k_swap_seq<<<1, 256, 0, st>>>(state, sm, b1, b2, W, S);
    const size_t n16 = seq_bytes / 16;
    unsigned gx = (unsigned)((n16 + 255) / 256);
    if (gx > 2048) gx = 2048;
    for (int which = 0; which < 2; ++which) {
        char* base = (char*)(which ? vc : kc);
        k_swap_chunks<<<dim3(gx, (unsigned)layers), 256, 0, st>>>((uint4*)(base + (size_t)b1 * seq_bytes), (uint4*)(base + (size_t)b2 * seq_bytes),
                                                                 n16, layer_stride_bytes / 16);
    }
    return hipGetLastError();
}
