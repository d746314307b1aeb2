// Device-resident decoding state shared by the per-pass kernels and the fused decode kernel.
#pragma once
#include "common.hpp"
#include "entropy.hpp"

namespace ead {

// Per-sequence decoding state, all device arrays indexed by sequence.
struct SeqState {
    int *tokens;            // [max_batch][max_seq] prompt + generated
    int *len;               // tokens present
    int *kvlen;             // [2][max_batch] positions each model has consumed
    int *model, *c, *ngen, *done, *last_step;
    int *goal;              // tokens a sequence may have generated before it pauses (<= the run's bound)
    float *ring;            // [max_batch][w_cap]
    int *out_tok; uint8_t *out_mid; float *out_H; float *out_Hbar; uint8_t *out_dec;   // [max_batch][cap]
    int *forced_tok; uint8_t *forced_mid;                                              // replay, [max_batch][cap]
    int *err;
    int max_batch, max_seq, cap;
};

struct Plan { int *hdr; int *row_seq, *row_pos, *lm_row, *lm_seq; };

struct FinArgs {
    SeqState s; Plan p; GateCfg cfg;
    const EntPartial *partials; int n_part; int unit;
    int score_mode; float *sc_H; int *sc_arg;      // score: indexed by position
    int model_id, max_new, eos_id, replay, n_new, force_model, step;
    int sampling;            // 1: the token is the sampled one (st.gidx), else the arg max
    int *host_model, *host_done;   // pinned host memory, [max_batch]: next model and done flag of the sequences this pass finalizes
};

// Algorithm 1's bookkeeping for sequence b once the entropy statistics of its logits are
// known: record the token, its model and entropy, push the window, apply the switch rule,
// append the token.  Called by one thread.
__device__ __forceinline__ void lm_finalize_seq(const FinArgs &a, int b, const EntStat &st, float H) {
    const int n = a.s.ngen[b], cur = a.model_id;
    int next = cur, c = a.s.c[b];
    const float hb = gate_update(a.s.ring + (size_t)b * a.cfg.w, n, H, a.cfg, &next, &c);
    const size_t o = (size_t)b * a.s.cap + n;
    const int choice = a.sampling ? st.gidx : st.idx;
    a.s.out_tok[o] = choice; a.s.out_mid[o] = (uint8_t)cur; a.s.out_H[o] = H; a.s.out_Hbar[o] = hb;
    a.s.out_dec[o] = (uint8_t)next;
    int tok = choice;
    if (a.replay) {
        tok = a.s.forced_tok[o];
        const int nxt = (n + 1 < a.n_new) ? a.s.forced_mid[o + 1] : cur;
        if (nxt != cur) c = 0;
        next = nxt;
    }
    if (a.force_model >= 0) next = a.force_model;
    const int L = a.s.len[b];
    a.s.tokens[(size_t)b * a.s.max_seq + L] = tok;
    a.s.len[b] = L + 1; a.s.ngen[b] = n + 1;
    const int done = (n + 1 >= a.max_new) || (a.eos_id >= 0 && tok == a.eos_id);
    a.s.done[b] = done;
    a.s.model[b] = next; a.s.c[b] = c; a.s.last_step[b] = a.step;
    // what the host's mirror needs after the pass, written where it can read it without a copy
    if (a.host_model) { a.host_model[b] = next; a.host_done[b] = done; }
    if (!isfinite(H)) atomicOr(a.s.err, 1);
}

// One wave per sequence that gets logits this pass: finish entropy and arg max from the
// LM-head partials, then run the bookkeeping above.
__global__ __launch_bounds__(64) void k_lm_finalize(FinArgs a) {
    const int i = blockIdx.x;
    if (i >= a.p.hdr[1]) return;
    const EntStat st = merge_partials(a.partials + (size_t)i * a.n_part, a.n_part);
    const float H = entropy_from(st, a.unit);
    if (threadIdx.x != 0) return;
    const int b = a.p.lm_seq[i];
    if (a.score_mode) {
        const int pos = a.p.row_pos[a.p.lm_row[i]];
        a.sc_H[pos] = H; a.sc_arg[pos] = st.idx;
        return;
    }
    lm_finalize_seq(a, b, st, H);
}

}  // namespace ead
