// Kernels: the fused whole-model decode step, the per-operation baseline, and the loaders.
#pragma once
#include "ff_phases.h"
#include "ff_glu.h"
#include "ff_dense.h"
#include "ff_wide.h"

namespace ff {

constexpr int kTagsPerLayer = 5;   // phase instances (= exchange tags) per layer of the fused kernel

// status codes written by kernels (mirror the C ABI's FF_ERR_*)
constexpr int kStatusRange = -3;
constexpr int kStatusTimeout = -5;

// tokens / pos point to the first sequence of the current pass; the check covers every sequence of
// the whole decode step (all passes), so that a bad token or position anywhere skips every pass.
__device__ __forceinline__ bool inputs_ok(const DevModel& M, const DevKV& KV, const int* tokens, const int* pos) {
    bool ok = true;
    for (int b = -KV.seq0; b < KV.step_batch - KV.seq0; b++) {
        int p = pos[b], t = tokens[b];
        ok = ok && (t == kTokenSkip || (p >= 0 && p < KV.max_ctx && t >= 0 && t < M.V));
    }
    return ok;
}

// Attention work distribution: the items (sequence b, kv head j, split s) of all sequences form
// one list that is dealt round-robin to the workgroups (a per-layer work queue with a static
// owner per entry; the split count follows each sequence's current length).
template <int NW>
__device__ void attention_phase_plain(const DevModel& M, const DevKV& KV, const int* tokens, const int* pos, int batch, int layer, uint8_t* lds) {
    const int G = M.Hq / M.Hkv;
    const int share = max(1, (int)gridDim.x / (batch * M.Hkv));
    int base = 0;
    PlainAttnIO xio;
    for (int b = 0; b < batch; b++) {
        const int T = max(step_pos(tokens, pos, b), 0);
        const int ns = attn_nsplit(T, share);
        const int nitems = M.Hkv * ns;
        int first = ((int)blockIdx.x - base) % (int)gridDim.x;
        if (first < 0) first += gridDim.x;
        for (int it = first; it < nitems; it += gridDim.x) {
            int j = it / ns, s = it % ns;
            int t0 = (int)((long)T * s / ns), t1 = (int)((long)T * (s + 1) / ns);
            bool cur = s == ns - 1;
            if (M.hd == 64 && G == 4) attn_item<64, 4, NW>(M, KV, xio, layer, b, j, t0, t1, cur, s, lds);
            else if (M.hd == 128 && G == 4) attn_item<128, 4, NW>(M, KV, xio, layer, b, j, t0, t1, cur, s, lds);
            else if (M.hd == 128 && G == 8) attn_item<128, 8, NW>(M, KV, xio, layer, b, j, t0, t1, cur, s, lds);
        }
        base = (base + nitems) % (int)gridDim.x;
    }
}

// Fused kernel: queries / current k,v are awaited through their tags; the workgroup that owns the
// last split of (b, j) also merges all splits of that head group (paper Section 4.2: the reduction
// is fused into the attention pass instead of a separate kernel).  The head geometry is a template
// parameter here (one kernel instance per geometry) to keep the register footprint of the fused
// kernel down to what the model at hand needs.  `pos` points to the positions staged in LDS and
// ncta is the grid size: both are read often, and fetching them from global memory here would make
// the wave wait for every load it has in flight, weight tiles included.
// Workgroups per (sequence, kv head) for a step's attention, by the sequences' lengths: every
// sequence gets one per kv head, and what is left of the grid is dealt out in proportion to the
// rows each has to read (cached rows + its own).  A sequence much longer than its neighbours is cut
// into correspondingly more slices, so the slices of a ragged batch come out about equally long
// instead of the long sequence's being as many times longer as it is (the paper names load balance
// at variable context as the reason for scheduling at run time, Section 6); with equal lengths this
// is the equal division n_workgroups / (batch * Hkv).  The shares sum to at most n_workgroups / Hkv.
// Every workgroup computes the same list from the step's positions: the work list is rebuilt each
// step, its entries have fixed owners, nothing is claimed with atomics.
__device__ __forceinline__ int attn_share_of(const int* tokens, const int* pos, int batch, int b, int ncta, int Hkv, bool uniform) {
    const u32 floor_items = (u32)(batch * Hkv);
    const u32 budget = (u32)ncta > floor_items ? (u32)ncta - floor_items : 0u;
    if (uniform) return 1 + (int)(budget / floor_items);
    u32 tot = 0;
    for (int i = 0; i < batch; i++) tot += (u32)max(step_pos(tokens, pos, i), 0) + 1u;
    const u32 mine = (u32)max(step_pos(tokens, pos, b), 0) + 1u;
    return 1 + (int)((u32)((u64)budget * mine / tot) / (u32)Hkv);
}

// share: workgroups per kv head of each sequence (attn_share_of), staged in LDS like the positions.
template <int NW, int HD, int G, int MODE = 0>
__device__ __forceinline__ bool attention_phase_tagged(const DevModel& M, const DevKV& KV, const int* pos, const int* share, int batch, int layer,
                                                       uint8_t* lds, u32 in_tag, u32 out_tag, u32 out_cnt, const UDiv& nc, WgVote& vote, u64* ev = nullptr,
                                                       uint8_t* merged_img = nullptr) {
    constexpr int NT = NW * 64;
    const int ncta = (int)nc.n;
    int base = 0;
    bool ok = true;
    TaggedAttnIO xio{in_tag, out_tag, &vote};
    for (int b = 0; b < batch; b++) {
        const int T = max(pos[b], 0);   // (-1: the sequence sits this step out and is carried as a placeholder with an empty cache)
        const int ns = attn_nsplit(T, share[b]);
        const int nitems = M.Hkv * ns;
        // (32-bit unsigned arithmetic throughout: this runs between the end of the QKV projection
        // and the first cache loads, and 64-bit or signed divisions are long instruction sequences)
        const int first = (int)nc.mod((u32)blockIdx.x + (u32)ncta - (u32)base);   // base < ncta
        for (int it = first; it < nitems; it += ncta) {
            const int j = (int)((u32)it / (u32)ns), s = it - j * ns;
            const int t0 = (int)((u32)T * (u32)s / (u32)ns), t1 = (int)((u32)T * (u32)(s + 1) / (u32)ns);   // T * 64 < 2^32
            bool cur = s == ns - 1;
            ok = attn_item<HD, G, NW, TaggedAttnIO, MODE>(M, KV, xio, layer, b, j, t0, t1, cur, s, lds, ev) && ok;
            if (cur) ok = attn_merge_tagged<HD, G, NT>(M, b, j, ns, out_tag, out_cnt, (float*)lds, vote, ev, merged_img) && ok;
        }
        base = (int)nc.mod((u32)base + (u32)nitems);
    }
    return ok;
}

}  // namespace ff
