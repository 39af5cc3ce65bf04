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
template <int NW, int HD, int G, int MODE = 0>
__device__ __forceinline__ bool attention_phase_tagged(const DevModel& M, const DevKV& KV, const int* pos, int batch, int layer,
                                                       uint8_t* lds, u32 in_tag, u32 out_tag, u32 out_cnt, const UDiv& nc, WgVote& vote, u64* ev = nullptr,
                                                       uint8_t* merged_img = nullptr) {
    constexpr int NT = NW * 64;
    const int ncta = (int)nc.n;
    const int share = max(1, (int)((u32)ncta / (u32)(batch * M.Hkv)));
    int base = 0;
    bool ok = true;
    TaggedAttnIO xio{in_tag, out_tag, &vote};
    for (int b = 0; b < batch; b++) {
        const int T = max(pos[b], 0);   // (-1: the sequence sits this step out and is carried as a placeholder with an empty cache)
        const int ns = attn_nsplit(T, share);
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
