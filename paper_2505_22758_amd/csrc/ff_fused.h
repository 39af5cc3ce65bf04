// The fused whole-model decode kernel (one persistent launch per decode step).
#pragma once
#include <mutex>
#include "ff_kernels.h"

namespace ff {

// Workgroup shape of the fused kernel: one wave per SIMD, so that each wave may use the whole
// 512-entry register file of its SIMD for its tile ring.
constexpr int kFusedWaves = 4;
constexpr int kFusedThreads = kFusedWaves * 64;

__device__ __forceinline__ void compiler_fence() { asm volatile("" ::: "memory"); }

// ---------------------------------------------------------------- the fused whole-model kernel
// One launch = one decode step for all layers (paper abstract, Section 4).  Phases per layer:
// [RMSNorm + QKV projection + RoPE + cache append] [split-KV attention + merge] [output projection]
// [residual + RMSNorm + gate/up projection + SwiGLU] [down projection]; then residual + final norm
// + LM head.  The residual additions are folded into the staging of the next normalised
// projection, so no projection epilogue reads global memory.
//
// Synchronisation between phases is by dataflow on tagged values (see tagged_t): a phase starts in
// a workgroup as soon as the vector it consumes carries the producing phase's tag.  The paper's
// kernel separates the same phases with an atomic device-wide barrier plus fences (Section 4.1);
// on this chip a barrier round trip, the wait for store acknowledgements before it and the input
// load after it are three dependent trips through a memory pipeline that is full of weight
// traffic, so the dependency is carried by the data instead.
//
// Memory pipeline (the paper's cross-layer overlap, Section 4.1, re-designed for CDNA4): each of
// wave owns a ring of kDepth register stages of 16-byte non-temporal weight loads.  When a phase
// ends, the first kDepth stages of the NEXT weight matrix are issued at once and the loads of the
// next input vector right behind them, speculatively: by the time they return (results come back
// in issue order) the other workgroups have usually published their part, so HBM keeps streaming
// while the dependency resolves.
//
// The projections of all phases run through ONE instance of the streaming loop; what differs per
// phase (input, epilogue) is selected at run time once per row pair.
enum { PH_QKV = 0, PH_O = 1, PH_GU = 2, PH_DOWN = 3, PH_LM = 4 };
// Measurement switches of a launch (debug entry points): tiles requested only after the input has
// arrived; attention shares equal for every sequence instead of by length (attn_share_of).
enum { kSwNoOverlap = 1, kSwUniformShares = 2 };
enum { TAG_QKV = 0, TAG_ATT = 1, TAG_O = 2, TAG_GU = 3, TAG_DOWN = 4 };

// Optional profile (100 MHz wall clock), written only while a buffer is set through the debug entry
// point.  Layout in uint64 words, P = number of projection phases, W = workgroups:
//   [0, 12P)             workgroup 0, wave 0: kEvSlots stamps per phase (EV_* below)
//   [12P, 12P + 32W)     layer 1, every wave: 8 words per wave = run end of QKV/O/GU/DOWN (0..3),
//                        run start of the same (4..7)
//   [.. , .. + 40W)      layer 1, every workgroup: 8 words per projection kind about the staging of
//                        its input: 0 entered, 1 first load checked, 2 last light wait done,
//                        3 all tags fresh, 4 staged, 5 number of stale passes; then 8 words about
//                        its attention work: 0 start, 1 queries seen, 2 rows done, 3 partial stored,
//                        4 (merging workgroups) split maxima seen, 5 merged output stored, 6 end
enum { EV_SYNCED = 0, EV_RUN_DONE = 1, EV_PF_ISSUED = 2, EV_H_START = 3, EV_ATT_START = 6, EV_ATT_END = 7, kEvSlots = 12 };
__device__ __forceinline__ void dbg_event(const DevModel& M, int ph, int ev, int lane) {
    if (M.dbg && blockIdx.x == 0 && lane == 0) as_global(M.dbg)[ph * kEvSlots + ev] = wall_clock64();
}
__device__ __forceinline__ u64* dbg_wave_slots(const DevModel& M, int n_phases, int layer, int wave) {
    return M.dbg && layer == 1 ? M.dbg + (size_t)n_phases * kEvSlots + ((size_t)blockIdx.x * kFusedWaves + wave) * 8 : nullptr;
}
__device__ __forceinline__ u64* dbg_stage_slots(const DevModel& M, int n_phases, int ncta, int layer, int kind) {
    return M.dbg && layer == 1 && kind < 5 ? M.dbg + (size_t)n_phases * kEvSlots + (size_t)ncta * kFusedWaves * 8 + ((size_t)blockIdx.x * 5 + kind) * 8
                                           : nullptr;
}

struct EpiFused {
    int kind; u32 tag; u32 cnt;   // tag: 32-bit tag of q / k,v; cnt: write counter of the compact output vector
    const DevModel& M; const DevKV& KV; const int* pos; int layer; const float2* rope; float* logits;
    int pair0 = 0;   // LM head in row blocks (wide pass): first row pair of the block
    __device__ __forceinline__ void operator()(int pair, int b, float v0, float v1) const {
        switch (kind) {
            case PH_QKV: EpiQKVTagged{M, KV, pos, layer, rope, tag}(pair, b, v0, v1); break;
            case PH_GU: EpiSwiGLUTagged{M.ch, M.F, cnt, M.gu}(pair, b, v0, v1); break;
            case PH_LM: if (pos[b] >= 0) EpiStore{logits, M.V}(pair + pair0, b, v0, v1); break;   // (no logits for a sequence that sits the step out)
            default: EpiDeltaTagged{M.cdelta, M.d, cnt}(pair, b, v0, v1); break;
        }
    }
};

// Everything that distinguishes one projection phase from another.
struct PhaseDesc {
    int kind, layer;
    TSrc src;
    PMat W;
    u32 out_tag;     // 32-bit tag of this phase's tagged outputs (q, k, v; attention partials)
    u32 out_cnt;     // write counter of this phase's compact output vector
};
struct PhaseState {   // the residual stream's ping-pong buffers
    cword_t* xcur; cword_t* xnext;
};
// The buffers swap roles after every QKV and every GU phase (each publishes the updated stream into
// xnext), so which is which follows from the phase number alone.
__device__ __forceinline__ PhaseState phase_state(const DevModel& M, int ph) {
    const int k = ph & 3;
    const bool odd = k == 1 || k == 2;
    return odd ? PhaseState{M.cx2, M.cx} : PhaseState{M.cx, M.cx2};
}
__device__ __forceinline__ u32 tag_of(u32 tag_base, int l, int k) { return tag_base + 1u + (u32)(l * kTagsPerLayer + k); }

// `sl` = (steps executed so far) * L: the write counters of the compact vectors are sl + layer for the
// buffers written once per layer and 2 * (sl + layer) + {0, 1} for the sublayer output (O, then DOWN).
__device__ __forceinline__ PhaseDesc phase_desc(const DevModel& M, const int* tokens, u32 tb, u32 sl, int ph, int lm_in_kernel, const PhaseState& X, bool eager_attn) {
    PhaseDesc D;
    const int l = ph >> 2;
    const FF_CONST PLayer* Lp = as_const(M.layers) + min(l, M.L - 1);   // scalar loads (see as_const)
    D.layer = l;
    D.kind = ph == 4 * M.L ? PH_LM : (ph & 3);
    D.out_tag = 0;
    D.out_cnt = 0;
    TSrc& src = D.src;
    if (D.kind == PH_QKV) {
        if (l == 0) { src.embed = M.embed; src.tokens = tokens; src.tag = 0; }   // embedding rows are synthesised with tag 0
        else {
            src.base = X.xcur; src.stride = M.d; src.tag = sl + l - 1;
            src.add = M.cdelta; src.add_stride = M.d; src.add_tag = 2 * (sl + l - 1) + 1;
        }
        src.wb = X.xnext; src.wb_stride = M.d; src.wb_tag = sl + l;
        src.gain = Lp->g1; src.eps = M.eps;
        D.out_tag = tag_of(tb, l, TAG_QKV);
        D.W = FF_PMAT_FIELDS(Lp->qkv);
    } else if (D.kind == PH_O) {
        src.base = M.cattn_o; src.stride = (size_t)M.Hq * M.hd; src.tag = sl + l;
        src.eager = eager_attn;
        D.out_cnt = 2 * (sl + l);
        D.W = FF_PMAT_FIELDS(Lp->o);
    } else if (D.kind == PH_GU) {
        src.base = X.xcur; src.stride = M.d; src.tag = sl + l;
        src.add = M.cdelta; src.add_stride = M.d; src.add_tag = 2 * (sl + l);
        src.wb = X.xnext; src.wb_stride = M.d; src.wb_tag = sl + l;
        src.gain = Lp->g2; src.eps = M.eps;
        D.out_cnt = sl + l;
        D.W = FF_PMAT_FIELDS(Lp->gu);
    } else if (D.kind == PH_DOWN) {
        src.base = M.ch; src.stride = M.F; src.tag = sl + l;
        D.out_cnt = 2 * (sl + l) + 1;
        D.W = FF_PMAT_FIELDS(Lp->down);
    } else {
        src.base = X.xcur; src.stride = M.d; src.tag = sl + M.L - 1;
        src.add = M.cdelta; src.add_stride = M.d; src.add_tag = 2 * (sl + M.L - 1) + 1;
        src.gain = M.gf; src.eps = M.eps;
        D.W = M.lm;
    }
    return D;
}

// The whole step of a wide pass (see ff_wide.h): the same phases, with activations exchanged as
// images of the consumers' LDS layout, epochs instead of per-word counters, and the residual stream
// kept by the workgroups that own its rows.  The step's embedding rows (residual rows, first image,
// partial sums of squares) are prepared by k_wide_embed, launched in front of the fused kernel.
// n_lm: LM-head phases (row blocks of at most kDenseMaxTiles tiles per workgroup), 0 = not here.
// Returns false after a time-out (status is set).
#ifndef FF_WIDE_SPLIT
#define FF_WIDE_SPLIT 1   // K split of the wide pass's output and down projections (0: every workgroup multiplies its own rows over all of K)
#endif
template <int WD, int HD, int G>
__device__ __forceinline__ bool wide_loop(const DevModel& M, const DevKV& KV, const int* pos_lds, const int* share_lds, const float2* rope_lds, float* logits, int batch,
                                          int n_lm, int ncta, uint8_t* lds, WgVote& vote, u32 steps_done, u32 sl, u32 tag_base) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const UDiv n_ctas = UDiv::of((u32)ncta);
    float4* xs = (float4*)lds;
    float* rs = (float*)(lds + kLdsActBytes);   // aux region: 1/rms per sequence, scratch of the reduction, verdict word
    float* part = rs + 16;
    const WideSync sync{M.wflag, ncta, (lds_u32*)(part + 256), M.wpflag};
    float* ssl = (float*)(lds + 64 * 1024);     // behind the partial tiles of the reduction (at most 56 KB)
    const u32 ebase = steps_done * (u32)(4 * M.L);   // epochs of this step: ebase + 4 l + {1: attention, 2: O, 3: gate/up, 4: down}
    const int n_phases = 4 * M.L + n_lm;
    mfma_f4 acc[kDenseMaxTiles];
    typename WideStageOf<WD>::type ring[2];
    DenseCursor cur{0, 0};   // int8, int4: next stage to load
    for (int ph = 0; ph < n_phases; ph++) {
        const int lm_block = max(ph - 4 * M.L, 0);
        PhaseDesc D = phase_desc(M, nullptr, tag_base, sl, ph - lm_block, 1, phase_state(M, ph - lm_block), true);
        EpiFused epf{D.kind, D.out_tag, D.out_cnt, M, KV, pos_lds, D.layer, rope_lds, logits};
        if (D.kind == PH_LM) {
            const int block_rows = kDenseMaxTiles * 16 * ncta, row0 = lm_block * block_rows;
            D.W.w += (size_t)row0 * D.W.row_bytes();
            if constexpr (WD == W_INT8) D.W.s += row0;   // row scales of the block
            if constexpr (WD == W_INT4) { D.W.s += (size_t)row0 * (D.W.k / 128); D.W.z += (size_t)row0 * (D.W.k / 128); }   // group scales and zeros
            D.W.n = min(block_rows, D.W.n - row0);
            epf.pair0 = row0 >> 1;
        }
        const int l = D.layer;
        const FF_CONST PLayer* Lp = as_const(M.layers) + min(l, M.L - 1);
        // output and down projection: K split between the workgroups of a pair where the shapes allow (see DenseStream)
        const bool split = FF_WIDE_SPLIT && (D.kind == PH_O || D.kind == PH_DOWN) && DenseStream::can_split(D.W, n_ctas);
        DenseStream DS = DenseStream::make<WD>(D.W, 0, n_ctas, split);
        const int seg0 = DS.seg0, seg1 = DS.seg1;
        DS = DenseStream::make<WD>(D.W, seg0, n_ctas, split);
        if constexpr (WD == W_INT4) dense_prefetch_i4(DS, cur, ring, wave, lane);
        else if constexpr (WD == W_INT8) dense_prefetch_i8(DS, cur, ring, wave, lane);
        else dense_prefetch(DS, ring, wave, lane);
        u32 wait_epoch = 0;
        const uint8_t* img = M.wimg_x;
        bool normed = true;
        if (D.kind == PH_QKV) wait_epoch = l > 0 ? ebase + 4u * (u32)l : 0u;
        else if (D.kind == PH_O) {
            __syncthreads();   // the previous projection's epilogue has read its sums out of LDS
            const bool ok = attention_phase_tagged<kFusedWaves, HD, G, 2>(M, KV, pos_lds, share_lds, batch, l, lds, tag_of(tag_base, l, TAG_QKV), tag_of(tag_base, l, TAG_ATT),
                                                                      sl + l, n_ctas, vote, nullptr, M.wimg_a);
            if (!ok) return false;
            sync.arrive(ebase + 4u * (u32)l + 1u);
            wait_epoch = ebase + 4u * (u32)l + 1u; img = M.wimg_a; normed = false;
        } else if (D.kind == PH_GU) wait_epoch = ebase + 4u * (u32)l + 2u;
        else if (D.kind == PH_DOWN) { wait_epoch = ebase + 4u * (u32)l + 3u; img = M.wimg_h; normed = false; }
        else wait_epoch = ebase + 4u * (u32)M.L;
        if (wait_epoch) {
            if (!sync.wait(wait_epoch, wave, lane)) {
                if (threadIdx.x == 0) atomicCAS(M.status, 0, -55 - 10 * ph);
                return false;
            }
        } else __syncthreads();
        if (normed) wide_rms(M.wsspart, ncta, D.W.k, M.eps, part, rs, threadIdx.x);
#pragma unroll
        for (int t = 0; t < kDenseMaxTiles; t++) acc[t] = mfma_f4{0.f, 0.f, 0.f, 0.f};
        bool run_ok = true;
        for (int seg = seg0; seg < seg1; seg++) {
            DS = DenseStream::make<WD>(D.W, seg, n_ctas, split);
            if (DS.T > 0) wide_copy_quarter(img + (size_t)seg * kWideSegBytes, lds, wave, lane, batch);   // (private to the wave: no barrier)
            const float* rsp = normed ? rs : nullptr;
            const int par = ((seg - seg0) * (WD == W_INT4 ? (DS.T + 1) >> 1 : DS.T)) & 1;   // int8, int4: ring slot of the segment's first stage
            if (D.kind == PH_GU) dense_run_wide<WD>(DS, ring, xs, acc, batch, wave, lane, WideEpiSwiGLU{M.wimg_h, M.gu}, rsp, nullptr, nullptr, 0u, &cur, par);
            else if (D.kind == PH_O)
                run_ok = dense_run_wide<WD>(DS, ring, xs, acc, batch, wave, lane, WideEpiResidual{M.wxres, M.d, Lp->g2, M.wimg_x, ssl, DS.own0}, rsp,
                                            M.wxch, &sync, ebase + 4u * (u32)l + 2u, &cur, par);
            else if (D.kind == PH_DOWN)
                run_ok = dense_run_wide<WD>(DS, ring, xs, acc, batch, wave, lane,
                                            WideEpiResidual{M.wxres, M.d, l + 1 < M.L ? (as_const(M.layers) + l + 1)->g1 : M.gf, M.wimg_x, ssl, DS.own0}, rsp,
                                            M.wxch, &sync, ebase + 4u * (u32)l + 4u, &cur, par);
            else dense_run_wide<WD>(DS, ring, xs, acc, batch, wave, lane, WideEpiPairs<EpiFused>{epf}, rsp, nullptr, nullptr, 0u, &cur, par);
        }
        if (!run_ok) {   // (uniform) the partner of a K-split projection did not deliver
            if (threadIdx.x == 0) atomicCAS(M.status, 0, -58 - 10 * ph);
            return false;
        }
        if (D.kind == PH_O || D.kind == PH_DOWN) {
            // this workgroup's share of every sequence's sum of squares of the new residual rows
            __syncthreads();
            if (threadIdx.x < kMaxBatchWide) {
                float t = 0.f;
                const int ngrp = (DS.own1 - DS.own0) >> 2;
                if ((int)threadIdx.x < batch) for (int q = 0; q < ngrp; q++) t += ssl[q * kMaxBatchWide + threadIdx.x];
                xst(M.wsspart + (size_t)blockIdx.x * kMaxBatchWide + threadIdx.x, t);
            }
        }
        if (D.kind == PH_O) sync.arrive(ebase + 4u * (u32)l + 2u);
        else if (D.kind == PH_GU) sync.arrive(ebase + 4u * (u32)l + 3u);
        else if (D.kind == PH_DOWN) sync.arrive(ebase + 4u * (u32)l + 4u);
    }
    return true;
}

// Attention form of the passes of up to four sequences (see attn_item): 0 = row by row on the vector
// ALU, 1 = scores of 16 cached rows at a time on the matrix cores (head dimension 128 only).  With
// eight query heads per KV head the row-wise form is bound by the vector ALU (the 70B shape at batch
// 1: 23.8 -> 23.3 ms per step with form 1); with four, form 1 is ahead by 0.2 % (8B bf16, batch 1,
// context 1024) to 1.1 % (context 6144).  FF_ATTN_MODE / FF_ATTN_MODE_I4 override at build time.
#ifndef FF_ATTN_MODE
#define FF_ATTN_MODE 1
#endif
#ifndef FF_ATTN_MODE_I4
#define FF_ATTN_MODE_I4 0   // int4 instances: form 1 spills a few registers at batch 2-4 and measured 1 % slower there
#endif
template <int WD> constexpr int kAttnModeOf = WD == W_INT4 ? FF_ATTN_MODE_I4 : FF_ATTN_MODE;
template <int WD, int B, int HD, int G>
__global__ void __launch_bounds__(kFusedThreads) fused_decode_kernel(DevModel M, DevKV KV, const int* __restrict__ tokens,
                                                                     const int* __restrict__ pos, float* __restrict__ logits,
                                                                     int batch, int lm_in_kernel, int ncta, int mute_wg, int switches, int glu_off) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    if (!inputs_ok(M, KV, tokens, pos)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicExch(M.status, kStatusRange);
        return;
    }
    // Test hook for the time-out path: the muted workgroup publishes nothing, so every workgroup
    // that needs its output runs into its own bounded wait, records the time-out and leaves.
    if ((int)blockIdx.x == mute_wg) return;
    constexpr int EPU = WTraits<WD>::EPU;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float4* xs = (float4*)lds;
    // The wide instance (up to 16 sequences, bf16 weights) keeps its RoPE rows in the tail of the aux
    // region that only int4 weights use plus the regular RoPE region behind it, and its positions
    // in the mailbox region (no wave pairs share a row group there).
    constexpr bool kWide = B > kMaxBatchFused;
    static_assert(!kWide || (kLdsXsumBytes + kLdsRopeBytes >= B * 64 * (int)sizeof(float2) && kLdsPairBytes >= B * 4 && B <= kMaxBatchWide),
                  "LDS layout of the wide pass");
    float2* rope_lds = (float2*)(lds + kLdsActBytes + kLdsAuxBytes - (kWide ? kLdsXsumBytes : 0));   // [batch][hd/2]
    for (int i = threadIdx.x; i < batch * (M.hd / 2); i += kFusedThreads) {
        int b = i / (M.hd / 2), f = i % (M.hd / 2);
        rope_lds[i] = KV.rope[(size_t)max(step_pos(tokens, pos, b), 0) * (M.hd / 2) + f];
    }
    // Launch dimensions and positions are read again and again below; a vector load of them would
    // make the wave wait for everything it has in flight (its prefetched weight tiles included), so
    // the grid size is a kernel argument and the positions are staged in LDS once.
    static_assert(kLdsRopeBytes == kMaxBatchFused * 64 * sizeof(float2) && kLdsMiscBytes >= (16 + 2 * (1 + WgVote::kMaxSums) * kFusedWaves) * 4, "LDS layout");
    int* pos_lds = kWide ? (int*)(lds + kLdsActBytes + kLdsAuxBytes + kLdsRopeBytes + kLdsMiscBytes)
                         : (int*)((float*)(lds + kLdsActBytes + kLdsAuxBytes) + 2 * kMaxBatchFused * 64 + 8);
    int* share_lds = pos_lds + (kWide ? kMaxBatchWide : kMaxBatch);   // workgroups per kv head of each sequence's attention (attn_share_of)
    static_assert(kLdsPairBytes >= 2 * kMaxBatchWide * 4 && 2 * kMaxBatch <= 8, "positions and attention shares in LDS");
    if ((int)threadIdx.x < batch) {
        pos_lds[threadIdx.x] = step_pos(tokens, pos, threadIdx.x);   // -1: the sequence sits this step out
        share_lds[threadIdx.x] = attn_share_of(tokens, pos, batch, threadIdx.x, ncta, M.Hkv, (switches & kSwUniformShares) != 0);
    }
    if (!kWide && threadIdx.x < 2) ((lds_u32*)(pairbox_of(xs) + 4 * kPairBoxFloats))[threadIdx.x] = 0u;
    if (B == 1 && threadIdx.x < kGluMaxChunks) ((lds_u32*)pairbox_of(xs))[threadIdx.x] = 0u;   // arrival counters of the staged h chunks (glu_run)
    __syncthreads();
    // projections only; attention runs right after each PH_QKV.  The LM head runs here unless its
    // weight type differs from the layers' (then the host launches it separately).
    // (lm_in_kernel: number of LM-head phases; 1, or with a wide pass the number of row blocks)
    const int n_phases = 4 * M.L + (kWide ? lm_in_kernel : lm_in_kernel ? 1 : 0);
    const int dbg_phases = 4 * M.L + (lm_in_kernel ? 1 : 0);   // phases the optional timeline buffer has slots for (further LM blocks share the last)
    // steps executed so far on the compact buffers (kept on the device: a skipped step does not count)
    const u32 steps_done = (u32)__builtin_amdgcn_readfirstlane(xld_u32(M.stepctr));
    const u32 sl = steps_done * (u32)M.L;
    // The 32-bit tags of this step's queries, keys, values and attention partials: a fresh range
    // per executed step, derived from the same device-side counter, so that a launch carries no
    // host-side step state (a launch recorded into a HIP graph replays correctly).  Tags wrap after
    // 2^32 / (5 L + 1) steps; a slot could only be mistaken for fresh if it had not been rewritten
    // for exactly that many steps, and every slot a step reads is rewritten by that step first.
    const u32 tag_base = steps_done * (u32)(kTagsPerLayer * M.L + 1);

    const int gwave = blockIdx.x * kFusedWaves + wave;
    const UDiv n_gwaves = UDiv::of((u32)ncta * kFusedWaves), n_ctas = UDiv::of((u32)ncta);
    float* myacc = (float*)(lds + kLdsActBytes) + (size_t)wave * kAccFloatsPerWave;
    float* red = (float*)(lds + kLdsActBytes + kLdsAuxBytes) + 2 * kMaxBatchFused * 64;   // behind the RoPE rows
    WgVote vote{(u32*)(red + 16), 0u};   // behind the reduction scratch and the positions
    // One iteration = one K segment of one projection; only (phase, segment) are carried from one
    // iteration to the next.  With kScalarState they are pinned to scalar registers, so that all
    // that derives from them (the layer's descriptor, the wave's share) is fetched and computed on
    // the scalar unit, the next descriptor is touched ahead of time, and the wait for the merged
    // attention output re-reads eagerly.  Each of the three shortens the path from the end of one
    // projection to the first tile requests of the next; with several sequences per pass that
    // pays (8B bf16, batch 4: 5.70 -> 5.61 ms); with a single one the step measured slower
    // (3.26 -> 3.30 ms; presumably the earlier requests compete with the workgroups still finishing
    // the previous projection), so batch 1 keeps the unpinned form.
    constexpr bool kScalarState = B > 1;
    constexpr bool kQuad = kQuadOf<WD, B>;   // matrix-core GEMV on groups of four rows, split-bf16 staged input
    if constexpr (kWide) {
        if (!wide_loop<WD, HD, G>(M, KV, pos_lds, share_lds, rope_lds, logits, batch, lm_in_kernel, ncta, lds, vote, steps_done, sl, tag_base)) return;
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            xst_u32(M.stepctr + 1, 0u);   // the compact exchange rows were not written: the next narrow pass re-initialises its rows
            xst_u32(M.stepctr, steps_done + 1u);
        }
        return;
    } else {
    int ph = 0, seg = 0;
    for (;;) {
        if constexpr (kScalarState) {
            ph = __builtin_amdgcn_readfirstlane(ph);
            seg = __builtin_amdgcn_readfirstlane(seg);
        }
        const PhaseDesc D = phase_desc(M, tokens, tag_base, sl, ph, lm_in_kernel, phase_state(M, ph), kScalarState);
        EpiFused epi{D.kind, D.out_tag, D.out_cnt, M, KV, pos_lds, D.layer, rope_lds, logits};
        const Stream<WD, B> S = Stream<WD, B>::make(D.W, seg, gwave, n_gwaves, kQuad);
        // The wave's first tiles of this projection are requested before anything it has to wait
        // for (its input vector; for the output projection the whole attention), so the memory
        // pipe has work while the dependency resolves.  The ring lives from here to the end of
        // gemv_run only: keeping it out of the loop-carried state lets it stay in the registers
        // the loads were issued to (a copy would have to wait for the data).
        TSrc src = D.src;
        src.ncta = n_ctas;
        if (seg > 0) src.wb = nullptr;
        const bool att_first = D.kind == PH_O && seg == 0;
        Stage<WD> ring[kDepthOf<WD>];
        // (ablation switch, single-sequence bf16 instances only: with kSwNoOverlap the tiles are requested
        // after the input has arrived, as in a fused kernel without cross-layer memory overlap)
        constexpr bool kHasSwitch = B == 1 && WD == W_BF16;
        if (!kHasSwitch || !(switches & kSwNoOverlap)) prefetch_stream<kQuad>(S, ring, lane, 0, kPrefetchOf<WD>);
        if (wave == 0) dbg_event(M, min(ph, dbg_phases - 1), EV_PF_ISSUED, lane);
        // Touch the descriptor the NEXT phase will fetch, so that it sits in the scalar cache by
        // then instead of costing a trip to memory at the head of that phase.
        u32 warm = 0;
        if constexpr (kScalarState) {
            const FF_CONST u32* nd = (const FF_CONST u32*)(as_const(M.layers) + min((ph + 1) >> 2, M.L - 1));
            warm = nd[0] ^ nd[16] ^ nd[32] ^ nd[sizeof(PLayer) / 4 - 1];
        }
        if (att_first) {
            // split-KV attention + merge of this layer (the ring holds the output projection's tiles)
            __syncthreads();   // every wave has finished reading the staged input: LDS is free
            if (wave == 0) dbg_event(M, min(ph, dbg_phases - 1), EV_ATT_START, lane);
            u64* aev = dbg_stage_slots(M, dbg_phases, ncta, D.layer, 4);
            if (aev && threadIdx.x == 0) { as_global(aev)[0] = wall_clock64(); as_global(aev)[4] = 0; as_global(aev)[5] = 0; }
            const bool ok = attention_phase_tagged<kFusedWaves, HD, G, kAttnModeOf<WD>>(M, KV, pos_lds, share_lds, batch, D.layer, lds, tag_of(tag_base, D.layer, TAG_QKV),
                                                                tag_of(tag_base, D.layer, TAG_ATT), sl + D.layer, n_ctas, vote, aev);
            if (aev && threadIdx.x == 0) as_global(aev)[6] = wall_clock64();
            if (wave == 0) dbg_event(M, min(ph, dbg_phases - 1), EV_ATT_END, lane);
            if (!ok) return;
        }
        if (wave == 0) dbg_event(M, min(ph, dbg_phases - 1), EV_H_START, lane);
        bool ok;
        u64* ev = dbg_stage_slots(M, dbg_phases, ncta, D.layer, D.kind);
        if (src.add) ok = stage_tagged<EPU, true, kFusedThreads, kQuad, B>(src, batch, S.K, S.j0 * EPU, S.nunits, S.nup, xs, red, threadIdx.x, vote, ev);
        else ok = stage_tagged<EPU, false, kFusedThreads, kQuad, B>(src, batch, S.K, S.j0 * EPU, S.nunits, S.nup, xs, red, threadIdx.x, vote, ev);
        if (ev && threadIdx.x == 0) as_global(ev)[4] = wall_clock64();
        if (!ok) {
            if (threadIdx.x == 0) atomicCAS(M.status, 0, -55 - 10 * ph);
            return;
        }
        if (wave == 0) dbg_event(M, min(ph, dbg_phases - 1), EV_SYNCED, lane);
        if (kHasSwitch && (switches & kSwNoOverlap)) prefetch_stream<kQuad>(S, ring, lane, 0, kPrefetchOf<WD>);
        if constexpr (kPrefetchOf<WD> < kDepthOf<WD>) prefetch_stream<kQuad>(S, ring, lane, kPrefetchOf<WD>, kDepthOf<WD>);   // the rest of the ring, behind the input
        u64* wv = D.kind < 4 ? dbg_wave_slots(M, dbg_phases, D.layer, wave) : nullptr;
        if (wv && lane == 0) as_global(wv)[4 + D.kind] = wall_clock64();
        bool glu_done = false;
        if constexpr (B == 1) {
            if (glu_off >= 0 && D.kind == PH_GU) {
                // gate/up, SwiGLU and down projection as one stream, the down projection's input
                // staged chunk by chunk on the way (glu_run); the DOWN phase below is skipped
                const PhaseDesc Dd = phase_desc(M, tokens, tag_base, sl, ph + 1, lm_in_kernel, phase_state(M, ph + 1), false);
                const Stream<WD, B> Sd = Stream<WD, B>::make(Dd.W, 0, gwave, n_gwaves, false);
                const int pd = (int)n_gwaves.div((u32)(M.d / 2) + n_gwaves.n - 1u);   // most down-projection row pairs a wave owns
                float* lacc = (float*)(lds + kLdsActBytes + kLdsAuxBytes) - (size_t)(kFusedWaves - wave) * pd * 128;
                GluStager<WD> stg{M.ch, sl + (u32)D.layer, M.F, Sd.nup, Sd.cpr, (float4*)(lds + glu_off), (lds_u32*)pairbox_of(xs)};
                EpiSwiGLUTagged epig{M.ch, M.F, D.out_cnt, M.gu};
                EpiDeltaTagged epid{M.cdelta, M.d, Dd.out_cnt};
                const bool okg = glu_run<WD>(S, Sd, ring, xs, stg, lacc, (u32)kFusedWaves * (u32)(D.layer + 1),
                                             kChunkUnitsOf<WD> * WTraits<WD>::EPU / M.gu.nw, lane, epig, epid);
                if (!okg) {
                    if (lane == 0) atomicCAS(M.status, 0, -57 - 10 * ph);
                    return;
                }
                if (wv && lane == 0) as_global(wv)[PH_DOWN] = wall_clock64();
                glu_done = true;
            }
        }
        if (glu_done) { /* both projections are finished */ }
        else if constexpr (kQuad) gemv_run_quad<WD, B>(S, ring, xs, myacc, batch, lane, epi);
        else gemv_run<WD, B>(S, ring, xs, myacc, batch, lane, epi);
        asm volatile("" ::"s"(warm));   // keeps the touch alive
        if (wave == 0) dbg_event(M, min(ph, dbg_phases - 1), EV_RUN_DONE, lane);
        if (wv && lane == 0) as_global(wv)[D.kind] = wall_clock64();
        // next iteration: further K segment of the same projection, or the next projection
        if (glu_done) ++ph;   // the down projection ran inside glu_run
        if (seg + 1 < S.nseg) ++seg;
        else if (ph + 1 < n_phases) { ++ph; seg = 0; }
        else break;
    }
    // this step has been executed: the next one uses the next write counters (workgroup 0 can only
    // get here after every workgroup has taken part in every phase, i.e. has read the counter)
    // Word 1 of the counter block: sequences whose compact exchange rows this launch has written
    // (k_scrub_rows re-initialises further rows before a larger batch runs).
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        xst_u32(M.stepctr + 1, (u32)batch);
        xst_u32(M.stepctr, steps_done + 1u);
    }
    }   // (!kWide)
}

// Host-side launcher of one weight-type family; defined once per weight type in its own
// translation unit so that the instances compile in parallel.
struct FusedLaunch {
    DevModel M; DevKV KV; const int* tokens; const int* pos; float* logits;
    int batch; int lm_in_kernel; int n_cta; size_t lds_bytes; hipStream_t stream; int mute_wg; int switches;   // switches: kSw* bits
    int glu_off;   // >= 0: single-sequence passes run gate/up + down as one stream (glu_run), staged h at this LDS offset
    int wide;      // the pass runs on the wide instance (K-segmented inputs, LM head outside the kernel)
};
template <int WD, int B, int HD, int G>
inline hipError_t launch_fused_instance(const FusedLaunch& a, const char** what) {
    auto kern = fused_decode_kernel<WD, B, HD, G>;
    // one-time set-up per instance (thread-safe; a failure is remembered and reported by every call)
    static std::once_flag once;
    static hipError_t setup_err = hipSuccess;
    static const char* setup_what = "";
    std::call_once(once, [&] {
        setup_err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.lds_bytes);
        if (setup_err != hipSuccess) { setup_what = "hipFuncSetAttribute"; return; }
        int occ = 0;
        setup_err = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kern, kFusedThreads, a.lds_bytes);
        if (setup_err != hipSuccess) { setup_what = "hipOccupancyMaxActiveBlocksPerMultiprocessor"; return; }
        if (occ < 1) { setup_what = "fused kernel does not fit on a compute unit"; setup_err = hipErrorLaunchOutOfResources; }
    });
    if (setup_err != hipSuccess) { *what = setup_what; return setup_err; }
    kern<<<a.n_cta, kFusedThreads, a.lds_bytes, a.stream>>>(a.M, a.KV, a.tokens, a.pos, a.logits, a.batch, a.lm_in_kernel, a.n_cta, a.mute_wg, a.switches, a.glu_off);
    *what = "fused kernel launch";
    return hipGetLastError();
}
template <int WD, int HD, int G>
inline hipError_t launch_fused_family(const FusedLaunch& a, const char** what) {
    if (a.wide) return launch_fused_instance<WD, kMaxBatchWide, HD, G>(a, what);   // (the host decides, and sizes lm_in_kernel and the buffers for it)
    if (a.batch == 1) return launch_fused_instance<WD, 1, HD, G>(a, what);
    if (a.batch == 2) return launch_fused_instance<WD, 2, HD, G>(a, what);
    if (a.batch > kMaxBatch) {
        *what = "more than four sequences per pass without the wide instance";
        return hipErrorInvalidValue;
    }
    return launch_fused_instance<WD, 4, HD, G>(a, what);
}
// One definition per (weight type, head geometry), each in its own translation unit.
#define FF_FUSED_FAMILIES(X) \
    X(bf16, W_BF16, 64, 4) X(bf16, W_BF16, 128, 4) X(bf16, W_BF16, 128, 8) \
    X(int8, W_INT8, 64, 4) X(int8, W_INT8, 128, 4) X(int8, W_INT8, 128, 8) \
    X(int4, W_INT4, 64, 4) X(int4, W_INT4, 128, 4) X(int4, W_INT4, 128, 8)
#define FF_DECLARE_FAMILY(name, wd, hd, g) hipError_t launch_fused_##name##_hd##hd##_g##g(const FusedLaunch& a, const char** what);
FF_FUSED_FAMILIES(FF_DECLARE_FAMILY)
#undef FF_DECLARE_FAMILY

}  // namespace ff
