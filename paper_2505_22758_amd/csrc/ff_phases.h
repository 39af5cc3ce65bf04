// Split-KV attention and the projection epilogues of the decode step.  Workgroup-collective
// device functions used by the fused kernel (ordered by tagged dataflow) and, with launch
// boundaries as the ordering, by the per-operation baseline kernels.
#pragma once
#include <type_traits>
#include "ff_gemv.h"

namespace ff {

// ---------------------------------------------------------------- tagged exchange format
// Inside the fused kernel the small exchanged values (queries, the step's own k and v, attention
// partials) travel as 8-byte pairs (fp32 bits, tag) written with one coherent 8-byte store; the big
// vectors use the compact format further down.  The tag names the phase instance that
// produced the value (it grows monotonically over phases and over decode steps), so a consumer can
// tell from the data itself whether its producer has run: it simply re-reads until every tag it
// needs matches.  Dependencies are thereby resolved by dataflow -- no device-wide barrier, no
// waiting for store acknowledgements -- and a vector is on the critical path for one store->load
// hop only (paper Section 4.1 needs a fence + global barrier on its hardware for the same RAW hazard).
#ifndef FF_TLD_AUX
#define FF_TLD_AUX 17   /* sc0 | sc1 */
#endif
typedef u32x2 tagged_t;
constexpr int kPollLanes = 8;
__device__ __forceinline__ void tst(tagged_t* p, float v, u32 tag) { xst2((float*)p, v, __uint_as_float(tag)); }
__device__ __forceinline__ void tst2(tagged_t* p, float v0, float v1, u32 tag) {
    tst(p, v0, tag);
    tst(p + 1, v1, tag);
}
__device__ __forceinline__ u32x2 tld1(const tagged_t* base, int i) {
    u64 a = __hip_atomic_load(as_global((const u64*)(base + i)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return u32x2{(u32)a, (u32)(a >> 32)};
}
// Two consecutive tagged values (base + i, i even) as (v0, tag0, v1, tag1).  8-byte agent-scope
// atomic loads are used on purpose: 16-byte buffer loads with the same cache-policy bits were
// observed to keep returning a stale copy while polling, and inline-assembly loads cannot be kept
// asynchronous safely (the compiler may copy their destination registers before the data lands).
__device__ __forceinline__ u32x4 tld2(const tagged_t* base, int i) {
    u32x2 a = tld1(base, i), b = tld1(base, i + 1);
    return u32x4{a.x, a.y, b.x, b.y};
}

// ---------------------------------------------------------------- compact exchange format
// The vectors that every workgroup reads whole (residual stream, sublayer outputs, merged attention
// output, SwiGLU output) travel as 4-byte words: the fp32 value rounded to 22 mantissa bits, with
// the low 2 bits of a per-buffer WRITE COUNTER in the freed bits.  Every element of such a buffer
// (for the sequences of the step) is rewritten each time the buffer is written, and the counter
// grows by exactly one per write, so whatever a reader can find in a slot is either the value it
// waits for or the previous write, whose counter bits differ (one bit would tell the two apart; two
// leave a margin and cost a quarter of an fp32 ulp).  The counter is derived from the number of
// steps EXECUTED on the buffers (kept on the device: a skipped step changes nothing), the layer and
// the phase.  Rows of sequences beyond the previous step's batch are re-initialised by the host
// side (a small fill) before a larger batch runs.  Two elements move per 8-byte coherent access.
typedef u32 cword_t;
constexpr u32 kCntMask = 3u;   // counter bits of a compact word
__device__ __forceinline__ u32 cpack(float v, u32 cnt) {
    const u32 b = __float_as_uint(v);
    const u32 r = (b & 0x7F800000u) == 0x7F800000u ? b : b + (kCntMask + 1u) / 2u;   // round to nearest; infinities and NaNs keep their class
    return (r & ~kCntMask) | (cnt & kCntMask);
}
__device__ __forceinline__ float cvalue(u32 w) { return __uint_as_float(w & ~kCntMask); }
__device__ __forceinline__ bool cfresh(u32 w, u32 cnt) { return ((w ^ cnt) & kCntMask) == 0; }
__device__ __forceinline__ void cst1(cword_t* p, float v, u32 cnt) { xst_u32(p, cpack(v, cnt)); }
__device__ __forceinline__ void cst2(cword_t* p, float v0, float v1, u32 cnt) {   // p 8-byte aligned
    xst2((float*)p, __uint_as_float(cpack(v0, cnt)), __uint_as_float(cpack(v1, cnt)));
}
__device__ __forceinline__ u32 cld1(const cword_t* base, int i) { return xld_u32(base + i); }
__device__ __forceinline__ u32x2 cld2(const cword_t* base, int i) {   // elements i, i+1 (i even)
    u64 a = __hip_atomic_load(as_global((const u64*)(base + i)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return u32x2{(u32)a, (u32)(a >> 32)};
}

// Workgroup-wide AND of a predicate with ONE barrier: every wave votes with a ballot, its first
// lane drops the result into an LDS slot, and after the barrier every thread reads all slots.
// Consecutive votes alternate between two sets of slots, so a wave that runs ahead to the next vote
// cannot overwrite a slot another wave has yet to read (the vote after that lies behind the next
// vote's barrier, which that other wave only reaches after its read).  All threads must take part
// in every vote, in the same order.
struct WgVote {
    static constexpr int kMaxSums = 4;
    u32* slots;   // LDS, 2 * (1 + kMaxSums) * (waves per workgroup) words
    u32 par;
    template <int NT>
    __device__ __forceinline__ bool all(bool ok) {
        const float none[1] = {0.f};
        float unused[1];
        return all_sum<NT, 1>(ok, none, unused);
    }
    // The same vote, which also adds up N (wave-uniform) floats per wave over the workgroup.
    template <int NT, int N>
    __device__ __forceinline__ bool all_sum(bool ok, const float (&part)[N], float (&total)[N]) {
        static_assert(N <= kMaxSums, "too many sums");
        constexpr int NW = NT / 64;
        const u32 w = __all(ok) ? 1u : 0u;
        u32* f = slots + par * (1 + kMaxSums) * NW;
        par ^= 1u;
        if ((threadIdx.x & 63) == 0) {
            f[threadIdx.x >> 6] = w;
#pragma unroll
            for (int n = 0; n < N; n++) f[(1 + n) * NW + (threadIdx.x >> 6)] = __float_as_uint(part[n]);
        }
        __syncthreads();
        u32 r = 1u;
#pragma unroll
        for (int i = 0; i < NW; i++) r &= f[i];
#pragma unroll
        for (int n = 0; n < N; n++) {
            float t = 0.f;
#pragma unroll
            for (int i = 0; i < NW; i++) t += __uint_as_float(f[(1 + n) * NW + i]);
            total[n] = t;
        }
        return __builtin_amdgcn_readfirstlane(r) != 0;
    }
};

// Input of a projection inside the fused kernel.
struct TSrc {
    const cword_t* base = nullptr; size_t stride = 0; u32 tag = 0;         // compact vector [B][stride] (tag = write counter) ...
    const bf16_t* embed = nullptr; const int* tokens = nullptr;            // ... or rows of the embedding table
    const cword_t* add = nullptr; size_t add_stride = 0; u32 add_tag = 0;  // optional: + sublayer output
    cword_t* wb = nullptr; size_t wb_stride = 0; u32 wb_tag = 0;           // optional: publish the sum (residual stream)
    const bf16_t* gain = nullptr; float eps = 0.f;                         // optional: RMSNorm
    UDiv ncta = {1, 0};                                                    // workgroups in the grid (each publishes 1/ncta of wb)
    bool eager = false;   // re-read the whole vector while waiting instead of polling samples (see stage_tagged_onepass)
};

// Waits (bounded) until kPollLanes sampled elements of the source vector(s) carry their tags: a
// cheap way to sit out a producer that is still running -- a few 8-byte loads with pauses in
// between cost the memory system next to nothing even with every workgroup waiting at once.
template <bool HAS_ADD>
__device__ __forceinline__ bool light_wait(const TSrc& S, int batch, int k0, int nel, int lane) {
    const int sample = min(k0 + (int)(((long)(lane % kPollLanes) * nel) / kPollLanes) + (int)(blockIdx.x % 16) * 2, k0 + nel - 1);
    const cword_t* sb = S.base + (size_t)(batch - 1) * S.stride;
    const cword_t* sa = HAS_ADD ? S.add + (size_t)(batch - 1) * S.add_stride : nullptr;
    for (int spins = 0; spins < kSpinLimit; spins++) {
        bool ok = true;
        if (lane < kPollLanes) {
            ok = cfresh(cld1(sb, sample), S.tag);
            if constexpr (HAS_ADD) ok = ok && cfresh(cld1(sa, sample), S.add_tag);
        }
        if (__all(ok)) return true;
        __builtin_amdgcn_s_sleep(4);
    }
    return false;
}

// (a, b) rounded to bf16 (nearest even) and packed, a in the low half: v_cvt_pk_bf16_f32.
typedef float pk_f2 __attribute__((ext_vector_type(2)));
typedef __bf16 pk_bf2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32 pack_bf16(float a, float b) {
    return __builtin_bit_cast(u32, __builtin_convertvector(pk_f2{a, b}, pk_bf2));
}
// fp32 pair -> packed bf16 heads and packed bf16 remainders, both round to nearest even:
// |error| <= 2^-18 |v|.
__device__ __forceinline__ void split_bf16x2(float a, float b, u32& hi, u32& lo) {
    hi = pack_bf16(a, b);
    lo = pack_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xFFFF0000u));
}
// Wide pass (see ff_wide.h): byte offset of column `col` of sequence n in a global image of the
// consumers' LDS layout (plane 0: heads, 1: remainders): K segment of 2048 columns, then plane-major
// with 16-byte unit j at index j ^ n.
constexpr int kWideSegUnits = 256;
constexpr int kWideSegBytes = kLdsActBytes;
__device__ __forceinline__ size_t wide_img_off(int n, int plane, int col) {
    const int j = col >> 3;
    return (size_t)(j >> 8) * kWideSegBytes + ((size_t)((2 * n + plane) * kWideSegUnits + ((j & 255) ^ n))) * 16 + (size_t)(col & 7) * 2;
}

// Writes quad qi (elements 4*qi .. 4*qi+3) of sequence b into the staged vector.  Plain form: the
// quad-planar fp32 layout of stage_act.  SPLIT form (input of gemv_run_quad): every value v is
// stored as bf16 head h = v rounded to nearest and bf16 remainder = v - h rounded to nearest (the
// pair carries 17 significant bits), heads in plane 2b and remainders in plane 2b+1, element order as in a weight unit.
//   bf16 weights (8 elements = 16 bytes per unit and plane): unit j at index j ^ ((b & 3) << 2);
//   int8 weights (16 elements = two 16-byte chunks): chunk q of unit j at index
//   2 (j ^ ((b & 2) << 1)) + (q ^ (b & 1));
//   int4 weights (32 elements = four 16-byte chunks per unit and plane): chunk q of unit j at
//   index 4 j + (q ^ (b & 3)), and the sum of the unit's 32 values in xsum_of(xs)[b * nup + j].
// Either way the four lanes of a matrix-core block (same j, sequences 0..3) hit different banks.
// All lanes of a unit must call together (int4: eight consecutive quads = eight consecutive lanes).
template <int EPU, bool SPLIT>
__device__ __forceinline__ void stage_store(float4* xs, int nup, int b, int qi, const float4& t) {
    constexpr int NQ = EPU / 4;
    if constexpr (!SPLIT) {
        xs[((size_t)b * NQ + qi % NQ) * nup + qi / NQ] = t;
    } else {
        static_assert(EPU == 8 || EPU == 16 || EPU == 32, "bf16, int8 or int4 weights");
        // heads and remainders with the packed conversion (two values per instruction, round to
        // nearest even): |error| <= 2^-18 |v|
        u32 h01, l01, h23, l23;
        split_bf16x2(t.x, t.y, h01, l01);
        split_bf16x2(t.z, t.w, h23, l23);
        const u32 h[4] = {h01 << 16, h01 & 0xFFFF0000u, h23 << 16, h23 & 0xFFFF0000u};   // (only the int4 unit sums below look at these)
        const u32 l[4] = {l01 << 16, l01 & 0xFFFF0000u, l23 << 16, l23 & 0xFFFF0000u};
        u32x2 *ph, *pl;
        if constexpr (EPU == 8) {
            const int j = (qi >> 1) ^ ((b & 3) << 2);
            ph = (u32x2*)(xs + (size_t)(2 * b) * nup + j) + (qi & 1);
            pl = (u32x2*)(xs + (size_t)(2 * b + 1) * nup + j) + (qi & 1);
        } else if constexpr (EPU == 16) {
            const int j = (qi >> 2) ^ ((b & 2) << 1), q = ((qi >> 1) & 1) ^ (b & 1);
            ph = (u32x2*)(xs + ((size_t)(2 * b) * nup + j) * 2 + q) + (qi & 1);
            pl = (u32x2*)(xs + ((size_t)(2 * b + 1) * nup + j) * 2 + q) + (qi & 1);
        } else {
            const int j = qi >> 3, q = ((qi >> 1) & 3) ^ (b & 3);
            ph = (u32x2*)(xs + ((size_t)(2 * b) * nup + j) * 4 + q) + (qi & 1);
            pl = (u32x2*)(xs + ((size_t)(2 * b + 1) * nup + j) * 4 + q) + (qi & 1);
            // the sum of the values as the matrix cores will see them (head + stored remainder)
            float hv[4];
#pragma unroll
            for (int e = 0; e < 4; e++) hv[e] = __uint_as_float(h[e]) + __uint_as_float(l[e]);
            const float us = group_sum<8>((hv[0] + hv[1]) + (hv[2] + hv[3]));
            if ((qi & 7) == 0) xsum_of(xs)[(size_t)b * nup + j] = us;
        }
        *ph = u32x2{h01, h23};
        *pl = u32x2{l01, l23};
    }
}

// Several-pass form (vectors longer than one pass of stage_tagged_onepass; one row at a time).
// The workgroup stages elements [k0, k0 + nunits*EPU) of every batch row into LDS in the
// quad-planar layout of stage_act, re-reading the tagged sources until their producers have
// written them.  Every thread issues all loads of its share of a batch at once and speculatively
// (a load issued behind a wave's weight prefetch takes microseconds to return, so round trips are
// what count); only if some tag in the workgroup is stale does it fall back to light polling.
// The first workgroup barrier inside doubles as the hand-over of the LDS region from the previous
// projection.  NT = threads of the workgroup.  Returns false (uniformly) on a time-out.
// QB = quads per thread and pass (2 8-byte loads per quad and source, all in flight at once; their
// 4*QB destination registers per source must fit beside the wave's prefetched weight tiles, or the
// compiler parks those tiles elsewhere and has to wait for them first).
template <int EPU, bool HAS_ADD, bool HAS_GAIN, int NT, int QB, bool SPLIT>
__device__ __forceinline__ bool stage_tagged_multipass(const TSrc& S, int batch, int K, int k0, int nunits, int nup, float4* xs, float* red, int tid, WgVote& vote, u64* ev) {
    constexpr int NQ = EPU / 4;
    if (ev && tid == 0) { as_global(ev)[0] = wall_clock64(); as_global(ev)[2] = 0; as_global(ev)[5] = 0; }
    const int lane = tid & 63;
    const int nquads = nunits * NQ;
    const int padquads = nup * NQ;
    const u32 wb_lo = S.ncta.div((u32)nquads * blockIdx.x), wb_hi = S.ncta.div((u32)nquads * (blockIdx.x + 1));
    for (int b = 0; b < batch; b++) {
        float4* xb = xs + (size_t)b * NQ * nup;
        const cword_t* src = S.base + (size_t)b * S.stride;
        const cword_t* add = HAS_ADD ? S.add + (size_t)b * S.add_stride : nullptr;
        const bf16_t* erow = nullptr;   // embedding rows only come through the (no add, gain) instance
        if constexpr (!HAS_ADD && HAS_GAIN) erow = S.tokens ? S.embed + (size_t)max(as_global(S.tokens)[b], 0) * K : nullptr;
        float ss = 0.f;
        for (int q0 = tid; q0 < padquads; q0 += NT * QB) {
            u32x4 v[QB], a[HAS_ADD ? QB : 1];   // four compact words per quad and source
            u32x2 g[HAS_GAIN ? QB : 1];
            bool all_ok = false;
            u32 stale = (1u << QB) - 1;   // quads (bit u) this lane still has to (re)load
            for (int spins = 0; spins < kSpinLimit && !all_ok; spins++) {
                // first pass: every quad of every lane; later passes: only what came back stale, so
                // a vector that was mostly complete is not fetched twice
#pragma unroll
                for (int u = 0; u < QB; u++) {
                    const int k = k0 + min(q0 + u * NT, nquads - 1) * 4;   // clamped: every load is issued
                    if (spins == 0 || ((stale >> u) & 1)) {
                        if (erow) {   // bf16 values are exact in the compact format: mark them fresh
                            u32x2 w = *as_global((const u32x2*)(erow + k));
                            const u32 t = S.tag & kCntMask;
                            v[u] = u32x4{(w.x << 16) | t, (w.x & 0xFFFF0000u) | t, (w.y << 16) | t, (w.y & 0xFFFF0000u) | t};
                        } else {
                            const u32x2 lo = cld2(src, k), hi = cld2(src, k + 2);
                            v[u] = u32x4{lo.x, lo.y, hi.x, hi.y};
                        }
                        if constexpr (HAS_ADD) {
                            const u32x2 lo = cld2(add, k), hi = cld2(add, k + 2);
                            a[u] = u32x4{lo.x, lo.y, hi.x, hi.y};
                        }
                    }
                    if constexpr (HAS_GAIN) { if (spins == 0) g[u] = *as_global((const u32x2*)(S.gain + k)); }
                }
                stale = 0;
#pragma unroll
                for (int u = 0; u < QB; u++) {
                    bool ok = cfresh(v[u].x, S.tag) && cfresh(v[u].y, S.tag) && cfresh(v[u].z, S.tag) && cfresh(v[u].w, S.tag);
                    if constexpr (HAS_ADD)
                        ok = ok && cfresh(a[u].x, S.add_tag) && cfresh(a[u].y, S.add_tag) && cfresh(a[u].z, S.add_tag) && cfresh(a[u].w, S.add_tag);
                    if (!ok) stale |= 1u << u;
                }
                all_ok = vote.all<NT>(stale == 0);
                if (ev && tid == 0 && spins == 0 && b == 0) as_global(ev)[1] = wall_clock64();
                if (!all_ok) {
                    bool lw = true;
                    if (tid < 64) lw = light_wait<HAS_ADD>(S, batch, k0, nunits * EPU, lane);
                    if (!vote.all<NT>(lw)) return false;
                    if (ev && tid == 0) { as_global(ev)[2] = wall_clock64(); as_global(ev)[5] += 1; }
                }
            }
            if (!all_ok) return false;
            if (ev && tid == 0) as_global(ev)[3] = wall_clock64();
#pragma unroll
            for (int u = 0; u < QB; u++) {
                const int qi = q0 + u * NT;
                if (qi < padquads) {
                    float4 t = make_float4(cvalue(v[u].x), cvalue(v[u].y), cvalue(v[u].z), cvalue(v[u].w));
                    if constexpr (HAS_ADD) { t.x += cvalue(a[u].x); t.y += cvalue(a[u].y); t.z += cvalue(a[u].z); t.w += cvalue(a[u].w); }
                    if (qi >= nquads) t = make_float4(0.f, 0.f, 0.f, 0.f);
                    else if (S.wb && (u32)qi >= wb_lo && (u32)qi < wb_hi) {   // this workgroup's slice of the published sum
                        cword_t* w = S.wb + (size_t)b * S.wb_stride + k0 + qi * 4;
                        cst2(w, t.x, t.y, S.wb_tag);
                        cst2(w + 2, t.z, t.w, S.wb_tag);
                    }
                    if constexpr (HAS_GAIN) {
                        if (qi < nquads) {
                            ss += t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
                            t.x *= bf_lo(g[u].x); t.y *= bf_hi(g[u].x); t.z *= bf_lo(g[u].y); t.w *= bf_hi(g[u].y);
                        }
                    }
                    stage_store<EPU, SPLIT>(xs, nup, b, qi, t);
                }
            }
        }
        if constexpr (HAS_GAIN) {
            static_assert(!SPLIT, "the rescaling pass below works on the fp32 layout");
            ss = wave_sum_uniform(ss);
            if (lane == 0) red[tid >> 6] = ss;
            __syncthreads();
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < NT / 64; w++) tot += red[w];
            const float r = rsqrtf(tot / (float)K + S.eps);
            for (int qi = tid; qi < nquads; qi += NT) {   // each thread rescales the quads it wrote
                int j = qi / NQ, qd = qi % NQ;
                float4 v4 = xb[(size_t)qd * nup + j];
                v4.x *= r; v4.y *= r; v4.z *= r; v4.w *= r;
                xb[(size_t)qd * nup + j] = v4;
            }
            if (b + 1 < batch) __syncthreads();   // `red` is rewritten for the next row
        }
    }
    __syncthreads();
    return true;
}

// The common case, where one pass of QB quads per thread covers the whole vector (nup * EPU / 4 <=
// NT * QB): every thread keeps its quads in registers from the load to the LDS write, and the sums
// of squares of the normalisation travel with the freshness vote, so a group of RB batch rows costs
// a single workgroup barrier and the staged vectors are written once, already scaled.  The loads
// of all RB rows are in flight together: behind a wave's weight prefetch a round trip takes
// microseconds, and one per row would make the hand-over grow with the batch.
template <int EPU, bool HAS_ADD, bool HAS_GAIN, int NT, int QB, bool SPLIT, int RB>
__device__ __forceinline__ bool stage_tagged_onepass(const TSrc& S, int batch, int K, int k0, int nunits, int nup, float4* xs, int tid, WgVote& vote, u64* ev) {
    constexpr int NQ = EPU / 4;
    if (ev && tid == 0) { as_global(ev)[0] = wall_clock64(); as_global(ev)[2] = 0; as_global(ev)[5] = 0; }
    const int lane = tid & 63;
    const int nquads = nunits * NQ;
    const int padquads = nup * NQ;
    const u32 wb_lo = S.ncta.div((u32)nquads * blockIdx.x), wb_hi = S.ncta.div((u32)nquads * (blockIdx.x + 1));
    for (int b0 = 0; b0 < batch; b0 += RB) {
        // rows b0 .. b0+RB-1; a row past the batch repeats the last one (loaded and checked, never written)
        const cword_t* src[RB];
        const cword_t* add[RB];
        const bf16_t* erow[RB];   // embedding rows only come through the (no add, gain) instance
#pragma unroll
        for (int r = 0; r < RB; r++) {
            const int b = min(b0 + r, batch - 1);
            src[r] = S.base + (size_t)b * S.stride;
            add[r] = HAS_ADD ? S.add + (size_t)b * S.add_stride : nullptr;
            erow[r] = nullptr;
            if constexpr (!HAS_ADD && HAS_GAIN) erow[r] = S.tokens ? S.embed + (size_t)max(as_global(S.tokens)[b], 0) * K : nullptr;
        }
        u32x4 v[RB][QB], a[HAS_ADD ? RB : 1][HAS_ADD ? QB : 1];   // four compact words per quad and source
        u32x2 g[HAS_GAIN ? QB : 1];
        bool all_ok = false;
        float tot[RB];
        u32 stale[RB];   // quads (bit u) of row r this lane still has to (re)load
#pragma unroll
        for (int r = 0; r < RB; r++) { stale[r] = (1u << QB) - 1; tot[r] = 0.f; }
        // first every quad of every lane, unconditionally (no per-lane branches on the way to the
        // first request); after a failed vote only what came back stale, so a vector that was
        // mostly complete is not fetched twice
        auto load_quads = [&](auto ALL) {
            constexpr bool kAll = decltype(ALL)::value;
#pragma unroll
            for (int r = 0; r < RB; r++) {
#pragma unroll
                for (int u = 0; u < QB; u++) {
                    const int k = k0 + min(tid + u * NT, nquads - 1) * 4;   // clamped: every load is issued
                    if (kAll || ((stale[r] >> u) & 1)) {
                        if (erow[r]) {   // bf16 values are exact in the compact format: mark them fresh
                            u32x2 w = *as_global((const u32x2*)(erow[r] + k));
                            const u32 t = S.tag & kCntMask;
                            v[r][u] = u32x4{(w.x << 16) | t, (w.x & 0xFFFF0000u) | t, (w.y << 16) | t, (w.y & 0xFFFF0000u) | t};
                        } else {
                            const u32x2 lo = cld2(src[r], k), hi = cld2(src[r], k + 2);
                            v[r][u] = u32x4{lo.x, lo.y, hi.x, hi.y};
                        }
                        if constexpr (HAS_ADD) {
                            const u32x2 lo = cld2(add[r], k), hi = cld2(add[r], k + 2);
                            a[r][u] = u32x4{lo.x, lo.y, hi.x, hi.y};
                        }
                    }
                    if constexpr (HAS_GAIN && kAll) { if (r == 0) g[u] = *as_global((const u32x2*)(S.gain + k)); }
                }
            }
        };
        load_quads(std::true_type{});
        for (int spins = 0; spins < kSpinLimit && !all_ok; spins++) {
            float ss[RB];   // only meaningful if the vote passes
            bool mine = true;
            // With a single row in flight the lane first ORs the counter mismatches of all its
            // words together (one operation per word) and looks at single quads only if something
            // is stale; with several rows that form needs more registers than there are beside
            // the weight tiles (it spills), so they test quad by quad.
            u32 dirty = 0;
            if constexpr (RB == 1) {
#pragma unroll
                for (int u = 0; u < QB; u++) {
                    dirty |= (v[0][u].x ^ S.tag) | (v[0][u].y ^ S.tag) | (v[0][u].z ^ S.tag) | (v[0][u].w ^ S.tag);
                    if constexpr (HAS_ADD) dirty |= (a[0][u].x ^ S.add_tag) | (a[0][u].y ^ S.add_tag) | (a[0][u].z ^ S.add_tag) | (a[0][u].w ^ S.add_tag);
                }
                dirty &= kCntMask;
            }
#pragma unroll
            for (int r = 0; r < RB; r++) {
                stale[r] = 0;
                ss[r] = 0.f;
#pragma unroll
                for (int u = 0; u < QB; u++) {
                    if (RB > 1 || dirty) {
                        bool ok = cfresh(v[r][u].x, S.tag) && cfresh(v[r][u].y, S.tag) && cfresh(v[r][u].z, S.tag) && cfresh(v[r][u].w, S.tag);
                        if constexpr (HAS_ADD)
                            ok = ok && cfresh(a[r][u].x, S.add_tag) && cfresh(a[r][u].y, S.add_tag) && cfresh(a[r][u].z, S.add_tag) && cfresh(a[r][u].w, S.add_tag);
                        if (!ok) stale[r] |= 1u << u;
                    }
                    if constexpr (HAS_GAIN) {
                        float4 t = make_float4(cvalue(v[r][u].x), cvalue(v[r][u].y), cvalue(v[r][u].z), cvalue(v[r][u].w));
                        if constexpr (HAS_ADD) { t.x += cvalue(a[r][u].x); t.y += cvalue(a[r][u].y); t.z += cvalue(a[r][u].z); t.w += cvalue(a[r][u].w); }
                        if (tid + u * NT < nquads) ss[r] += t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
                    }
                }
                mine = mine && stale[r] == 0;
                if constexpr (HAS_GAIN) ss[r] = wave_sum_uniform(ss[r]);
            }
            if constexpr (HAS_GAIN) all_ok = vote.all_sum<NT, RB>(mine, ss, tot);
            else all_ok = vote.all<NT>(mine);
            if (ev && tid == 0 && spins == 0 && b0 == 0) as_global(ev)[1] = wall_clock64();
            if (!all_ok && !S.eager) {
                // A producer that is still streaming weights should not have to compete with 256
                // workgroups re-reading its output: wait on a few samples.  An eager source is
                // written by a handful of workgroups while the rest of the chip idles (the merged
                // attention output): there the stale quads are simply read again, which saves the
                // round trip between "sample seen" and "vector loaded".
                bool lw = true;
                if (tid < 64) lw = light_wait<HAS_ADD>(S, batch, k0, nunits * EPU, lane);
                if (!vote.all<NT>(lw)) return false;
                if (ev && tid == 0) { as_global(ev)[2] = wall_clock64(); as_global(ev)[5] += 1; }
            }
            if (!all_ok) load_quads(std::false_type{});
        }
        if (!all_ok) return false;
        if (ev && tid == 0) as_global(ev)[3] = wall_clock64();
        // Usually every (lane, u) holds a real quad (the vector is a whole number of NT*QB quads,
        // no padding): that case runs without the per-lane range tests, each of which is a
        // divergent branch -- expensive for a wave that has its SIMD to itself.
        const bool exact = nquads == padquads && padquads == QB * NT;
        auto write_quad = [&](auto EX, int r, int u, int b, float rs) {
            constexpr bool kExact = decltype(EX)::value;
            const int qi = tid + u * NT;
            if (kExact || qi < padquads) {
                float4 t = make_float4(cvalue(v[r][u].x), cvalue(v[r][u].y), cvalue(v[r][u].z), cvalue(v[r][u].w));
                if constexpr (HAS_ADD) { t.x += cvalue(a[r][u].x); t.y += cvalue(a[r][u].y); t.z += cvalue(a[r][u].z); t.w += cvalue(a[r][u].w); }
                if (!kExact && qi >= nquads) t = make_float4(0.f, 0.f, 0.f, 0.f);
                else {
                    if (S.wb && (u32)qi >= wb_lo && (u32)qi < wb_hi) {   // this workgroup's slice of the published sum
                        cword_t* w = S.wb + (size_t)b * S.wb_stride + k0 + qi * 4;
                        cst2(w, t.x, t.y, S.wb_tag);
                        cst2(w + 2, t.z, t.w, S.wb_tag);
                    }
                    if constexpr (HAS_GAIN) {
                        t.x *= bf_lo(g[u].x) * rs; t.y *= bf_hi(g[u].x) * rs; t.z *= bf_lo(g[u].y) * rs; t.w *= bf_hi(g[u].y) * rs;
                    }
                }
                stage_store<EPU, SPLIT>(xs, nup, b, qi, t);
            }
        };
#pragma unroll
        for (int r = 0; r < RB; r++) {
            const int b = b0 + r;
            if (b < batch) {
                const float rs = HAS_GAIN ? rsqrtf(tot[r] / (float)K + S.eps) : 1.f;
                if (exact) {
#pragma unroll
                    for (int u = 0; u < QB; u++) write_quad(std::true_type{}, r, u, b, rs);
                } else {
#pragma unroll
                    for (int u = 0; u < QB; u++) write_quad(std::false_type{}, r, u, b, rs);
                }
            }
        }
    }
    __syncthreads();
    return true;
}

// Picks the pass size that covers the vector in one pass with the fewest registers, and how many
// batch rows are loaded together (RBMAX = the kernel's batch capacity; four rows of a short
// vector, two of a long one, to keep the quads of all rows in registers beside the weight tiles).
// SPLIT selects the staged format (see stage_store); a normalised vector too long for one pass has
// no SPLIT form (the host rejects such configurations).
template <int EPU, bool HAS_ADD, int NT, bool SPLIT, int RBMAX>
__device__ __forceinline__ bool stage_tagged(const TSrc& S, int batch, int K, int k0, int nunits, int nup, float4* xs, float* red, int tid,
                                             WgVote& vote, u64* ev = nullptr) {
    constexpr int RB4 = RBMAX < 4 ? RBMAX : 4, RB2 = RBMAX < 2 ? RBMAX : 2;
    const int per_thread = (nup * (EPU / 4) + NT - 1) / NT;
    if constexpr (HAS_ADD) {   // residual stream + sublayer output, always normalised
        if (per_thread <= 4) return stage_tagged_onepass<EPU, true, true, NT, 4, SPLIT, RB4>(S, batch, K, k0, nunits, nup, xs, tid, vote, ev);
        if (per_thread <= 8) return stage_tagged_onepass<EPU, true, true, NT, 8, SPLIT, RB2>(S, batch, K, k0, nunits, nup, xs, tid, vote, ev);
        if constexpr (SPLIT) return false;
        else return stage_tagged_multipass<EPU, true, true, NT, 8, false>(S, batch, K, k0, nunits, nup, xs, red, tid, vote, ev);
    } else if (S.gain) {       // embedding rows
        if (per_thread <= 8) return stage_tagged_onepass<EPU, false, true, NT, 8, SPLIT, RB2>(S, batch, K, k0, nunits, nup, xs, tid, vote, ev);
        if constexpr (SPLIT) return false;
        else return stage_tagged_multipass<EPU, false, true, NT, 8, false>(S, batch, K, k0, nunits, nup, xs, red, tid, vote, ev);
    } else {
        if (per_thread <= 4) return stage_tagged_onepass<EPU, false, false, NT, 4, SPLIT, RB4>(S, batch, K, k0, nunits, nup, xs, tid, vote, ev);
        if (per_thread <= 8) return stage_tagged_onepass<EPU, false, false, NT, 8, SPLIT, RB4>(S, batch, K, k0, nunits, nup, xs, tid, vote, ev);
        if (per_thread <= 14) return stage_tagged_onepass<EPU, false, false, NT, 14, SPLIT, RB2>(S, batch, K, k0, nunits, nup, xs, tid, vote, ev);
        return stage_tagged_multipass<EPU, false, false, NT, 14, SPLIT>(S, batch, K, k0, nunits, nup, xs, red, tid, vote, ev);
    }
}

// 2^x straight from the hardware unit (v_exp_f32, about 1 ulp): the library routine wraps it in a
// rescaling sequence so that results below the normal range come out as denormals; here the
// arguments are differences to a running maximum (<= 0) and the results softmax weights, for which
// a flush to zero at 2^-126 is immaterial, and the sequence would be executed dozens of times on
// the attention's critical path.
__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

// ---------------------------------------------------------------- split-KV attention
// One work item = (sequence b, kv head j, rows [t0, t1) of its cache [+ this step's own k,v]).
// All G query heads that share kv head j are processed together, so each cached K and V element
// is read exactly once (paper Section 4.2, core attention: workgroups are split among KV heads and
// hold the queries of that head; the current token's k,v are taken from the exchange buffer, not
// from the cache).  Result: per query head the partial (max score, denominator, unnormalised
// output) of a FlashDecoding-style split, in base-2 exponent units.
//
// Thread mapping: a cache row is hd*2 bytes = LPR lanes x 16 bytes, so one wave load covers
// 64/LPR rows; lane (grp, sub) holds dims [8*sub, 8*sub+8) of row grp.  Every (wave, grp) keeps its
// own online-softmax state; the NW*64/LPR states are merged through LDS at the end (NW = waves of
// the workgroup, all of which take part).  XIO supplies the exchange accesses (plain buffers for
// the per-operation kernels, tagged buffers for the fused kernel); returns false on a time-out.
struct PlainAttnIO {
    // Workgroup-collective: the G query rows of kv head j, then (with_cur) this step's own key and
    // value row, as floats into dst[G*HD + 2*HD] (LDS); ends with a workgroup barrier.
    template <int HD, int G, int NT>
    __device__ __forceinline__ bool stage_inputs(const DevModel& M, int b, int j, bool with_cur, float* dst) const {
        const int nq = G * HD, n = nq + (with_cur ? 2 * HD : 0);
        for (int e = threadIdx.x; e < n; e += NT) {
            float v;
            if (e < nq) v = PlainIO::ld(M.q, (b * M.Hq + j * G) * HD + e);
            else v = PlainIO::ld(M.kvcur, ((b * 2 + (e - nq) / HD) * M.Hkv + j) * HD + (e - nq) % HD);
            dst[e] = v;
        }
        __syncthreads();
        return true;
    }
    template <int HD>
    __device__ __forceinline__ void store_partial(const DevModel& M, size_t hs, int dim, float ot, float mx, float lt) const {
        PlainIO::st(M.part_o + hs * HD + dim, ot);
        if (dim == 0) { PlainIO::st(M.part_m + hs, mx); PlainIO::st(M.part_l + hs, lt); }
    }
};
struct TaggedAttnIO {
    u32 in_tag;    // tag of q / kvcur (this layer's QKV projection)
    u32 out_tag;   // tag of the partials and of attn_o (this layer's attention)
    WgVote* vote;
    // Workgroup-collective, same contract as PlainAttnIO::stage_inputs.  The whole input of an
    // item is a few kilobytes (one or two 16-byte pairs per thread), so the workgroup simply
    // re-reads it until the QKV projection's tag is on every element; returns false on a time-out.
    template <int HD, int G, int NT>
    __device__ __forceinline__ bool stage_inputs(const DevModel& M, int b, int j, bool with_cur, float* dst) const {
        constexpr int NQ2 = G * HD / 2, NK2 = HD / 2;       // pairs of queries, of one k or v row
        constexpr int PP = (NQ2 + 2 * NK2 + NT - 1) / NT;   // pairs per thread
        const int np = NQ2 + (with_cur ? 2 * NK2 : 0);
        const tagged_t* qb = M.tq + (size_t)(b * M.Hq + j * G) * HD;
        const tagged_t* kb = M.tkvcur + (size_t)((b * 2 + 0) * M.Hkv + j) * HD;
        const tagged_t* vb = M.tkvcur + (size_t)((b * 2 + 1) * M.Hkv + j) * HD;
        u32x4 r[PP];
        bool done = false;
        for (int spins = 0; spins < kSpinLimit && !done; spins++) {
            bool ok = true;
#pragma unroll
            for (int u = 0; u < PP; u++) {
                const int p = min((int)threadIdx.x + u * NT, np - 1);   // clamped: every load is issued
                const tagged_t* src = p < NQ2 ? qb + 2 * p : p < NQ2 + NK2 ? kb + 2 * (p - NQ2) : vb + 2 * (p - NQ2 - NK2);
                r[u] = tld2(src, 0);
            }
#pragma unroll
            for (int u = 0; u < PP; u++) ok = ok && r[u].y == in_tag && r[u].w == in_tag;
            done = vote->all<NT>(ok);
            if (!done) __builtin_amdgcn_s_sleep(2);
        }
        if (!done) { atomicCAS(M.status, 0, -51); return false; }
#pragma unroll
        for (int u = 0; u < PP; u++) {
            const int p = (int)threadIdx.x + u * NT;
            if (p < np) { dst[2 * p] = __uint_as_float(r[u].x); dst[2 * p + 1] = __uint_as_float(r[u].z); }
        }
        __syncthreads();
        return true;
    }
    template <int HD>
    __device__ __forceinline__ void store_partial(const DevModel& M, size_t hs, int dim, float ot, float mx, float lt) const {
        tst(M.tpart_o + hs * HD + dim, ot, out_tag);
        if (dim == 0) { tst(M.tpart_m + hs, mx, out_tag); tst(M.tpart_l + hs, lt, out_tag); }
    }
};

#ifndef FF_ATTN_BATCH
#define FF_ATTN_BATCH 4   // wave loads of K and of V in flight per wave (can be overridden at build time for sweeps; 8 measured no faster)
#endif
// MM (head dimension 128; built for the wide pass with its hundreds of cached rows per wave and item,
// where the vector ALUs and not the memory set the pace, and also used by the bf16 and int8 passes of
// up to four sequences, with one batch of loads in flight): the scores of a batch of 16 rows come
// from the matrix cores, and the running maximum is updated once per batch instead of once per row.
//   * v_mfma_f32_16x16x32_bf16 with A = 16 cached key rows (lane (r, g4) loads dims [32 kk + 8 g4, + 8)
//     of row r for the k-steps kk = 0..3) and B = the queries as bf16 head (columns 0..G-1) and bf16
//     remainder (columns 8..8+G-1), so the products are as accurate as the fp32 ones of the row-wise
//     path; column n + 8 is added to column n, the scores are scaled and handed through a small LDS
//     area of the wave to the lane groups that hold the value rows (row r = 4 i + grp of the batch is
//     value load i of group grp, as in the row-wise path);
//   * per head: one maximum over the batch's four rows of the group, one rescaling of the running
//     output, then four multiply-adds per output element (rows past the item's end get weight 0).
// In the wide pass two batches of loads are kept in flight, the refills issued unconditionally (behind the item's
// last row they repeat that row), like the refills of the weight ring: where code paths that issued
// different numbers of loads meet, the compiler waits for all.
typedef __bf16 attn_bf8 __attribute__((ext_vector_type(8)));
template <int HD, int G, int NW, class XIO, int MODE = 0>   // 0: row-wise; 1: MM, one batch of loads in flight; 2: MM, two
__device__ __forceinline__ bool attn_item(const DevModel& M, const DevKV& KV, const XIO& xio, int layer, int b, int j, int t0, int t1, bool with_cur,
                          int split, uint8_t* lds, u64* ev = nullptr) {
    constexpr bool MM = MODE > 0 && HD == 128 && G <= 8;
    constexpr bool PIPE = MODE == 2;
    constexpr int LPR = HD / 8;        // lanes per cache row
    constexpr int RPW = 64 / LPR;      // rows per wave load
    constexpr int NS = NW * RPW;       // partial states per workgroup
    constexpr int NT = NW * 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPR, sub = lane % LPR;
    const float sc = 1.4426950408889634f / sqrtf((float)HD);   // alpha * log2(e)

    float m[G], l[G], o[G][8];
#pragma unroll
    for (int g = 0; g < G; g++) {
        m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e++) o[g][e] = 0.f;
    }
    const bf16_t* Kp = KV.plane(M, layer, b, j, 0);
    const bf16_t* Vp = KV.plane(M, layer, b, j, 1);
    float qr[G][8];
    auto update = [&](const float (&kf)[8], const float (&vf)[8], bool valid) {
#pragma unroll
        for (int g = 0; g < G; g++) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; e++) s = fmaf(qr[g][e], kf[e], s);
            s = group_sum<LPR>(s) * sc;
            if (valid) {
                float mn = fmaxf(m[g], s);
                float corr = exp2_hw(m[g] - mn), p = exp2_hw(s - mn);
                l[g] = l[g] * corr + p;
#pragma unroll
                for (int e = 0; e < 8; e++) o[g][e] = fmaf(p, vf[e], o[g][e] * corr);
                m[g] = mn;
            }
        }
    };
    // Cached rows do not depend on this step: the first kAttnBatch wave-loads are issued BEFORE the
    // queries are waited for, so the wait for the QKV projection overlaps them.
    constexpr int kAttnBatch = FF_ATTN_BATCH;
    constexpr int kStride = NW * RPW * kAttnBatch;
    static_assert(!MM || (kAttnBatch == 4 && 64 / (HD / 8) == 4), "a batch is 16 rows: four value loads of four rows");
    u32x4 kw[MM ? 2 * kAttnBatch : kAttnBatch], vw[MM ? 2 * kAttnBatch : kAttnBatch];   // MM: two batches ([buffer][load]); keys in matrix-core layout
    // MM: loads of the batch that starts at row tb (for this wave) into buffer bf
    auto issue_mm = [&](int bf, int tb) {
        const int r = lane & 15, g4 = lane >> 4;
        const int tk = min(tb + (r >> 2) * NW * RPW + (r & 3), t1 - 1);   // clamped: every load is issued
#pragma unroll
        for (int kk = 0; kk < 4; kk++) kw[bf * 4 + kk] = ldg_stream(Kp + (size_t)tk * HD + 32 * kk + 8 * g4);
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int t = min(tb + i * NW * RPW + grp, t1 - 1);
            vw[bf * 4 + i] = ldg_stream(Vp + (size_t)t * HD + sub * 8);
        }
    };
    auto issue = [&](int tb0) {
#pragma unroll
        for (int i = 0; i < kAttnBatch; i++) {
            const int t = min(tb0 + i * NW * RPW + grp, t1 - 1);   // clamped: every load is issued
            kw[i] = ldg_stream(Kp + (size_t)t * HD + sub * 8);
            vw[i] = ldg_stream(Vp + (size_t)t * HD + sub * 8);
        }
    };
    int tb0 = t0 + wave * RPW;
    if constexpr (MM) {
        if (PIPE ? t0 < t1 : tb0 < t1) {   // (an empty range has no row to clamp to)
            issue_mm(0, tb0);
            if (PIPE) issue_mm(1, tb0 + kStride);
        }
    } else {
        if (tb0 < t1) issue(tb0);
    }
    // queries of the G heads and this step's own k, v: staged once per workgroup behind the state
    // merge area, then read by every lane from LDS
    float* xin = (float*)lds + 2 * NS * G + (size_t)NS * G * HD;
    const bool ok = xio.template stage_inputs<HD, G, NT>(M, b, j, with_cur, xin);
    if (ev && threadIdx.x == 0) as_global(ev)[1] = wall_clock64();
    if (!ok) return false;   // uniform
    auto load_qr = [&]() {
#pragma unroll
        for (int g = 0; g < G; g++) {
            const float4 q0 = *(const float4*)(xin + g * HD + sub * 8), q1 = *(const float4*)(xin + g * HD + sub * 8 + 4);
            qr[g][0] = q0.x; qr[g][1] = q0.y; qr[g][2] = q0.z; qr[g][3] = q0.w;
            qr[g][4] = q1.x; qr[g][5] = q1.y; qr[g][6] = q1.z; qr[g][7] = q1.w;
        }
    };
    if constexpr (MM) {
        // queries as matrix-core B operand: column n = head n % 8, bf16 head (n < 8) or remainder (n >= 8)
        const int n = lane & 15, g4 = lane >> 4;
        u32x4 qb[4];
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
            const float* qp = xin + min(n & 7, G - 1) * HD + 32 * kk + 8 * g4;
            const float4 a = *(const float4*)qp, c = *(const float4*)(qp + 4);
            u32 h0, l0, h1, l1, h2, l2, h3, l3;
            split_bf16x2(a.x, a.y, h0, l0); split_bf16x2(a.z, a.w, h1, l1);
            split_bf16x2(c.x, c.y, h2, l2); split_bf16x2(c.z, c.w, h3, l3);
            qb[kk] = n < 8 ? u32x4{h0, h1, h2, h3} : u32x4{l0, l1, l2, l3};
        }
        float* sx = xin + (G + 2) * HD + wave * 128;   // this wave's score exchange: [16 rows][8 heads]
        auto consume = [&](int bf, int tb) {
            mfma_f4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; kk++)
                c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(attn_bf8, kw[bf * 4 + kk]), __builtin_bit_cast(attn_bf8, qb[kk]), c, 0, 0, 0);
            // lane (n, g4), element i: row 4 g4 + i of the batch, column n; heads + remainders
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const float v = c[i] + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(c[i]), 0x128, 0xF, 0xF, true));   // row_ror:8
                if (n < 8) sx[(4 * g4 + i) * 8 + n] = v * sc;
            }
            float vf[4][8];
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const u32x4 w = vw[bf * 4 + i];
                vf[i][0] = bf_lo(w.x); vf[i][1] = bf_hi(w.x); vf[i][2] = bf_lo(w.y); vf[i][3] = bf_hi(w.y);
                vf[i][4] = bf_lo(w.z); vf[i][5] = bf_hi(w.z); vf[i][6] = bf_lo(w.w); vf[i][7] = bf_hi(w.w);
            }
            float sr[4][8];   // scores of this group's four rows (row 4 i + grp), all heads
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const float4 s0 = *(const float4*)(sx + (4 * i + grp) * 8), s1 = *(const float4*)(sx + (4 * i + grp) * 8 + 4);
                const bool valid = tb + i * NW * RPW + grp < t1;
                sr[i][0] = valid ? s0.x : -INFINITY; sr[i][1] = valid ? s0.y : -INFINITY; sr[i][2] = valid ? s0.z : -INFINITY; sr[i][3] = valid ? s0.w : -INFINITY;
                sr[i][4] = valid ? s1.x : -INFINITY; sr[i][5] = valid ? s1.y : -INFINITY; sr[i][6] = valid ? s1.z : -INFINITY; sr[i][7] = valid ? s1.w : -INFINITY;
            }
#pragma unroll
            for (int g = 0; g < G; g++) {
                const float mn = fmaxf(fmaxf(m[g], fmaxf(sr[0][g], sr[1][g])), fmaxf(sr[2][g], sr[3][g]));
                const float mref = mn == -INFINITY ? 0.f : mn;   // nothing valid so far: all weights 0
                const float corr = exp2_hw(m[g] - mref);
                const float p0 = exp2_hw(sr[0][g] - mref), p1 = exp2_hw(sr[1][g] - mref), p2 = exp2_hw(sr[2][g] - mref), p3 = exp2_hw(sr[3][g] - mref);
                l[g] = fmaf(l[g], corr, (p0 + p1) + (p2 + p3));
#pragma unroll
                for (int e = 0; e < 8; e++)
                    o[g][e] = fmaf(p3, vf[3][e], fmaf(p2, vf[2][e], fmaf(p1, vf[1][e], fmaf(p0, vf[0][e], o[g][e] * corr))));
                m[g] = mn;
            }
        };
        if constexpr (!PIPE) {
            for (bool first = true; tb0 < t1; tb0 += kStride, first = false) {
                if (!first) issue_mm(0, tb0);
                consume(0, tb0);
            }
        } else
        for (; tb0 < t1; tb0 += 2 * kStride) {
            consume(0, tb0);
            __builtin_amdgcn_sched_barrier(0);
            issue_mm(0, tb0 + 2 * kStride);
            __builtin_amdgcn_sched_barrier(0);
            if (tb0 + kStride < t1) consume(1, tb0 + kStride);
            __builtin_amdgcn_sched_barrier(0);
            issue_mm(1, tb0 + 3 * kStride);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        load_qr();
        for (bool first = true; tb0 < t1; tb0 += kStride, first = false) {
            if (!first) issue(tb0);
#pragma unroll
            for (int i = 0; i < kAttnBatch; i++) {
                const bool valid = tb0 + i * NW * RPW + grp < t1;
                float kf[8] = {bf_lo(kw[i].x), bf_hi(kw[i].x), bf_lo(kw[i].y), bf_hi(kw[i].y), bf_lo(kw[i].z), bf_hi(kw[i].z), bf_lo(kw[i].w), bf_hi(kw[i].w)};
                float vf[8] = {bf_lo(vw[i].x), bf_hi(vw[i].x), bf_lo(vw[i].y), bf_hi(vw[i].y), bf_lo(vw[i].z), bf_hi(vw[i].z), bf_lo(vw[i].w), bf_hi(vw[i].w)};
                update(kf, vf, valid);
            }
        }
    }
    if constexpr (MM) { if (with_cur && wave == 0) load_qr(); }   // (the row-wise update below needs the queries per lane)
    if (with_cur && wave == 0) {   // this step's own key/value (uniform branch per wave)
        float kf[8], vf[8];
        const float* kc = xin + G * HD + sub * 8;
        const float* vc = kc + HD;
#pragma unroll
        for (int e = 0; e < 8; e++) { kf[e] = kc[e]; vf[e] = vc[e]; }
        update(kf, vf, grp == 0);   // scores reduce over the lanes of one row group: only group 0 is valid
    }
    // ---- merge the NS states of this workgroup ----
    float* sm = (float*)lds;              // [NS][G]
    float* sl = sm + NS * G;              // [NS][G]
    float* so = sl + NS * G;              // [NS][G][HD]
    const int si = wave * RPW + grp;
    if (ev && threadIdx.x == 0) as_global(ev)[2] = wall_clock64();
    __syncthreads();
#pragma unroll
    for (int g = 0; g < G; g++) {
        if (sub == 0) { sm[si * G + g] = m[g]; sl[si * G + g] = l[g]; }
#pragma unroll
        for (int e = 0; e < 8; e++) so[((size_t)si * G + g) * HD + sub * 8 + e] = o[g][e];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * HD; idx += NT) {
        int g = idx / HD, dim = idx % HD;
        float mx = -INFINITY;
        for (int s = 0; s < NS; s++) mx = fmaxf(mx, sm[s * G + g]);
        float lt = 0.f, ot = 0.f;
        for (int s = 0; s < NS; s++) {
            float w = exp2_hw(sm[s * G + g] - mx);   // empty states have m = -inf -> weight 0
            lt = fmaf(sl[s * G + g], w, lt);
            ot = fmaf(so[((size_t)s * G + g) * HD + dim], w, ot);
        }
        size_t hs = ((size_t)b * M.Hq + (j * G + g)) * kMaxSplits + split;
        xio.template store_partial<HD>(M, hs, dim, ot, mx, lt);
    }
    if (ev && threadIdx.x == 0) as_global(ev)[3] = wall_clock64();
    return ok;
}

// Final merge for (b, kv head j) over nsplit partials (paper Section 4.2: combine per-block maximum
// and denominator, rescale by own/global denominator ratio, sum): writes attn_o[b][h][:].
// Workgroup-collective; uses 2*G*kMaxSplits floats of LDS.
template <int HD, int G, int NT>
__device__ void attn_merge(const DevModel& M, int b, int j, int nsplit, float* lds) {
    typedef PlainIO IO;
    float* ms = lds;                       // [G][nsplit] maxima, then normalised weights
    float* ls = lds + G * kMaxSplits;      // [G][nsplit] denominators
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * nsplit; idx += NT) {
        int g = idx / nsplit, s = idx % nsplit;
        int hs = (b * M.Hq + (j * G + g)) * kMaxSplits + s;
        ms[g * kMaxSplits + s] = IO::ld(M.part_m, hs);
        ls[g * kMaxSplits + s] = IO::ld(M.part_l, hs);
    }
    __syncthreads();
    if (threadIdx.x < G) {
        int g = threadIdx.x;
        float mx = -INFINITY;
        for (int s = 0; s < nsplit; s++) mx = fmaxf(mx, ms[g * kMaxSplits + s]);
        float lt = 0.f;
        for (int s = 0; s < nsplit; s++) {
            float w = exp2_hw(ms[g * kMaxSplits + s] - mx);
            ms[g * kMaxSplits + s] = w;
            lt = fmaf(ls[g * kMaxSplits + s], w, lt);
        }
        float inv = 1.0f / lt;
        for (int s = 0; s < nsplit; s++) ms[g * kMaxSplits + s] *= inv;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * HD / 4; idx += NT) {
        int g = idx / (HD / 4), d4 = (idx % (HD / 4)) * 4;
        int hs = (b * M.Hq + (j * G + g)) * kMaxSplits;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
        for (int s = 0; s < nsplit; s++) {
            float4 o = IO::ld4(M.part_o, (hs + s) * HD + d4);
            float w = ms[g * kMaxSplits + s];
            acc.x = fmaf(o.x, w, acc.x); acc.y = fmaf(o.y, w, acc.y); acc.z = fmaf(o.z, w, acc.z); acc.w = fmaf(o.w, w, acc.w);
        }
        IO::st4(M.attn_o + ((size_t)b * M.Hq + (j * G + g)) * HD + d4, acc);
    }
}

// The same merge on tagged partials (fused kernel): the workgroup that computed the LAST split of
// (b, j) gathers all splits, re-reading until every partial carries this layer's attention tag,
// and publishes attn_o with the same tag.  Returns false on a time-out.
template <int HD, int G, int NT>
// img (wide pass): the merged output goes into the output projection's input image as bf16 head +
// remainder instead of the compact vector.
__device__ __forceinline__ bool attn_merge_tagged(const DevModel& M, int b, int j, int nsplit, u32 tag, u32 out_cnt, float* lds, WgVote& vote, u64* ev = nullptr,
                                                  uint8_t* img = nullptr) {
    float* ms = lds;
    float* ls = lds + G * kMaxSplits;
    constexpr int kSB = 16;   // splits gathered per batch of loads
    constexpr u32 kAll = (1u << kSB) - 1;
    // (re)loads the partial outputs of splits s0.. (bit u of mask = split s0+u) for output pair d2
    auto issue = [&](u32x4 (&r)[kSB], int hs, int d2, int s0, u32 mask) {
#pragma unroll
        for (int u = 0; u < kSB; u++)
            if ((mask >> u) & 1) r[u] = tld2(M.tpart_o, (hs + min(s0 + u, nsplit - 1)) * HD + d2);
    };
    auto stale_of = [&](const u32x4 (&r)[kSB]) {
        u32 m = 0;
#pragma unroll
        for (int u = 0; u < kSB; u++) if (!(r[u].y == tag && r[u].w == tag)) m |= 1u << u;
        return m;
    };
    // The first batch of partial outputs is requested before the maxima and denominators are
    // waited for: all partials of a head group arrive in one round trip, and whatever is still
    // stale (the last split's rows, typically) is re-read selectively.
    u32x4 r[kSB];
    const bool pre = (int)threadIdx.x < G * HD / 2;
    if (pre) issue(r, (b * M.Hq + (j * G + (int)threadIdx.x / (HD / 2))) * kMaxSplits, ((int)threadIdx.x % (HD / 2)) * 2, 0, kAll);
    __syncthreads();
    bool done = false;
    for (int spins = 0; spins < kSpinLimit && !done; spins++) {
        bool ok = true;
        for (int idx = threadIdx.x; idx < G * nsplit; idx += NT) {
            int g = idx / nsplit, s = idx % nsplit;
            int hs = (b * M.Hq + (j * G + g)) * kMaxSplits + s;
            u32x2 pm = tld1(M.tpart_m, hs), pl = tld1(M.tpart_l, hs);
            ok = ok && pm.y == tag && pl.y == tag;
            ms[g * kMaxSplits + s] = __uint_as_float(pm.x);
            ls[g * kMaxSplits + s] = __uint_as_float(pl.x);
        }
        done = vote.all<NT>(ok);
        if (!done) __builtin_amdgcn_s_sleep(2);
    }
    if (!done) { atomicCAS(M.status, 0, -53); return false; }
    if (ev && threadIdx.x == 0) as_global(ev)[4] = wall_clock64();
    bool all_ok = true;
    for (int idx = threadIdx.x; idx < G * HD / 2; idx += NT) {
        int g = idx / (HD / 2), d2 = (idx % (HD / 2)) * 2;
        int hs = (b * M.Hq + (j * G + g)) * kMaxSplits;
        // every thread reduces the maxima and denominators of its head itself (independent LDS
        // reads; no serial section, no further barrier)
        float mx = -INFINITY;
        for (int s0 = 0; s0 < nsplit; s0 += kSB) {
#pragma unroll
            for (int u = 0; u < kSB; u++) mx = fmaxf(mx, ms[g * kMaxSplits + min(s0 + u, nsplit - 1)]);   // batched LDS reads
        }
        float lt = 0.f;
        for (int s0 = 0; s0 < nsplit; s0 += kSB) {
#pragma unroll
            for (int u = 0; u < kSB; u++) {
                const int s = min(s0 + u, nsplit - 1);
                const float w = exp2_hw(ms[g * kMaxSplits + s] - mx);
                lt = fmaf(ls[g * kMaxSplits + s], s0 + u < nsplit ? w : 0.f, lt);
            }
        }
        const float inv = 1.0f / lt;
        float a0 = 0.f, a1 = 0.f;
        for (int s0 = 0; s0 < nsplit; s0 += kSB) {
            u32 need = (idx == (int)threadIdx.x && s0 == 0) ? 0u : kAll;   // the first batch is already in flight
            bool ok = false;
            for (int spins = 0; spins < kSpinLimit && !ok; spins++) {
                issue(r, hs, d2, s0, need);
                need = stale_of(r);
                ok = need == 0;
            }
            all_ok = all_ok && ok;
            if (!ok) atomicCAS(M.status, 0, -54);
#pragma unroll
            for (int u = 0; u < kSB; u++) {
                const float mu = ms[g * kMaxSplits + min(s0 + u, nsplit - 1)];
                const float w = s0 + u < nsplit ? exp2_hw(mu - mx) * inv : 0.f;
                a0 = fmaf(__uint_as_float(r[u].x), w, a0);
                a1 = fmaf(__uint_as_float(r[u].z), w, a1);
            }
        }
        if (img) {
            u32 hi, lo;
            split_bf16x2(a0, a1, hi, lo);
            const int col = (j * G + g) * HD + d2;
            xst_u32((u32*)(img + wide_img_off(b, 0, col)), hi);
            xst_u32((u32*)(img + wide_img_off(b, 1, col)), lo);
        } else {
            cst2(M.cattn_o + ((size_t)b * M.Hq + (j * G + g)) * HD + d2, a0, a1, out_cnt);
        }
    }
    if (ev && threadIdx.x == 0) as_global(ev)[5] = wall_clock64();
    return vote.all<NT>(all_ok);
}

// Number of KV splits for a sequence with `ncache` cached rows when `share` workgroups are
// available per (sequence, kv head).
__device__ __forceinline__ int attn_nsplit(int ncache, int share) {
    int ns = ncache / kMinSplitLen;
    // The merge gathers the partials 16 at a time, and every further round is a serial round of loads:
    // 16 slices until they are 256 rows long, then whole rounds of 16 (measured at the 8B shape, batch 1,
    // us per step: context 3072 as 24 x 128 rows 3112, as 16 x 192 3062; 6144 as 32 x 192 3182, as
    // 24 x 256 3212, as 16 x 384 3199; 8192 as 32 x 256 3231, as 16 x 512 3285).
    constexpr int kRound = 16, kRoundRows = kRound * 256;
    if (ns > kRound) ns = kRound * ((ncache + kRoundRows - 1) / kRoundRows);
    ns = min(ns, min(share, kMaxSplits));
    return max(ns, 1);
}

// ---------------------------------------------------------------- epilogues
// No epilogue of the fused kernel issues a global LOAD: vector-memory operations of a wave complete
// in issue order, so a load in the middle of the weight stream would drain the whole prefetch
// pipeline.  What an epilogue needs beyond the dot products comes from LDS (RoPE cos/sin) or from
// scalar loads (positions).
//
// QKV rows in packed order: q heads then k heads with RoPE partners (i, i+hd/2) adjacent, then v.
template <class IO>
struct EpiQKV {
    const DevModel& M; const DevKV& KV; const int* tokens; const int* pos; int layer;
    const float2* rope;   // [batch][hd/2] (cos, sin) of each sequence's position; LDS in the fused kernel
    __device__ __forceinline__ void operator()(int pair, int b, float v0, float v1) const {
        const int half = M.hd / 2;
        const int nq = M.Hq * half, nk = M.Hkv * half;
        const int p = as_global(tokens)[b] == kTokenSkip ? -1 : as_global(pos)[b];   // -1: the cache of this sequence is not touched
        if (pair < nq + nk) {
            bool isq = pair < nq;
            int pp = isq ? pair : pair - nq;
            int head = pp / half, i = pp % half;
            float2 cs = rope[b * half + i];
            float a = v0 * cs.x - v1 * cs.y;
            float c = v1 * cs.x + v0 * cs.y;
            if (isq) {
                float* qp = M.q + ((size_t)b * M.Hq + head) * M.hd;
                IO::st(qp + i, a); IO::st(qp + i + half, c);
            } else {
                bf16_t ab = f_to_bf(a), cb = f_to_bf(c);
                bf16_t* row = KV.plane(M, layer, b, head, 0) + (size_t)p * M.hd;
                if (p >= 0) { as_global(row)[i] = ab; as_global(row)[i + half] = cb; }
                float* kc = M.kvcur + ((size_t)b * 2 + 0) * M.Hkv * M.hd + (size_t)head * M.hd;
                IO::st(kc + i, bf_to_f(ab)); IO::st(kc + i + half, bf_to_f(cb));
            }
        } else {
            int pp = pair - nq - nk;
            int head = pp / half, i = (pp % half) * 2;
            bf16_t ab = f_to_bf(v0), cb = f_to_bf(v1);
            bf16_t* row = KV.plane(M, layer, b, head, 1) + (size_t)p * M.hd;
            if (p >= 0) *as_global((u32*)(row + i)) = (u32)ab | ((u32)cb << 16);
            float* vc = M.kvcur + ((size_t)b * 2 + 1) * M.Hkv * M.hd + (size_t)head * M.hd;
            IO::st2(vc + i, bf_to_f(ab), bf_to_f(cb));
        }
    }
};
// Per-operation kernels: x[b][row] += W row . input
struct EpiResidual {
    float* x; int d;
    __device__ __forceinline__ void operator()(int pair, int b, float v0, float v1) const {
        FF_GLOBAL f32x2* p = as_global((f32x2*)(x + (size_t)b * d + 2 * pair));
        f32x2 o = *p;
        *p = f32x2{o.x + v0, o.y + v1};
    }
};
// packed rows (2i, 2i+1) = (gate_i, up_i):  h_i = silu(gate_i) * up_i
template <class IO>
struct EpiSwiGLU {
    float* h; int F; GuPerm perm;
    __device__ __forceinline__ void operator()(int pair, int b, float g, float u) const {
        float s = g / (1.0f + expf(-g));
        IO::st(h + (size_t)b * F + perm.unit_of_pair(pair), s * u);
    }
};
// ---- fused-kernel epilogues: outputs go to the tagged exchange buffers ----
struct EpiQKVTagged {   // pos: positions of this step, staged in LDS (-1: the sequence sits the step out, its cache is not touched)
    const DevModel& M; const DevKV& KV; const int* pos; int layer; const float2* rope; u32 tag;
    __device__ __forceinline__ void operator()(int pair, int b, float v0, float v1) const {
        const int half = M.hd / 2;
        const int nq = M.Hq * half, nk = M.Hkv * half;
        const int p = pos[b];
        if (pair < nq + nk) {
            bool isq = pair < nq;
            int pp = isq ? pair : pair - nq;
            int head = pp / half, i = pp % half;
            float2 cs = rope[b * half + i];
            float a = v0 * cs.x - v1 * cs.y;
            float c = v1 * cs.x + v0 * cs.y;
            if (isq) {
                tagged_t* qp = M.tq + ((size_t)b * M.Hq + head) * M.hd;
                tst(qp + i, a, tag); tst(qp + i + half, c, tag);
            } else {
                bf16_t ab = f_to_bf(a), cb = f_to_bf(c);
                bf16_t* row = KV.plane(M, layer, b, head, 0) + (size_t)p * M.hd;
                if (p >= 0) { as_global(row)[i] = ab; as_global(row)[i + half] = cb; }
                tagged_t* kc = M.tkvcur + ((size_t)b * 2 + 0) * M.Hkv * M.hd + (size_t)head * M.hd;
                tst(kc + i, bf_to_f(ab), tag); tst(kc + i + half, bf_to_f(cb), tag);
            }
        } else {
            int pp = pair - nq - nk;
            int head = pp / half, i = (pp % half) * 2;
            bf16_t ab = f_to_bf(v0), cb = f_to_bf(v1);
            bf16_t* row = KV.plane(M, layer, b, head, 1) + (size_t)p * M.hd;
            if (p >= 0) *as_global((u32*)(row + i)) = (u32)ab | ((u32)cb << 16);
            tagged_t* vc = M.tkvcur + ((size_t)b * 2 + 1) * M.Hkv * M.hd + (size_t)head * M.hd;
            tst2(vc + i, bf_to_f(ab), bf_to_f(cb), tag);
        }
    }
};
struct EpiDeltaTagged {   // projections feeding the residual stream: publish the output, the next
    cword_t* delta; int d; u32 tag;    // normalised staging adds it (paper Section 4.2: added to the residual)
    __device__ __forceinline__ void operator()(int pair, int b, float v0, float v1) const { cst2(delta + (size_t)b * d + 2 * pair, v0, v1, tag); }
};
struct EpiSwiGLUTagged {   // packed rows (2i, 2i+1) = (gate_i, up_i):  h_i = silu(gate_i) * up_i
    cword_t* h; int F; u32 tag; GuPerm perm;
    __device__ __forceinline__ void operator()(int pair, int b, float g, float u) const {
        float s = g / (1.0f + expf(-g));
        cst1(h + (size_t)b * F + perm.unit_of_pair(pair), s * u, tag);
    }
};
struct EpiStore {   // plain output rows (logits; per-op raw projections)
    float* y; int n;
    u32 skip = 0;   // bit b set: row b is not written (logits of a sequence that sits the step out)
    __device__ __forceinline__ void operator()(int pair, int b, float v0, float v1) const {
        if ((skip >> b) & 1u) return;
        FF_GLOBAL float* p = as_global(y + (size_t)b * n + 2 * pair);
        p[0] = v0;
        if (2 * pair + 1 < n) p[1] = v1;
    }
};

}  // namespace ff
