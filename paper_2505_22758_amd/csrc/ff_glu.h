// Gate/up projection, SwiGLU and down projection of one layer as ONE weight stream per wave, with
// the down projection's input staged chunk by chunk while the stream runs (single sequence).
//
// The paper fuses the GLU so that no device-wide synchronisation separates its two projections
// (Section 4.2 "GLU": every workgroup multiplies its slice of the intermediate vector at once and
// the partial sums are reduced at the end).  Here the down projection stays row-partitioned (no
// partial vectors to reduce), and the synchronisation between the two projections is dissolved
// instead: the gate/up row pairs are interleaved over the waves of the grid (GuPerm), so the
// i-th pair of every wave together produce the contiguous units [i nw, (i + 1) nw) of the SwiGLU
// output h, and a K chunk of the down projection (kChunkUnits units of 16 bytes) is complete once
// every wave has finished a fixed few of its pairs -- long before the gate/up projection ends.  Each
// wave therefore
//   * streams its gate/up pairs, then its down-projection rows CHUNK-major (all its rows over chunk
//     0, then over chunk 1, ...; the per-lane partial sums of a row pair wait in LDS between chunks),
//     as one flat sequence of ring stages (the slot a gate/up stage frees is refilled with the
//     first down-projection stages);
//   * every other stage, asynchronously, requests its quarter of the next chunk of h (a few 8-byte
//     coherent loads per lane, issued behind the tile refill and looked at two stages later, when
//     they have come back in the shadow of the tile loads), checks the write counters, writes the
//     values to the h region in LDS and bumps the chunk's arrival counter.
// By the time a wave reaches chunk c of the down projection the chunk has normally been staged
// for thousands of cycles; if not, the wave finishes its own quarter synchronously and waits
// (bounded) for the other three.  The hand-over between the two projections and the idle tail of
// the gate/up projection (waves that finish early start on the down projection at once) disappear.
#pragma once
#include "ff_phases.h"

namespace ff {

constexpr int kGluMaxChunks = 16;   // K chunks of the down projection (d_ffn <= 16 chunks)

template <int WD>
struct GluStager {
    static constexpr int EPU = WTraits<WD>::EPU;
    static constexpr int kChunkQuads = kChunkUnitsOf<WD> * EPU / 4;      // quads (4 values) per chunk
    static constexpr int NQT = kChunkQuads / kThreads;                   // quads per thread and chunk
    static_assert(kChunkQuads % kThreads == 0 && NQT >= 1, "a chunk is a whole number of quads per thread");
    const cword_t* src;   // h in the compact exchange format (one sequence)
    u32 cnt;              // its write counter for this layer
    int F, nup, n_chunks; // d_ffn, staged units of the down projection (padded), chunks
    float4* hs;           // LDS region of the staged h
    lds_u32* flags;       // per chunk: quarters staged so far (monotonic over layers)
    int staged = 0;       // chunks this wave has staged
    bool inflight = false;
    u32x4 v[NQT];
    __device__ __forceinline__ void issue(int tid) {
#pragma unroll
        for (int u = 0; u < NQT; u++) {
            const int k = min((staged * kChunkQuads + tid + u * kThreads) * 4, F - 4);   // clamped: every load is issued
            const u32x2 lo = cld2(src, k), hi = cld2(src, k + 2);
            v[u] = u32x4{lo.x, lo.y, hi.x, hi.y};
        }
        inflight = true;
    }
    // the loads of `issue` have come back: all four waves' words fresh?  (wave-uniform)
    __device__ __forceinline__ bool fresh() const {
        u32 dirty = 0;
#pragma unroll
        for (int u = 0; u < NQT; u++) dirty |= (v[u].x ^ cnt) | (v[u].y ^ cnt) | (v[u].z ^ cnt) | (v[u].w ^ cnt);
        return __all((dirty & kCntMask) == 0);
    }
    __device__ __forceinline__ void commit(int tid, int lane) {
#pragma unroll
        for (int u = 0; u < NQT; u++) {
            const int qi = staged * kChunkQuads + tid + u * kThreads;
            float4 t = make_float4(cvalue(v[u].x), cvalue(v[u].y), cvalue(v[u].z), cvalue(v[u].w));
            if (qi * 4 >= F) t = make_float4(0.f, 0.f, 0.f, 0.f);   // padding behind a ragged last chunk
            if (qi < nup * (EPU / 4)) stage_store<EPU, false>(hs, nup, 0, qi, t);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (lane == 0) __hip_atomic_fetch_add(flags + staged, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        ++staged;
        inflight = false;
    }
    // One asynchronous step: look at what was requested last time, request the next chunk if its
    // producers ought to be done (`ready_chunks` = chunks whose gate/up pairs this wave itself has
    // finished, one pair of slack included).
    __device__ __forceinline__ void step(int ready_chunks, int tid, int lane) {
        if (inflight) {
            if (fresh()) commit(tid, lane);
            else { issue(tid); return; }   // still being written: read it again
        }
        if (staged < n_chunks && staged < ready_chunks) issue(tid);
    }
    // Synchronous: stage this wave's quarter of chunk c now.  False on a time-out.
    __device__ __forceinline__ bool finish(int c, int tid, int lane) {
        for (int spins = 0; staged <= c; spins++) {
            if (spins > kSpinLimit) return false;
            if (!inflight) issue(tid);
            if (fresh()) commit(tid, lane);
            else { inflight = false; __builtin_amdgcn_s_sleep(2); }
        }
        return true;
    }
};

// Runs gate/up + SwiGLU + down projection of one layer for this wave.  On entry ring[s] holds
// iteration s of the gate/up stream (s < kDepth <= Sg.n_it), xs the staged, normalised input.
// epig / epid: epilogues of the two projections.  Returns false on a time-out.
template <int WD, class EpiG, class EpiD>
__device__ __forceinline__ bool glu_run(const Stream<WD, 1>& Sg, const Stream<WD, 1>& Sd, Stage<WD> (&ring)[kDepthOf<WD>], const float4* xs,
                                        GluStager<WD>& stg, float* lacc, u32 flag_target, int ipc, int lane, EpiG& epig, EpiD& epid) {
    constexpr int kDepth = kDepthOf<WD>;
    const int tid = threadIdx.x;
    const int pg_end = Sg.p0 + Sg.n_it / Sg.cpr, pd_end = Sd.p0 + Sd.n_it / Sd.cpr;
    const int n_total = Sg.n_it + Sd.n_it;
    struct Cur { int down, pair, chunk; };
    auto advance = [&](Cur& c) {
        if (!c.down) {
            if (++c.chunk == Sg.cpr) {
                c.chunk = 0;
                if (++c.pair == pg_end) { c.down = 1; c.pair = Sd.p0; }
            }
        } else if (++c.pair == pd_end) {
            c.pair = Sd.p0;
            ++c.chunk;
        }
    };
    Cur cc{0, Sg.p0, 0}, lc{0, Sg.p0, 0};
    for (int s = 0; s < kDepth; s++) advance(lc);
    float acc[2][1] = {{0.f}, {0.f}};
    int pairs_done = 0;   // gate/up pairs this wave has finished
    bool ok = true;

    constexpr int kUnr = kUnrOf<WD>, kParts = kRefillPartsOf<WD, 1>;
    float4 xr[kUnr][kXQuadsOf<WD>];   // (kXPreloadOf) the stage's inputs, read ahead of their multiply-accumulates
    auto compute = [&](const Stage<WD>& st, auto units) {   // units: the StageUnits range multiplied by this call (first: the chunk's checks, last: the iteration's end)
        constexpr int U0 = decltype(units)::u0, U1 = decltype(units)::u1;
        if (!cc.down) {
            if constexpr (kXPreloadOf<WD, 1>) {
                stage_x_load<WD, U0, U1>(xs, Sg.nup, cc.chunk, lane, xr);
                stage_fma_x<WD, U0, U1>(st, xr, acc);
            } else
            stage_fma<WD, 1, U0, U1>(st, xs, Sg.nup, cc.chunk, lane, acc);
            if constexpr (U1 < kUnr) return;
            if (cc.chunk == Sg.cpr - 1) {
                float v0 = wave_sum_uniform(acc[0][0]), v1 = wave_sum_uniform(acc[1][0]);
                acc[0][0] = acc[1][0] = 0.f;
                if constexpr (WD == W_INT8) { v0 *= f16_to_f((f16_t)st.rs[0]); v1 *= f16_to_f((f16_t)st.rs[1]); }
                if (lane == 0) epig(cc.pair, 0, v0, v1);
                ++pairs_done;
            }
        } else {
            const int pl = cc.pair - Sd.p0;
            if (U0 == 0 && pl == 0) {
                // first row pair of a chunk: the chunk must be staged (normally it has been for a while)
                if (__builtin_expect(stg.staged <= cc.chunk, 0)) ok = stg.finish(cc.chunk, tid, lane) && ok;
                bool there = false;
                for (int spins = 0; spins < (kSpinLimit << 4) && !there; spins++) {
                    there = (int)(__hip_atomic_load(stg.flags + cc.chunk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) - flag_target) >= 0;
                    if (!there) __builtin_amdgcn_s_sleep(1);
                }
                asm volatile("" ::: "memory");
                ok = ok && there;
            }
            float* la = lacc + (size_t)pl * 128 + lane;
            if (U0 == 0 && cc.chunk > 0) { acc[0][0] = la[0]; acc[1][0] = la[64]; }
            if constexpr (kXPreloadOf<WD, 1>) {
                stage_x_load<WD, U0, U1>(stg.hs, Sd.nup, cc.chunk, lane, xr);
                stage_fma_x<WD, U0, U1>(st, xr, acc);
            } else
            stage_fma<WD, 1, U0, U1>(st, stg.hs, Sd.nup, cc.chunk, lane, acc);
            if constexpr (U1 < kUnr) return;
            if (cc.chunk == Sd.cpr - 1) {
                float v0 = wave_sum_uniform(acc[0][0]), v1 = wave_sum_uniform(acc[1][0]);
                if constexpr (WD == W_INT8) { v0 *= f16_to_f((f16_t)st.rs[0]); v1 *= f16_to_f((f16_t)st.rs[1]); }
                if (lane == 0) epid(cc.pair, 0, v0, v1);
            } else {
                la[0] = acc[0][0]; la[64] = acc[1][0];
            }
            acc[0][0] = acc[1][0] = 0.f;
        }
        advance(cc);
    };
    auto load = [&](Stage<WD>& st, auto units) {
        constexpr int U0 = decltype(units)::u0, U1 = decltype(units)::u1;
        if (!lc.down) load_stage<WD, 1, U0, U1>(Sg, lc.pair, lc.chunk, st, lane);
        else load_stage<WD, 1, U0, U1>(Sd, lc.pair, lc.chunk, st, lane);
        if constexpr (U1 == kUnr) advance(lc);
    };
    // chunks of h whose producing pairs this wave itself has finished, with one pair of slack (the
    // other waves are usually within a pair of this one)
    auto ready_chunks = [&]() { return cc.down ? stg.n_chunks : max(pairs_done - 1, 0) / ipc; };
    int it = 0;
    for (; it + 2 * kDepth <= n_total && ok; it += kDepth) {
#pragma unroll
        for (int s = 0; s < kDepth; s++) {
            static_for<0, kParts>([&](auto part) {
                constexpr int P = decltype(part)::u0;
                typedef StageUnits<P * kUnr / kParts, (P + 1) * kUnr / kParts> Units;
                compute(ring[s], Units{});
                __builtin_amdgcn_sched_barrier(0);
                load(ring[s], Units{});
                __builtin_amdgcn_sched_barrier(0);
            });
            if (s == 0) stg.step(ready_chunks(), tid, lane);
        }
    }
    for (; it < n_total && ok; it += kDepth) {
#pragma unroll
        for (int s = 0; s < kDepth; s++) {
            if (it + s < n_total) {
                compute(ring[s], StageUnits<0, kUnr>{});
                __builtin_amdgcn_sched_barrier(0);
                if (it + s + kDepth < n_total) load(ring[s], StageUnits<0, kUnr>{});
                __builtin_amdgcn_sched_barrier(0);
                if (s == 0) stg.step(ready_chunks(), tid, lane);
            }
        }
    }
    // a wave without rows of the down projection still owes the workgroup its quarter of every chunk
    return stg.finish(stg.n_chunks - 1, tid, lane) && ok;
}

}  // namespace ff
