// Weight-streaming GEMV engine: activation staging into LDS, a register ring of weight tiles kept
// in flight ahead of the FMAs, and the per-format dot products.  Used by the fused whole-model
// kernel (which requests a projection's first tiles before it waits for the projection's input)
// and by the per-operation baseline kernels.
#pragma once
#include "ff_device.h"

namespace ff {

template <int WD> struct WTraits;
template <> struct WTraits<W_BF16> { static constexpr int EPU = 8; };   // elements per 16-byte unit
template <> struct WTraits<W_INT8> { static constexpr int EPU = 16; };
template <> struct WTraits<W_INT4> { static constexpr int EPU = 32; };

// 16-byte units per row and pipeline stage (per lane).  A unit of int4 weights spans 32 columns, so
// four units per lane would cover 8192 columns per stage: rows of 4096 columns would leave half
// the lanes multiplying padding.  int4 stages are therefore half as wide and its ring twice as deep.
#ifndef FF_UNR
#define FF_UNR 4   // 16-byte units per row, lane and stage for bf16 / int8 weights (can be overridden at build time for sweeps)
#endif
template <int WD> constexpr int kUnrOf = WD == W_INT4 ? 2 : FF_UNR;
// Pipeline stages (register ring slots) per wave.  Two stages (16 loads of 16 bytes per lane) keep
// the memory pipe full; deeper rings measured slower in the fused kernel, because every byte
// prefetched across a projection boundary queues in front of the loads of the next input vector
// (a wave's loads return in issue order).  FF_DEPTH can be overridden at build time for sweeps.
#ifndef FF_DEPTH
#define FF_DEPTH 2
#endif
template <int WD> constexpr int kDepthOf = WD == W_INT4 ? 2 * FF_DEPTH : FF_DEPTH;
template <int WD> constexpr int kChunkUnitsOf = 64 * kUnrOf<WD>;   // units of one row covered by one stage of one wave
// Refill granularity of the single-sequence streams: a ring slot is refilled in kRefillParts parts,
// each right behind the multiply-accumulates that freed its registers, so that 16 - 8 / parts of
// the wave's 16 loads stay in flight while a stage is being multiplied (8 with whole-stage refills).
#ifndef FF_REFILL_PARTS
#define FF_REFILL_PARTS 2
#endif
#ifndef FF_REFILL_PARTS_I4
#define FF_REFILL_PARTS_I4 1
#endif
template <int WD, int B> constexpr int kRefillPartsOf = B != 1 ? 1 : WD == W_INT4 ? FF_REFILL_PARTS_I4 : (kUnrOf<WD> % FF_REFILL_PARTS == 0 ? FF_REFILL_PARTS : 1);
#ifndef FF_REFILL_PARTS_QUAD
#define FF_REFILL_PARTS_QUAD 2
#endif
template <int WD> constexpr int kQuadRefillPartsOf = WD == W_INT4 ? 1 : FF_REFILL_PARTS_QUAD;   // the same for the matrix-core streams of 2-4 sequences
template <int U0, int U1> struct StageUnits { static constexpr int u0 = U0, u1 = U1; };   // units [U0, U1) of a stage
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(StageUnits<I, N>{});   // (I of N: the callee derives its unit range)
        static_for<I + 1, N>(f);
    }
}
// With two or more sequences per pass the projections run on the matrix cores in groups of four
// rows (gemv_run_quad below) instead of row pairs on the vector ALUs.
template <int WD, int B> constexpr bool kQuadOf = B > 1;
template <int WD> constexpr int kQuadLoadsOf = WD == W_INT4 ? 4 : 8;       // 16-byte loads per lane and stage in that mode ...
template <int WD> constexpr int kQuadChunkUnitsOf = 16 * kQuadLoadsOf<WD>; // ... = units of one row covered by one stage of one wave
constexpr int kAccFloatsPerWave = (kLdsAuxBytes - kLdsXsumBytes) / 4 / kWaves;   // partial sums a wave can carry between K segments
// Per-unit input sums of the int4 matrix-core path live at the end of the aux region (xs = start of LDS).
__device__ __forceinline__ float* xsum_of(const float4* xs) { return (float*)((uint8_t*)xs + kLdsActBytes + kLdsAuxBytes - kLdsXsumBytes); }
// Mailboxes of the wave pairs (0,1) and (2,3) of a workgroup: [pair][side][16 x 8 floats], then one flag word per pair.
typedef __attribute__((address_space(3))) float lds_float;
typedef __attribute__((address_space(3))) u32 lds_u32;
__device__ __forceinline__ lds_float* pairbox_of(const float4* xs) {
    return (lds_float*)((uint8_t*)xs + kLdsActBytes + kLdsAuxBytes + kLdsRopeBytes + kLdsMiscBytes);
}
constexpr int kPairBoxFloats = 32;   // per (pair, side): 4 rows x 8 sequences

// ---------------------------------------------------------------- reductions
// Sum over the 64 lanes with DPP row operations; the result is wave-uniform.
__device__ __forceinline__ float wave_sum_uniform(float v) {
    int x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, true));   // row_half_mirror
    x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x140, 0xF, 0xF, true));   // row_mirror
    x = __float_as_int(v);
    float r0 = __int_as_float(__builtin_amdgcn_readlane(x, 0));
    float r1 = __int_as_float(__builtin_amdgcn_readlane(x, 16));
    float r2 = __int_as_float(__builtin_amdgcn_readlane(x, 32));
    float r3 = __int_as_float(__builtin_amdgcn_readlane(x, 48));
    return (r0 + r1) + (r2 + r3);
}

// Sum over aligned groups of W lanes (W = 8 or 16), every lane of a group receiving the group's sum:
// DPP steps inside one 16-lane row, no LDS permute traffic.
template <int W>
__device__ __forceinline__ float group_sum(float v) {
    static_assert(W == 8 || W == 16, "group width");
    int x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    x = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, true));   // row_half_mirror
    if constexpr (W == 16) {
        x = __float_as_int(v);
        v += __int_as_float(__builtin_amdgcn_update_dpp(0, x, 0x140, 0xF, 0xF, true));   // row_mirror
    }
    return v;
}

// ---------------------------------------------------------------- staging
// Where a GEMV phase takes its input vector(s) from, and what is folded into the staging.
struct ActSrc {
    const float* base = nullptr;    // fp32 exchange buffer [B][stride] ...
    size_t stride = 0;
    const bf16_t* embed = nullptr;  // ... or (tokens != null) rows of the bf16 embedding table
    const int* tokens = nullptr;
    const float* add = nullptr;     // optional second fp32 vector added element-wise (residual + sublayer output)
    size_t add_stride = 0;
    float* wb = nullptr;            // optional: the summed, un-normalised vector is written back here,
    size_t wb_stride = 0;           //   each workgroup storing an interleaved slice
    const bf16_t* gain = nullptr;   // non-null: RMSNorm with this gain is applied while staging
    float eps = 0.f;
};

// Stage elements [k0, k0 + nunits*EPU) of every batch row into LDS, quad-planar so that a wave's
// 64 lanes read 64 consecutive float4: quad qd of unit j of row b lives at xs[(b*NQ + qd)*nup + j].
// Units [nunits, nup) are zero filled (the weight stream reads clamped addresses there).  With a
// gain, RMSNorm (paper Section 2.1: pre-RMSNorm in front of the QKV and GLU in/gate projections) is
// applied; that needs k0 == 0 and the whole row.  NT threads take part (tid in [0, NT)): 64 = one
// wave (reduction by DPP), otherwise the whole workgroup (reduction through `red` in LDS, with
// __syncthreads).  All global loads of a batch of kStageBatch quads per thread are issued before any
// is used.  The caller synchronises before the staged vector is read.
constexpr int kStageBatch = 8;
template <int EPU, class IO, int NT>
__device__ void stage_act(const ActSrc& S, int batch, int K, int k0, int nunits, int nup, float4* xs, float* red, int tid) {
    constexpr int NQ = EPU / 4;
    const int nquads = nunits * NQ;
    const int padquads = nup * NQ;
    for (int b = 0; b < batch; b++) {
        float4* xb = xs + (size_t)b * NQ * nup;
        const float* src = S.base + (size_t)b * S.stride;
        const float* add = S.add ? S.add + (size_t)b * S.add_stride : nullptr;
        const bf16_t* erow = S.tokens ? S.embed + (size_t)max(as_global(S.tokens)[b], 0) * K : nullptr;
        float ss = 0.f;
        for (int q0 = tid; q0 < padquads; q0 += NT * kStageBatch) {
            float4 v[kStageBatch], a[kStageBatch];
            u32x2 g[kStageBatch];
#pragma unroll
            for (int u = 0; u < kStageBatch; u++) {
                int qi = min(q0 + u * NT, nquads - 1);   // clamped: the load is always issued
                int k = k0 + qi * 4;
                if (erow) {
                    u32x2 w = *as_global((const u32x2*)(erow + k));
                    v[u] = make_float4(bf_lo(w.x), bf_hi(w.x), bf_lo(w.y), bf_hi(w.y));
                } else {
                    v[u] = IO::ld4(src, k);
                }
                if (add) a[u] = IO::ld4(add, k);
                if (S.gain) g[u] = *as_global((const u32x2*)(S.gain + k));
            }
#pragma unroll
            for (int u = 0; u < kStageBatch; u++) {
                int qi = q0 + u * NT;
                if (qi < padquads) {
                    float4 t = v[u];
                    if (add) { t.x += a[u].x; t.y += a[u].y; t.z += a[u].z; t.w += a[u].w; }
                    if (qi >= nquads) t = make_float4(0.f, 0.f, 0.f, 0.f);
                    else if (S.wb && (qi % (int)gridDim.x) == (int)blockIdx.x) IO::st4(S.wb + (size_t)b * S.wb_stride + k0 + qi * 4, t);
                    if (S.gain && qi < nquads) {
                        ss += t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
                        t.x *= bf_lo(g[u].x); t.y *= bf_hi(g[u].x); t.z *= bf_lo(g[u].y); t.w *= bf_hi(g[u].y);
                    }
                    xb[(size_t)(qi % NQ) * nup + qi / NQ] = t;
                }
            }
        }
        if (S.gain) {
            float tot;
            if constexpr (NT == 64) {
                tot = wave_sum_uniform(ss);
            } else {
                ss = wave_sum_uniform(ss);
                __syncthreads();
                if ((tid & 63) == 0) red[tid >> 6] = ss;
                __syncthreads();
                tot = 0.f;
#pragma unroll
                for (int w = 0; w < NT / 64; w++) tot += red[w];
            }
            float r = 1.0f / sqrtf(tot / (float)K + S.eps);
            for (int qi = tid; qi < nquads; qi += NT) {   // each thread rescales the quads it wrote
                int j = qi / NQ, qd = qi % NQ;
                float4 v = xb[(size_t)qd * nup + j];
                v.x *= r; v.y *= r; v.z *= r; v.w *= r;
                xb[(size_t)qd * nup + j] = v;
            }
        }
    }
}

// ---------------------------------------------------------------- one stage of weights
template <int WD> struct Stage {
    u32x4 w[2][kUnrOf<WD>];
};
template <> struct Stage<W_INT8> {
    u32x4 w[2][kUnrOf<W_INT8>];
    u32 rs[2];                 // raw fp16 row scales (loaded with the row's last chunk)
};
template <> struct Stage<W_INT4> {
    u32x4 w[2][kUnrOf<W_INT4>];
    u32 s[2][kUnrOf<W_INT4>], z[2][kUnrOf<W_INT4>];   // raw fp16 group scale / zero of each unit
};

__device__ __forceinline__ float dot_bf16(const u32x4& w, const float4& a, const float4& b, float acc) {
    acc = fmaf(bf_lo(w.x), a.x, acc);
    acc = fmaf(bf_hi(w.x), a.y, acc);
    acc = fmaf(bf_lo(w.y), a.z, acc);
    acc = fmaf(bf_hi(w.y), a.w, acc);
    acc = fmaf(bf_lo(w.z), b.x, acc);
    acc = fmaf(bf_hi(w.z), b.y, acc);
    acc = fmaf(bf_lo(w.w), b.z, acc);
    acc = fmaf(bf_hi(w.w), b.w, acc);
    return acc;
}
__device__ __forceinline__ float dot_i8x4(u32 w, const float4& x, float acc) {
    acc = fmaf((float)(int)(int8_t)(w), x.x, acc);
    acc = fmaf((float)(int)(int8_t)(w >> 8), x.y, acc);
    acc = fmaf((float)(int)(int8_t)(w >> 16), x.z, acc);
    acc = fmaf((float)((int)w >> 24), x.w, acc);
    return acc;
}
// int4 group-128: a 16-byte unit holds 32 codes of ONE group, so its contribution is
//   sum_i (code_i - z) s x_i  =  s (sum_i code_i x_i  -  z sum_i x_i):
// the inner loop only converts codes and multiplies (about 2.4 operations per weight); scale and
// zero are applied once per unit.  Even codes of a word are isolated with one mask, odd ones with a
// shift and the same mask, and the byte-to-float conversions pick them up.
__device__ __forceinline__ float dot_i4x8_codes(u32 w, const float4& x0, const float4& x1, float acc) {
    u32 e = w & 0x0F0F0F0Fu, o = (w >> 4) & 0x0F0F0F0Fu;
    // value barriers (no instruction): keep the compiler from folding the masks back into one
    // bit-field extract per code, which would cost an extra operation per weight
    asm("" : "+v"(e));
    asm("" : "+v"(o));
    acc = fmaf((float)(e & 0xFFu), x0.x, acc);
    acc = fmaf((float)(o & 0xFFu), x0.y, acc);
    acc = fmaf((float)((e >> 8) & 0xFFu), x0.z, acc);
    acc = fmaf((float)((o >> 8) & 0xFFu), x0.w, acc);
    acc = fmaf((float)((e >> 16) & 0xFFu), x1.x, acc);
    acc = fmaf((float)((o >> 16) & 0xFFu), x1.y, acc);
    acc = fmaf((float)(e >> 24), x1.z, acc);
    acc = fmaf((float)(o >> 24), x1.w, acc);
    return acc;
}
__device__ __forceinline__ float sum4(const float4& v) { return (v.x + v.y) + (v.z + v.w); }

// Division by a launch constant (waves or workgroups in the grid) that is a power of two on the
// usual 256-workgroup launch: a shift there, a division otherwise.  It sits on the path between two
// projections, where a 32-bit division is a thirty-instruction sequence.
struct UDiv {
    u32 n; int sh;   // sh >= 0: n == 1 << sh
    __device__ __forceinline__ static UDiv of(u32 n) { return UDiv{n, (n & (n - 1)) == 0 ? (int)__builtin_ctz(n) : -1}; }
    __device__ __forceinline__ u32 div(u32 x) const { return sh >= 0 ? x >> sh : x / n; }
    __device__ __forceinline__ u32 mod(u32 x) const { return sh >= 0 ? x & (n - 1) : x % n; }
};

// ---------------------------------------------------------------- per-wave view of one GEMV
// A projection is cut along K into segments whose staged input fits the LDS activation region
// (one segment except for the widest inputs at batch 4); along N every wave of the grid owns a
// contiguous range of row pairs.  All fields are wave-uniform.
template <int WD, int B>
struct Stream {
    const uint8_t* w; const f16_t* s; const f16_t* z;
    size_t rowb;
    int N, K, ng;
    int nseg, seg, j0, nunits, cpr, nup;
    int p0, c0, n_it;   // first row pair (or group) and first chunk of it, iterations

    static constexpr int EPU = WTraits<WD>::EPU;
    static constexpr int kChunkUnits = kChunkUnitsOf<WD>;
    static constexpr int seg_units = (kLdsActBytes / (B * EPU * 4)) / kChunkUnits * kChunkUnits;

    // quad: rows are dealt out in groups of four (p0 counts groups) and a stage covers
    // kQuadChunkUnitsOf units of each of the four rows instead of kChunkUnits units of two rows.
    __device__ __forceinline__ static Stream make(const PMat& M, int seg, int gwave, const UDiv& n_gwaves, bool quad = false) {
        Stream S;
        S.w = M.w; S.s = M.s; S.z = M.z; S.N = M.n; S.K = M.k; S.ng = M.k / 128;
        S.rowb = WD == W_BF16 ? (size_t)M.k * 2 : WD == W_INT8 ? (size_t)M.k : (size_t)M.k / 2;
        const int total_units = M.k / EPU;
        S.nseg = (total_units + seg_units - 1) / seg_units;
        S.seg = seg;
        S.j0 = seg * seg_units;
        S.nunits = min(seg_units, total_units - S.j0);
        S.nup = (S.nunits + kChunkUnits - 1) / kChunkUnits * kChunkUnits;
        S.cpr = S.nup / (quad ? kQuadChunkUnitsOf<WD> : kChunkUnits);
        // row pairs (groups) [p0, p1) of this wave; the products fit 32 bits (rows * waves < 2^32)
        const u32 npairs = quad ? (u32)(M.n + 3) / 4 : (u32)(M.n + 1) / 2;
        S.p0 = (int)n_gwaves.div(npairs * (u32)gwave);
        S.c0 = 0;
        S.n_it = ((int)n_gwaves.div(npairs * (u32)(gwave + 1)) - S.p0) * S.cpr;
        // Groups of four rows that come out as an odd number of HALF groups per wave (the 8B QKV
        // projection: 1.5) are dealt out in halves along K instead: the wave's work is the flat
        // range [gwave * h, (gwave + 1) * h) of (group, chunk) iterations, h = chunks per wave, so
        // an odd wave starts in the middle of the group its even neighbour (same workgroup)
        // began; the two exchange their partial sums through LDS (gemv_run_quad).
        if (quad && S.nseg == 1 && (S.cpr & 1) == 0 && n_gwaves.mod(2 * npairs) == 0 && (n_gwaves.div(2 * npairs) & 1)) {
            const int h = (int)n_gwaves.div(2 * npairs) * (S.cpr / 2);
            S.p0 = gwave * h / S.cpr;
            S.c0 = gwave * h % S.cpr;
            S.n_it = h;
        }
        return S;
    }
};

// Issue the loads of iteration (pair, chunk).  Every load is issued unconditionally from a clamped
// address: out-of-range units meet zeros in the staged input, out-of-range rows are dropped by the
// epilogue.  Nothing is converted here, so no load result is waited for at issue time.
template <int WD, int B, int U0 = 0, int U1 = kUnrOf<WD>>
__device__ __forceinline__ void load_stage(const Stream<WD, B>& S, int pair, int chunk, Stage<WD>& st, int lane) {
    constexpr int kUnr = kUnrOf<WD>;
#pragma unroll
    for (int u = U0; u < U1; u++) {
        const int j = min((chunk * kUnr + u) * 64 + lane, S.nunits - 1);
#pragma unroll
        for (int r = 0; r < 2; r++) {
            const int row = min(2 * pair + r, S.N - 1);
            st.w[r][u] = ldg_stream(S.w + (size_t)row * S.rowb + (size_t)(S.j0 + j) * 16);
            if constexpr (WD == W_INT4) {
                const size_t gi = (size_t)row * S.ng + (S.j0 + j) / 4;
                st.s[r][u] = as_global(S.s)[gi];
                st.z[r][u] = as_global(S.z)[gi];
            }
        }
    }
    if constexpr (WD == W_INT8 && U1 == kUnr) {
        if (chunk == S.cpr - 1) {
            st.rs[0] = as_global(S.s)[min(2 * pair, S.N - 1)];
            st.rs[1] = as_global(S.s)[min(2 * pair + 1, S.N - 1)];
        }
    }
}

// The same for a group of four rows: lane (blk = lane / 4, r = lane % 4) loads unit blk of row r of
// each of the stage's 16-unit slices, i.e. a wave load covers 256 contiguous bytes of four rows.
template <int WD, int B, int U0 = 0, int U1 = kQuadLoadsOf<WD>>
__device__ __forceinline__ void load_stage_quad(const Stream<WD, B>& S, int grp, int chunk, Stage<WD>& st, int lane) {
    constexpr int NL = kQuadLoadsOf<WD>, kUnr = kUnrOf<WD>;
    const int row = min(4 * grp + (lane & 3), S.N - 1);
    const uint8_t* rp = S.w + (size_t)row * S.rowb + (size_t)S.j0 * 16;
#pragma unroll
    for (int u = U0; u < U1; u++) {
        const int j = min((chunk * NL + u) * 16 + (lane >> 2), S.nunits - 1);
        st.w[u / kUnr][u % kUnr] = ldg_stream(rp + (size_t)j * 16);
        if constexpr (WD == W_INT4) {
            const size_t gi = (size_t)row * S.ng + (S.j0 + j) / 4;
            st.s[u / kUnr][u % kUnr] = as_global(S.s)[gi];
            st.z[u / kUnr][u % kUnr] = as_global(S.z)[gi];
        }
    }
    if constexpr (WD == W_INT8 && U1 == NL) {
        st.rs[0] = as_global(S.s)[row];   // this lane's row (every stage: a wave may end in the middle of a group)
    }
}

// Issue iterations [s0, min(s1, n_it)) of a stream into ring slots of the same index (by default the
// whole ring: the first min(kDepth, n_it) iterations).
// FF_PREFETCH_STAGES: how many of them the fused kernel requests BEFORE it waits for a projection's
// input (what is requested across a hand-over queues in front of the input's loads); the rest of the
// ring is requested once the input is there.
#ifndef FF_PREFETCH_STAGES
#define FF_PREFETCH_STAGES FF_DEPTH
#endif
template <int WD> constexpr int kPrefetchOf = (WD == W_INT4 ? 2 : 1) * (FF_PREFETCH_STAGES < FF_DEPTH ? FF_PREFETCH_STAGES : FF_DEPTH);
template <bool QUAD, int WD, int B>
__device__ __forceinline__ void prefetch_stream(const Stream<WD, B>& S, Stage<WD> (&ring)[kDepthOf<WD>], int lane, int s0 = 0, int s1 = kDepthOf<WD>) {
    constexpr int kDepth = kDepthOf<WD>;
    int pair = S.p0, chunk = S.c0;
#pragma unroll
    for (int s = 0; s < kDepth; s++) {
        if (s >= s0 && s < s1 && s < S.n_it) {
            if constexpr (QUAD) load_stage_quad(S, pair, chunk, ring[s], lane);
            else load_stage(S, pair, chunk, ring[s], lane);
        }
        if (++chunk == S.cpr) { chunk = 0; ++pair; }
    }
}

// The multiply-accumulates of one stage: chunk cc of a row pair against the staged input.
template <int WD, int B, int U0 = 0, int U1 = kUnrOf<WD>>
__device__ __forceinline__ void stage_fma(const Stage<WD>& st, const float4* xs, int nup, int cc, int lane, float (&acc)[2][B]) {
    constexpr int kUnr = kUnrOf<WD>;
    constexpr int NQ = WTraits<WD>::EPU / 4;
#pragma unroll
    for (int u = U0; u < U1; u++) {
        const int j = (cc * kUnr + u) * 64 + lane;
#pragma unroll
        for (int b = 0; b < B; b++) {
            const float4* xq = xs + (size_t)b * NQ * nup + j;
            if constexpr (WD == W_BF16) {
                float4 x0 = xq[0], x1 = xq[nup];
                acc[0][b] = dot_bf16(st.w[0][u], x0, x1, acc[0][b]);
                acc[1][b] = dot_bf16(st.w[1][u], x0, x1, acc[1][b]);
            } else if constexpr (WD == W_INT8) {
                float4 x0 = xq[0], x1 = xq[nup], x2 = xq[2 * nup], x3 = xq[3 * nup];
#pragma unroll
                for (int r = 0; r < 2; r++) {
                    float a = acc[r][b];
                    a = dot_i8x4(st.w[r][u].x, x0, a); a = dot_i8x4(st.w[r][u].y, x1, a);
                    a = dot_i8x4(st.w[r][u].z, x2, a); a = dot_i8x4(st.w[r][u].w, x3, a);
                    acc[r][b] = a;
                }
            } else {
                float4 x[8];
#pragma unroll
                for (int q = 0; q < 8; q++) x[q] = xq[q * nup];
                const float xsum = ((sum4(x[0]) + sum4(x[1])) + (sum4(x[2]) + sum4(x[3]))) + ((sum4(x[4]) + sum4(x[5])) + (sum4(x[6]) + sum4(x[7])));
#pragma unroll
                for (int r = 0; r < 2; r++) {
                    const float sc = f16_to_f((f16_t)st.s[r][u]), zp = f16_to_f((f16_t)st.z[r][u]);
                    float t = dot_i4x8_codes(st.w[r][u].x, x[0], x[1], 0.f);
                    t = dot_i4x8_codes(st.w[r][u].y, x[2], x[3], t);
                    t = dot_i4x8_codes(st.w[r][u].z, x[4], x[5], t);
                    t = dot_i4x8_codes(st.w[r][u].w, x[6], x[7], t);
                    acc[r][b] = fmaf(sc, fmaf(-zp, xsum, t), acc[r][b]);
                }
            }
        }
    }
}

// The staged inputs of a whole stage read from LDS ahead of its multiply-accumulates (single
// sequence): with one wave per SIMD nothing else hides the latency of an LDS read,
// and a read issued right in front of its use costs that latency once per unit.  With
// FF_X_PRELOAD the reads of all units of a stage (int8: of a part) are issued when its first part
// (the part) starts (8B bf16, batch 1: 2968 -> 2946 us per step; issuing them a whole stage ahead
// gained nothing further).
#ifndef FF_X_PRELOAD
#define FF_X_PRELOAD 1
#endif
#ifndef FF_X_PRELOAD_I4
#define FF_X_PRELOAD_I4 1   // int4: both units of a stage (8B int4, batch 1: 2395 -> 2384 us per step)
#endif
template <int WD, int B> constexpr bool kXPreloadOf = FF_X_PRELOAD && (WD == W_BF16 || WD == W_INT8 || (WD == W_INT4 && FF_X_PRELOAD_I4)) && B == 1;
template <int WD> constexpr int kXQuadsOf = WTraits<WD>::EPU / 4;   // float4 reads per unit (bf16: 2, int8: 4)
// Units [U0, U1) of a stage: bf16 reads the whole stage's inputs with its first part (16 registers per
// part), int8 each part's inputs when the part starts (its units are twice as wide).
template <int WD, int U0, int U1>
__device__ __forceinline__ void stage_x_load(const float4* xs, int nup, int cc, int lane, float4 (&xr)[kUnrOf<WD>][kXQuadsOf<WD>]) {
    constexpr int kUnr = kUnrOf<WD>, NX = kXQuadsOf<WD>;
    constexpr int L0 = WD == W_INT8 ? U0 : 0, L1 = WD == W_INT8 ? U1 : (U0 == 0 ? kUnr : 0);   // int4 (whole-stage parts only): like bf16
#pragma unroll
    for (int u = L0; u < L1; u++) {
        const float4* xq = xs + (cc * kUnr + u) * 64 + lane;
#pragma unroll
        for (int q = 0; q < NX; q++) xr[u][q] = xq[q * nup];
    }
}
template <int WD, int U0, int U1>
__device__ __forceinline__ void stage_fma_x(const Stage<WD>& st, const float4 (&xr)[kUnrOf<WD>][kXQuadsOf<WD>], float (&acc)[2][1]) {
#pragma unroll
    for (int u = U0; u < U1; u++) {
        if constexpr (WD == W_BF16) {
            acc[0][0] = dot_bf16(st.w[0][u], xr[u][0], xr[u][1], acc[0][0]);
            acc[1][0] = dot_bf16(st.w[1][u], xr[u][0], xr[u][1], acc[1][0]);
        } else if constexpr (WD == W_INT8) {
#pragma unroll
            for (int r = 0; r < 2; r++) {
                float a = acc[r][0];
                a = dot_i8x4(st.w[r][u].x, xr[u][0], a); a = dot_i8x4(st.w[r][u].y, xr[u][1], a);
                a = dot_i8x4(st.w[r][u].z, xr[u][2], a); a = dot_i8x4(st.w[r][u].w, xr[u][3], a);
                acc[r][0] = a;
            }
        } else {
            const float4 (&x)[8] = xr[u];
            const float xsum = ((sum4(x[0]) + sum4(x[1])) + (sum4(x[2]) + sum4(x[3]))) + ((sum4(x[4]) + sum4(x[5])) + (sum4(x[6]) + sum4(x[7])));
#pragma unroll
            for (int r = 0; r < 2; r++) {
                const float sc = f16_to_f((f16_t)st.s[r][u]), zp = f16_to_f((f16_t)st.z[r][u]);
                float t = dot_i4x8_codes(st.w[r][u].x, x[0], x[1], 0.f);
                t = dot_i4x8_codes(st.w[r][u].y, x[2], x[3], t);
                t = dot_i4x8_codes(st.w[r][u].z, x[4], x[5], t);
                t = dot_i4x8_codes(st.w[r][u].w, x[6], x[7], t);
                acc[r][0] = fmaf(sc, fmaf(-zp, xsum, t), acc[r][0]);
            }
        }
    }
}

// Weight-streaming GEMV over one stream for up to B batch rows (paper Section 4.2: batch-one
// projections are matrix-vector products with the input cached on chip and each workgroup owning
// some rows of W; Section 5.2: at batch 2-4 the weights are still read exactly once and the inputs
// replicated).  On entry ring[s] holds iteration s (s < min(kDepth, n_it)); iteration i+kDepth is
// issued into the slot iteration i has just freed, so 2*kDepth*kUnr 16-byte non-temporal loads
// per lane stay in flight across row boundaries.  epi(pair, b, v0, v1) runs on lane 0 with the two
// finished dot products of rows (2*pair, 2*pair+1); partial sums of earlier K segments are carried
// in `myacc` (LDS, private to the wave).
template <int WD, int B, class Epi>
__device__ __forceinline__ void gemv_run(const Stream<WD, B>& S, Stage<WD> (&ring)[kDepthOf<WD>], const float4* xs, float* myacc,
                                         int batch, int lane, Epi& epi) {
    constexpr int kDepth = kDepthOf<WD>;
    const int nup = S.nup;
    float acc[2][B];
#pragma unroll
    for (int b = 0; b < B; b++) acc[0][b] = acc[1][b] = 0.f;
    int pc = S.p0, cc = 0;          // (pair, chunk) of the next compute
    int pl = S.p0, cl = 0;          // (pair, chunk) of the next load = iteration kDepth
    for (int s = 0; s < kDepth; s++) if (++cl == S.cpr) { cl = 0; ++pl; }

    constexpr int kUnr = kUnrOf<WD>, kParts = kRefillPartsOf<WD, B>;
    float4 xr[kUnr][kXQuadsOf<WD>];   // (kXPreloadOf) the stage's inputs, read ahead of their multiply-accumulates
    auto compute = [&](const Stage<WD>& st, auto units) {   // units: the StageUnits range multiplied by this call; the last one finishes the iteration
        constexpr int U0 = decltype(units)::u0, U1 = decltype(units)::u1;
        if constexpr (kXPreloadOf<WD, B>) {
            stage_x_load<WD, U0, U1>(xs, nup, cc, lane, xr);
            stage_fma_x<WD, U0, U1>(st, xr, acc);
        } else stage_fma<WD, B, U0, U1>(st, xs, nup, cc, lane, acc);
        if constexpr (U1 < kUnr) return;
        if (cc == S.cpr - 1) {   // row pair finished (for this K segment)
            const int lp = pc - S.p0;
#pragma unroll
            for (int b = 0; b < B; b++) {
                float v0 = wave_sum_uniform(acc[0][b]), v1 = wave_sum_uniform(acc[1][b]);
                acc[0][b] = acc[1][b] = 0.f;
                if constexpr (WD == W_INT8) { v0 *= f16_to_f((f16_t)st.rs[0]); v1 *= f16_to_f((f16_t)st.rs[1]); }
                if (lane == 0 && b < batch) {
                    if (S.nseg > 1) {
                        float* a = myacc + ((size_t)lp * B + b) * 2;
                        if (S.seg > 0) { v0 += a[0]; v1 += a[1]; }
                        if (S.seg < S.nseg - 1) { a[0] = v0; a[1] = v1; }
                    }
                    if (S.seg == S.nseg - 1) epi(pc, b, v0, v1);
                }
            }
        }
        if (++cc == S.cpr) { cc = 0; ++pc; }
    };
    auto load = [&](Stage<WD>& st, auto units) {
        constexpr int U0 = decltype(units)::u0, U1 = decltype(units)::u1;
        load_stage<WD, B, U0, U1>(S, pl, cl, st, lane);
        if constexpr (U1 < kUnr) return;
        if (++cl == S.cpr) { cl = 0; ++pl; }
    };
    int it = 0;
    // steady state: every slot is consumed and refilled
    for (; it + 2 * kDepth <= S.n_it; it += kDepth) {
#pragma unroll
        for (int s = 0; s < kDepth; s++) {
            // keep the instruction scheduler from hoisting a slot's refill above the FMAs that
            // still read the slot: that doubles the live tile registers and ends in spills
            static_for<0, kParts>([&](auto part) {
                constexpr int P = decltype(part)::u0;
                typedef StageUnits<P * kUnr / kParts, (P + 1) * kUnr / kParts> Units;
                compute(ring[s], Units{});
                __builtin_amdgcn_sched_barrier(0);
                load(ring[s], Units{});
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    }
    // tail
    for (; it < S.n_it; it += kDepth) {
#pragma unroll
        for (int s = 0; s < kDepth; s++) {
            if (it + s < S.n_it) {
                compute(ring[s], StageUnits<0, kUnr>{});
                __builtin_amdgcn_sched_barrier(0);
                if (it + s + kDepth < S.n_it) load(ring[s], StageUnits<0, kUnr>{});
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
}

// ---------------------------------------------------------------- matrix-core variant (bf16, batch >= 2)
// The same stream for groups of FOUR rows on v_mfma_f32_4x4x4_16b_bf16, which multiplies sixteen
// independent 4x4x4 blocks per wave: in block blk = lane / 4, lane r = lane % 4 supplies row r of
// A (four k values) and column r of B, and receives column r of the 4x4 result (register i = row
// i).  Here A = the four weight rows over four consecutive k (half of the lane's 16-byte unit) and
// B = the staged inputs of sequences 0..3 over the same k, so one instruction does the 64
// multiply-adds that cost 16 vector FMAs plus conversions in gemv_run, and the cost no longer
// grows with the batch (paper Section 5.2 keeps the weights read once at batch 2-4; this keeps the
// arithmetic from becoming the limit there).  The inputs stay fp32-accurate: staging splits every
// value into a bf16 head and a bf16 remainder (two planes per sequence, see stage_store), and both
// are multiplied.  Unit j of sequence b sits at index (j ^ ((b & 3) << 2)) of its plane, which spreads
// the four lanes of a block over different LDS banks.  More than four sequences take one
// accumulator pair per set of four (the weights in registers are reused).
// Value of lane I of every aligned group of four lanes (DPP quad permute).
template <int I>
__device__ __forceinline__ float quad_bcast(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), I * 0x55, 0xF, 0xF, true));
}
typedef short mfma_s4 __attribute__((ext_vector_type(4)));
typedef float mfma_f4 __attribute__((ext_vector_type(4)));

template <int WD, int B, class Epi>
__device__ __forceinline__ void gemv_run_quad(const Stream<WD, B>& S, Stage<WD> (&ring)[kDepthOf<WD>], const float4* xs,
                                              float* myacc, int batch, int lane, Epi& epi) {
    static_assert(WD == W_BF16 || B <= 4, "more than one set of four sequences: bf16 only");
    constexpr int kDepth = kDepthOf<WD>;
    constexpr int NL = kQuadLoadsOf<WD>, kUnr = kUnrOf<WD>;
    constexpr int NC = (B + 3) / 4;   // sets of four sequences (one accumulator pair each)
    const int nup = S.nup;
    const int r4 = lane & 3;
    const u32x4* xh[NC];
#pragma unroll
    for (int c = 0; c < NC; c++) {
        const int bl = min(4 * c + r4, B - 1);   // sequence whose inputs this lane feeds (columns >= B are never read back)
        if constexpr (WD == W_BF16) xh[c] = (const u32x4*)xs + (size_t)(2 * bl) * nup + ((lane >> 2) ^ ((bl & 3) << 2));
        else if constexpr (WD == W_INT8) xh[c] = (const u32x4*)xs + ((size_t)(2 * bl) * nup + ((lane >> 2) ^ ((bl & 2) << 1))) * 2;
        else xh[c] = (const u32x4*)xs + ((size_t)(2 * bl) * nup + (lane >> 2)) * 4;
    }
    const int bl0 = min(r4, B - 1);
    const float* xsum = xsum_of(xs) + (size_t)bl0 * nup + (lane >> 2);   // int4 only
    mfma_f4 acc0[NC], acc1[NC];
#pragma unroll
    for (int c = 0; c < NC; c++) { acc0[c] = mfma_f4{0.f, 0.f, 0.f, 0.f}; acc1[c] = mfma_f4{0.f, 0.f, 0.f, 0.f}; }
    int pc = S.p0, cc = S.c0;       // (group, chunk) of the next compute
    int pl = S.p0, cl = S.c0;       // (group, chunk) of the next load = iteration kDepth
    for (int s = 0; s < kDepth; s++) if (++cl == S.cpr) { cl = 0; ++pl; }

    auto half = [](u32 a, u32 b) { u32x2 v{a, b}; return __builtin_bit_cast(mfma_s4, v); };
    constexpr int kParts = kQuadRefillPartsOf<WD>;
    auto compute = [&](const Stage<WD>& st, bool last, auto units) {   // units: the StageUnits range of the stage's loads multiplied by this call; the last one finishes the iteration
        constexpr int U0 = decltype(units)::u0, U1 = decltype(units)::u1;
        // int4: the staged inputs of unit u+1 are requested from LDS before unit u is multiplied
        // (with one wave per SIMD nothing else hides the LDS latency, and a unit needs nine reads)
        u32x4 hx[2][4], lx[2][4];
        float Xs[2];
        auto fetch = [&](int u, int slot) {
            const size_t off = (size_t)(cc * NL + u) * 16;
#pragma unroll
            for (int q = 0; q < 4; q++) {
                hx[slot][q] = xh[0][off * 4 + (q ^ r4)];
                lx[slot][q] = xh[0][((size_t)nup + off) * 4 + (q ^ r4)];
            }
            Xs[slot] = xsum[off];
        };
        if constexpr (WD == W_INT4) fetch(0, 0);
#pragma unroll
        for (int u = U0; u < U1; u++) {
            const int off = (cc * NL + u) * 16;
            const u32x4 w = st.w[u / kUnr][u % kUnr];
            if constexpr (WD == W_INT4) {
                if (u + 1 < NL) fetch(u + 1, (u + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (WD == W_BF16) {
#pragma unroll
                for (int c = 0; c < NC; c++) {
                    const u32x4 h = xh[c][off], l = xh[c][off + nup];
                    acc0[c] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(w.x, w.y), half(h.x, h.y), acc0[c], 0, 0, 0);
                    acc1[c] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(w.x, w.y), half(l.x, l.y), acc1[c], 0, 0, 0);
                    acc0[c] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(w.z, w.w), half(h.z, h.w), acc0[c], 0, 0, 0);
                    acc1[c] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(w.z, w.w), half(l.z, l.w), acc1[c], 0, 0, 0);
                }
            } else if constexpr (WD == W_INT8) {
                // int8 per-channel: a signed byte is exact in bf16 (8 significant bits), so the
                // unit's 16 codes are converted (sign-extending byte conversion, then the upper
                // halves of two floats packed into one register) and multiplied like bf16
                // weights; the row scale is applied to the finished sums.
                const u32 ww[4] = {w.x, w.y, w.z, w.w};
                auto pack = [](float lo, float hi) { return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u); };
#pragma unroll
                for (int q = 0; q < 2; q++) {   // 8 codes = one 16-byte chunk of heads and one of remainders
                    const int qq = q ^ (bl0 & 1);
                    const u32x4 h = xh[0][(size_t)off * 2 + qq], l = xh[0][((size_t)nup + off) * 2 + qq];
                    const u32 wa = ww[2 * q], wb = ww[2 * q + 1];
                    const u32 a0 = pack((float)(int)(int8_t)wa, (float)(int)(int8_t)(wa >> 8));
                    const u32 a1 = pack((float)(int)(int8_t)(wa >> 16), (float)((int)wa >> 24));
                    const u32 a2 = pack((float)(int)(int8_t)wb, (float)(int)(int8_t)(wb >> 8));
                    const u32 a3 = pack((float)(int)(int8_t)(wb >> 16), (float)((int)wb >> 24));
                    acc0[0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(a0, a1), half(h.x, h.y), acc0[0], 0, 0, 0);
                    acc1[0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(a0, a1), half(l.x, l.y), acc1[0], 0, 0, 0);
                    acc0[0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(a2, a3), half(h.z, h.w), acc0[0], 0, 0, 0);
                    acc1[0] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(a2, a3), half(l.z, l.w), acc1[0], 0, 0, 0);
                }
            } else {
                // int4 group-128: the unit's 32 codes n become the bf16 numbers 128 + n by bit
                // operations alone (0x4300 | n: exponent 2^7, n in the mantissa), so the blocks
                // deliver d = sum (128 + n) x, and with X = sum of the unit's x (staged beside it)
                //   sum s (n - z) x  =  s (d - (128 + z) X).
                // Scale s and zero z belong to the ROW, which the lanes of a block hold one each:
                // they are passed round the four lanes with quad permutes.
                const u32 ww[4] = {w.x, w.y, w.z, w.w};
                mfma_f4 dh = {0.f, 0.f, 0.f, 0.f}, dl = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int q = 0; q < 4; q++) {   // 8 codes = one 16-byte chunk of heads and one of remainders
                    const u32x4 h = hx[u & 1][q], l = lx[u & 1][q];
                    const u32 e = ww[q] & 0x0F0F0F0Fu, o = (ww[q] >> 4) & 0x0F0F0F0Fu;   // codes 0,2,4,6 / 1,3,5,7 as bytes
                    const u32 a0 = __builtin_amdgcn_perm(o, e, 0x0c040c00u) | 0x43004300u;   // codes 0, 1
                    const u32 a1 = __builtin_amdgcn_perm(o, e, 0x0c050c01u) | 0x43004300u;   // codes 2, 3
                    const u32 a2 = __builtin_amdgcn_perm(o, e, 0x0c060c02u) | 0x43004300u;   // codes 4, 5
                    const u32 a3 = __builtin_amdgcn_perm(o, e, 0x0c070c03u) | 0x43004300u;   // codes 6, 7
                    dh = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(a0, a1), half(h.x, h.y), dh, 0, 0, 0);
                    dl = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(a0, a1), half(l.x, l.y), dl, 0, 0, 0);
                    dh = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(a2, a3), half(h.z, h.w), dh, 0, 0, 0);
                    dl = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(half(a2, a3), half(l.z, l.w), dl, 0, 0, 0);
                }
                const float X = Xs[u & 1];
                const float sc = f16_to_f((f16_t)st.s[u / kUnr][u % kUnr]);
                const float zp = 128.f + f16_to_f((f16_t)st.z[u / kUnr][u % kUnr]);
                // row i of the block: scale and zero held by lane i of the quad
                acc0[0][0] = fmaf(quad_bcast<0>(sc), fmaf(-quad_bcast<0>(zp), X, dh[0] + dl[0]), acc0[0][0]);
                acc0[0][1] = fmaf(quad_bcast<1>(sc), fmaf(-quad_bcast<1>(zp), X, dh[1] + dl[1]), acc0[0][1]);
                acc0[0][2] = fmaf(quad_bcast<2>(sc), fmaf(-quad_bcast<2>(zp), X, dh[2] + dl[2]), acc0[0][2]);
                acc0[0][3] = fmaf(quad_bcast<3>(sc), fmaf(-quad_bcast<3>(zp), X, dh[3] + dl[3]), acc0[0][3]);
            }
        }
        if constexpr (U1 < NL) return;
        if (cc == S.cpr - 1 || last) {   // group finished (for this K segment, or this wave's part of it): add up the sixteen blocks
            float t[NC][4];
#pragma unroll
            for (int c = 0; c < NC; c++) {
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    float v = acc0[c][i] + acc1[c][i];
                    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xF, 0xF, true));   // row_ror:8
                    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x124, 0xF, 0xF, true));   // row_ror:4
                    v += __shfl_xor(v, 16);
                    v += __shfl_xor(v, 32);
                    t[c][i] = v;   // row 4*group + i, sequence 4*c + lane % 4
                }
                if constexpr (WD == W_INT8) {   // row scales: lane r of a quad holds that of row r
                    const float rs = f16_to_f((f16_t)st.rs[0]);
                    t[c][0] *= quad_bcast<0>(rs); t[c][1] *= quad_bcast<1>(rs); t[c][2] *= quad_bcast<2>(rs); t[c][3] *= quad_bcast<3>(rs);
                }
                acc0[c] = mfma_f4{0.f, 0.f, 0.f, 0.f};
                acc1[c] = mfma_f4{0.f, 0.f, 0.f, 0.f};
            }
            // A group shared with the neighbouring wave (see Stream::make): each of the two drops
            // its sums into its side of the pair's mailbox and then bumps the pair's flag; the
            // one that finds the flag already bumped adds the other's sums and finishes the rows.
            // LDS executes a wave's operations in order, so the sums are in place before the flag
            // moves; nobody waits for anybody.
            const bool ended_early = cc != S.cpr - 1, started_late = pc == S.p0 && S.c0 != 0;
            bool finish = true;
            if (ended_early || started_late) {
                const int pair = (int)(threadIdx.x >> 7), side = ended_early ? 0 : 1;
                lds_float* box = pairbox_of(xs);
                lds_u32* flag = (lds_u32*)(box + 4 * kPairBoxFloats) + pair;
                lds_float* mine = box + (pair * 2 + side) * kPairBoxFloats;
                lds_float* other = box + (pair * 2 + (1 - side)) * kPairBoxFloats;
                if (lane < 4) {
#pragma unroll
                    for (int c = 0; c < NC; c++)
#pragma unroll
                        for (int i = 0; i < 4; i++) mine[(c * 4 + lane) * 4 + i] = t[c][i];
                }
                asm volatile("" ::: "memory");
                u32 seen = 0;
                if (lane == 0) seen = __hip_atomic_fetch_add(flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                seen = (u32)__builtin_amdgcn_readfirstlane((int)seen);
                asm volatile("" ::: "memory");
                finish = seen != 0;
                if (finish) {
                    if (lane < 4) {
#pragma unroll
                        for (int c = 0; c < NC; c++)
#pragma unroll
                            for (int i = 0; i < 4; i++) t[c][i] += other[(c * 4 + lane) * 4 + i];
                    }
                    if (lane == 0) *flag = 0u;   // next use: a later projection, behind workgroup barriers
                }
            }
#pragma unroll
            for (int c = 0; c < NC; c++) {
                const int b = 4 * c + lane;
                if (finish && lane < 4 && b < batch) {   // lanes 0..3 finish one sequence each
                    if (S.nseg > 1) {
                        float* a = myacc + ((size_t)(pc - S.p0) * B + b) * 4;
#pragma unroll
                        for (int i = 0; i < 4; i++) {
                            if (S.seg > 0) t[c][i] += a[i];
                            if (S.seg < S.nseg - 1) a[i] = t[c][i];
                        }
                    }
                    if (S.seg == S.nseg - 1) {
                        epi(2 * pc, b, t[c][0], t[c][1]);
                        if (4 * pc + 2 < S.N) epi(2 * pc + 1, b, t[c][2], t[c][3]);
                    }
                }
            }
        }
        if (++cc == S.cpr) { cc = 0; ++pc; }
    };
    auto load = [&](Stage<WD>& st, auto units) {
        constexpr int U0 = decltype(units)::u0, U1 = decltype(units)::u1;
        load_stage_quad<WD, B, U0, U1>(S, pl, cl, st, lane);
        if constexpr (U1 < NL) return;
        if (++cl == S.cpr) { cl = 0; ++pl; }
    };
    int it = 0;
    for (; it + 2 * kDepth <= S.n_it; it += kDepth) {
#pragma unroll
        for (int s = 0; s < kDepth; s++) {
            static_for<0, kParts>([&](auto part) {
                constexpr int P = decltype(part)::u0;
                typedef StageUnits<P * NL / kParts, (P + 1) * NL / kParts> Units;
                compute(ring[s], false, Units{});
                __builtin_amdgcn_sched_barrier(0);
                load(ring[s], Units{});
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    }
    for (; it < S.n_it; it += kDepth) {
#pragma unroll
        for (int s = 0; s < kDepth; s++) {
            if (it + s < S.n_it) {
                compute(ring[s], it + s == S.n_it - 1, StageUnits<0, NL>{});
                __builtin_amdgcn_sched_barrier(0);
                if (it + s + kDepth < S.n_it) load(ring[s], StageUnits<0, NL>{});
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
}

}  // namespace ff
