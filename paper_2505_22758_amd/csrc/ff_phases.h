// Phase bodies of the decode step: activation staging, weight-streaming GEMV, split-KV attention.
// Each is a workgroup-collective device function used by the fused kernel (between grid barriers)
// and, with launch boundaries instead of barriers, by the per-operation baseline kernels.
#pragma once
#include "ff_device.h"

namespace ff {

template <int WD> struct WTraits;
template <> struct WTraits<W_BF16> { static constexpr int EPU = 8; };   // elements per 16-byte unit
template <> struct WTraits<W_INT8> { static constexpr int EPU = 16; };
template <> struct WTraits<W_INT4> { static constexpr int EPU = 32; };

constexpr int kUnr = 4;   // 16-byte loads per row kept in flight per lane and pipeline stage

// Where a GEMV phase takes its input vector(s) from.
struct ActSrc {
    const void* base;     // fp32 exchange buffer, or bf16 embedding table
    const int* tokens;    // non-null: row b is base(bf16)[tokens[b]][K]
    size_t stride;        // elements between batch rows (fp32 source)
    const bf16_t* gain;   // non-null: RMSNorm with this gain is applied while staging
    float eps;
};

__device__ __forceinline__ float block_sum(float v, float* red /*LDS, >= kWaves floats*/) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; w++) t += red[w];
    return t;
}

// Stage elements [k0, k0 + nunits*EPU) of every batch row into LDS, quad-planar so that a wave's
// 64 lanes read 64 consecutive float4: quad qd of unit j of row b lives at xs[(b*NQ + qd)*nup + j].
// Units [nunits, nup) are zero filled.  With a gain, RMSNorm (paper Section 2.1: pre-RMSNorm in
// front of the QKV and GLU in/gate projections) is applied; that needs k0 == 0 and the whole row.
template <int EPU, class IO>
__device__ void stage_act(const ActSrc& S, int batch, int K, int k0, int nunits, int nup, float4* xs, float* red) {
    constexpr int NQ = EPU / 4;
    const int nquads = nunits * NQ;
    const int padquads = nup * NQ;
    for (int b = 0; b < batch; b++) {
        float4* xb = xs + (size_t)b * NQ * nup;
        float ss = 0.f;
        for (int qi = threadIdx.x; qi < padquads; qi += kThreads) {
            int j = qi / NQ, qd = qi % NQ;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (qi < nquads) {
                int k = k0 + qi * 4;
                if (S.tokens) {
                    const bf16_t* row = (const bf16_t*)S.base + (size_t)S.tokens[b] * K;
                    u32x2 w = *(const u32x2*)(row + k);
                    v = make_float4(bf_lo(w.x), bf_hi(w.x), bf_lo(w.y), bf_hi(w.y));
                } else {
                    const float* row = (const float*)S.base + (size_t)b * S.stride;
                    float2 a = IO::ld2(row + k), c = IO::ld2(row + k + 2);
                    v = make_float4(a.x, a.y, c.x, c.y);
                }
                if (S.gain) {
                    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
                    u32x2 g = *(const u32x2*)(S.gain + k);
                    v.x *= bf_lo(g.x); v.y *= bf_hi(g.x); v.z *= bf_lo(g.y); v.w *= bf_hi(g.y);
                }
            }
            xb[(size_t)qd * nup + j] = v;
        }
        if (S.gain) {
            float tot = block_sum(ss, red);
            float r = 1.0f / sqrtf(tot / (float)K + S.eps);
            for (int qi = threadIdx.x; qi < nquads; qi += kThreads) {
                int j = qi / NQ, qd = qi % NQ;
                float4 v = xb[(size_t)qd * nup + j];
                v.x *= r; v.y *= r; v.z *= r; v.w *= r;
                xb[(size_t)qd * nup + j] = v;
            }
        }
    }
    __syncthreads();
}

// ---- one 16-byte unit of weights against the staged activations ----
template <int WD> struct UnitAux {};                       // per-unit side data (int4 scale/zero)
template <> struct UnitAux<W_INT4> { float s, z; };

template <int WD>
__device__ __forceinline__ float unit_dot(const u32x4& w, const UnitAux<WD>& aux, const float4* xq, int nup);

template <>
__device__ __forceinline__ float unit_dot<W_BF16>(const u32x4& w, const UnitAux<W_BF16>&, const float4* xq, int nup) {
    float4 a = xq[0], b = xq[nup];
    float acc = bf_lo(w.x) * a.x;
    acc = fmaf(bf_hi(w.x), a.y, acc);
    acc = fmaf(bf_lo(w.y), a.z, acc);
    acc = fmaf(bf_hi(w.y), a.w, acc);
    acc = fmaf(bf_lo(w.z), b.x, acc);
    acc = fmaf(bf_hi(w.z), b.y, acc);
    acc = fmaf(bf_lo(w.w), b.z, acc);
    acc = fmaf(bf_hi(w.w), b.w, acc);
    return acc;
}
__device__ __forceinline__ float i8dot4(u32 w, const float4& x, float acc) {
    acc = fmaf((float)(int)(int8_t)(w), x.x, acc);
    acc = fmaf((float)(int)(int8_t)(w >> 8), x.y, acc);
    acc = fmaf((float)(int)(int8_t)(w >> 16), x.z, acc);
    acc = fmaf((float)((int)w >> 24), x.w, acc);
    return acc;
}
template <>
__device__ __forceinline__ float unit_dot<W_INT8>(const u32x4& w, const UnitAux<W_INT8>&, const float4* xq, int nup) {
    float acc = 0.f;
    acc = i8dot4(w.x, xq[0], acc);
    acc = i8dot4(w.y, xq[nup], acc);
    acc = i8dot4(w.z, xq[2 * nup], acc);
    acc = i8dot4(w.w, xq[3 * nup], acc);
    return acc;
}
// (code - z) * s is formed exactly as the dequantisation definition, then multiplied by x.
__device__ __forceinline__ float i4dot8(u32 w, const float4& x0, const float4& x1, float s, float z, float acc) {
    acc = fmaf(((float)(w & 15u) - z) * s, x0.x, acc);
    acc = fmaf(((float)((w >> 4) & 15u) - z) * s, x0.y, acc);
    acc = fmaf(((float)((w >> 8) & 15u) - z) * s, x0.z, acc);
    acc = fmaf(((float)((w >> 12) & 15u) - z) * s, x0.w, acc);
    acc = fmaf(((float)((w >> 16) & 15u) - z) * s, x1.x, acc);
    acc = fmaf(((float)((w >> 20) & 15u) - z) * s, x1.y, acc);
    acc = fmaf(((float)((w >> 24) & 15u) - z) * s, x1.z, acc);
    acc = fmaf(((float)(w >> 28) - z) * s, x1.w, acc);
    return acc;
}
template <>
__device__ __forceinline__ float unit_dot<W_INT4>(const u32x4& w, const UnitAux<W_INT4>& a, const float4* xq, int nup) {
    float acc = 0.f;
    acc = i4dot8(w.x, xq[0], xq[nup], a.s, a.z, acc);
    acc = i4dot8(w.y, xq[2 * nup], xq[3 * nup], a.s, a.z, acc);
    acc = i4dot8(w.z, xq[4 * nup], xq[5 * nup], a.s, a.z, acc);
    acc = i4dot8(w.w, xq[6 * nup], xq[7 * nup], a.s, a.z, acc);
    return acc;
}

template <int WD> struct PipeBuf {
    u32x4 w[2][kUnr];
    UnitAux<WD> aux[2][kUnr];
};

// Weight-streaming GEMV for up to B batch rows (paper Section 3.2: batch-one projections are
// matrix-vector products with the input cached on chip and each workgroup owning some rows of W;
// Section 4.2: at batch 2-4 the weights are still read exactly once and the inputs replicated).
// Rows are handled in adjacent pairs (2p, 2p+1); every wave of the grid owns a contiguous range
// of pairs and keeps 2*kUnr 16-byte non-temporal loads per lane in flight, one pipeline stage
// ahead of the FMAs, across row boundaries.  epi(pair, b, v0, v1) runs on lane 0 with the two
// finished dot products.
template <int WD, int B, class IO, class Epi>
__device__ void gemv_phase(const PMat& M, const ActSrc& S, int batch, uint8_t* lds, Epi& epi) {
    constexpr int EPU = WTraits<WD>::EPU;
    constexpr int NQ = EPU / 4;
    float4* xs = (float4*)lds;
    float* accbuf = (float*)(lds + kLdsActBytes);
    float* red = (float*)(lds + kLdsActBytes + kLdsAuxBytes - 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int K = M.k, N = M.n;
    const size_t rowb = M.row_bytes();
    const int total_units = K / EPU;
    constexpr int chunk_units = 64 * kUnr;
    int seg_units = (kLdsActBytes / (B * EPU * 4)) / chunk_units * chunk_units;
    const int nseg = (total_units + seg_units - 1) / seg_units;
    const long npairs = (N + 1) / 2;
    const long nwg = (long)gridDim.x * kWaves, gw = (long)blockIdx.x * kWaves + wave;
    const int p0 = (int)(npairs * gw / nwg), p1 = (int)(npairs * (gw + 1) / nwg);
    const int my_pairs = p1 - p0;
    float* myacc = accbuf + (size_t)wave * ((kLdsAuxBytes - 64) / 4 / kWaves);

    for (int seg = 0; seg < nseg; seg++) {
        const int j0 = seg * seg_units;
        const int nunits = min(seg_units, total_units - j0);
        const int cpr = (nunits + chunk_units - 1) / chunk_units;
        const int nup = cpr * chunk_units;
        if (seg > 0) __syncthreads();
        stage_act<EPU, IO>(S, batch, K, j0 * EPU, nunits, nup, xs, red);

        const int n_it = my_pairs * cpr;
        PipeBuf<WD> bufA, bufB;
        auto load_it = [&](PipeBuf<WD>& buf, int pair, int chunk) {
#pragma unroll
            for (int u = 0; u < kUnr; u++) {
                int j = (chunk * kUnr + u) * 64 + lane;
                bool valid = j < nunits;
#pragma unroll
                for (int r = 0; r < 2; r++) {
                    int row = 2 * pair + r;
                    bool ok = valid && row < N;
                    const uint8_t* p = M.w + (size_t)row * rowb + (size_t)(j0 + j) * 16;
                    buf.w[r][u] = ok ? ldg_stream(p) : u32x4{0u, 0u, 0u, 0u};
                    if constexpr (WD == W_INT4) {
                        int g = (j0 + j) / 4, ng = K / 128;
                        buf.aux[r][u].s = ok ? f16_to_f(M.s[(size_t)row * ng + g]) : 0.f;
                        buf.aux[r][u].z = ok ? f16_to_f(M.z[(size_t)row * ng + g]) : 0.f;
                    }
                }
            }
        };
        float acc[2][B];
#pragma unroll
        for (int b = 0; b < B; b++) acc[0][b] = acc[1][b] = 0.f;
        auto compute_it = [&](const PipeBuf<WD>& buf, int pair, int chunk) {
#pragma unroll
            for (int u = 0; u < kUnr; u++) {
                int j = (chunk * kUnr + u) * 64 + lane;
#pragma unroll
                for (int b = 0; b < B; b++) {
                    const float4* xq = xs + (size_t)b * NQ * nup + j;
                    acc[0][b] += unit_dot<WD>(buf.w[0][u], buf.aux[0][u], xq, nup);
                    acc[1][b] += unit_dot<WD>(buf.w[1][u], buf.aux[1][u], xq, nup);
                }
            }
            if (chunk == cpr - 1) {
                int lp = pair - p0;
#pragma unroll
                for (int b = 0; b < B; b++) {
                    float v0 = wave_sum(acc[0][b]), v1 = wave_sum(acc[1][b]);
                    acc[0][b] = acc[1][b] = 0.f;
                    if (lane == 0 && b < batch) {
                        if (nseg > 1) {
                            float* a = myacc + ((size_t)lp * B + b) * 2;
                            if (seg > 0) { v0 += a[0]; v1 += a[1]; }
                            if (seg < nseg - 1) { a[0] = v0; a[1] = v1; }
                        }
                        if (seg == nseg - 1) {
                            if constexpr (WD == W_INT8) {
                                v0 *= f16_to_f(M.s[2 * pair]);
                                if (2 * pair + 1 < N) v1 *= f16_to_f(M.s[2 * pair + 1]);
                            }
                            epi(pair, b, v0, v1);
                        }
                    }
                }
            }
        };
        if (n_it > 0) {
            int pl = p0, cl = 0;   // (pair, chunk) of the next load
            int pc = p0, cc = 0;   // (pair, chunk) of the next compute
            auto adv = [&](int& p, int& c) { if (++c == cpr) { c = 0; ++p; } };
            load_it(bufA, pl, cl); adv(pl, cl);
            for (int it = 0; it < n_it; it += 2) {
                if (it + 1 < n_it) { load_it(bufB, pl, cl); adv(pl, cl); }
                compute_it(bufA, pc, cc); adv(pc, cc);
                if (it + 1 < n_it) {
                    if (it + 2 < n_it) { load_it(bufA, pl, cl); adv(pl, cl); }
                    compute_it(bufB, pc, cc); adv(pc, cc);
                }
            }
        }
    }
}

// ---------------------------------------------------------------- split-KV attention
// One work item = (sequence b, kv head j, rows [t0, t1) of its cache [+ this step's own k,v]).
// All G query heads that share kv head j are processed together, so each cached K and V element
// is read exactly once (paper Section 3.2, core attention: workgroups are split among KV heads and
// hold the queries of that head; the current token's k,v are taken from the exchange buffer, not
// from the cache).  Result: per query head the partial (max score, denominator, unnormalised
// output) of a FlashDecoding-style split, in base-2 exponent units.
//
// Thread mapping: a cache row is hd*2 bytes = LPR lanes x 16 bytes, so one wave load covers
// 64/LPR rows; lane (grp, sub) holds dims [8*sub, 8*sub+8) of row grp.  Every (wave, grp) keeps its
// own online-softmax state; the kWaves*64/LPR states are merged through LDS at the end.
template <int HD, int G, class IO>
__device__ void attn_item(const DevModel& M, const DevKV& KV, int layer, int b, int j, int t0, int t1, bool with_cur,
                          int split, uint8_t* lds) {
    constexpr int LPR = HD / 8;        // lanes per cache row
    constexpr int RPW = 64 / LPR;      // rows per wave load
    constexpr int NS = kWaves * RPW;   // partial states per workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPR, sub = lane % LPR;
    const float sc = 1.4426950408889634f / sqrtf((float)HD);   // alpha * log2(e)

    float qr[G][8];
#pragma unroll
    for (int g = 0; g < G; g++) {
        const float* qp = M.q + ((size_t)b * M.Hq + (j * G + g)) * HD + sub * 8;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            float2 v = IO::ld2(qp + e);
            qr[g][e] = v.x; qr[g][e + 1] = v.y;
        }
    }
    float m[G], l[G], o[G][8];
#pragma unroll
    for (int g = 0; g < G; g++) {
        m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e++) o[g][e] = 0.f;
    }
    auto update = [&](const float (&kf)[8], const float (&vf)[8], bool valid) {
#pragma unroll
        for (int g = 0; g < G; g++) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; e++) s = fmaf(qr[g][e], kf[e], s);
#pragma unroll
            for (int off = LPR / 2; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
            s *= sc;
            if (valid) {
                float mn = fmaxf(m[g], s);
                float corr = exp2f(m[g] - mn), p = exp2f(s - mn);
                l[g] = l[g] * corr + p;
#pragma unroll
                for (int e = 0; e < 8; e++) o[g][e] = fmaf(p, vf[e], o[g][e] * corr);
                m[g] = mn;
            }
        }
    };
    const bf16_t* Kp = KV.plane(M, layer, b, j, 0);
    const bf16_t* Vp = KV.plane(M, layer, b, j, 1);
    for (int tb = t0 + wave * RPW; tb < t1; tb += kWaves * RPW) {
        int t = tb + grp;
        bool valid = t < t1;
        u32x4 kw = {0u, 0u, 0u, 0u}, vw = {0u, 0u, 0u, 0u};
        if (valid) {
            kw = ldg_stream(Kp + (size_t)t * HD + sub * 8);
            vw = ldg_stream(Vp + (size_t)t * HD + sub * 8);
        }
        float kf[8] = {bf_lo(kw.x), bf_hi(kw.x), bf_lo(kw.y), bf_hi(kw.y), bf_lo(kw.z), bf_hi(kw.z), bf_lo(kw.w), bf_hi(kw.w)};
        float vf[8] = {bf_lo(vw.x), bf_hi(vw.x), bf_lo(vw.y), bf_hi(vw.y), bf_lo(vw.z), bf_hi(vw.z), bf_lo(vw.w), bf_hi(vw.w)};
        update(kf, vf, valid);
    }
    if (with_cur && wave == 0) {   // this step's own key/value (uniform branch per wave)
        const float* kc = M.kvcur + ((size_t)b * 2 + 0) * M.Hkv * HD + (size_t)j * HD + sub * 8;
        const float* vc = M.kvcur + ((size_t)b * 2 + 1) * M.Hkv * HD + (size_t)j * HD + sub * 8;
        float kf[8], vf[8];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            float2 a = IO::ld2(kc + e), c = IO::ld2(vc + e);
            bool mine = grp == 0;
            kf[e] = mine ? a.x : 0.f; kf[e + 1] = mine ? a.y : 0.f;
            vf[e] = c.x; vf[e + 1] = c.y;
        }
        update(kf, vf, grp == 0);
    }
    // ---- merge the NS states of this workgroup ----
    float* sm = (float*)lds;              // [NS][G]
    float* sl = sm + NS * G;              // [NS][G]
    float* so = sl + NS * G;              // [NS][G][HD]
    const int si = wave * RPW + grp;
    __syncthreads();
#pragma unroll
    for (int g = 0; g < G; g++) {
        if (sub == 0) { sm[si * G + g] = m[g]; sl[si * G + g] = l[g]; }
#pragma unroll
        for (int e = 0; e < 8; e++) so[((size_t)si * G + g) * HD + sub * 8 + e] = o[g][e];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * HD; idx += kThreads) {
        int g = idx / HD, dim = idx % HD;
        float mx = -INFINITY;
        for (int s = 0; s < NS; s++) mx = fmaxf(mx, sm[s * G + g]);
        float lt = 0.f, ot = 0.f;
        for (int s = 0; s < NS; s++) {
            float w = exp2f(sm[s * G + g] - mx);   // empty states have m = -inf -> weight 0
            lt = fmaf(sl[s * G + g], w, lt);
            ot = fmaf(so[((size_t)s * G + g) * HD + dim], w, ot);
        }
        size_t hs = ((size_t)b * M.Hq + (j * G + g)) * kMaxSplits + split;
        IO::st(M.part_o + hs * HD + dim, ot);
        if (dim == 0) { IO::st(M.part_m + hs, mx); IO::st(M.part_l + hs, lt); }
    }
}

// Final merge for (b, kv head j) over nsplit partials (paper Section 3.2: combine per-block maximum
// and denominator, rescale by own/global denominator ratio, sum): writes attn_o[b][h][:].
template <int HD, int G, class IO>
__device__ void attn_merge(const DevModel& M, int b, int j, int nsplit) {
    for (int idx = threadIdx.x; idx < G * HD; idx += kThreads) {
        int g = idx / HD, dim = idx % HD;
        size_t hs = ((size_t)b * M.Hq + (j * G + g)) * kMaxSplits;
        float mx = -INFINITY;
        for (int s = 0; s < nsplit; s++) mx = fmaxf(mx, IO::ld(M.part_m + hs + s));
        float lt = 0.f, ot = 0.f;
        for (int s = 0; s < nsplit; s++) {
            float w = exp2f(IO::ld(M.part_m + hs + s) - mx);
            lt = fmaf(IO::ld(M.part_l + hs + s), w, lt);
            ot = fmaf(IO::ld(M.part_o + (hs + s) * HD + dim), w, ot);
        }
        IO::st(M.attn_o + ((size_t)b * M.Hq + (j * G + g)) * HD + dim, ot / lt);
    }
}

// Number of KV splits for a sequence with `ncache` cached rows when `share` workgroups are
// available per (sequence, kv head).
__device__ __forceinline__ int attn_nsplit(int ncache, int share) {
    int ns = ncache / kMinSplitLen;
    ns = min(ns, min(share, kMaxSplits));
    return max(ns, 1);
}

// ---------------------------------------------------------------- epilogues
// QKV rows in packed order: q heads then k heads with RoPE partners (i, i+hd/2) adjacent, then v.
template <class IO>
struct EpiQKV {
    const DevModel& M; const DevKV& KV; const int* pos; int layer;
    __device__ void operator()(int pair, int b, float v0, float v1) const {
        const int half = M.hd / 2;
        const int nq = M.Hq * half, nk = M.Hkv * half;
        const int p = pos[b];
        if (pair < nq + nk) {
            bool isq = pair < nq;
            int pp = isq ? pair : pair - nq;
            int head = pp / half, i = pp % half;
            float2 cs = KV.rope[(size_t)p * half + i];
            float a = v0 * cs.x - v1 * cs.y;
            float c = v1 * cs.x + v0 * cs.y;
            if (isq) {
                float* qp = M.q + ((size_t)b * M.Hq + head) * M.hd;
                IO::st(qp + i, a); IO::st(qp + i + half, c);
            } else {
                bf16_t ab = f_to_bf(a), cb = f_to_bf(c);
                bf16_t* row = KV.plane(M, layer, b, head, 0) + (size_t)p * M.hd;
                row[i] = ab; row[i + half] = cb;
                float* kc = M.kvcur + ((size_t)b * 2 + 0) * M.Hkv * M.hd + (size_t)head * M.hd;
                IO::st(kc + i, bf_to_f(ab)); IO::st(kc + i + half, bf_to_f(cb));
            }
        } else {
            int pp = pair - nq - nk;
            int head = pp / half, i = (pp % half) * 2;
            bf16_t ab = f_to_bf(v0), cb = f_to_bf(v1);
            bf16_t* row = KV.plane(M, layer, b, head, 1) + (size_t)p * M.hd;
            *(u32*)(row + i) = (u32)ab | ((u32)cb << 16);
            float* vc = M.kvcur + ((size_t)b * 2 + 1) * M.Hkv * M.hd + (size_t)head * M.hd;
            IO::st2(vc + i, bf_to_f(ab), bf_to_f(cb));
        }
    }
};
// x[b][row] += W row . input   (attention output projection and GLU output projection: both add
// straight into the residual stream, paper Section 3.2)
template <class IO>
struct EpiResidual {
    float* x; int d;
    __device__ void operator()(int pair, int b, float v0, float v1) const {
        float* p = x + (size_t)b * d + 2 * pair;
        float2 o = IO::ld2(p);
        IO::st2(p, o.x + v0, o.y + v1);
    }
};
// packed rows (2i, 2i+1) = (gate_i, up_i):  h_i = silu(gate_i) * up_i
template <class IO>
struct EpiSwiGLU {
    float* h; int F;
    __device__ void operator()(int pair, int b, float g, float u) const {
        float s = g / (1.0f + expf(-g));
        IO::st(h + (size_t)b * F + pair, s * u);
    }
};
struct EpiStore {   // plain output rows (logits; per-op raw projections)
    float* y; int n;
    __device__ void operator()(int pair, int b, float v0, float v1) const {
        float* p = y + (size_t)b * n + 2 * pair;
        p[0] = v0;
        if (2 * pair + 1 < n) p[1] = v1;
    }
};

}  // namespace ff
