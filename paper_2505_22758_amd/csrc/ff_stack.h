// Stacked square linear layers on one input vector: the ablation of the paper's preliminary study
// (Section 3, latency table of stacked linear layers): "Baseline" = one launch per layer, "Fused" =
// all layers in one persistent kernel with a tagged hand-over between layers, "+ Overlap" = the same
// with a layer's first weight tiles requested before its input is waited for.  Built from the
// building blocks of the decode kernel (static row partition, register tile ring, tagged compact
// exchange vectors, one-pass staging), so what it measures is what those blocks cost and gain.
#pragma once
#include "ff_fused.h"

namespace ff {

struct StackArgs {
    const uint8_t* w;     // [n_layers][d][d] bf16, row-major [out][in]
    int d, n_layers;
    cword_t* buf[2];      // ping-pong compact vectors [d]; layer l reads buf[l & 1] (write counter l), writes buf[(l + 1) & 1] (counter l + 1)
    int* status;
};

// input x (fp32) -> compact words with write counter 0 in buf[0]; both buffers' counter bits are
// first set to "one before" what their first reader expects, so a stale word can never pass
__global__ void k_stack_pack(StackArgs A, const float* x) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < A.d; i += gridDim.x * blockDim.x) {
        as_global(A.buf[0])[i] = cpack(x[i], 0u);
        as_global(A.buf[1])[i] = 2u;   // counter 2 (value 0): layer 0 writes counter 1 there
    }
}
__global__ void k_stack_unpack(StackArgs A, float* y) {
    const cword_t* src = A.buf[A.n_layers & 1];
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < A.d; i += gridDim.x * blockDim.x) y[i] = cvalue(as_global(src)[i]);
}

template <bool OVERLAP>
__global__ void __launch_bounds__(kFusedThreads) stack_linear_kernel(StackArgs A, int ncta) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int EPU = WTraits<W_BF16>::EPU;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float4* xs = (float4*)lds;
    float* myacc = (float*)(lds + kLdsActBytes) + (size_t)wave * kAccFloatsPerWave;
    float* red = (float*)(lds + kLdsActBytes + kLdsAuxBytes) + 2 * kMaxBatchFused * 64;
    WgVote vote{(u32*)(red + 16), 0u};
    const int gwave = blockIdx.x * kFusedWaves + wave;
    const UDiv n_gwaves = UDiv::of((u32)ncta * kFusedWaves), n_ctas = UDiv::of((u32)ncta);
    for (int l = 0; l < A.n_layers; l++) {
        PMat W;
        W.w = A.w + (size_t)l * A.d * A.d * 2; W.s = nullptr; W.z = nullptr; W.n = A.d; W.k = A.d; W.wd = W_BF16;
        const Stream<W_BF16, 1> S = Stream<W_BF16, 1>::make(W, 0, gwave, n_gwaves);
        Stage<W_BF16> ring[kDepthOf<W_BF16>];
        if constexpr (OVERLAP) prefetch_stream<false>(S, ring, lane);
        TSrc src;
        src.base = A.buf[l & 1]; src.stride = (size_t)A.d; src.tag = (u32)l;
        src.ncta = n_ctas;
        if (l > 0) __syncthreads();   // every wave has finished reading the previous staged input
        const bool ok = stage_tagged<EPU, false, kFusedThreads, false, 1>(src, 1, S.K, 0, S.nunits, S.nup, xs, red, threadIdx.x, vote);
        if (!ok) {
            if (threadIdx.x == 0) atomicCAS(A.status, 0, -55 - 10 * l);
            return;
        }
        if constexpr (!OVERLAP) prefetch_stream<false>(S, ring, lane);
        EpiDeltaTagged epi{A.buf[(l + 1) & 1], A.d, (u32)(l + 1)};
        gemv_run<W_BF16, 1>(S, ring, xs, myacc, 1, lane, epi);
    }
}

}  // namespace ff
