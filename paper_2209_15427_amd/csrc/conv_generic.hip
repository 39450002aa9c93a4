// Direct convolution for every geometry, dtype and zero-point combination the MFMA kernels do
// not cover (small or odd channel counts; int16 layers that are small, carry a weight zero-point
// or come without the optional workspace; weight zero-points in expert-grouped launches).  One thread per
// (output pixel, 4 output channels); differences-first accumulation
//   acc = sum (x - z_x)(w - z_w)      (first quantized-multiply equation, section
//                                      "Quantized Operations")
// in int64 for integers (exact for int16 as well) and in fp32, index order, for fp16.
#include "common.h"
#include "epilogue.h"

namespace mpq {

namespace {

constexpr int kThreads = 256;
constexpr int kCh = 4;   // output channels per thread

template <typename T, typename AccT>
__global__ void __launch_bounds__(kThreads) conv_generic_kernel(ConvArgs a) {
    const Plan &pl = a.plan;
    const int PQ = a.P * a.Q;
    const size_t M = (size_t)a.N * PQ;
    const int kq = (a.K + kCh - 1) / kCh;
    const size_t total = M * kq;
    size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t nthreads = (size_t)gridDim.x * blockDim.x;
    const T *x = (const T *)a.x;
    for (size_t i = tid; i < total; i += nthreads) {
        int k0 = (int)(i % kq) * kCh;
        size_t m = i / kq;
        int q = (int)(m % a.Q);
        size_t np = m / a.Q;
        int p = (int)(np % a.P);
        int n = (int)(np / a.P);

        // grouped (MoE) launch: sample n belongs to the expert whose offset range holds it
        const char *wbase = (const char *)a.w;
        const char *bias = (const char *)a.bias;
        Epi epi = a.epi;
        if (a.seg.offsets) {
            int e = 0;
            while (e + 1 < a.seg.num_experts && n >= a.seg.offsets[e + 1]) ++e;
            if (n >= a.seg.offsets[a.seg.num_experts]) continue;
            wbase += (size_t)e * a.seg.w_stride;
            if (bias) bias += (size_t)e * a.seg.bias_stride * 4;
            epi = a.seg.epi[e];
        }
        const T *w = (const T *)wbase;

        AccT acc[kCh];
#pragma unroll
        for (int j = 0; j < kCh; ++j) acc[j] = 0;
        // all kCh channels of a thread lie in one group when Kg % kCh == 0; otherwise handle each
        // channel's group separately (rare, tiny layers)
        const int h0 = p * a.stride_h - a.pad_h, w0 = q * a.stride_w - a.pad_w;
        for (int j = 0; j < kCh; ++j) {
            int k = k0 + j;
            if (k >= a.K) break;
            int g = k / pl.Kg;
            const T *wk = w + (size_t)k * pl.Kp;
            AccT s = 0;
            for (int r = 0; r < a.R; ++r) {
                int h = h0 + r;
                if (h < 0 || h >= a.H) continue;
                for (int sx = 0; sx < a.S; ++sx) {
                    int ww = w0 + sx;
                    if (ww < 0 || ww >= a.W) continue;
                    const T *xp = x + (((size_t)n * a.H + h) * a.W + ww) * a.C + (size_t)g * pl.Cg;
                    const T *wp = wk + r * pl.row_pitch + sx * pl.s_pitch;
                    if constexpr (sizeof(AccT) == 8) {
                        for (int c = 0; c < pl.Cg; ++c)
                            s += (AccT)((int)xp[c] - epi.zx) * (AccT)((int)wp[c] - epi.zw);
                    } else {
                        for (int c = 0; c < pl.Cg; ++c) s += (float)xp[c] * (float)wp[c];
                    }
                }
            }
            acc[j] = s;
        }
#pragma unroll
        for (int j = 0; j < kCh; ++j) {
            int k = k0 + j;
            if (k >= a.K) break;
            size_t o = m * a.K + k;
            if constexpr (sizeof(AccT) == 8) {
                long long t = acc[j] + (bias ? (long long)((const int *)bias)[k] : 0ll);
                if (epi.kind == kEpiRawI32) {
                    ((int *)a.y)[o] = (int)t;
                } else {
                    int v = requant64(t, epi);
                    if (a.out_dtype == MPQ_INT8) ((int8_t *)a.y)[o] = (int8_t)v;
                    else ((int16_t *)a.y)[o] = (int16_t)v;
                }
            } else {
                float t = acc[j] + (bias ? ((const float *)bias)[k] : 0.f);
                if (epi.relu) t = t > 0.f ? t : 0.f;
                if (epi.kind == kEpiRawF32) ((float *)a.y)[o] = t;
                else ((_Float16 *)a.y)[o] = (_Float16)t;
            }
        }
    }
}

}  // namespace

hipError_t launch_conv_generic(const ConvArgs &a, hipStream_t st) {
    size_t M = (size_t)a.N * a.P * a.Q;
    size_t total = M * ((a.K + kCh - 1) / kCh);
    if (total == 0) return hipSuccess;
    size_t blocks = (total + kThreads - 1) / kThreads;
    if (blocks > 256 * 64) blocks = 256 * 64;
    if (a.in_dtype == MPQ_INT8)
        conv_generic_kernel<int8_t, long long><<<(int)blocks, kThreads, 0, st>>>(a);
    else if (a.in_dtype == MPQ_INT16)
        conv_generic_kernel<int16_t, long long><<<(int)blocks, kThreads, 0, st>>>(a);
    else
        conv_generic_kernel<_Float16, float><<<(int)blocks, kThreads, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace mpq
