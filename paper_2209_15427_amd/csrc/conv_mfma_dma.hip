// Implicit-GEMM convolution / fully-connected kernel on the gfx950 matrix cores, fast variant:
// operand tiles travel HBM/L2 -> LDS directly (buffer_load ... lds), several reduction steps in
// flight, so that the MFMA pipe only ever waits on LDS.
//
// Same arithmetic as conv_mfma.hip (expanded-form accumulate of section "Quantized Operations",
// then the fused bias + ReLU + requantize epilogue); this file differs in data movement only:
//   - NST LDS stages, each one 64-byte reduction step of the weight tile (BC rows) and of the
//     gathered input tile (BP rows).  Stage k + NST - 1 is requested while stage k is multiplied.
//   - a wavefront-wide direct-to-LDS load writes 64 consecutive 16-byte slots (16 tile rows);
//     which 16-byte global chunk a lane fetches is chosen so that the slot it lands in is the
//     XOR-swizzled position the MFMA fragment reads expect (chunk c of row r at slot
//     c ^ ((r >> 2) & 3)): no bank conflicts, no register staging, no ds_write.
//   - buffer addressing: a lane whose tap falls outside the image (or whose row is past the
//     tile's end) is pointed beyond the buffer and the hardware writes zeros.  That is the
//     right padding value only when the input zero-point is 0 (or the layer has no padding);
//     other cases run on the register-staged kernel.
//   - synchronisation is explicit: a wavefront counts its own outstanding loads (s_waitcnt
//     vmcnt), then a bare s_barrier makes every wavefront's loads of that step visible.  The
//     fragment reads are issued as inline ds_read_b128 so that the compiler, which cannot tell
//     the stages apart, does not drain all outstanding loads in front of them.
#include <type_traits>

#include "common.h"
#include "epilogue.h"

namespace mpq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

#define MPQ_LDS(p) ((__attribute__((address_space(3))) void *)(p))

template <typename T> struct Mma;
template <> struct Mma<int8_t> {
    typedef v16i Acc;
    static __device__ __forceinline__ Acc run(v4i a, v4i b, Acc c) {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    }
};
template <> struct Mma<_Float16> {
    typedef v16f Acc;
    static __device__ __forceinline__ Acc run(v4i a, v4i b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c,
                                                      0, 0, 0);
    }
};

constexpr int kThreads = 256;
constexpr unsigned kOob = 0x7ffffff0u;   // beyond any buffer this kernel accepts (< 2 GiB)

// LDS fragment read the compiler does not model as a memory access (see the header).  The value
// arrives asynchronously: lds_arrived() must come between the read and the first use.
template <int OFF> __device__ __forceinline__ v4i lds_read(unsigned addr) {
    v4i r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}
__device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
// ties a fragment's uses to the wait that precedes this statement
__device__ __forceinline__ void lds_arrived(v4i &f) { asm volatile("" : "+v"(f)); }

// wait until at most n of this wavefront's vector-memory operations are outstanding
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xf) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

template <typename T, int BC, int BP, int WGC, int WGP, int NST, int WPE>
__global__ void __launch_bounds__(kThreads, WPE) conv_mfma_dma_kernel(ConvArgs a) {
    static_assert(WGC * WGP == 4, "four wavefronts per workgroup");
    static_assert(BC % 64 == 0 && BP % 64 == 0, "tile rows come in groups of 64");
    static_assert(NST == 3 || NST == 4, "three or four stages");
    constexpr int WTC = BC / WGC, WTP = BP / WGP;
    constexpr int TC = WTC / 32, TP = WTP / 32;
    constexpr int LW = BC / 64, LX = BP / 64;        // loads per thread and step: weights, input
    constexpr int LPT = LW + LX;
    constexpr int STAGE = (BC + BP) * kStepBytes;
    constexpr int ES = (int)sizeof(T);
    typedef typename Mma<T>::Acc Acc;

    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wc = wave % WGC, wp = wave / WGC;
    const Plan &pl = a.plan;
    const int PQ = a.P * a.Q;

    // ---- which tile: consecutive workgroups land on different XCDs, so hand each XCD a
    // contiguous range of tiles (neighbouring tiles share input rows and weights in its L2) ----
    const int ctiles = (pl.Kg + BC - 1) / BC;
    const int nblk = gridDim.x;
    int bid = blockIdx.x;
    {
        const int per = nblk / 8, rem = nblk % 8, x = bid % 8, j = bid / 8;
        bid = x * per + (x < rem ? x : rem) + j;
    }
    const int ct = bid % ctiles;
    bid /= ctiles;
    int pt = bid % a.ptiles;
    const int g = bid / a.ptiles;

    int m_begin = 0, m_end = a.N * PQ;
    const char *wbase = (const char *)a.w;
    const char *bias = (const char *)a.bias;
    Epi epi = a.epi;
    if (a.seg.offsets) {
        int e = 0, tile_base = 0;
        bool found = false;
        for (; e < a.seg.num_experts; ++e) {
            int lo = a.seg.offsets[e], hi = a.seg.offsets[e + 1];
            int tiles = ((hi - lo) * PQ + BP - 1) / BP;
            if (pt < tile_base + tiles) {
                m_begin = lo * PQ;
                m_end = hi * PQ;
                pt -= tile_base;
                found = true;
                break;
            }
            tile_base += tiles;
        }
        if (!found) return;
        wbase += (size_t)e * a.seg.w_stride;
        if (bias) bias += (size_t)e * a.seg.bias_stride * 4;
        epi = a.seg.epi[e];
    }
    const int m0 = m_begin + pt * BP;
    const int ch0 = ct * BC;
    if (m0 >= m_end) return;

    const __amdgpu_buffer_rsrc_t wrs =
        __builtin_amdgcn_make_buffer_rsrc((void *)wbase, (short)0, (int)pl.wsum_off, 0x00020000);
    const __amdgpu_buffer_rsrc_t xrs =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.x, (short)0, (int)a.x_bytes, 0x00020000);

    // ---- per-thread load coordinates: lane l of a wavefront-wide load fills slot l, i.e. row
    // l / 4 of a 16-row group, physical chunk l % 4 ------------------------------------------------
    const int lrow = lane >> 2;
    const int lchunk = (lane & 3) ^ ((lane >> 4) & 3);      // logical chunk that belongs in this slot
    const int S_eff = a.s_eff, cpt = a.cpt;

    unsigned woff[LW];
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        const int ch = ch0 + (i * 4 + wave) * 16 + lrow;
        woff[i] = ch < pl.Kg ? (unsigned)(((size_t)(g * pl.Kg + ch) * pl.Kp) * ES + lchunk * kChunkBytes) : kOob;
    }
    int xoff[LX];
    unsigned hmask[LX], wmask[LX];
#pragma unroll
    for (int i = 0; i < LX; ++i) {
        const int m = m0 + (i * 4 + wave) * 16 + lrow;
        const bool mv = m < m_end;
        const int mm = mv ? m : m_begin;
        const int n = mm / PQ, rem = mm % PQ;
        const int p = rem / a.Q, q = rem % a.Q;
        const int h0 = p * a.stride_h - a.pad_h, w0 = q * a.stride_w - a.pad_w;
        xoff[i] = (((n * a.H + h0) * a.W + w0) * a.C + g * pl.Cg) * ES;
        unsigned hm = 0, wm = 0;
        for (int r = 0; r < a.R; ++r) hm |= (unsigned)(h0 + r >= 0 && h0 + r < a.H) << r;
        for (int s = 0; s < S_eff; ++s) wm |= (unsigned)(w0 + s >= 0 && w0 + s + a.tap_px <= a.W) << s;
        hmask[i] = mv ? hm : 0u;
        wmask[i] = wm;
    }

    int kc = lchunk, cc = kc % cpt, tap = kc / cpt;
    int tr = tap / S_eff, ts = tap % S_eff;
    const int tap_stride_r = a.W * a.C * ES, tap_stride_s = a.C * ES;
    // phased order (taps wider than one step): the reduction axis is walked 64-byte channel block
    // by channel block, all taps inside a block, so that consecutive steps re-read the lines the
    // neighbouring pixels just fetched (they are still in the vector L1) instead of coming back
    // to them R*S*C/64 steps later.  The packed weights are addressed in the same order.
    const bool phased = a.phased != 0;
    int ph = 0;    // uniform counters of the phased walk: channel block; (tr, ts) is the tap
    if (phased) {
        tr = 0;
        ts = 0;
    }

    // request reduction step `kt` into stage buffer `dst`
    auto request = [&](unsigned char *dst, int kt) {
        // steps past the end are requested too (it keeps the outstanding-load count uniform); they
        // are never multiplied, and the range-checked buffer makes any offset harmless
        unsigned kbyte = (unsigned)kt * kStepBytes;
        int ccx = cc;
        bool kval = kc < a.nchunks;
        if (phased) {
            ccx = ph * 4 + lchunk;
            kbyte = (unsigned)((tr * S_eff + ts) * cpt + ph * 4) * kChunkBytes;
            kval = ph * 4 < cpt;
        }
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            const unsigned vo = woff[i] + kbyte;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wrs, MPQ_LDS(dst + (i * 4 + wave) * 1024), 16, vo, 0, 0, 0);
        }
        const int tapoff = tr * tap_stride_r + ts * tap_stride_s + ccx * kChunkBytes;
#pragma unroll
        for (int i = 0; i < LX; ++i) {
            const bool ok = kval && (((hmask[i] >> tr) & (wmask[i] >> ts) & 1u) != 0u);
            const unsigned vo = ok ? (unsigned)(xoff[i] + tapoff) : kOob;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xrs, MPQ_LDS(dst + BC * kStepBytes + (i * 4 + wave) * 1024), 16,
                                                     vo, 0, 0, 0);
        }
        if (phased) {
            if (++ts == S_eff) {
                ts = 0;
                if (++tr == a.R) {
                    tr = 0;
                    ++ph;
                }
            }
        } else {
            kc += 4;
            cc += 4;
            while (cc >= cpt) {
                cc -= cpt;
                if (++ts == S_eff) {
                    ts = 0;
                    ++tr;
                }
            }
        }
    };

    // Accumulators start at the epilogue's per-channel constant: the bias, minus z_x * sum(w) for
    // int8 (register v of lane l in a 32x32 tile holds channel 8*(v/4) + 4*(l/32) + v%4).
    const int *wsum = reinterpret_cast<const int *>(wbase + pl.wsum_off);
    Acc acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; ++i) {
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            const int ch = ch0 + wc * WTC + i * 32 + vq * 8 + (lane >> 5) * 4;
            const int kabs = g * pl.Kg + (ch < pl.Kg ? ch : 0);
            if constexpr (ES == 1) {
                v4i b4 = {0, 0, 0, 0};
                if (bias) b4 = *reinterpret_cast<const v4i *>(bias + (size_t)kabs * 4);
                if (epi.zx != 0) b4 -= *reinterpret_cast<const v4i *>(wsum + kabs) * epi.zx;
#pragma unroll
                for (int j = 0; j < TP; ++j)
#pragma unroll
                    for (int u = 0; u < 4; ++u) acc[i][j][vq * 4 + u] = b4[u];
            } else {
                float4 bb = make_float4(0.f, 0.f, 0.f, 0.f);
                if (bias) bb = *reinterpret_cast<const float4 *>(bias + (size_t)kabs * 4);
#pragma unroll
                for (int j = 0; j < TP; ++j) {
                    acc[i][j][vq * 4 + 0] = bb.x;
                    acc[i][j][vq * 4 + 1] = bb.y;
                    acc[i][j][vq * 4 + 2] = bb.z;
                    acc[i][j][vq * 4 + 3] = bb.w;
                }
            }
        }
    }

    // fragment addresses: lane l reads row l % 32 of a 32-row sub-tile, chunk (2 ks + l / 32) at its
    // swizzled slot; sub-tiles are 32 rows = 2048 bytes apart (an immediate offset)
    const int frow = lane & 31, fk = lane >> 5;
    const unsigned sw = (unsigned)((frow >> 2) & 3);
    const unsigned fa0 = (unsigned)((wc * WTC + frow) * kStepBytes) + ((0u + fk) ^ sw) * kChunkBytes;
    const unsigned fa1 = (unsigned)((wc * WTC + frow) * kStepBytes) + ((2u + fk) ^ sw) * kChunkBytes;
    const unsigned fb0 = (unsigned)((BC + wp * WTP + frow) * kStepBytes) + ((0u + fk) ^ sw) * kChunkBytes;
    const unsigned fb1 = (unsigned)((BC + wp * WTP + frow) * kStepBytes) + ((2u + fk) ^ sw) * kChunkBytes;
    auto read_frags = [&](unsigned base, unsigned fa, unsigned fb, v4i(&af)[TC], v4i(&bf)[TP]) {
        static_assert(TC <= 2 && TP <= 4, "fragment reads are written out for up to 2 x 4 sub-tiles");
        af[0] = lds_read<0>(base + fa);
        if constexpr (TC > 1) af[1] = lds_read<2048>(base + fa);
        bf[0] = lds_read<0>(base + fb);
        if constexpr (TP > 1) bf[1] = lds_read<2048>(base + fb);
        if constexpr (TP > 2) bf[2] = lds_read<4096>(base + fb);
        if constexpr (TP > 3) bf[3] = lds_read<6144>(base + fb);
    };
    auto arrived = [&](v4i(&af)[TC], v4i(&bf)[TP]) {
        lds_wait();
#pragma unroll
        for (int i = 0; i < TC; ++i) lds_arrived(af[i]);
#pragma unroll
        for (int j = 0; j < TP; ++j) lds_arrived(bf[j]);
    };
    auto multiply = [&](const unsigned char *src) {
        const unsigned base = (unsigned)(size_t)MPQ_LDS(src);
        v4i a0[TC], b0[TP], a1[TC], b1[TP];
        read_frags(base, fa0, fb0, a0, b0);
        read_frags(base, fa1, fb1, a1, b1);      // second half in flight while the first multiplies
        arrived(a0, b0);                         // (reads return in order; one wait covers both)
        arrived(a1, b1);
#pragma unroll
        for (int i = 0; i < TC; ++i)
#pragma unroll
            for (int j = 0; j < TP; ++j) acc[i][j] = Mma<T>::run(a0[i], b0[j], acc[i][j]);
#pragma unroll
        for (int i = 0; i < TC; ++i)
#pragma unroll
            for (int j = 0; j < TP; ++j) acc[i][j] = Mma<T>::run(a1[i], b1[j], acc[i][j]);
    };

    // one pipeline step: stage `cur` holds step kt; `refill` (the stage multiplied one step ago)
    // receives step kt + NST - 1
    auto step = [&](unsigned char *cur, unsigned char *refill, int kt) {
        wait_vmcnt<LPT *(NST - 2)>();    // this wavefront's loads of step kt have landed
        asm volatile("s_barrier" ::: "memory");   // everyone's have, and everyone is done with `refill`
        request(refill, kt + NST - 1);
        multiply(cur);
    };

    const int ksteps = a.ksteps;
#pragma unroll
    for (int p = 0; p < NST - 1; ++p) request(lds + p * STAGE, p);
    int cur = 0, refill = NST - 1;
    for (int kt = 0; kt < ksteps; ++kt) {
        step(lds + cur * STAGE, lds + refill * STAGE, kt);
        cur = cur + 1 == NST ? 0 : cur + 1;
        refill = refill + 1 == NST ? 0 : refill + 1;
    }
    wait_vmcnt<0>();    // drain the trailing all-zero requests before the LDS is released

    asm volatile("s_barrier" ::: "memory");   // every wavefront is done with the stages

    // ---- epilogue ---------------------------------------------------------------------------
    // Register v of lane l in a 32x32 tile holds channel 8*(v/4) + 4*(l/32) + v%4 of pixel l%32:
    // four consecutive channels of one pixel.  Storage-type outputs are first laid out in LDS as
    // the tile's [pixel][channel] image (16-byte chunks XOR-swizzled by the pixel index), then
    // written with 16-byte stores in which consecutive lanes cover consecutive channels of a
    // pixel, so that every store instruction fills whole cache lines.  Raw accumulator outputs
    // (gating logits) are stored directly.
    const bool raw = epi.kind == kEpiRawI32 || epi.kind == kEpiRawF32;
    constexpr int ROWB = BC * ES, CH16 = ROWB / 16;
    static_assert(BP * ROWB <= NST * STAGE, "output tile must fit the stage buffers");
    static_assert((CH16 & (CH16 - 1)) == 0, "chunks per row must be a power of two");
    // FAST: int8 with ReLU and a right shift of at least one bit.  Negative accumulators clamp to
    // the zero-point whatever their rounding, and for t >= 0 truncate-then-floor is one floor:
    // floor(t * mult / 2^(31 + shift)) = mulhi(t, mult) >> (shift - 1).
    auto run_epilogue = [&](auto fast_tag) {
        constexpr bool FAST = decltype(fast_tag)::value;
        const FastRequant fr = make_fast_requant(epi);
#pragma unroll
        for (int i = 0; i < TC; ++i) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int chl = wc * WTC + i * 32 + vq * 8 + fk * 4;     // channel within the tile
                const int ch = ch0 + chl;
                const bool chv = ch < pl.Kg;
                const int kabs = g * pl.Kg + (chv ? ch : 0);
                const unsigned cb = (unsigned)(chl * ES);
#pragma unroll
                for (int j = 0; j < TP; ++j) {
                    const int row = wp * WTP + j * 32 + frow;
                    const int m = m0 + row;
                    const unsigned la = (unsigned)(row * ROWB) + (((cb >> 4) ^ (unsigned)(row & (CH16 - 1))) << 4) + (cb & 15u);
                    if constexpr (ES == 1) {
                        int t[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) t[u] = acc[i][j][vq * 4 + u];
                        if (raw) {
                            if (chv && m < m_end)
                                *reinterpret_cast<v4i *>((int *)a.y + (size_t)m * a.K + kabs) = v4i{t[0], t[1], t[2], t[3]};
                        } else {
                            unsigned packed = 0;
                            if constexpr (FAST) {
                                packed = requant4_fast(t[0], t[1], t[2], t[3], fr);
                            } else {
#pragma unroll
                                for (int u = 0; u < 4; ++u) packed |= ((unsigned)requant32(t[u], epi) & 0xffu) << (8 * u);
                            }
                            *reinterpret_cast<unsigned *>(lds + la) = packed;
                        }
                    } else {
                        float t[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            t[u] = acc[i][j][vq * 4 + u];
                            if (epi.relu) t[u] = t[u] > 0.f ? t[u] : 0.f;
                        }
                        if (raw) {
                            if (chv && m < m_end)
                                *reinterpret_cast<float4 *>((float *)a.y + (size_t)m * a.K + kabs) =
                                    make_float4(t[0], t[1], t[2], t[3]);
                        } else {
                            typedef _Float16 v4h __attribute__((ext_vector_type(4)));
                            v4h hv = {(_Float16)t[0], (_Float16)t[1], (_Float16)t[2], (_Float16)t[3]};
                            *reinterpret_cast<v4h *>(lds + la) = hv;
                        }
                    }
                }
            }
        }
    };
    const bool fast = ES == 1 && fast_requant_ok(epi);
    if (fast) run_epilogue(std::true_type{});
    else run_epilogue(std::false_type{});
    if (raw) return;
    __syncthreads();
    constexpr int CHUNK_ELEMS = 16 / ES;
    char *yb = (char *)a.y;
#pragma unroll 4
    for (int idx = tid; idx < BP * CH16; idx += kThreads) {
        const int row = idx / CH16, c16 = idx % CH16;
        const int m = m0 + row;
        const int ch = ch0 + c16 * CHUNK_ELEMS;
        if (m >= m_end || ch >= pl.Kg) continue;
        const v4i v = *reinterpret_cast<const v4i *>(lds + row * ROWB + ((c16 ^ (row & (CH16 - 1))) << 4));
        char *dst = yb + ((size_t)m * a.K + (size_t)(g * pl.Kg + ch)) * ES;
        if (a.y_vec16 && ch + CHUNK_ELEMS <= pl.Kg) {
            *reinterpret_cast<v4i *>(dst) = v;
        } else {
            // ragged or unaligned tail: 4 bytes at a time (channel counts are multiples of 4)
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (ch + (u * 4 + 3) / ES < pl.Kg) *reinterpret_cast<int *>(dst + u * 4) = v[u];
        }
    }
}

template <typename T, int BC, int BP, int WGC, int WGP, int NST, int WPE>
hipError_t launch_one(ConvArgs a, hipStream_t st) {
    const int PQ = a.P * a.Q;
    const int ctiles = (a.plan.Kg + BC - 1) / BC;
    long long rows = (long long)a.N * PQ;
    int ptiles = (int)((rows + BP - 1) / BP);
    if (a.seg.offsets) ptiles += a.seg.num_experts;
    a.ptiles = ptiles;
    long long blocks = (long long)ptiles * ctiles * a.groups;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7fffffffll) return hipErrorInvalidValue;
    conv_mfma_dma_kernel<T, BC, BP, WGC, WGP, NST, WPE><<<(unsigned)blocks, kThreads, 0, st>>>(a);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_typed(const ConvArgs &a, hipStream_t st) {
    const int Kg = a.plan.Kg;
    if (Kg % 128 == 0 || (Kg > 128 && Kg % 64 != 0)) return launch_one<T, 128, 256, 2, 2, 3, 2>(a, st);
    return launch_one<T, 64, 256, 1, 4, 3, 2>(a, st);
}

}  // namespace

// The direct-to-LDS kernel zero-fills out-of-image taps and addresses buffers with 32-bit offsets.
bool conv_mfma_dma_eligible(const ConvArgs &a) {
    if (a.x_bytes >= 0x7ffffff0ull || a.plan.wsum_off >= 0x7ffffff0ull) return false;
    if (a.R > 32 || a.s_eff > 32) return false;
    const bool padded = a.pad_h != 0 || a.pad_w != 0;
    if (a.in_dtype == MPQ_INT8 && padded) {
        if (a.epi.zx != 0) return false;
        if (a.seg.offsets)
            for (int e = 0; e < a.seg.num_experts; ++e)
                if (a.seg.epi[e].zx != 0) return false;
    }
    return true;
}

hipError_t launch_conv_mfma_dma(const ConvArgs &a, hipStream_t st) {
    if (a.in_dtype == MPQ_INT8) return launch_typed<int8_t>(a, st);
    return launch_typed<_Float16>(a, st);
}

}  // namespace mpq
