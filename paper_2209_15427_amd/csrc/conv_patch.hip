// Stride-1 convolution on the gfx950 matrix cores with the input patch resident in LDS.
//
// Same arithmetic as the other MFMA kernels (expanded-form accumulate of section "Quantized
// Operations", fused bias + ReLU + requantize epilogue).  What changes is where the im2col
// expansion happens.  An implicit-GEMM kernel that gathers its B operand from global memory
// fetches every input element R*S times; at these layer sizes that traffic, not the matrix
// cores, sets the pace (measured: the L2 -> LDS path saturates).  Here a workgroup's BP output
// pixels (a contiguous run in n, p, q order) read a contiguous run of the zero-padded "virtual"
// input (rows of W + 2 pad pixels, H + 2 pad rows per image): output pixel (n, p, q) tap (r, s)
// is virtual pixel (n Hv + p + r) Wv + q + s.  That run is loaded into LDS once per channel
// block (CB <= 96 bytes of every pixel; double buffered), and the B fragment of tap (r, s) is
// the same LDS rows shifted by r Wv + s.  Only the weights stream through a small LDS ring,
// one 64-byte reduction step (4 chunks of 16 bytes, walking (tap, chunk) inside the channel
// block) per barrier.
//
// LDS: 2 patch buffers + NSTW weight stages = 80 KiB for BC = 128, i.e. two workgroups per CU.
// Loads are direct-to-LDS (buffer_load ... lds); halo pixels outside the image are pointed past
// the buffer and arrive as zeros, so an int8 layer with padding needs z_x = 0.
// Synchronisation as in conv_mfma_dma.hip: counted s_waitcnt vmcnt + bare s_barrier per step;
// loads complete in order, so a patch requested at the start of a phase is resident before the
// phase ends without ever being waited for.
#include "mfma_tile.h"

namespace mpq {

namespace {

using namespace tile;

constexpr int kMaxPatchSlots = 8;

__device__ __forceinline__ unsigned udiv_magic(unsigned v, unsigned magic) {
    return (unsigned)(((unsigned long long)v * magic) >> 32);
}

template <typename T, int BC, int BP, int WGC, int WGP, int NSTW, int NSLOT, int WPE>
__global__ void __launch_bounds__(kThreads, WPE) conv_patch_kernel(ConvArgs a) {
    typedef Tile<T, BC, BP, WGC, WGP> TL;
    constexpr int WTC = TL::WTC, WTP = TL::WTP, TC = TL::TC, TP = TL::TP, ES = TL::ES;
    constexpr int LW = BC / 64;                       // weight loads per thread and step
    // NSLOT: patch loads per thread and phase
    constexpr int PATCH_BYTES = NSLOT * kThreads * kChunkBytes;
    constexpr int WSTAGE = BC * kStepBytes;
    constexpr int LDS_BYTES = 2 * PATCH_BYTES + NSTW * WSTAGE;
    static_assert(TL::kImageBytes <= LDS_BYTES, "output tile must fit the LDS");
    static_assert(TC <= 2 && TP <= 4, "fragment reads are written out for up to 2 x 4 sub-tiles");
    static_assert(NSTW == 3, "the outstanding-load counts below are derived for three weight stages");
    typedef typename TL::Acc Acc;

    __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];
    unsigned char *wring = lds + 2 * PATCH_BYTES;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wc = wave % WGC, wp = wave / WGC;
    const Plan &pl = a.plan;
    const int PQ = a.P * a.Q;

    TileCtx t;
    if (!decode_tile<BC, BP>(a, t)) return;
    const int g = t.g, m0 = t.m0, m_end = t.m_end, ch0 = t.ch0;

    const __amdgpu_buffer_rsrc_t wrs =
        __builtin_amdgcn_make_buffer_rsrc((void *)t.wbase, (short)0, (int)pl.wsum_off, 0x00020000);
    const __amdgpu_buffer_rsrc_t xrs =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.x, (short)0, (int)a.x_bytes, 0x00020000);

    // ---- geometry of the virtual (zero-padded) input ------------------------------------------
    const int Hv = a.H + 2 * a.pad_h, Wv = a.W + 2 * a.pad_w, HWv = Hv * Wv;
    const int cbc = a.cbc, CB = cbc * kChunkBytes;     // chunks / bytes per pixel per channel block
    const int CgB = pl.Cg * ES;                        // bytes per pixel per group
    const int NT = a.R * a.S;                          // taps
    const unsigned swm = cbc == 4 ? 3u : 0u;           // 64-byte rows need the XOR swizzle
    auto virt = [&](int m) {                           // virtual pixel of output pixel m at tap (0, 0)
        const int n = m / PQ, rem = m - n * PQ;
        const int p = rem / a.Q, q = rem - p * a.Q;
        return (n * Hv + p) * Wv + q;
    };
    const int v0 = virt(m0);
    const int m_last = (m0 + BP < m_end ? m0 + BP : m_end) - 1;
    const int PV = virt(m_last) + (a.R - 1) * Wv + (a.S - 1) - v0 + 1;    // rows of the patch in use

    // ---- patch fill: this thread's slots (16-byte chunk slots tid, tid + 256, ...) ---------------
    // (array bound not dependent on a template parameter: with `xoff[NSLOT]` hipcc's host pass
    // silently emitted no launch stub for this kernel)
    unsigned xoff[kMaxPatchSlots];
    static_assert(NSLOT <= kMaxPatchSlots, "more patch loads per thread than slots");
#pragma unroll
    for (int k = 0; k < NSLOT; ++k) {
        const unsigned cs = (unsigned)(k * kThreads + tid);
        const unsigned row = udiv_magic(cs, a.magic_cbc);
        const unsigned phys = cs - row * cbc;
        unsigned off = kOob;
        if ((int)row < PV) {
            const unsigned v = (unsigned)v0 + row;
            const unsigned n = udiv_magic(v, a.magic_hw);
            const unsigned rem = v - n * HWv;
            const unsigned hv = udiv_magic(rem, a.magic_wv);
            const int h = (int)hv - a.pad_h, w = (int)(rem - hv * Wv) - a.pad_w;
            if ((int)n < a.N && h >= 0 && h < a.H && w >= 0 && w < a.W)
                off = (unsigned)((((int)n * a.H + h) * a.W + w) * a.C * ES + g * CgB) + ((phys ^ ((row >> 2) & swm)) << 4);
        }
        xoff[k] = off;
    }
    auto request_patch = [&](int buf, int cb) {
        unsigned char *dst = lds + buf * PATCH_BYTES;
#pragma unroll
        for (int k = 0; k < NSLOT; ++k)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xrs, MPQ_LDS(dst + (k * kThreads + wave * 64) * kChunkBytes), 16,
                                                     xoff[k] + (unsigned)(cb * CB), 0, 0, 0);
    };

    // ---- weight stream: lane l fills slot l of a 16-row group (row l / 4, physical chunk l % 4);
    // the chunk it fetches is kc = 4 kstep + logical chunk -> (tap, chunk within the channel block)
    const int lrow = lane >> 2;
    const int lchunk = (lane & 3) ^ ((lane >> 4) & 3);
    unsigned woff[LW];
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        const int ch = ch0 + (i * 4 + wave) * 16 + lrow;
        woff[i] = ch < pl.Kg ? (unsigned)(((size_t)(g * pl.Kg + ch) * pl.Kp) * ES) : kOob;
    }
    const int KSP = a.ksp;                             // steps per phase
    int w_cb = 0, w_step = 0;                          // next weight step to request: (phase, step)
    int w_tap = lchunk / cbc, w_cc = lchunk - w_tap * cbc;
    auto request_weights = [&](int stage) {
        // past the last phase the requests continue (uniform outstanding-load count) and read zeros
        const bool ok = w_tap < NT && w_cb < a.nphase;
        const unsigned kbyte = (unsigned)(w_tap * CgB + w_cb * CB + w_cc * kChunkBytes);
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            const unsigned vo = ok ? woff[i] + kbyte : kOob;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wrs, MPQ_LDS(wring + stage * WSTAGE + (i * 4 + wave) * 1024), 16,
                                                     vo, 0, 0, 0);
        }
        if (++w_step == KSP) {
            w_step = 0;
            ++w_cb;
            w_tap = lchunk / cbc;
            w_cc = lchunk - w_tap * cbc;
        } else {
            w_cc += 4;
            while (w_cc >= cbc) {
                w_cc -= cbc;
                ++w_tap;
            }
        }
    };

    Acc acc[TC][TP];
    TL::init_acc(acc, a, t);

    // ---- fragment addressing -------------------------------------------------------------------
    const int frow = lane & 31, fk = lane >> 5;
    const unsigned sw = (unsigned)((frow >> 2) & 3);
    const unsigned fa0 = (unsigned)((wc * WTC + frow) * kStepBytes) + ((0u + fk) ^ sw) * kChunkBytes;
    const unsigned fa1 = (unsigned)((wc * WTC + frow) * kStepBytes) + ((2u + fk) ^ sw) * kChunkBytes;
    // B: patch row of this lane's pixel in each 32-pixel sub-tile (tap (0,0)); pixels past the
    // tile's end reuse the last valid one (their results are never stored)
    int vrow[TP];
#pragma unroll
    for (int j = 0; j < TP; ++j) {
        int m = m0 + wp * WTP + j * 32 + frow;
        m = m <= m_last ? m : m_last;
        vrow[j] = virt(m) - v0;
    }
    // this lane's chunk for sub-step ks is kc = 4 kstep + 2 ks + fk -> (tap, cc); delta = r Wv + s
    int b_tap[2], b_cc[2], b_s[2], b_delta[2];
    auto reset_b = [&]() {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int kc = 2 * ks + fk;
            b_tap[ks] = kc / cbc;
            b_cc[ks] = kc - b_tap[ks] * cbc;
            const int r = b_tap[ks] / a.S;
            b_s[ks] = b_tap[ks] - r * a.S;
            b_delta[ks] = r * Wv + b_s[ks];
        }
    };
    auto advance_b = [&]() {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            b_cc[ks] += 4;
            while (b_cc[ks] >= cbc) {
                b_cc[ks] -= cbc;
                ++b_tap[ks];
                ++b_delta[ks];
                if (++b_s[ks] == a.S) {
                    b_s[ks] = 0;
                    b_delta[ks] += Wv - a.S;
                }
            }
        }
    };
    reset_b();

    auto multiply = [&](int stage, int pbuf) {
        const unsigned wbase_l = (unsigned)(size_t)MPQ_LDS(wring + stage * WSTAGE);
        const unsigned pbase_l = (unsigned)(size_t)MPQ_LDS(lds + pbuf * PATCH_BYTES);
        v4i af[2][TC], bf[2][TP];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const unsigned fa = ks == 0 ? fa0 : fa1;
            af[ks][0] = lds_read<0>(wbase_l + fa);
            if constexpr (TC > 1) af[ks][1] = lds_read<2048>(wbase_l + fa);
            // a lane whose chunk lies past the last tap multiplies zero weights: keep its address valid
            const int delta = b_tap[ks] < NT ? b_delta[ks] : 0;
#pragma unroll
            for (int j = 0; j < TP; ++j) {
                const unsigned row = (unsigned)(vrow[j] + delta);
                const unsigned addr = pbase_l + row * (unsigned)CB + (((unsigned)b_cc[ks] ^ ((row >> 2) & swm)) << 4);
                bf[ks][j] = lds_read<0>(addr);
            }
        }
        lds_wait();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int i = 0; i < TC; ++i) lds_arrived(af[ks][i]);
#pragma unroll
            for (int j = 0; j < TP; ++j) lds_arrived(bf[ks][j]);
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int i = 0; i < TC; ++i)
#pragma unroll
                for (int j = 0; j < TP; ++j) acc[i][j] = Mma<T>::run(af[ks][i], bf[ks][j], acc[i][j]);
        advance_b();
    };

    // ---- pipeline ---------------------------------------------------------------------------------
    request_patch(0, 0);
#pragma unroll
    for (int p = 0; p < NSTW - 1; ++p) request_weights(p);
    int cur = 0, refill = NSTW - 1;
    for (int cb = 0; cb < a.nphase; ++cb) {
        for (int ks = 0; ks < KSP; ++ks) {
            // the weights of this step have landed when at most the later steps' loads -- and, for
            // the two steps after a patch request, that patch's loads -- are outstanding
            if (ks >= 1 && ks <= NSTW - 1 && cb + 1 < a.nphase) wait_vmcnt<LW *(NSTW - 2) + NSLOT>();
            else wait_vmcnt<LW *(NSTW - 2)>();
            bare_barrier();              // everyone's have; everyone is done with `refill` (and, at
                                         // a phase start, with the patch buffer of two phases ago)
            request_weights(refill);
            if (ks == 0 && cb + 1 < a.nphase) request_patch((cb + 1) & 1, cb + 1);
            multiply(cur, cb & 1);
            cur = cur + 1 == NSTW ? 0 : cur + 1;
            refill = refill + 1 == NSTW ? 0 : refill + 1;
        }
        reset_b();
    }
    wait_vmcnt<0>();
    bare_barrier();

    TL::finish(acc, lds, a, t);
}

template <typename T, int BC, int BP, int WGC, int WGP, int NSTW, int NSLOT, int WPE>
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
    conv_patch_kernel<T, BC, BP, WGC, WGP, NSTW, NSLOT, WPE><<<(unsigned)blocks, kThreads, 0, st>>>(a);
    return hipGetLastError();
}

constexpr int kPatchSlots = 7;                                  // 16-byte loads per thread
constexpr int kPatchBytes = kPatchSlots * 256 * kChunkBytes;    // 28 KiB per patch buffer
constexpr int kBP = 256;

unsigned magic_for(unsigned d) { return (unsigned)(((1ull << 32) + d - 1) / d); }

}  // namespace

// Fills the patch-kernel fields of `a` and says whether the layer fits: stride 1, tap-mode plan,
// zero padding value (see the header), every tile's virtual run within one patch buffer.
bool conv_patch_prepare(ConvArgs &a) {
    const Plan &pl = a.plan;
    if (pl.mode != kModeTap || a.stride_h != 1 || a.stride_w != 1) return false;
    if (!conv_mfma_dma_eligible(a)) return false;
    const int CgB = pl.Cg * pl.esize;
    int CB;
    if (CgB <= 96) CB = CgB;
    else if (CgB % 64 == 0) CB = 64;
    else return false;
    if (CB % kChunkBytes != 0 || CB < 32) return false;
    a.cbc = CB / kChunkBytes;
    a.nphase = CgB / CB;
    const int NT = a.R * a.S;                          // taps
    a.ksp = (NT * a.cbc + 3) / 4;
    if (a.ksp < 4) return false;                 // too few steps per phase to hide the patch load
    const int Hv = a.H + 2 * a.pad_h, Wv = a.W + 2 * a.pad_w, PQ = a.P * a.Q;
    // largest virtual run any tile of kBP consecutive output pixels can need
    long long worst = 0;
    auto virt = [&](long long m) {
        const long long n = m / PQ, rem = m % PQ;
        return (n * Hv + rem / a.Q) * Wv + rem % a.Q;
    };
    for (int s0 = 0; s0 < PQ; ++s0) {
        const long long span = virt((long long)s0 + kBP - 1) + (long long)(a.R - 1) * Wv + (a.S - 1) - virt(s0) + 1;
        if (span > worst) worst = span;
    }
    if (worst * CB > kPatchBytes) return false;
    const unsigned long long vmax = (unsigned long long)(a.N + 1) * Hv * Wv + kPatchBytes;
    if (vmax * (unsigned long long)(Hv * Wv) >= (1ull << 32)) return false;    // exactness of the magic division
    a.magic_wv = magic_for((unsigned)Wv);
    a.magic_hw = magic_for((unsigned)(Hv * Wv));
    a.magic_cbc = magic_for((unsigned)a.cbc);
    return true;
}

hipError_t launch_conv_patch(const ConvArgs &a, hipStream_t st) {
    const int Kg = a.plan.Kg;
    const bool wide = Kg % 128 == 0 || (Kg > 128 && Kg % 64 != 0);
    if (a.in_dtype == MPQ_INT8) {
        if (wide) return launch_one<int8_t, 128, kBP, 2, 2, 3, kPatchSlots, 2>(a, st);
        return launch_one<int8_t, 64, kBP, 1, 4, 3, kPatchSlots, 2>(a, st);
    }
    if (wide) return launch_one<_Float16, 128, kBP, 2, 2, 3, kPatchSlots, 2>(a, st);
    return launch_one<_Float16, 64, kBP, 1, 4, 3, kPatchSlots, 2>(a, st);
}

}  // namespace mpq
