// conv2 / conv3 forward and input-gradient passes for large bf16 batches with the layer's input held in LDS.
//
// The tile kernel of gemm.hpp gathers every (position, tap) slice of the im2col matrix from L2 -- an activation is
// fetched once per tap that touches it, and with 32 or 64 output channels there is little to do per fetched byte, so
// those kernels are bound by L2 traffic.  Here a workgroup keeps the activations (forward) or output gradients
// (input gradient) of G samples and the whole weight matrix in LDS; a wavefront takes 32 output positions, builds the
// position operand of each tap straight from the resident rows (16 bytes per lane, no im2col in memory), reads the
// weight operand from the resident matrix and keeps a 32 x 32 (x2 for 64 columns) accumulator.
//
// Both passes are  out[row][col] = sum_{tap, c} in[row_of(row, tap)][c] * w[col][tap][c]:
//   forward         rows = output positions, row_of = (oy*s + u, ox*s + v), always inside the input
//   input gradient  rows = input positions of one parity class (y % s, x % s); only the taps u = y%s + s*a,
//                   v = x%s + s*b reach them, row_of = ((y-u)/s, (x-v)/s) when inside the output, else a zero row
// The geometry is a template parameter (every index division is by a constant).  The forward pass adds its products
// in the same k order and the same segments as the other forward kernels (segment sums formed in a fresh accumulator
// and added in order), so its output bits are theirs.
#pragma once
#include "gemm.hpp"

namespace hts {

struct ImgConvArgs {
    const bf16_t *in;      // resident operand [B][PIN][CIN]
    const bf16_t *w;       // weight copy [NCOL][KTOT], k = (tap, c)
    const bf16_t *mask;    // input gradient: post-ReLU output of the layer below, laid out like out
    const float *bias;     // forward
    bf16_t *out;
    bf16_t *out2;          // forward with FLAT: optional channel-innermost copy of the output
    int B;
};

// forward pass of a layer with CIN input channels, 64 output channels, on an HIN x WIN input
template <int CIN_, int KSZ_, int STRIDE_, int HIN_, int WIN_, int G_, int SEG_, bool FLAT_> struct ImgFwd {
    static constexpr bool FWD = true, FLAT = FLAT_;
    static constexpr int CIN = CIN_, NCOL = 64, G = G_;
    static constexpr int HO = (HIN_ - KSZ_) / STRIDE_ + 1, WO = (WIN_ - KSZ_) / STRIDE_ + 1;
    static constexpr int PIN = HIN_ * WIN_, POUT_ALL = HO * WO;
    static constexpr int TAPS = KSZ_ * KSZ_, NCLS = 1, KTOT = TAPS * CIN_;
    static constexpr int SEGSTEPS = SEG_ / 16;                      // matrix instructions per segment
    static constexpr int cls_h(int) { return HO; }
    static constexpr int cls_w(int) { return WO; }
    static constexpr int src_tap(int, int tap) { return tap; }
    static HTS_HD int in_row(int, int yy, int xx, int tap)
    {
        return (yy * STRIDE_ + tap / KSZ_) * WIN_ + xx * STRIDE_ + tap % KSZ_;
    }
    static HTS_HD int out_pos(int, int yy, int xx) { return yy * WO + xx; }
};

// input gradient of a layer with NCOL_ input channels and 64 output channels on an HIN x WIN input; the resident
// operand is the layer's output gradient [HO*WO][64]
template <int NCOL_, int KSZ_, int STRIDE_, int HIN_, int WIN_, int G_> struct ImgDgrad {
    static constexpr bool FWD = false, FLAT = false;
    static constexpr int CIN = 64, NCOL = NCOL_, G = G_;
    static constexpr int HO = (HIN_ - KSZ_) / STRIDE_ + 1, WO = (WIN_ - KSZ_) / STRIDE_ + 1;
    static constexpr int PIN = HO * WO, POUT_ALL = HIN_ * WIN_;
    static constexpr int TK = KSZ_ / STRIDE_, TAPS = TK * TK, NCLS = STRIDE_ * STRIDE_, KTOT = KSZ_ * KSZ_ * 64;
    static constexpr int SEGSTEPS = 0;
    static_assert(KSZ_ % STRIDE_ == 0 && NCLS <= 4, "parity classes");
    static constexpr int cls_h(int c) { return (HIN_ - c / STRIDE_ + STRIDE_ - 1) / STRIDE_; }
    static constexpr int cls_w(int c) { return (WIN_ - c % STRIDE_ + STRIDE_ - 1) / STRIDE_; }
    static constexpr int src_tap(int c, int tap)
    {
        return (c / STRIDE_ + STRIDE_ * (tap / TK)) * KSZ_ + c % STRIDE_ + STRIDE_ * (tap % TK);
    }
    static HTS_HD int in_row(int, int yy, int xx, int tap)
    {
        const int oy = yy - tap / TK, ox = xx - tap % TK;
        return (oy >= 0 && ox >= 0 && oy < HO && ox < WO) ? oy * WO + ox : -1;
    }
    static HTS_HD int out_pos(int c, int yy, int xx) { return (yy * STRIDE_ + c / STRIDE_) * WIN_ + xx * STRIDE_ + c % STRIDE_; }
};

template <class S> constexpr int imgconv_tiles(int cls)            // 32-row tiles of classes 0 .. cls-1
{
    int t = 0;
    for (int c = 0; c < cls; ++c) t += (S::G * S::cls_h(c) * S::cls_w(c) + 31) / 32;
    return t;
}
// elements of the LDS copy of a group's channel-major output (forward pass with FLAT), else 0
template <class S> constexpr size_t imgconv_stage_elems() { return S::FWD && S::FLAT ? (size_t)S::G * S::NCOL * S::POUT_ALL : 0; }
template <class S> constexpr size_t imgconv_lds_bytes()
{
    return ((size_t)S::NCLS * S::NCOL * (S::TAPS * S::CIN + 8) + (size_t)(S::G * S::PIN + 1) * (S::CIN + 8) + imgconv_stage_elems<S>()) * sizeof(bf16_t)
           + (S::FWD ? S::NCOL * sizeof(float) : 0);          // the biases
}

constexpr int IMGCONV_THREADS = 512;     // (16 wavefronts on the 32-column input gradient's short tiles: no faster, measured)

template <class S> __global__ __launch_bounds__(IMGCONV_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void imgconv_kernel(const ImgConvArgs a)
{
    constexpr int CIN = S::CIN, NCOL = S::NCOL, TAPS = S::TAPS, NCLS = S::NCLS, G = S::G, TN = NCOL / 32;
    constexpr int KC = TAPS * CIN, WP = KC + 8, IP = CIN + 8, PIN = S::PIN, ZR = G * PIN;   // pitches; the zero row
    constexpr int NT = IMGCONV_THREADS, NWV = NT / 64;
    constexpr int NVEC = G * PIN * CIN / 8, NPF = (NVEC + NT - 1) / NT;       // 16-byte vectors of a group of samples
    constexpr int TILES = imgconv_tiles<S>(NCLS);
    static_assert(CIN % 16 == 0 && NCOL % 32 == 0 && imgconv_lds_bytes<S>() <= 160 * 1024, "shape");
    extern __shared__ __attribute__((aligned(16))) unsigned char ic_smem[];
    bf16_t *wl = reinterpret_cast<bf16_t *>(ic_smem);                // [NCLS][NCOL][WP]
    bf16_t *inl = wl + NCLS * NCOL * WP;                             // [G*PIN + 1][IP]
    bf16_t *stg = inl + (G * PIN + 1) * IP;                          // FLAT: [G][NCOL][POUT_ALL], the group's output as it lies in memory
    float *biasl = reinterpret_cast<float *>(stg + imgconv_stage_elems<S>());   // forward: [NCOL]
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lrow = lane & 31, kg = lane >> 5;

    // The weight matrix, class by class (a class keeps the taps that reach it, in tap order).  All of it is requested
    // before anything is waited for, and the first group of samples right behind it: one memory round trip, not two.
    constexpr int WV = NCLS * NCOL * TAPS * (CIN / 8), NWPF = (WV + NT - 1) / NT;
    bf16x8 wpf[NWPF];
    auto wslot = [&](int v, int *lds_off) {                          // source offset in a.w; LDS offset in wl
        const int c8 = v % (CIN / 8);
        int t = v / (CIN / 8);
        const int tap = t % TAPS;
        t /= TAPS;
        const int col = t % NCOL, cls = t / NCOL;
        *lds_off = (cls * NCOL + col) * WP + tap * CIN + c8 * 8;
        return col * S::KTOT + S::src_tap(cls, tap) * CIN + c8 * 8;
    };
#pragma unroll
    for (int i = 0; i < NWPF; ++i) {
        const int v = tid + i * NT;
        int lo;
        if (v < WV) wpf[i] = *reinterpret_cast<const bf16x8 *>(a.w + wslot(v, &lo));
    }

    bf16x8 pf[NPF];
    const long long in_elems = (long long)a.B * PIN * CIN;
    auto fetch = [&](int grp) {
        const long long base = (long long)grp * G * PIN * CIN;
#pragma unroll
        for (int i = 0; i < NPF; ++i) {
            const int v = tid + i * NT;
            if (v < NVEC && base + (long long)v * 8 < in_elems) pf[i] = *reinterpret_cast<const bf16x8 *>(a.in + base + (long long)v * 8);
        }
    };
    const int ngroups = (a.B + G - 1) / G;
    if ((int)blockIdx.x < ngroups) fetch(blockIdx.x);
#pragma unroll
    for (int i = 0; i < NWPF; ++i) {
        const int v = tid + i * NT;
        int lo;
        if (v < WV) { wslot(v, &lo); *reinterpret_cast<bf16x8 *>(wl + lo) = wpf[i]; }
    }
    if (tid < CIN / 8) *reinterpret_cast<bf16x8 *>(inl + ZR * IP + tid * 8) = zero_vec<bf16_t, 8>();
    if constexpr (S::FWD) { if (tid >= NT - NCOL) biasl[tid - (NT - NCOL)] = a.bias[tid - (NT - NCOL)]; }   // (an epilogue that fetched them would wait a memory round trip)

    for (int grp = blockIdx.x; grp < ngroups; grp += gridDim.x) {
#pragma unroll
        for (int i = 0; i < NPF; ++i) {
            const int v = tid + i * NT;
            if (v < NVEC) *reinterpret_cast<bf16x8 *>(inl + (v / (CIN / 8)) * IP + (v % (CIN / 8)) * 8) = pf[i];
        }
        __syncthreads();
        if (grp + (int)gridDim.x < ngroups) fetch(grp + gridDim.x);          // the next group travels meanwhile
        const int ng = min(G, a.B - grp * G);                                 // samples of this group that exist

        auto do_tile = [&](auto cls_tag, int t) {
            constexpr int CLS = decltype(cls_tag)::value;
            constexpr int HC = S::cls_h(CLS), WC = S::cls_w(CLS), PC = HC * WC, ROWS = G * PC;
            const int idx = t * 32 + lrow;
            const bool rvalid = idx < ROWS;
            const int ic = rvalid ? idx : ROWS - 1;
            const int g = ic / PC, p = ic - g * PC, yy = p / WC, xx = p - yy * WC;
            int ra[TAPS];                                                    // LDS offset of this lane's row per tap
#pragma unroll
            for (int tap = 0; tap < TAPS; ++tap) {
                const int r = S::in_row(CLS, yy, xx, tap);
                ra[tap] = (r >= 0 ? g * PIN + r : ZR) * IP + 8 * kg;
            }
            const bf16_t *wrow = wl + (CLS * NCOL + lrow) * WP + 8 * kg;
            const bool store_row = rvalid && g < ng;
            const long long b = (long long)grp * G + (store_row ? g : 0);
            // What the epilogue needs from memory (the ReLU masks of the input gradient) is requested now, so that it
            // travels while the products are formed: fetched after them, every tile would end with a bare memory
            // round trip.
            // (a lane reads and writes 16 consecutive channels of each 32, see the epilogue)
            const long long o = (b * S::POUT_ALL + S::out_pos(CLS, yy, xx)) * NCOL + 16 * kg;
            bf16x8 mk[TN][2];
            if constexpr (!S::FWD) {
                if (store_row) {
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int h = 0; h < 2; ++h) mk[j][h] = *reinterpret_cast<const bf16x8 *>(a.mask + o + j * 32 + 8 * h);
                }
            }
            f32x16 acc[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
            constexpr int CS = CIN / 16, STEPS = TAPS * CS, SEGS = S::SEGSTEPS;
            static_assert(SEGS == 0 || STEPS % SEGS == 0, "whole segments");
            // Software pipeline over the matrix-instruction steps: the operands of step ks+PD are read before the
            // products of step ks are issued (an LDS read takes a few hundred cycles to return when eight wavefronts
            // read at once, a step's products 32-64), and the scheduling barriers keep the reads from drifting
            // further ahead (all of them at once would not fit the register file).  The ring of PD operand sets is
            // indexed at compile time: the step loops are written out.
            constexpr int PD = 3;
            static_assert(STEPS >= PD && (SEGS == 0 || SEGS % PD == 0), "pipeline depth");
            bf16x8 av_q[PD], bv_q[PD][TN];
            auto read_step = [&](int ks, int slot) {              // both compile-time constants after unrolling
                const int tap = ks / CS, cs = ks % CS;
                av_q[slot] = *reinterpret_cast<const bf16x8 *>(inl + ra[tap] + cs * 16);
#pragma unroll
                for (int j = 0; j < TN; ++j) bv_q[slot][j] = *reinterpret_cast<const bf16x8 *>(wrow + j * 32 * WP + tap * CIN + cs * 16);
            };
#pragma unroll
            for (int q = 0; q < PD; ++q) read_step(q, q);
            if constexpr (SEGS > 0) {
                // Forward: a fresh accumulator per segment, added in order.  The segment loop is a real loop (written
                // out, the compiler moves all the additions to the end and runs out of registers); its step index
                // is the same in all lanes, and a forward row's tap offsets are affine in the tap, so nothing needs
                // a run-time index into registers.
                static_assert(S::FWD, "segments are a forward-pass matter");
                const int ra0 = ra[0];
                auto read_rt = [&](int ks, int slot) {            // ks: run-time, wavefront-uniform
                    const int tap = ks / CS, cs = ks % CS;
                    av_q[slot] = *reinterpret_cast<const bf16x8 *>(inl + ra0 + (S::in_row(0, 0, 0, tap) - S::in_row(0, 0, 0, 0)) * IP + cs * 16);
#pragma unroll
                    for (int j = 0; j < TN; ++j) bv_q[slot][j] = *reinterpret_cast<const bf16x8 *>(wrow + j * 32 * WP + ks * 16);
                };
#pragma unroll 1
                for (int sg = 0; sg < STEPS / SEGS; ++sg) {
                    f32x16 sacc[TN];
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) sacc[j][r] = 0.0f;
#pragma unroll
                    for (int u = 0; u < SEGS; ++u) {
                        const bf16x8 av = av_q[u % PD];
                        bf16x8 bv[TN];
#pragma unroll
                        for (int j = 0; j < TN; ++j) bv[j] = bv_q[u % PD][j];
                        read_rt(min(sg * SEGS + u + PD, STEPS - 1), u % PD);     // (past the end: the last step again)
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int j = 0; j < TN; ++j) sacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv[j], av, sacc[j], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[j][r] += sacc[j][r];
                }
            } else {
#pragma unroll
                for (int ks = 0; ks < STEPS; ++ks) {
                    const bf16x8 av = av_q[ks % PD];
                    bf16x8 bv[TN];
#pragma unroll
                    for (int j = 0; j < TN; ++j) bv[j] = bv_q[ks % PD][j];
                    if (ks + PD < STEPS) read_step(ks + PD, ks % PD);
                    __builtin_amdgcn_sched_barrier(0);
                    // the weights are the first operand: a lane's accumulator registers are 16 output columns of ONE row
#pragma unroll
                    for (int j = 0; j < TN; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv[j], av, acc[j], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (!store_row) return;
            // register 4q+e of accumulator j is column j*32 + 8q + 4kg + e
            // The two lanes of a row hold alternate groups of four columns.  They trade halves so that one has columns
            // 0-15 and the other 16-31 of each 32: two 16-byte stores (and mask loads) per lane and 32 columns instead
            // of four 8-byte ones -- half the cache-line visits of these memory-bound passes.
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            auto trade = [&](const u32x2 (&pk)[4], int h) {                    // columns 16 kg + 8 h .. + 7 of the 32
                const u32x2 mine = kg ? pk[2 + h] : pk[h], send = kg ? pk[h] : pk[2 + h];
                u32x2 got;
                got.x = __shfl_xor(send.x, 32, 64);
                got.y = __shfl_xor(send.y, 32, 64);
                const u32x4 v = kg ? u32x4{got.x, got.y, mine.x, mine.y} : u32x4{mine.x, mine.y, got.x, got.y};
                return __builtin_bit_cast(bf16x8, v);
            };
            if constexpr (S::FWD) {
                const long long m = b * S::POUT_ALL + p;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    u32x2 pk[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int ch = j * 32 + 8 * q + 4 * kg;
                        const f32x4 bn = *reinterpret_cast<const f32x4 *>(biasl + ch);
                        Vec<bf16_t, 4> y;
#pragma unroll
                        for (int e = 0; e < 4; ++e) { const float tv = acc[j][4 * q + e] + bn[e]; y[e] = from_f32<bf16_t>(tv > 0.0f ? tv : 0.0f); }
                        if constexpr (S::FLAT) {
                            // channel-major: a lane's 32 values lie POUT_ALL apart, so they go to the LDS copy of the
                            // group's output and leave from there in whole vectors (two-byte stores to memory, 32
                            // instructions per tile, were a third of this kernel's time)
#pragma unroll
                            for (int e = 0; e < 4; ++e) stg[(g * NCOL + ch + e) * S::POUT_ALL + p] = y[e];
                        }
                        pk[q] = __builtin_bit_cast(u32x2, y);
                    }
                    bf16_t *rowmajor = S::FLAT ? a.out2 : a.out;               // [row][NCOL]
                    if (rowmajor) {
#pragma unroll
                        for (int h = 0; h < 2; ++h) *reinterpret_cast<bf16x8 *>(rowmajor + m * NCOL + j * 32 + 16 * kg + 8 * h) = trade(pk, h);
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    u32x2 pk[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        Vec<bf16_t, 4> y;
#pragma unroll
                        for (int e = 0; e < 4; ++e) y[e] = from_f32<bf16_t>(acc[j][4 * q + e]);
                        pk[q] = __builtin_bit_cast(u32x2, y);
                    }
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        bf16x8 y = trade(pk, h);
#pragma unroll
                        for (int i = 0; i < 8; ++i) y[i] = to_f32(mk[j][h][i]) > 0.0f ? y[i] : from_f32<bf16_t>(0.0f);
                        *reinterpret_cast<bf16x8 *>(a.out + o + j * 32 + 8 * h) = y;
                    }
                }
            }
        };
        for (int tile = w; tile < TILES; tile += NWV) {                       // `tile` is the same in all lanes of a wavefront
            if constexpr (NCLS == 1) do_tile(std::integral_constant<int, 0>{}, tile);
            else {
                if (tile < imgconv_tiles<S>(1)) do_tile(std::integral_constant<int, 0>{}, tile);
                else if (tile < imgconv_tiles<S>(2)) do_tile(std::integral_constant<int, 1>{}, tile - imgconv_tiles<S>(1));
                else if (NCLS > 2 && tile < imgconv_tiles<S>(NCLS > 2 ? 3 : 2)) do_tile(std::integral_constant<int, (NCLS > 2 ? 2 : 0)>{}, tile - imgconv_tiles<S>(2));
                else if (NCLS > 3) do_tile(std::integral_constant<int, (NCLS > 3 ? 3 : 0)>{}, tile - imgconv_tiles<S>(NCLS > 3 ? 3 : 2));
            }
        }
        __syncthreads();          // the resident rows are overwritten by the next group
        if constexpr (S::FWD && S::FLAT) {
            // (the next group's tiles write the copy only after the barrier that follows its rows' arrival)
            constexpr int PER = NCOL * S::POUT_ALL;
            static_assert(PER % 8 == 0, "whole vectors per sample");
            bf16_t *dst = a.out + (long long)grp * G * PER;
            for (int v = tid; v < ng * (PER / 8); v += NT) *reinterpret_cast<bf16x8 *>(dst + v * 8) = *reinterpret_cast<const bf16x8 *>(stg + v * 8);
        }
    }
}

template <class S> inline hipError_t launch_imgconv(const ImgConvArgs &a, hipStream_t stream)
{
    if (a.B <= 0) return hipSuccess;
    auto kern = imgconv_kernel<S>;
    static std::atomic<bool> attr_set{false};       // raise the dynamic-LDS limit once per instantiation (setting it twice is harmless)
    if (!attr_set.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)imgconv_lds_bytes<S>());
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    const int ngroups = (a.B + S::G - 1) / S::G;
    const int grid = ngroups < 256 ? ngroups : 256;          // one workgroup per compute unit walks the groups
    hipLaunchKernelGGL(kern, dim3(grid), dim3(IMGCONV_THREADS), imgconv_lds_bytes<S>(), stream, a);
    return hipGetLastError();
}

}  // namespace hts
