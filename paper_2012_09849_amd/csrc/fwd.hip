// Forward pass of the policy/value network (appendix "Implementation Details") as four tiled contractions:
// conv1 (uint8 gather, 1/255 folded in), conv2, conv3, FC.  The heads run in misc.hip.
#include "internal.hpp"
#include "imgconv.hpp"

#include <atomic>

namespace hts {

// ------------------------------------------------------------------------------------------------------------
// conv1 for large batches of small 4-channel frames (bf16, image <= 64 KiB of LDS, e.g. 4x84x84): one workgroup per
// observation.
// The frame is converted to bf16 ONCE into an LDS image [(c,y)][Wp] (the tile kernel converts every pixel four times,
// once per patch that contains it, and spends most of its issue slots on that and on gather addresses); the matrix
// instruction's position operand is then read straight from the image -- 8 consecutive k of conv1.w's (c,u,v) order
// are 8 neighbouring pixels of one row -- and the 32 x 64C weight operand lives in registers for the whole kernel.
// Same k order, same 64-wide segments (one input channel each) and the same epilogue as Conv1Fwd, so the output bits
// equal those of the other conv1 kernels.
// ------------------------------------------------------------------------------------------------------------
struct Conv1ImgArgs {
    const uint8_t *obs;
    const int32_t *index;
    const bf16_t *w;        // [32][64*C]
    const float *bias;
    bf16_t *out;            // [B][P1][32]
    int B, H, W, W1, P1, Wp;
    FastDiv dGpr, dW1;      // division by W/4 (4-pixel groups per image row) and by W1
};
constexpr int C1IMG_THREADS = 256;        // 4 wavefronts (one per SIMD); two workgroups share a compute unit, one converting while the other multiplies
constexpr int C1IMG_MAX_PASSES = 32;      // passes of a wavefront over its share of the image rows

// HC, WPC: frame height and image pitch as compile-time constants (0: taken from the arguments).  With them every
// image offset of the multiply loop is an immediate of the LDS instruction.  NP: passes of a wavefront over its share
// of the image rows (registers that hold the next frame while this one is multiplied).
template <int C, int HC, int WPC, int NP> __global__ __launch_bounds__(C1IMG_THREADS, 2) void conv1_image_kernel(const Conv1ImgArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char c1_smem[];
    bf16_t *img = reinterpret_cast<bf16_t *>(c1_smem);
    constexpr int K = 64 * C;
    const int H = HC ? HC : a.H, Wp = WPC ? WPC : a.Wp;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lrow = lane & 31, lk = lane >> 5;
    bf16x8 breg[K / 16];
#pragma unroll
    for (int t = 0; t < K / 16; ++t) breg[t] = *reinterpret_cast<const bf16x8 *>(a.w + lrow * K + 16 * t + 8 * lk);
    // The weights are the FIRST operand of the matrix instruction, so a lane's accumulator registers are 16 output
    // channels (8g + 4 lk + j, g and j < 4) of ONE position and leave as four 8-byte stores.
    const int rows = C * H, gpr = a.W >> 2;
    float *lbias = reinterpret_cast<float *>(img + ((rows * Wp + 7) & ~7));     // conv1.b behind the image, 16-byte aligned
    if (tid < 32) lbias[tid] = a.bias[tid];
    const int ntiles = (a.P1 + 31) >> 5;
    // Frame -> image: a wavefront takes 64/gpr image rows per pass, one 4-pixel group per lane, so neighbouring lanes
    // load neighbouring dwords and write neighbouring 8-byte LDS slots; a lane's (row-in-pass, group) never changes.
    const int rpp = 64 / gpr;                                    // image rows per wavefront pass
    const int lr = a.dGpr.div(lane), xg = lane - lr * gpr;
    const bool lane_on = lr < rpp;
    constexpr int NW = C1IMG_THREADS / 64;
    uint32_t raw[NP];
    auto fetch = [&](int b) {
        const uint8_t *src = a.obs + (long long)(a.index ? a.index[b] : b) * rows * a.W + 4 * xg;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int row = (w + i * NW) * rpp + lr;
            if (lane_on && row < rows) raw[i] = *reinterpret_cast<const uint32_t *>(src + row * a.W);
        }
    };
    if ((int)blockIdx.x < a.B) fetch(blockIdx.x);
    for (int b = blockIdx.x; b < a.B; b += gridDim.x) {
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int row = (w + i * NW) * rpp + lr;
            if (!lane_on || row >= rows) continue;
            Vec<bf16_t, 4> px;
#pragma unroll
            for (int e = 0; e < 4; ++e) px[e] = from_f32<bf16_t>((float)((raw[i] >> (8 * e)) & 0xFFu));
            *reinterpret_cast<Vec<bf16_t, 4> *>(img + row * Wp + 4 * xg) = px;
        }
        __syncthreads();
        if (b + (int)gridDim.x < a.B) fetch(b + gridDim.x);      // the next frame travels while this one is multiplied
        for (int mt = w; mt < ntiles; mt += C1IMG_THREADS / 64) {
            const int m = mt * 32 + lrow, mc = m < a.P1 ? m : a.P1 - 1;
            const int oy = a.dW1.div(mc), ox = mc - oy * a.W1;
            const bf16_t *base = img + (4 * oy + lk) * Wp + 4 * ox;      // image row u = 2t + lk of the patch, t = 0
            // One 64-long segment per input channel.  The C segment chains are independent until they are added, so
            // their matrix instructions are interleaved (t outer, channel inner): no instruction waits for its
            // predecessor, and within a segment k still ascends.
            // (Two chains at a time: enough to hide the instruction's latency, and half the accumulator registers.)
            // The segment sums are added in channel order; a segment sum is never -0, so the total starts as the first.
            static_assert(C % 2 == 0, "channel pairs");
            f32x16 tot;
#pragma unroll
            for (int c0 = 0; c0 < C; c0 += 2) {
                f32x16 acc[2];
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[c][r] = 0.0f;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    bf16x8 av[2];
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        const bf16_t *pa = base + ((c0 + c) * H + 2 * t) * Wp;
                        const Vec<bf16_t, 4> lo = *reinterpret_cast<const Vec<bf16_t, 4> *>(pa),
                                             hi = *reinterpret_cast<const Vec<bf16_t, 4> *>(pa + 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) { av[c][e] = lo[e]; av[c][4 + e] = hi[e]; }
                    }
#pragma unroll
                    for (int c = 0; c < 2; ++c)
                        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(breg[(c0 + c) * 4 + t], av[c], acc[c], 0, 0, 0);
                }
                if (c0 == 0) tot = acc[0];
                else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) tot[r] += acc[0][r];
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) tot[r] += acc[1][r];
            }
            if (m < a.P1) {
                // (trading halves with the position's other lane for two 16-byte stores, which pays in the LDS-resident
                // conv2/conv3 kernels, changes nothing here: 22.2 vs 23.1 us at 1024 rows)
                bf16_t *dst = a.out + ((long long)b * a.P1 + m) * 32 + 4 * lk;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 bias = *reinterpret_cast<const f32x4 *>(lbias + 8 * g + 4 * lk);
                    Vec<bf16_t, 4> o;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float y = __builtin_fmaf(tot[4 * g + j], 1.0f / 255.0f, bias[j]);
                        o[j] = from_f32<bf16_t>(y > 0.0f ? y : 0.0f);
                    }
                    *reinterpret_cast<Vec<bf16_t, 4> *>(dst + 8 * g) = o;
                }
            }
        }
        __syncthreads();          // the image is overwritten by the next observation
    }
}

// Row pitch of the LDS image: a multiple of 4 pixels, and congruent to W1 modulo 32 so that a tile's positions keep
// their 8-byte bank stride when they wrap from one output row to the next (4 image rows further down).
static int conv1_image_pitch(const Geom &g)
{
    int wp = g.W;
    while ((wp - g.W1) % 32 != 0) wp += 4;
    return wp;
}

// true if the frame shape and pointers fit conv1_image_kernel
static bool conv1_image_fits(const Geom &g, const uint8_t *obs)
{
    if (g.C != 4 || g.W > 256 || (((uintptr_t)obs) & 3u)) return false;
    const int gpr = g.W / 4, rpp = 64 / gpr, rows = g.C * g.H;
    return rows <= C1IMG_MAX_PASSES * rpp * (C1IMG_THREADS / 64) && (size_t)rows * conv1_image_pitch(g) * 2 + 16 + 128 <= 65536;
}

static hipError_t launch_conv1_image(Ctx &c, const uint8_t *obs, const int32_t *index, int B)
{
    const Geom &g = c.g;
    Conv1ImgArgs a;
    a.obs = obs; a.index = index; a.w = (const bf16_t *)c.ws.w1s; a.bias = c.ws.hb + c.sh.b1; a.out = (bf16_t *)c.ws.act1;
    a.B = B; a.H = g.H; a.W = g.W; a.W1 = g.W1; a.P1 = g.P1; a.Wp = conv1_image_pitch(g);
    a.dGpr = FastDiv::make(g.W / 4); a.dW1 = FastDiv::make(g.W1);
    const size_t lds = (((size_t)g.C * g.H * a.Wp + 7) & ~(size_t)7) * sizeof(bf16_t) + 32 * sizeof(float);      // image + conv1.b
    const int grid = B < 512 ? B : 512;          // resident workgroups walk the batch
    if (g.H == 84 && g.W == 84 && a.Wp == 84)                 // the Atari frame of the paper's experiments
        hipLaunchKernelGGL((conv1_image_kernel<4, 84, 84, 28>), dim3(grid), dim3(C1IMG_THREADS), lds, c.stream, a);
    else
        hipLaunchKernelGGL((conv1_image_kernel<4, 0, 0, C1IMG_MAX_PASSES>), dim3(grid), dim3(C1IMG_THREADS), lds, c.stream, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------------
// conv1 for large bf16 batches of the two frame shapes of the paper's experiments (16x72x96, and 4x84x84 for the largest
// batches), whose four-channel slab (4*H*W bytes, about 27 KB) fits twice into LDS as bf16: one workgroup per compute
// unit walks a share of the observations.
// A frame passes in slabs of four channels.  Wavefronts 4-7 (producers) fetch slab q+2 into registers, convert slab q+1
// to bf16 once into one of two LDS images [(c,y)][W] and copy the 32 x 256 slice of conv1.w that belongs to its
// channels beside it; meanwhile wavefronts 0-3 (consumers, one per SIMD next to a producer) multiply slab q: position
// tiles w, w+4, ... of 32 positions each, the matrix instruction's weight operand read from the LDS slice (shared by two
// tiles; a four-channel frame is a single slab and its weights stay in the consumers' registers instead), its position
// operand straight from the image (8 consecutive k of conv1.w's (c,u,v) order are 8 neighbouring
// pixels of one row).  A tile's running total stays in the consumer's registers across the frame's slabs, so the
// channels' 64-long segment sums are added in channel order exactly as in Conv1Fwd: same bits as the other conv1
// kernels.  One barrier per slab.  (The tile kernel converts every pixel four times and fetches it in 8-byte pieces;
// with every wavefront doing both jobs in turn the compute unit alternates between a conversion phase and a multiply
// phase and is no faster than the tile kernel, 155 us for 2048 frames of 16x72x96; this way: 96 us.)
// ------------------------------------------------------------------------------------------------------------
struct Conv1SlabArgs {
    const uint8_t *obs;
    const int32_t *index;
    const bf16_t *w;        // [32][64*C]
    const float *bias;
    bf16_t *out;            // [B][P1][32]
    int B, W1, P1;
};
constexpr int C1S_THREADS = 512, C1S_PRODUCERS = 256;
constexpr int C1S_MAX_SAMPLES = 64;       // observations per workgroup (their row indices are read once, into LDS)
constexpr int C1S_WPITCH = 528;           // bytes per weight row in LDS: 512 + 16, so that rows start four banks apart
constexpr int C1S_WBUF = 32 * C1S_WPITCH;
constexpr int C1S_TILES = 4;              // position tiles per consumer wavefront

template <int H, int W> constexpr size_t conv1_slab_lds() { return (size_t)2 * (8 * H * W) + 2 * C1S_WBUF + 128 + C1S_MAX_SAMPLES * 4; }

// (LDS admits one workgroup per compute unit, two wavefronts per SIMD: the register budget is stated, or the compiler
// aims at three and keeps fewer loads in flight -- 107 -> 96 us)
template <int NG, int H, int W> __global__ __launch_bounds__(C1S_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void conv1_slab_kernel(const Conv1SlabArgs a)
{
    constexpr int C = 4 * NG, K = 64 * C, SLAB = 4 * H * W, NV = SLAB / 16, PT = C1S_PRODUCERS, NP = (NV + PT - 1) / PT;
    constexpr int IMG = 2 * SLAB;          // bytes of one bf16 image
    constexpr int D = 2;                   // slabs in flight in the producers' registers (four: no faster, 99 vs 96 us)
    static_assert(SLAB % 16 == 0 && (NG == 1 || NG % D == 0), "slab shape");
    extern __shared__ __attribute__((aligned(16))) unsigned char c1s_smem[];
    unsigned char *wl = c1s_smem + 2 * IMG;
    float *lbias = reinterpret_cast<float *>(wl + 2 * C1S_WBUF);
    int *rowid = reinterpret_cast<int *>(lbias + 32);
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), lrow = lane & 31, lk = lane >> 5;
    const int nsamp = (a.B - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    if (tid < nsamp) { const int b = blockIdx.x + tid * gridDim.x; rowid[tid] = a.index ? a.index[b] : b; }
    if (tid >= 64 && tid < 96) lbias[tid - 64] = a.bias[tid - 64];
    __syncthreads();
    const int nphase = nsamp * NG;          // slab q: observation q / NG of this workgroup, channels 4 (q % NG) .. + 3
    if (w >= 4) {
        // ---- producers ----
        const int pt = tid - (C1S_THREADS - PT);
        constexpr int NWV = NG > 1 ? 4 : 0;                // 16-byte vectors of the weight slice per producer thread
        uint4 raw[D][NP + NWV];                            // a slab's vectors, then its weight slice's
        // A thread's byte offsets inside a slab / a weight slice never change; what changes per slab is the same for the
        // whole workgroup and is kept in scalar registers, so a fetch is loads and nothing else.
        uint32_t ioff[NP], woffs[NWV ? NWV : 1];
#pragma unroll
        for (int i = 0; i < NP; ++i) { const int v = pt + i * PT; ioff[i] = 16u * (uint32_t)(NV % PT == 0 ? v : min(v, NV - 1)); }   // a vector behind the slab's end repeats its last one
#pragma unroll
        for (int i = 0; i < NWV; ++i) { const int v = pt + i * PT; woffs[i] = (uint32_t)((v >> 5) * (2 * K) + (v & 31) * 16); }       // row v / 32, 16-byte column v % 32 of the 32 x 256 slice
        auto fetch = [&](int q, uint4 (&r)[NP + NWV]) {
            const int s = q / NG, cg = q - s * NG;
            const long long row = __builtin_amdgcn_readfirstlane(rowid[s]);
            const uint8_t *src = a.obs + (row * C + 4 * cg) * (H * W);
#pragma unroll
            for (int i = 0; i < NP; ++i) r[i] = *reinterpret_cast<const uint4 *>(src + ioff[i]);
            if constexpr (NG > 1) {
                const unsigned char *wsrc = reinterpret_cast<const unsigned char *>(a.w) + cg * 512;
#pragma unroll
                for (int i = 0; i < NWV; ++i) r[NP + i] = *reinterpret_cast<const uint4 *>(wsrc + woffs[i]);
            }
        };
        auto convert = [&](const uint4 (&r)[NP + NWV], int buf) {
            unsigned char *dst = c1s_smem + buf * IMG + 32 * pt;
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                if (NV % PT != 0 && pt + i * PT >= NV) continue;
                const uint32_t x[4] = {r[i].x, r[i].y, r[i].z, r[i].w};
                bf16x8 lo, hi;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    lo[e] = from_f32<bf16_t>((float)((x[0] >> (8 * e)) & 0xFFu));
                    lo[4 + e] = from_f32<bf16_t>((float)((x[1] >> (8 * e)) & 0xFFu));
                    hi[e] = from_f32<bf16_t>((float)((x[2] >> (8 * e)) & 0xFFu));
                    hi[4 + e] = from_f32<bf16_t>((float)((x[3] >> (8 * e)) & 0xFFu));
                }
                *reinterpret_cast<bf16x8 *>(dst + i * PT * 32) = lo;
                *reinterpret_cast<bf16x8 *>(dst + i * PT * 32 + 16) = hi;
            }
            if constexpr (NG > 1) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int v = pt + i * PT;
                    *reinterpret_cast<uint4 *>(wl + buf * C1S_WBUF + (v >> 5) * C1S_WPITCH + (v & 31) * 16) = r[NP + i];
                }
            }
        };
#pragma unroll
        for (int d = 0; d < D; ++d) if (d < nphase) fetch(d, raw[d]);
        convert(raw[0], 0);
        if (D < nphase) fetch(D, raw[0]);
        __syncthreads();
        for (int q0 = 0; q0 < nphase; q0 += D) {
#pragma unroll
            for (int j = 0; j < D; ++j) {                      // slab q+1 sits in register set (j+1) % D
                const int q = q0 + j;
                if (NG % D != 0 && q >= nphase) break;         // (the same for the whole workgroup)
                if (q + 1 < nphase) convert(raw[(j + 1) % D], (q & 1) ^ 1);
                if (q + 1 + D < nphase) fetch(q + 1 + D, raw[(j + 1) % D]);
                __syncthreads();
            }
        }
        return;
    }
    // ---- consumers ----
    const int ntiles = (a.P1 + 31) >> 5;
    uint32_t toff[C1S_TILES];
    int tm[C1S_TILES];
#pragma unroll
    for (int i = 0; i < C1S_TILES; ++i) {
        const int m = (w + 4 * i) * 32 + lrow, mc = m < a.P1 ? m : a.P1 - 1;
        const int oy = mc / a.W1, ox = mc - oy * a.W1;
        toff[i] = 2u * (uint32_t)((4 * oy + lk) * W + 4 * ox);      // image row u = 2t + lk of the patch, t = 0
        tm[i] = m;
    }
    const int mytiles = w < ntiles ? (ntiles - w + 3) / 4 : 0;       // the same for the whole wavefront
    const uint32_t woff = (uint32_t)(lrow * C1S_WPITCH + 16 * lk);
    // a four-channel frame is one slab: its weights never change and stay in registers
    bf16x8 breg[NG == 1 ? 16 : 1];
    if constexpr (NG == 1) {
#pragma unroll
        for (int t = 0; t < 16; ++t) breg[t] = *reinterpret_cast<const bf16x8 *>(a.w + lrow * K + 16 * t + 8 * lk);
    }
    f32x16 tot[C1S_TILES];
    // 8 pixels of one image row (8-byte aligned) as two single 8-byte reads.  Left alone, the compiler merges them
    // (or reads of two steps) into one two-address read, which the LDS serves at half the rate of two single ones --
    // 8.0 against 2 x 2.4 ticks per wavefront -- and the LDS pipe is what the consumers wait for: hence volatile
    // reads on explicit LDS addresses (conv1 forward at 2048 frames of 16x72x96: 93 -> 84 us).
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    typedef const volatile u32x2 __attribute__((address_space(3))) *lds_u32x2;
    typedef __attribute__((address_space(3))) unsigned char *lds_bytes;
    const uint32_t smem0 = (uint32_t)(uintptr_t)(lds_bytes)c1s_smem;
    auto read16 = [&](uint32_t p) {
        const u32x2 lw = *(lds_u32x2)(uintptr_t)p, hw = *(lds_u32x2)(uintptr_t)(p + 8u);
        const Vec<bf16_t, 4> lo = __builtin_bit_cast(Vec<bf16_t, 4>, lw), hi = __builtin_bit_cast(Vec<bf16_t, 4>, hw);
        bf16x8 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[e] = lo[e]; v[4 + e] = hi[e]; }
        return v;
    };
    // tiles T0 .. T0+NT-1 of this wavefront against the slab in `buf`.  One 64-long segment per input channel, formed
    // in a fresh accumulator (k ascending) and added to the running total in channel order (a segment sum is never
    // -0, so the total of a frame starts as its first).
    // The 16 steps (channel, k-step) are written out as a software pipeline: a consumer is alone on its SIMD's matrix
    // pipe, so nothing hides an LDS round trip but its own earlier reads.  The operands of step e + PD are read before
    // the products of step e are issued; the channels alternate between two accumulators, and the 16 additions per
    // tile that fold a finished segment into the total are spread over the next channel's four steps, where they run
    // beside its matrix instructions.  (Left to the compiler, most matrix instructions waited for a read issued just
    // before them, and the additions of two channels ran in a block behind their products: 5400 ticks per slab for
    // the wavefront with four tiles, against 2048 of matrix instructions.)
    auto mult = [&](int buf, auto t0c, auto ntc, auto firstc) {
        constexpr int T0 = decltype(t0c)::value, NT = decltype(ntc)::value, PD = 3;
        constexpr bool FIRST = decltype(firstc)::value;
        const unsigned char *wb = wl + buf * C1S_WBUF + woff;
        uint32_t ib[NT][4];                               // per tile and channel, so that a step's offset is an immediate
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int ch = 0; ch < 4; ++ch) {
                ib[i][ch] = smem0 + buf * IMG + toff[T0 + i] + 2 * (ch * H * W);
                asm volatile("" : "+v"(ib[i][ch]));       // (kept in a register: folded back into one base plus a constant, the
            }                                             //  constant exceeds the instruction's offset field and costs an addition per read)
        bf16x8 wq[PD], aq[PD][NT];
        auto rd = [&](int e, int slot) {                  // both compile-time constants after unrolling
            const int ch = e >> 2, t = e & 3;
            if constexpr (NG == 1) wq[slot] = breg[ch * 4 + t];
            else wq[slot] = *reinterpret_cast<const bf16x8 *>(wb + 2 * (64 * ch + 16 * t));
#pragma unroll
            for (int i = 0; i < NT; ++i) aq[slot][i] = read16(ib[i][ch] + 2 * (2 * t * W));
        };
#pragma unroll
        for (int e = 0; e < PD; ++e) rd(e, e);
        f32x16 acc[NT][2], zero;
#pragma unroll
        for (int r = 0; r < 16; ++r) zero[r] = 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int ch = e >> 2, t = e & 3, par = ch & 1;
            const bf16x8 wv = wq[e % PD];
            bf16x8 av[NT];
#pragma unroll
            for (int i = 0; i < NT; ++i) av[i] = aq[e % PD][i];
            if (e + PD < 16) rd(e + PD, e % PD);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NT; ++i) acc[i][par] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, av[i], t == 0 ? zero : acc[i][par], 0, 0, 0);
            if (ch > 0) {                                  // a quarter of the previous channel's segment sum joins the total
#pragma unroll
                for (int i = 0; i < NT; ++i)
#pragma unroll
                    for (int r = 4 * t; r < 4 * t + 4; ++r) {
                        if (FIRST && ch == 1) tot[T0 + i][r] = acc[i][par ^ 1][r];
                        else tot[T0 + i][r] += acc[i][par ^ 1][r];
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) tot[T0 + i][r] += acc[i][1][r];
    };
    // The weights are the FIRST operand of the matrix instruction, so a lane's accumulator registers are 16 output
    // channels (8g + 4 lk + j, g and j < 4) of ONE position.  Lanes l and l + 32 hold the two interleaved halves of a
    // position's 64-byte row; they exchange two of their four 8-byte groups so that each writes 32 contiguous bytes
    // (as four 8-byte stores per lane the row left in 16-byte pieces, and the kernel wrote three times its output).
    auto finish = [&](int b, int m, const f32x16 &tt) {
        uint2 p[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 bias = *reinterpret_cast<const f32x4 *>(lbias + 8 * g + 4 * lk);
            Vec<bf16_t, 4> o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float y = __builtin_fmaf(tt[4 * g + j], 1.0f / 255.0f, bias[j]);
                o[j] = from_f32<bf16_t>(y > 0.0f ? y : 0.0f);
            }
            p[g] = __builtin_bit_cast(uint2, o);
        }
        // lane lk = 0 keeps groups 0, 1 (channels 0-3, 8-11) and receives its partner's (4-7, 12-15);
        // lane lk = 1 keeps groups 2, 3 (channels 20-23, 28-31) and receives its partner's (16-19, 24-27)
        const uint2 s0 = lk ? p[0] : p[2], s1 = lk ? p[1] : p[3];
        uint2 r0, r1;
        r0.x = __shfl_xor(s0.x, 32, 64); r0.y = __shfl_xor(s0.y, 32, 64);
        r1.x = __shfl_xor(s1.x, 32, 64); r1.y = __shfl_xor(s1.y, 32, 64);
        if (m < a.P1) {
            uint4 *dst = reinterpret_cast<uint4 *>(a.out + ((long long)b * a.P1 + m) * 32 + 16 * lk);
            dst[0] = lk ? make_uint4(r0.x, r0.y, p[2].x, p[2].y) : make_uint4(p[0].x, p[0].y, r0.x, r0.y);
            dst[1] = lk ? make_uint4(r1.x, r1.y, p[3].x, p[3].y) : make_uint4(p[1].x, p[1].y, r1.x, r1.y);
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    auto slab = [&](int buf, auto firstc, auto lastc, int b) {
        if (mytiles >= 2) mult(buf, I0{}, I2{}, firstc); else if (mytiles == 1) mult(buf, I0{}, I1{}, firstc);
        if (mytiles >= 4) mult(buf, I2{}, I2{}, firstc); else if (mytiles == 3) mult(buf, I2{}, I1{}, firstc);
        if constexpr (decltype(lastc)::value) {
#pragma unroll
            for (int i = 0; i < C1S_TILES; ++i) if (i < mytiles) finish(b, tm[i], tot[i]);
        }
    };
    __syncthreads();
    for (int s = 0; s < nsamp; ++s) {
        const int b = blockIdx.x + s * gridDim.x;
#pragma unroll
        for (int cg = 0; cg < NG; ++cg) {
            const int buf = (s * NG + cg) & 1;
            if (cg == 0) slab(buf, std::true_type{}, std::integral_constant<bool, NG == 1>{}, b);
            else if (cg == NG - 1) slab(buf, std::false_type{}, std::true_type{}, b);
            else slab(buf, std::false_type{}, std::false_type{}, b);
            __syncthreads();
        }
    }
}

// true if the frame shape and pointers fit conv1_slab_kernel as it is instantiated
static bool conv1_slab_fits(const Geom &g, const uint8_t *obs)
{
    const bool football = g.C == 16 && g.H == 72 && g.W == 96, atari = g.C == 4 && g.H == 84 && g.W == 84;
    return (football || atari) && (g.P1 + 31) / 32 <= 4 * C1S_TILES && !(((uintptr_t)obs) & 15u);
}

static hipError_t launch_conv1_slab(Ctx &c, const uint8_t *obs, const int32_t *index, int B)
{
    const Geom &g = c.g;
    Conv1SlabArgs a;
    a.obs = obs; a.index = index; a.w = (const bf16_t *)c.ws.w1s; a.bias = c.ws.hb + c.sh.b1; a.out = (bf16_t *)c.ws.act1;
    a.B = B; a.W1 = g.W1; a.P1 = g.P1;
    const bool football = g.C == 16;
    void (*kern)(const Conv1SlabArgs) = football ? conv1_slab_kernel<4, 72, 96> : conv1_slab_kernel<1, 84, 84>;
    const size_t lds = football ? conv1_slab_lds<72, 96>() : conv1_slab_lds<84, 84>();
    static std::atomic<bool> attr_set[2] = {};      // raise the dynamic-LDS limit once per instantiation (setting it twice is harmless)
    if (!attr_set[football ? 1 : 0].load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set[football ? 1 : 0].store(true, std::memory_order_release);
    }
    int grid = B < 256 ? B : 256;                    // one workgroup per compute unit (its LDS), walking the batch
    const int least = (B + C1S_MAX_SAMPLES - 1) / C1S_MAX_SAMPLES;
    if (grid < least) grid = least;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C1S_THREADS), lds, c.stream, a);
    return hipGetLastError();
}

template <typename T> static hipError_t forward_t(Ctx &c, const uint8_t *obs, const int32_t *index, int B, bool learn)
{
    const Geom &g = c.g;
    hipError_t e = hipSuccess;
    const bool small = B <= c.small_b;
    const float *hb = c.ws.hb;
    // Small batches whose layer has fewer 32x32 output tiles (workgroups) than a threshold take 16x16 tiles: four
    // times the workgroups, half the operand bytes per workgroup, the same bits.
    // Measured (act call, 16 rows, binary32): 34.7 -> 26.7 us.  The gain ends between 100 and 200 workgroups (conv3
    // at 32 rows, 98 workgroups: 12.6 -> 10.5 us; at 64 rows, 196: 13.2 -> 16.0 us); conv1 gains only with binary32
    // operands (its frame operand is bytes either way), up to about 200 workgroups.
    auto few32 = [&](int workgroups) { return workgroups < c.tile16_below; };
    {
        Conv1Fwd<T> p;
        p.M = B * g.P1; p.N = 32; p.K = g.K1; p.klen = g.K1;
        p.obs = obs; p.index = index; p.w = (const T *)c.ws.w1s; p.bias = hb + c.sh.b1; p.out = (T *)c.ws.act1;
        p.C = g.C; p.H = g.H; p.W = g.W; p.W1 = g.W1; p.P1 = g.P1;
        p.dP1 = FastDiv::make(g.P1); p.dW1 = FastDiv::make(g.W1);
        {
            SiteTimer tm(c, learn ? SITE_CONV1_FWD_LEARN : SITE_CONV1_FWD);
            // one wavefront per 64-long segment (= per input channel): 4 for a 4-channel frame; a 16-channel frame
            // gets 16 (binary32: with the weight operand straight from memory so that their panels still fit in LDS;
            // bfloat16 panels fit, and staging the weights is faster: 9.7 -> 8.3 us at 16 rows of 16x72x96)
            bool done = false;
            if constexpr (sizeof(T) == 4) {
                if (small && few32((p.M + 31) / 64)) {
                    e = g.K1 >= 1024 ? launch_wsgemm16<Conv1Fwd<T>, 16, Conv1Fwd<T>::SEG>(p, c.stream)
                                     : launch_wsgemm16<Conv1Fwd<T>, 4, Conv1Fwd<T>::SEG>(p, c.stream);
                    done = true;
                }
            }
            if (done) {}
            else if (small) e = g.K1 >= 1024 ? launch_wsgemm<Conv1Fwd<T>, 16, Conv1Fwd<T>::SEG, false, (sizeof(T) == 4)>(p, c.stream)
                                        : launch_wsgemm<Conv1Fwd<T>, 4, Conv1Fwd<T>::SEG, false>(p, c.stream);
            // (four-channel frames too: against the LDS-image kernel of that shape, conv1 at 1024 rows of 4x84x84
            // 21.7 -> 19.0 us, an act call at 256 / 4096 rows 38.8 -> 36.7 / 203 -> 188 us)
            else if (sizeof(T) == 2 && B >= c.conv1_slab_rows && conv1_slab_fits(g, obs)) e = launch_conv1_slab(c, obs, index, B);
            else if (sizeof(T) == 2 && conv1_image_fits(g, obs)) e = launch_conv1_image(c, obs, index, B);
            else e = launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    const bool atari_grid = g.H1 == 20 && g.W1 == 20;      // 84x84 frames: conv2 sees 20x20, conv3 9x9
    const bool foot_grid = g.H1 == 17 && g.W1 == 23;       // 72x96 frames: conv2 sees 17x23, conv3 7x10
    {
        ConvFwd<T, Layer2, false> p;
        p.M = B * g.P2; p.N = 64; p.K = 512; p.klen = 512;
        p.in = (const T *)c.ws.act1; p.wf = (const T *)c.ws.wf2; p.bias = hb + c.sh.b2; p.out = (T *)c.ws.act2; p.out2 = nullptr;
        p.Hin = g.H1; p.Win = g.W1; p.Wo = g.W2; p.Po = g.P2;
        p.dPo = FastDiv::make(g.P2); p.dWo = FastDiv::make(g.W2);
        {
            SiteTimer tm(c, learn ? SITE_CONV2_FWD_LEARN : SITE_CONV2_FWD);
            // (the LDS-resident kernel of imgconv.hpp measured slower here than the tile kernel: 20.4 vs 17.8 us at
            // B = 1024 -- this layer streams the large conv1 output once either way)
            if (small && few32(((p.M + 31) / 32) * 2))
                e = launch_wsgemm16<ConvFwd<T, Layer2, false>, 8, ConvFwd<T, Layer2, false>::SEG>(p, c.stream);
            else
            e = small ? launch_wsgemm<ConvFwd<T, Layer2, false>, 8, ConvFwd<T, Layer2, false>::SEG, false>(p, c.stream)
                      : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {
        ConvFwd<T, Layer3, true> p;
        p.M = B * g.P3; p.N = 64; p.K = 576; p.klen = 576;
        p.in = (const T *)c.ws.act2; p.wf = (const T *)c.ws.wf3; p.bias = hb + c.sh.b3; p.out = (T *)c.ws.a3;
        p.out2 = learn ? (T *)c.ws.a3n : nullptr;
        p.Hin = g.H2; p.Win = g.W2; p.Wo = g.W3; p.Po = g.P3;
        p.dPo = FastDiv::make(g.P3); p.dWo = FastDiv::make(g.W3);
        {
            SiteTimer tm(c, learn ? SITE_CONV3_FWD_LEARN : SITE_CONV3_FWD);
            if (small && few32(((p.M + 31) / 32) * 2))     // binary32: 6 segments of 96; bfloat16: 3 of 192 (the fold needs 4 wavefronts)
                e = launch_wsgemm16<ConvFwd<T, Layer3, true>, (sizeof(T) == 4 ? 6 : 4), ConvFwd<T, Layer3, true>::SEG>(p, c.stream);
            else if (small) e = launch_wsgemm<ConvFwd<T, Layer3, true>, (sizeof(T) == 4 ? 8 : 4), ConvFwd<T, Layer3, true>::SEG, false, true>(p, c.stream);
            else if (sizeof(T) == 2 && atari_grid) {       // large bf16 batch, 9x9 input: activations resident in LDS
                ImgConvArgs a = {};
                a.in = (const bf16_t *)c.ws.act2; a.w = (const bf16_t *)c.ws.wf3; a.bias = hb + c.sh.b3;
                a.out = (bf16_t *)c.ws.a3; a.out2 = learn ? (bf16_t *)c.ws.a3n : nullptr; a.B = B;
                e = launch_imgconv<ImgFwd<64, 3, 1, 9, 9, 4, ConvFwd<bf16_t, Layer3, true>::SEG, true>>(a, c.stream);
            } else if (sizeof(T) == 2 && foot_grid) {       // the same on the 7x10 input of 72x96 frames (20.0 -> 17.8 us at 2048 rows)
                ImgConvArgs a = {};
                a.in = (const bf16_t *)c.ws.act2; a.w = (const bf16_t *)c.ws.wf3; a.bias = hb + c.sh.b3;
                a.out = (bf16_t *)c.ws.a3; a.out2 = learn ? (bf16_t *)c.ws.a3n : nullptr; a.B = B;
                e = launch_imgconv<ImgFwd<64, 3, 1, 7, 10, 4, ConvFwd<bf16_t, Layer3, true>::SEG, true>>(a, c.stream);
            } else e = launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {   // groups of FC_GROUP_K inputs; the heads kernel adds them (same grouping and order on both paths)
        FcFwd<T> p;
        // With enough rows to fill the machine the tile kernel adds the groups itself (same order, same bits) and the
        // partial sums -- G x the FC output, written here and read back by the heads kernel -- shrink to one slice.
        // Measured: slower than G x the workgroups at 2048 rows (54 vs 52 us for FC + heads), faster at 4096 (69 vs 77).
        const bool fold = !small && B >= c.fc_fold_rows;
        p.M = B; p.N = 512; p.K = g.F; p.klen = fold ? g.F : FC_GROUP_K;
        c.fc_slices = fold ? 1 : c.fc_groups;
        p.a3 = (const T *)c.ws.a3; p.w = (const T *)c.ws.wfc; p.part = c.ws.fc_part;
        static_assert(FC_GROUP_K % FcFwd<T>::SEG == 0 && FcFwd<T>::GROUP == FC_GROUP_K, "a group is a whole number of segments");
        {
            SiteTimer tm(c, learn ? SITE_FC_FWD_LEARN : SITE_FC_FWD);
            // (also when 16-row tiles leave fewer padded rows: 80 rows are five tiles of 16 but three of 32; 13.8 -> 10.9 us)
            const bool less_padding = c.tile16_below > 0 && ((B + 15) / 16) * 16 < ((B + 31) / 32) * 32;
            if (small && (few32(((B + 31) / 32) * 16 * c.fc_groups) || less_padding))
                e = launch_wsgemm16<FcFwd<T>, 8, FcFwd<T>::SEG>(p, c.stream, FC_GROUP_K / FcFwd<T>::SEG);
            else
            e = small ? launch_wsgemm<FcFwd<T>, 8, FcFwd<T>::SEG, false>(p, c.stream, FC_GROUP_K / FcFwd<T>::SEG)
                      : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t run_forward(Ctx &c, const uint8_t *obs, const int32_t *index, int B, bool learn)
{
    return c.desc.precision == HTS_PRECISION_BF16 ? forward_t<bf16_t>(c, obs, index, B, learn)
                                                  : forward_t<float>(c, obs, index, B, learn);
}

template <typename T> static hipError_t plain_t(Ctx &c, const float *A, const float *Bm, float *C, int M, int N, int K)
{
    PlainGemm<T> p;
    p.M = M; p.N = N; p.K = K; p.klen = K; p.A = A; p.B = Bm; p.C = C;
    return launch_gemm(p, c.stream);
}

hipError_t run_plain_gemm(Ctx &c, int precision, const float *A, const float *B, float *C, int M, int N, int K)
{
    return precision == HTS_PRECISION_BF16 ? plain_t<bf16_t>(c, A, B, C, M, N, K) : plain_t<float>(c, A, B, C, M, N, K);
}

}  // namespace hts
